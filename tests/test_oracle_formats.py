"""Pins for the oracle's number formats and random bits (CPU only).

Each test ties one oracle function to something fixed outside it: the format
definitions of Sec. 3 / Table 1, an independent library cast, closed forms, or
the generator's published known-answer vectors.
"""
import os

import numpy as np
import pytest
import torch

import oracle


def _read_golden(golden_dir, name):
    with open(os.path.join(golden_dir, name)) as fh:
        return [ln.strip() for ln in fh if ln.strip() and not ln.startswith("#")]


def test_e2m1_grid(golden_dir):
    grid = [float(v) for v in _read_golden(golden_dir, "e2m1_grid.txt")[0].split()]
    assert len(grid) == 8
    for c in range(8):
        assert oracle.e2m1_decode(c) == grid[c]
        assert oracle.e2m1_decode(c | 8) == -grid[c]
    assert np.signbit(np.float32(oracle.e2m1_decode(8)))  # -0 keeps its sign


def test_e2m1_is_a_1_2_1_float():
    # Independent reading of "1 sign, 2 exponent, 1 mantissa": exactly the non-negative
    # numbers with <= 2 significant bits between the subnormal step 0.5 and 6.
    vals = sorted(oracle.e2m1_decode(c) for c in range(8))
    assert vals[1] - vals[0] == 0.5 and vals[-1] == 6.0
    for v in vals[1:]:
        m, _ = np.frexp(v)
        assert (m * 4) == int(m * 4)


def test_e4m3_decode_matches_library():
    b = torch.arange(0, 127, dtype=torch.uint8)
    ref = b.view(torch.float8_e4m3fn).float().numpy()
    ours = np.array([oracle.e4m3_decode(int(v)) for v in b])
    assert np.array_equal(ref, ours)
    assert oracle.e4m3_decode(0x7E) == 448.0 and oracle.e4m3_decode(0x38) == 1.0
    assert oracle.e4m3_decode(1) == 2.0 ** -9


def test_e4m3_encode_matches_library_cast():
    # every 509th binary32 pattern in [0, 448], plus every representable value, every midpoint
    # between neighbours and their binary32 neighbours
    hi = np.float32(448.0).view(np.uint32)
    pats = np.arange(0, int(hi) + 1, 509, dtype=np.uint32).view(np.float32)
    grid = np.array([oracle.e4m3_decode(b) for b in range(127)], dtype=np.float32)
    mids = ((grid[:-1].astype(np.float64) + grid[1:].astype(np.float64)) / 2).astype(np.float32)
    special = np.concatenate([grid, mids])
    special = np.concatenate([special, np.nextafter(special, np.float32(np.inf)),
                              np.nextafter(special, np.float32(-1))])
    special = special[(special >= 0) & (special <= 448)]
    x = np.concatenate([pats, special]).astype(np.float32)
    ref = torch.from_numpy(x).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    ours = oracle.e4m3_encode(x)
    assert np.array_equal(ref, ours)


def test_e4m3_encode_saturates_and_has_no_sign():
    for v in (449.0, 464.0, 465.0, 1e4, 3e38):
        assert oracle.e4m3_encode(v) == 0x7E
    x = np.abs(np.random.default_rng(0).standard_normal(10000).astype(np.float32)) * 100
    assert (oracle.e4m3_encode(x) & 0x80).max() == 0


def test_e8m0_closed_form():
    for b in (0, 1, 120, 127, 128, 200, 254):
        assert oracle.e8m0_decode(b) == float(np.ldexp(np.float32(1), b - 127))


def test_philox_known_answers(golden_dir):
    for ln in _read_golden(golden_dir, "philox4x32_10_kat.txt"):
        w = [int(t, 16) for t in ln.split()]
        out = oracle.philox4x32_10(w[0:4], w[4:6])
        assert [int(v) for v in out] == w[6:10]


def test_sr_bits_indexing():
    # word (e>>1)&3 of the draw for counter e>>3, low half first; high counter word used
    seed = 0x0123456789ABCDEF
    key = [seed & 0xFFFFFFFF, seed >> 32]
    for e in (0, 1, 2, 7, 8, 9, 1234567, (1 << 35) + 5, (1 << 40) + 14):
        c = e >> 3
        draw = oracle.philox4x32_10([c & 0xFFFFFFFF, c >> 32, 0, 0], key)
        w = int(draw[(e >> 1) & 3])
        assert oracle.sr_bits(seed, e) == ((w >> 16) if e & 1 else (w & 0xFFFF))
    a = oracle.sr_bits_range(seed, 40, 64)
    assert [int(v) for v in a] == [oracle.sr_bits(seed, 40 + t) for t in range(64)]


def test_sr_bits_are_uniform():
    u = oracle.sr_bits_range(7, 0, 1 << 20).astype(np.float64)
    assert u.max() < 65536
    assert abs(u.mean() - 32767.5) < 4 * 65536 / np.sqrt(12 * u.size)
    hist = np.bincount((u // 4096).astype(np.int64), minlength=16)
    assert np.all(np.abs(hist - u.size / 16) < 5 * np.sqrt(u.size / 16))
    # different seeds and neighbouring elements decorrelate
    v = oracle.sr_bits_range(8, 0, 1 << 20).astype(np.float64)
    assert abs(np.corrcoef(u, v)[0, 1]) < 0.01
    assert abs(np.corrcoef(u[:-1], u[1:])[0, 1]) < 0.01
