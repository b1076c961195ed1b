"""Pins for the oracle's quantization operation Q (Eqs. 1-6; formats of Sec. 3), CPU only."""
import os

import numpy as np
import pytest
import torch

import oracle
from oracle import MXFP4, NVFP4, RTN, SR, Format

GRID = np.array([0, 0.5, 1, 1.5, 2, 3, 4, 6], dtype=np.float64)


def unpack(codes):
    """[outer, K/2] bytes -> [outer, K] 4-bit codes (even position = low nibble)."""
    out = np.empty((codes.shape[0], codes.shape[1] * 2), np.uint8)
    out[:, 0::2] = codes & 15
    out[:, 1::2] = codes >> 4
    return out


def _read_golden(golden_dir):
    d = {}
    with open(os.path.join(golden_dir, "worked_blocks.txt")) as fh:
        for ln in fh:
            if ln.strip() and not ln.startswith("#"):
                k, v = ln.split(":")
                d[k.strip()] = v.split()
    return d


# ------------------------------------------------------------ scalar rounding
def test_rtn_is_nearest_value_brute_force():
    hi = int(np.float32(6.5).view(np.uint32))
    m = np.arange(0, hi, 127, dtype=np.uint32).view(np.float32)
    ties = np.array([0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0], dtype=np.float32)
    m = np.concatenate([m, GRID.astype(np.float32), ties, np.nextafter(ties, np.float32(9)),
                        np.nextafter(ties, np.float32(0))])
    m = np.minimum(m, np.float32(6))
    got = oracle.round_rtn(m)
    dist = np.abs(m.astype(np.float64)[:, None] - GRID[None, :])
    best = dist.min(axis=1)
    # the chosen value is a nearest one
    assert np.array_equal(dist[np.arange(m.size), got], best)
    # where two values are equally near, the even code is taken
    tie = (dist == best[:, None]).sum(axis=1) > 1
    assert tie.sum() >= 7 and np.all(got[tie] % 2 == 0)


def test_rtn_ties_listed():
    # midpoints of the grid: 0.25->0, 0.75->1, 1.25->1, 1.75->2, 2.5->2, 3.5->4, 5->4
    for m, val in ((0.25, 0), (0.75, 1.0), (1.25, 1.0), (1.75, 2.0), (2.5, 2.0), (3.5, 4.0), (5.0, 4.0)):
        assert GRID[oracle.round_rtn(m)] == val


def test_sr_support_and_exact_probability():
    # m = 2.4 lies 0.4 of the way from 2 to 3: exactly 26214 of the 65536 draws round up
    u = np.arange(65536, dtype=np.uint32)
    got = oracle.round_sr(np.full(65536, 2.4, np.float32), u)
    assert set(np.unique(got)) == {4, 5}
    assert int((got == 5).sum()) == 26214
    # monotone in u: small draws go up
    assert np.all(got[:26214] == 5) and np.all(got[26214:] == 4)
    # on-grid values and the saturated value never move
    for c in range(8):
        assert np.all(oracle.round_sr(np.full(65536, GRID[c], np.float32), u) == c)


def test_sr_tie_between_draw_and_position_rounds_up():
    # reading (the paper fixes neither the number of random bits nor this tie): a value whose
    # position between its neighbours falls exactly on a centred draw, 65536 t = u + 1/2, goes up
    # for that draw.  m = lo + step * 100.5 / 65536: draws 0..100 go up, 101.. stay.
    u = np.arange(65536, dtype=np.uint32)
    for lo, step in ((0.0, 0.5), (0.5, 0.5), (1.5, 0.5), (2.0, 1.0), (3.0, 1.0), (4.0, 2.0)):
        m = np.float32(lo + step * 100.5 / 65536)
        assert float(m) == lo + step * 100.5 / 65536  # exactly representable
        got = oracle.round_sr(np.full(65536, m, np.float32), u)
        base = int(np.searchsorted(GRID, lo))
        assert np.all(got[:101] == base + 1) and np.all(got[101:] == base)


def test_sr_probability_matches_distance_everywhere():
    rng = np.random.default_rng(3)
    u = np.arange(65536, dtype=np.uint32)
    for m in rng.uniform(0, 6, 40).astype(np.float32):
        got = oracle.round_sr(np.full(65536, m, np.float32), u)
        lo = np.searchsorted(GRID, m, side="right") - 1
        t = (float(m) - GRID[lo]) / (GRID[lo + 1] - GRID[lo])
        assert set(np.unique(got)) <= {lo, lo + 1}
        assert abs((got == lo + 1).mean() - t) <= 2.0 ** -16
        # expected value equals m to the draw's resolution: E[eps] = 0 (Sec. 4)
        assert abs(GRID[got].mean() - float(m)) <= (GRID[lo + 1] - GRID[lo]) * 2.0 ** -16


# ------------------------------------------------------------- worked blocks
@pytest.mark.parametrize("name", ["A", "B"])
def test_worked_block(golden_dir, name):
    g = _read_golden(golden_dir)
    x = np.array([float(v) for v in g[f"{name}_in"]], dtype=np.float32)[None, :]
    codes, scales, gs = oracle.quantize(x, 1, RTN, 0, NVFP4, g=1.0)
    assert gs == 1.0
    assert scales[0, 0] == int(g[f"{name}_scale"][0], 16)
    assert [int(c) for c in unpack(codes)[0]] == [int(c, 16) for c in g[f"{name}_codes"]]
    assert [int(b) for b in codes[0]] == [int(b, 16) for b in g[f"{name}_bytes"]]
    # the same block down a column gives the same bytes (transposed output)
    codes_t, scales_t, _ = oracle.quantize(np.ascontiguousarray(x.T), 0, RTN, 0, NVFP4, g=1.0)
    assert np.array_equal(codes_t, codes) and np.array_equal(scales_t, scales)


def test_block_B_decodes_to_saturated_value():
    x = np.zeros((1, 16), np.float32)
    x[0, 0] = 5.0
    c, s, g = oracle.quantize(x, 1, RTN, 0, NVFP4, g=1.0)
    assert oracle.dequantize(c, s, g)[0, 0] == 4.875


# -------------------------------------------------------------- tensor scale
def test_tensor_scale_closed_form():
    assert oracle.tensor_scale_from_amax(2688.0) == 1.0
    assert oracle.tensor_scale_from_amax(0.0) == 1.0
    assert oracle.tensor_scale_from_amax(1e-40) == 2.0 ** -117
    x = np.random.default_rng(0).standard_normal((32, 64)).astype(np.float32)
    x[5, 17] = -2688.0
    codes, scales, g = oracle.quantize(x, 1, RTN, 0, NVFP4)
    assert g == 1.0
    assert scales[5, 1] == 0x7E  # the block holding the tensor maximum gets 448
    assert unpack(codes)[5, 17] == 0xF
    assert scales.max() == 0x7E and (scales & 0x80).max() == 0


def test_all_zero_tensor_and_zero_blocks_keep_sign():
    x = np.zeros((16, 32), np.float32)
    x[3, 5] = -0.0
    codes, scales, g = oracle.quantize(x, 1, RTN, 0, NVFP4)
    assert g == 1.0 and scales.max() == 0
    u = unpack(codes)
    assert u[3, 5] == 8 and u.sum() == 8
    # a block that underflows the scale format: zero magnitudes, signs kept
    x = np.zeros((1, 32), np.float32)
    x[0, 0] = 2688.0
    x[0, 16:] = -1e-4  # r = 1e-4/6 < 2^-10 rounds to scale 0
    codes, scales, g = oracle.quantize(x, 1, SR, 5, NVFP4)
    assert scales[0, 1] == 0 and np.all(unpack(codes)[0, 16:] == 8)


# ----------------------------------------------------------------- invariants
def _representable(rng, rows, nblk, gexp=-3, bf16=False):
    """x = +-grid[c] * s * g with one code-7 element per block, one block at 448: Q(x) must
    return exactly (c, s, g) for RtN and for SR with any seed."""
    c = rng.integers(0, 16, (rows, nblk * 16)).astype(np.uint8)
    sb = rng.integers(0x08 if not bf16 else 0x20, 0x7F, (rows, nblk)).astype(np.uint8)
    if bf16:  # keep c*s within 8 significant bits: scale mantissa limited to multiples of 1/4
        sb &= 0xFE
    pos = rng.integers(0, 16, (rows, nblk))
    for r in range(rows):
        for b in range(nblk):
            c[r, b * 16 + pos[r, b]] = 7 | (c[r, b * 16 + pos[r, b]] & 8)
    sb[0, 0] = 0x7E
    g = 2.0 ** gexp
    s = np.array([oracle.e4m3_decode(int(v)) for v in range(127)])[sb]
    sign = np.where(c & 8, -1.0, 1.0)
    x = sign * GRID[c & 7] * np.repeat(s, 16, axis=1) * g
    assert np.array_equal(x.astype(np.float32).astype(np.float64), x)
    return x.astype(np.float32), c, sb, g


@pytest.mark.parametrize("rounding,seed", [(RTN, 0), (SR, 0), (SR, 12345)])
def test_idempotent_on_representable_tensors(rounding, seed):
    rng = np.random.default_rng(11)
    x, c, sb, g = _representable(rng, 24, 6)
    codes, scales, g2 = oracle.quantize(x, 1, rounding, seed, NVFP4)
    assert g2 == g
    assert np.array_equal(scales, sb)
    assert np.array_equal(unpack(codes), c)
    # and through the transposed path
    codes_t, scales_t, g3 = oracle.quantize(np.ascontiguousarray(x.T), 0, rounding, seed, NVFP4)
    assert g3 == g and np.array_equal(scales_t, sb) and np.array_equal(unpack(codes_t), c)
    # dequantize returns the tensor itself
    assert np.array_equal(oracle.dequantize(codes, scales, g2), x.astype(np.float64))


def test_idempotent_bf16():
    rng = np.random.default_rng(12)
    x, c, sb, g = _representable(rng, 8, 4, bf16=True)
    xb = torch.from_numpy(x).to(torch.bfloat16)
    assert torch.equal(xb.float(), torch.from_numpy(x))
    codes, scales, g2 = oracle.quantize(xb, 1, SR, 9, NVFP4)
    assert g2 == g and np.array_equal(scales, sb) and np.array_equal(unpack(codes), c)


@pytest.mark.parametrize("rounding", [RTN, SR])
@pytest.mark.parametrize("axis", [0, 1])
def test_power_of_two_covariance_and_sign_symmetry(rounding, axis):
    rng = np.random.default_rng(5)
    x = (rng.standard_t(3, (64, 96)) * 0.02).astype(np.float32)
    c0, s0, g0 = oracle.quantize(x, axis, rounding, 3, NVFP4)
    for n in (-7, 5):
        c1, s1, g1 = oracle.quantize(x * np.float32(2.0 ** n), axis, rounding, 3, NVFP4)
        assert np.array_equal(c0, c1) and np.array_equal(s0, s1) and g1 == g0 * 2.0 ** n
    c2, s2, g2 = oracle.quantize(-x, axis, rounding, 3, NVFP4)
    assert np.array_equal(c2, c0 ^ 0x88) and np.array_equal(s2, s0) and g2 == g0


def test_axis0_equals_axis1_of_transpose_for_rtn():
    x = np.random.default_rng(6).standard_normal((48, 80)).astype(np.float32)
    a = oracle.quantize(x, 0, RTN, 0, NVFP4)
    b = oracle.quantize(np.ascontiguousarray(x.T), 1, RTN, 0, NVFP4)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1]) and a[2] == b[2]
    assert a[0].shape == (80, 24) and a[1].shape == (80, 3)


def test_sr_draw_follows_the_element_not_the_axis():
    # the random bits of element (i, j) depend on i*cols + j only: quantizing along either
    # axis with a scale that makes both paths see the same y gives the same rounding decision
    rng = np.random.default_rng(8)
    x = rng.uniform(-6, 6, (32, 32)).astype(np.float32)
    x[:, ::16] = 6.0
    x[::16, :] = 6.0  # every row block and every column block has amax 6 -> scale 1 with g = 1
    a = unpack(oracle.quantize(x, 1, SR, 77, NVFP4, g=1.0)[0])
    b = unpack(oracle.quantize(x, 0, SR, 77, NVFP4, g=1.0)[0]).T
    assert np.array_equal(a, b)
    c = unpack(oracle.quantize(x, 1, SR, 78, NVFP4, g=1.0)[0])
    assert (a != c).mean() > 0.2  # another seed, another draw


def test_sr_codes_match_scalar_rule_and_are_unbiased():
    rng = np.random.default_rng(9)
    x = rng.uniform(-6, 6, (16, 64)).astype(np.float32)
    x[:, ::16] = 6.0
    acc = np.zeros(x.shape)
    S = 256
    for seed in range(S):
        codes, scales, g = oracle.quantize(x, 1, SR, seed, NVFP4, g=1.0)
        assert np.all(scales == 0x38)
        u = unpack(codes)
        if seed == 0:  # element-wise: code = scalar SR of |x| with the element's own bits
            bits = oracle.sr_bits_range(0, 0, x.size).reshape(x.shape)
            want = oracle.round_sr(np.abs(x), bits) | np.where(np.signbit(x), 8, 0).astype(np.uint8)
            assert np.array_equal(u, want)
        acc += np.where(u & 8, -1.0, 1.0) * GRID[u & 7]
    mean = acc / S
    lo = GRID[np.searchsorted(GRID, np.abs(x), side="right") - 1]
    hi = GRID[np.minimum(np.searchsorted(GRID, np.abs(x), side="right"), 7)]
    step = np.maximum(hi - lo, 1e-9)
    t = (np.abs(x) - lo) / step
    bound = 4.5 * step * np.sqrt(t * (1 - t) / S) + step * 2.0 ** -16 + 1e-12
    assert np.all(np.abs(mean - x) <= bound)
    # RtN on the same data is biased element-wise, SR is not: compare mean absolute error
    rt = unpack(oracle.quantize(x, 1, RTN, 0, NVFP4, g=1.0)[0])
    rt_val = np.where(rt & 8, -1.0, 1.0) * GRID[rt & 7]
    assert np.abs(mean - x).mean() < 0.2 * np.abs(rt_val - x).mean()


def test_rtn_error_bound_and_scale_rule():
    rng = np.random.default_rng(10)
    x = (rng.standard_t(3, (64, 128)) * 0.02).astype(np.float32)
    codes, scales, g = oracle.quantize(x, 1, RTN, 0, NVFP4)
    T = np.abs(x).max()
    assert g == float(np.float32(T) / np.float32(2688))
    s = np.array([oracle.e4m3_decode(int(v)) for v in range(127)])[scales]
    amax = np.abs(x.reshape(64, 8, 16)).max(axis=2).astype(np.float64)
    # the stored scale is the E4M3 value nearest to amax/(6g): within half an E4M3 step
    r = amax / (6.0 * g)
    assert np.all(np.abs(s - r) <= np.maximum(r * 2.0 ** -4, 2.0 ** -10) * (1 + 1e-6))
    v = oracle.dequantize(codes, scales, g)
    d = np.repeat(s * g, 16, axis=1)
    y = np.abs(x) / d
    unsat = y <= 6
    halfstep = np.where(y < 2, 0.25, np.where(y < 4, 0.5, 1.0))
    assert np.all(np.abs(v - x)[unsat] <= (halfstep * d)[unsat] * (1 + 1e-6))
    assert np.all(np.abs(v)[~unsat] == (6 * d)[~unsat])


def test_bf16_input_equals_its_fp32_widening():
    x = torch.from_numpy((np.random.default_rng(2).standard_t(3, (32, 64)) * 0.02).astype(np.float32))
    xb = x.to(torch.bfloat16)
    for axis in (0, 1):
        a = oracle.quantize(xb, axis, SR, 4, NVFP4)
        b = oracle.quantize(xb.float(), axis, SR, 4, NVFP4)
        assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1]) and a[2] == b[2]


# ------------------------------------------------------- MXFP4 and block sizes
def test_mxfp4_shared_exponent():
    x = np.zeros((4, 32), np.float32)
    x[0, 3] = 6.0      # floor(log2 6) = 2 -> e = 0 -> byte 127, values unchanged
    x[0, 4] = 1.25
    x[1, 0] = 7.9      # same exponent, 7.9 saturates at 6
    x[2, 7] = -1.0     # e = -2 -> byte 125 -> y = -4 -> code 0xE
    x[2, 8] = 0.3      # y = 1.2 -> 1.0
    codes, scales, g = oracle.quantize(x, 1, RTN, 0, MXFP4)
    assert g == 1.0
    assert [int(v) for v in scales[:, 0]] == [127, 127, 125, 0]
    u = unpack(codes)
    assert u[0, 3] == 7 and u[0, 4] == 2 and u[1, 0] == 7 and u[2, 7] == 0xE and u[2, 8] == 2
    assert u[3].sum() == 0
    v = oracle.dequantize(codes, scales, g, MXFP4)
    assert v[2, 7] == -1.0 and v[2, 8] == 0.25 and v[1, 0] == 6.0


def test_mxfp4_scale_is_power_of_two_and_covariant():
    rng = np.random.default_rng(4)
    x = (rng.standard_normal((32, 128)) * 3).astype(np.float32)
    c0, s0, _ = oracle.quantize(x, 1, SR, 1, MXFP4)
    amax = np.abs(x.reshape(32, 4, 32)).max(axis=2)
    assert np.array_equal(s0.astype(np.int64) - 127, np.floor(np.log2(amax)).astype(np.int64) - 2)
    c1, s1, _ = oracle.quantize(x * np.float32(16), 1, SR, 1, MXFP4)
    assert np.array_equal(c0, c1) and np.array_equal(s1.astype(int), s0.astype(int) + 4)
    assert oracle.quantize(x, 0, RTN, 0, MXFP4)[1].shape == (128, 1)


@pytest.mark.parametrize("block", [32, 64, 128])
def test_wider_e4m3_blocks(block):
    fmt = Format(block, oracle.SCALE_E4M3, 1)
    rng = np.random.default_rng(block)
    x = rng.standard_normal((16, 256)).astype(np.float32)
    codes, scales, g = oracle.quantize(x, 1, RTN, 0, fmt)
    assert scales.shape == (16, 256 // block)
    # a wider block is the NVFP4 computation with the maximum taken over more elements:
    # replicate each block's maximum into every 16-sub-block and NVFP4 must agree on the codes
    c16, s16, g16 = oracle.quantize(x, 1, RTN, 0, NVFP4)
    assert g16 == g
    amax_b = np.abs(x.reshape(16, -1, block)).max(axis=2)
    amax_16 = np.abs(x.reshape(16, -1, 16)).max(axis=2)
    same = np.repeat(amax_b, block // 16, axis=1) == amax_16
    assert np.array_equal(np.repeat(scales, block // 16, axis=1)[same], s16[same])
    same_el = np.repeat(same, 16, axis=1)
    assert np.array_equal(unpack(codes)[same_el], unpack(c16)[same_el])
    # mean squared error grows with the block size (Fig. 2's premise: finer blocks fit better)
    mse = np.mean((oracle.dequantize(codes, scales, g, fmt) - x) ** 2)
    mse16 = np.mean((oracle.dequantize(c16, s16, g16) - x) ** 2)
    assert mse >= mse16


def test_shape_errors():
    with pytest.raises(ValueError):
        oracle.quantize(np.zeros((4, 24), np.float32), 1)
    with pytest.raises(ValueError):
        oracle.quantize(np.zeros((24, 4), np.float32), 0)
