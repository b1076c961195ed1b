"""Pins for the oracle's quantization-noise statistics (the gradient-to-noise monitor of Sec. 4), CPU only.

The function under test is oracle.quant_noise -> (sum x^2, sum (Q(x) - x)^2).  Nothing here calls it to
produce its own expectation: values come from the E2M1 grid written out, the scale bytes decoded by hand,
closed forms and the unbiasedness / variance law of stochastic rounding.
"""
import numpy as np
import pytest
import torch

import oracle
from oracle import MXFP4, NVFP4, RTN, SR, Format

GRID = np.array([0, 0.5, 1, 1.5, 2, 3, 4, 6], dtype=np.float64)


def e4m3_value(b):
    """E4M3 byte (sign unused) -> value: bias 7, 3 mantissa bits, subnormals at exponent field 0."""
    e, m = int(b) >> 3 & 15, int(b) & 7
    return (m / 8.0) * 2.0 ** -6 if e == 0 else (1 + m / 8.0) * 2.0 ** (e - 7)


def by_hand(x, q, axis, fmt):
    """The definition written out with python loops over a tiny tensor."""
    codes, scales, g = q
    x = np.asarray(x, dtype=np.float64)
    rows, cols = x.shape
    sx = se = 0.0
    for i in range(rows):
        for j in range(cols):
            o, n = (i, j) if axis == 1 else (j, i)
            byte = int(codes[o, n // 2])
            code = (byte >> 4) if n & 1 else (byte & 15)
            sb = int(scales[o, n // fmt.block])
            s = e4m3_value(sb) if fmt.scale_fmt == oracle.SCALE_E4M3 else 2.0 ** (sb - 127)
            v = (-1.0 if code & 8 else 1.0) * GRID[code & 7] * s * (g if fmt.tensor_scale else 1.0)
            sx += x[i, j] ** 2
            se += (v - x[i, j]) ** 2
    return sx, se


@pytest.mark.parametrize("axis", [0, 1])
@pytest.mark.parametrize("fmt", [NVFP4, MXFP4, Format(64, oracle.SCALE_E4M3, 1)], ids=["nvfp4", "mxfp4", "b64"])
@pytest.mark.parametrize("rounding", [RTN, SR])
def test_matches_the_definition_written_out(axis, fmt, rounding):
    rng = np.random.default_rng(3 + axis)
    x = (rng.standard_normal((64, 128)) * np.exp(rng.standard_normal((64, 128)))).astype(np.float32)
    q = oracle.quantize(x, axis, rounding, 11, fmt)
    sx, se = oracle.quant_noise(x, q, axis, fmt)
    hx, he = by_hand(x, q, axis, fmt)
    assert sx == pytest.approx(hx, rel=1e-13) and se == pytest.approx(he, rel=1e-12)
    assert se > 0 and sx > se


def test_representable_tensor_has_zero_noise_and_known_energy():
    # every block holds the whole grid with both signs and has maximum 6, scales are exact powers of two
    # (tensor maximum 6 * 2^k * 448 is not needed: g is preset so that block scale bytes decode to 2^k)
    rng = np.random.default_rng(5)
    rows, cols = 48, 64
    mags = np.tile(np.concatenate([GRID, GRID]), (rows, cols // 16))
    sign = np.where(rng.random((rows, cols)) < 0.5, -1.0, 1.0)
    k = rng.integers(-3, 4, size=(rows, cols // 16)).repeat(16, axis=1)
    x = (sign * mags * 2.0 ** k).astype(np.float32)
    for rounding in (RTN, SR):
        q = oracle.quantize(x, 1, rounding, 2, NVFP4, g=1.0)
        sx, se = oracle.quant_noise(x, q, 1, NVFP4)
        assert se == 0.0
        assert sx == float((mags ** 2 * 4.0 ** k).sum())  # exact: dyadic rationals, small sum


def test_bf16_input_and_leading_dimension_free_definition():
    x = torch.randn(32, 96, dtype=torch.float32, generator=torch.Generator().manual_seed(1)).to(torch.bfloat16)
    q = oracle.quantize(x, 1, RTN, 0, NVFP4)
    sx, se = oracle.quant_noise(x, q, 1, NVFP4)
    hx, he = by_hand(x.to(torch.float64).numpy(), q, 1, NVFP4)
    assert sx == pytest.approx(hx, rel=1e-13) and se == pytest.approx(he, rel=1e-12)


def test_rtn_noise_obeys_the_half_step_bound():
    # |Q(x) - x| <= half the local grid step times the block's decoded scale (the scale byte is
    # chosen so that block max / scale <= 6 up to the scale's own rounding, which saturating
    # elements can exceed: those are excluded by bounding with the 6-saturation distance too)
    rng = np.random.default_rng(8)
    x = rng.standard_normal((32, 256)).astype(np.float32)
    codes, scales, g = q = oracle.quantize(x, 1, RTN, 0, NVFP4)
    d = oracle.dequantize(*q)
    s = np.array([e4m3_value(b) for b in scales.ravel()]).reshape(scales.shape).repeat(16, axis=1) * g
    y = np.abs(x.astype(np.float64)) / s
    step = np.where(y < 2, 0.5, np.where(y < 4, 1.0, 2.0))
    bound = np.where(y <= 6, step / 2, y - 6) * s
    assert np.all(np.abs(d - x) <= bound * (1 + 1e-12))
    sx, se = oracle.quant_noise(x, q, 1, NVFP4)
    assert se <= float((bound ** 2).sum()) * (1 + 1e-12)
    assert se == pytest.approx(float(((d - x) ** 2).sum()), rel=1e-12)


def test_sr_noise_energy_follows_the_two_point_variance_law():
    # For stochastic rounding between neighbours lo <= y <= hi, E[(Q - y)^2] = (y - lo)(hi - y):
    # averaged over seeds, the measured noise energy must approach that sum (g preset, so the block
    # scales do not depend on the seed).
    rng = np.random.default_rng(13)
    x = rng.standard_normal((16, 64)).astype(np.float32)
    codes, scales, g = oracle.quantize(x, 1, RTN, 0, NVFP4)
    s = np.array([e4m3_value(b) for b in scales.ravel()]).reshape(scales.shape).repeat(16, axis=1) * g
    y = np.minimum(np.abs(x.astype(np.float64)) / s, 6.0)
    lo = GRID[np.searchsorted(GRID, y, side="right") - 1]
    hi = GRID[np.minimum(np.searchsorted(GRID, y, side="left"), 7)]
    clip = np.maximum(np.abs(x.astype(np.float64)) / s - 6.0, 0.0)  # saturated elements: deterministic error
    expect = float((((y - lo) * (hi - y) + clip ** 2) * s ** 2).sum())
    got = np.mean([oracle.quant_noise(x, oracle.quantize(x, 1, SR, seed, NVFP4, g=g), 1, NVFP4)[1]
                   for seed in range(400)])
    assert got == pytest.approx(expect, rel=0.03)
    # and SR is noisier than RtN on the same tensor (RtN minimises the error element by element)
    assert got > oracle.quant_noise(x, (codes, scales, g), 1, NVFP4)[1]


def test_ratio_is_invariant_under_power_of_two_rescaling():
    rng = np.random.default_rng(21)
    x = rng.standard_normal((32, 64)).astype(np.float32)
    a = oracle.quant_noise(x, oracle.quantize(x, 0, SR, 4, NVFP4), 0, NVFP4)
    x8 = (x * np.float32(2.0 ** -9)).astype(np.float32)
    b = oracle.quant_noise(x8, oracle.quantize(x8, 0, SR, 4, NVFP4), 0, NVFP4)
    assert b[0] == a[0] * 4.0 ** -9 and b[1] == a[1] * 4.0 ** -9
