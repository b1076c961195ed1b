"""Parity of nvfp4_quant_noise (quantization-noise statistics of the Sec. 4 monitor) with the oracle, on the GPU."""
import numpy as np
import pytest
import torch

import oracle
from paper_2505_19115_amd import binding as nv
from paper_2505_19115_amd import synth

pytestmark = pytest.mark.gpu

# fp32 partial sums over 8 squares, fp64 above: a few 1e-7 relative in practice; the bar is the GEMM's
REL = 1e-5


def ofmt(fmt):
    return oracle.Format(fmt.block, fmt.scale, fmt.tensor_scale)


def run(x, axis, rounding, seed, fmt, what, ld=None):
    print(f"[case] quant_noise {what} shape={tuple(x.shape)} {x.dtype} axis={axis} rounding={rounding} fmt={fmt} ld={ld}", flush=True)
    if ld is None:
        xg = x.cuda()
    else:  # rows padded to ld elements on the device
        xg = torch.zeros((x.shape[0], ld), dtype=x.dtype, device="cuda")[:, : x.shape[1]]
        xg.copy_(x)
    q = nv.quantize(xg, axis, rounding, seed, fmt)
    got = nv.quant_noise(xg, q, axis, fmt).cpu().numpy()
    oq = oracle.quantize(x, axis, rounding, seed, ofmt(fmt))
    assert np.array_equal(q[0].cpu().numpy(), oq[0]) and np.array_equal(q[1].cpu().numpy(), oq[1])
    ref = oracle.quant_noise(x, oq, axis, ofmt(fmt))
    assert got[0] == pytest.approx(ref[0], rel=REL), what
    assert got[1] == pytest.approx(ref[1], rel=REL), what
    return got


FORMATS = [nv.NVFP4, nv.MXFP4, nv.Format(32, nv.SCALE_E4M3, 1), nv.Format(128, nv.SCALE_E4M3, 1)]


@pytest.mark.parametrize("fmt", FORMATS, ids=["nvfp4", "mxfp4", "b32", "b128"])
@pytest.mark.parametrize("axis", [0, 1])
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_ragged_shapes_all_formats(fmt, axis, dtype):
    # several workgroups in both kernels, a ragged last tile in both directions
    rows, cols = (384, 328) if axis == 0 else (203, 1152)
    x = synth.student_t_outliers(rows, cols, seed=7 + axis, dtype=dtype)
    run(x, axis, nv.SR, 5, fmt, "ragged")
    run(x, axis, nv.RTN, 0, fmt, "ragged")


@pytest.mark.parametrize("fmt", FORMATS[:2], ids=["nvfp4", "mxfp4"])
@pytest.mark.parametrize("cols", [328, 330], ids=["4-columns-per-lane", "1-column-per-lane"])
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_column_kernel_variants_with_a_short_last_span(fmt, cols, dtype):
    # 416 rows = one full 256-row tile, two full 64-row spans and one of 32 rows (four groups of 8);
    # 330 columns (rows padded to 336 elements for the 16-byte row alignment every entry point asks for)
    # rule out four columns per lane, so the one-column-per-lane kernel runs
    x = synth.student_t_outliers(416, cols, seed=11, dtype=dtype)
    run(x, 0, nv.SR, 3, fmt, "short span", ld=336)
    run(x, 0, nv.RTN, 0, fmt, "short span", ld=336)


def test_tiny_and_empty():
    run(synth.normal(1, 16, 1.0, 1, torch.float32), 1, nv.RTN, 0, nv.NVFP4, "one block")
    run(synth.normal(16, 4, 1.0, 2, torch.float32), 0, nv.RTN, 0, nv.NVFP4, "one block down each of 4 columns")
    x = torch.empty((0, 64), dtype=torch.bfloat16, device="cuda")
    q = nv.quantize(x, 1)
    out = nv.quant_noise(x, q, 1).cpu().numpy()
    assert out[0] == 0.0 and out[1] == 0.0


def test_representable_tensor_has_zero_noise():
    grid = torch.tensor([0, 0.5, 1, 1.5, 2, 3, 4, 6, 0, -0.5, -1, -1.5, -2, -3, -4, -6], dtype=torch.float32)
    x = grid.repeat(64, 8).contiguous()
    xg = x.cuda()
    g = torch.ones(1, device="cuda")
    q = nv.quantize(xg, 1, nv.SR, 3, tensor_scale=g)
    out = nv.quant_noise(xg, q, 1).cpu().numpy()
    assert out[1] == 0.0 and out[0] == float((x.double() ** 2).sum())


def test_window_of_a_wider_tensor_and_determinism():
    big = synth.normal(256, 512, 1.0, 9, torch.bfloat16).cuda()
    x = big[:, 64:64 + 256]
    q = nv.quantize(x, 0, nv.SR, 8)
    a = nv.quant_noise(x, q, 0).cpu().numpy()
    b = nv.quant_noise(x, q, 0).cpu().numpy()
    assert np.array_equal(a, b)
    xc = x.contiguous().cpu()
    ref = oracle.quant_noise(xc, tuple(t.cpu().numpy() if t.numel() > 1 else float(t) for t in q), 0)
    assert a[0] == pytest.approx(ref[0], rel=REL) and a[1] == pytest.approx(ref[1], rel=REL)


def test_gradient_like_tensor_at_7b_shape_ratio():
    # dY of the 7B down projection: the monitored ratio, both orientations the backward pass quantizes
    x = synth.gradient_like(4096, 4096, 77)
    for axis in (1, 0):
        got = run(x, axis, nv.SR, 21, nv.NVFP4, "7b-dY")
        ratio = float(np.sqrt(got[0] / got[1]))
        print(f"[info] gradient-to-noise ratio axis {axis}: {ratio:.3f} (threshold sqrt(3) = 1.732)", flush=True)
        assert ratio > 1.0
