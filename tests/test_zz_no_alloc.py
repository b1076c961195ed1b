"""nvfp4_quantize_static -- the entry point that allocates nothing -- against nvfp4_quantize, through the C ABI:
same bits on two calls in a row (the second on a smaller input, so the scratch still holds the first call's
partial maxima), for the dense and the strided tensor-maximum paths, and its size limit."""
import ctypes as C

import numpy as np
import pytest
import torch

from paper_2505_19115_amd import synth

pytestmark = pytest.mark.gpu


def _call_static(nv, x, axis, rounding, seed, fmt, codes, scales, g):
    f = fmt.c()
    rows, cols = x.shape
    return nv.lib.nvfp4_quantize_static(x.data_ptr(), nv.BF16 if x.dtype == torch.bfloat16 else nv.F32, rows, cols,
                                        x.stride(0), axis, rounding, seed, C.byref(f), codes.data_ptr(),
                                        scales.data_ptr(), g.data_ptr(), 0, torch.cuda.current_stream().cuda_stream)


def test_static_scratch_entry_matches_the_workspace_entry():
    assert torch.cuda.is_available(), "this test needs the MI355X"
    from paper_2505_19115_amd import binding as nv
    big = synth.student_t_outliers(1024, 4096, seed=61).cuda()        # dense: 512 partial maxima
    small = synth.student_t_outliers(96, 256, seed=62).cuda() * 0.25   # dense, one partial, smaller maximum
    wide = synth.student_t_outliers(320, 1056, seed=63).cuda()
    for fmt in (nv.NVFP4, nv.Format(32, nv.SCALE_E4M3, 1)):
        for axis, rounding, seed in ((1, nv.RTN, 0), (0, nv.SR, 9)):
            # two calls in a row on the static scratch, the second smaller; outputs allocated beforehand
            outs = []
            for x in (big, small, wide[:, 16:16 + 1024], small[:64, 32:32 + 128]):   # dense, dense, strided, strided
                rows, cols = x.shape
                outer, inner = (rows, cols) if axis == 1 else (cols, rows)
                outs.append((x, torch.zeros((outer, inner // 2), dtype=torch.uint8, device="cuda"),
                             torch.zeros((outer, inner // fmt.block), dtype=torch.uint8, device="cuda"),
                             torch.zeros(1, dtype=torch.float32, device="cuda")))
            torch.cuda.synchronize()
            for x, codes, scales, g in outs:
                print(f"[case] quantize_static fmt={fmt} axis={axis} rounding={rounding} shape={tuple(x.shape)} ld={x.stride(0)}", flush=True)
                assert _call_static(nv, x, axis, rounding, seed, fmt, codes, scales, g) == nv.OK
            torch.cuda.synchronize()
            for x, codes, scales, g in outs:
                want = nv.quantize(x, axis, rounding, seed, fmt)
                torch.cuda.synchronize()
                assert torch.equal(codes, want[0]) and torch.equal(scales, want[1]) and torch.equal(g, want[2]), tuple(x.shape)


def test_static_scratch_limit_and_binding():
    from paper_2505_19115_amd import binding as nv
    # a strided tensor with more row spans than the array holds partial maxima is refused, nothing enqueued
    x = torch.zeros((16400, 24), dtype=torch.bfloat16, device="cuda")[:, :16]
    codes = torch.zeros((16400, 8), dtype=torch.uint8, device="cuda")
    scales = torch.zeros((16400, 1), dtype=torch.uint8, device="cuda")
    g = torch.full((1,), -1.0, device="cuda")
    assert _call_static(nv, x, 1, nv.RTN, 0, nv.NVFP4, codes, scales, g) == nv.EWORKSPACE
    torch.cuda.synchronize()
    assert float(g) == -1.0
    # one row fewer than the limit works (16384 spans), and the thin binding gives the same as quantize()
    y = synth.normal(16384, 24, 1.0, 5).cuda()[:, :16]
    a, b = nv.quantize_static(y, 1, nv.SR, 3), nv.quantize(y, 1, nv.SR, 3)
    torch.cuda.synchronize()
    assert all(torch.equal(p, q) for p, q in zip(a, b))
