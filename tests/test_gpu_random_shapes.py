"""Seeded sweeps over random shapes: GEMM outputs within the stated tolerance of the oracle, quantizer
outputs (single-orientation and dual entries) bit-identical to it, whatever tile, edge and fallback
path a shape selects."""
import numpy as np
import pytest
import torch

import oracle
from paper_2505_19115_amd import synth
from gpu_util import assert_quant_equal, to_np

pytestmark = pytest.mark.gpu

nv = None


@pytest.fixture(scope="module", autouse=True)
def _binding():
    global nv
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2505_19115_amd import binding
    nv = binding
    yield


def test_gemm_random_shapes():
    rng = np.random.default_rng(2024)
    for it in range(36):
        big = it % 9 == 0  # >= 128 tiles of 256 x 256: the 8-wave NVFP4 kernel / the direct-to-LDS MXFP4 kernel
        M = int(rng.integers(2300, 3300)) if big else int(rng.integers(1, 700))
        N = int(rng.integers(2300, 3300)) if big else int(rng.integers(1, 700))
        mx = it % 2 == 1
        K = int(rng.integers(1, 5)) * 128 if big else int(rng.integers(1, 9)) * (128 if it % 3 == 0 else 32)
        fmt, of, blk = (nv.MXFP4, oracle.MXFP4, 32) if mx else (nv.NVFP4, oracle.NVFP4, 16)

        def operand(rows):
            codes = rng.integers(0, 256, (rows, K // 2)).astype(np.uint8)
            scales = (rng.integers(118, 136, (rows, K // blk)) if mx else rng.integers(0x28, 0x50, (rows, K // blk))).astype(np.uint8)
            return codes, scales, 1.0 if mx else float(rng.uniform(0.1, 2.0))

        A, B = operand(M), operand(N)
        dt = torch.bfloat16 if it % 4 < 2 else torch.float32
        print(f"[case] random gemm {it}: M={M} N={N} K={K} {'mxfp4' if mx else 'nvfp4'} {dt}", flush=True)
        dev = lambda o: (torch.from_numpy(o[0]).cuda(), torch.from_numpy(o[1]).cuda(),
                         torch.tensor([o[2]], dtype=torch.float32, device="cuda"))
        Y = nv.gemm(dev(A), dev(B), fmt, dt)
        torch.cuda.synchronize()
        ref, ra = oracle.gemm_nt(A, B, of), oracle.gemm_nt(A, B, of, take_abs=True)
        got = to_np(Y.float()).astype(np.float64)
        tol = (2.0 ** -8 * np.abs(ref) + 1e-5 * ra) if dt == torch.bfloat16 else 1e-5 * ra + 1e-300
        assert np.all(np.abs(got - ref) <= tol), (it, M, N, K)


def test_quantizers_random_shapes():
    rng = np.random.default_rng(7)
    fmts = [(nv.NVFP4, oracle.NVFP4), (nv.MXFP4, oracle.MXFP4), (nv.Format(32, 0, 1), oracle.Format(32, 0, 1)),
            (nv.Format(64, 0, 1), oracle.Format(64, 0, 1))]
    gens = [lambda r, c, seed, d: synth.normal(r, c, 1.0, seed, d),
            lambda r, c, seed, d: synth.student_t_outliers(r, c, seed, dtype=d),
            lambda r, c, seed, d: synth.gradient_like(r, c, seed, dtype=d)]
    for it in range(32):
        f, of = fmts[it % 4]
        B = f.block
        rows = int(rng.integers(1, 12)) * B * (1 + 3 * (it % 5 == 0))
        cols = int(rng.integers(1, 20)) * B * (1 + 2 * (it % 7 == 0))
        dt = torch.bfloat16 if it % 3 else torch.float32
        x = gens[it % 3](rows, cols, 100 + it, dt)
        rr, rc = [(0, 0), (1, 1), (0, 1), (1, 0)][(it // 4) % 4]
        print(f"[case] random quantize {it}: {rows}x{cols} block={B} scale={f.scale} {dt} rounding=({rr},{rc})", flush=True)
        xg = x.cuda()
        qr, qc = nv.quantize_dual(xg, rr, 31 + it, rc, 77 + it, f)
        a, b = nv.quantize(xg, 1, rr, 31 + it, f), nv.quantize(xg, 0, rc, 77 + it, f)
        torch.cuda.synchronize()
        wr, wc = oracle.quantize(x, 1, rr, 31 + it, of), oracle.quantize(x, 0, rc, 77 + it, of)
        assert_quant_equal(qr, wr, "dual rows")
        assert_quant_equal(qc, wc, "dual cols")
        assert_quant_equal(a, wr, "rows")
        assert_quant_equal(b, wc, "cols")
