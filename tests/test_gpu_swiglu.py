"""GPU parity of the SwiGLU backward fused with the quantizers of its results (nvfp4_swiglu_bwd_quantize) and of the
backward call that takes an already quantized upstream gradient (nvfp4_linear_bwd_dyq): the four operands per
result must equal, bit for bit, the oracle's quantization of the oracle's SwiGLU backward, and the GEMMs on them
must equal the ones of the unfused path."""
import numpy as np
import pytest
import torch

import oracle
from paper_2505_19115_amd import synth
from gpu_util import assert_bf16_gemm_close, assert_quant_equal, ofmt, to_np

pytestmark = pytest.mark.gpu

nv = None


@pytest.fixture(scope="module", autouse=True)
def _binding():
    global nv
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2505_19115_amd import binding
    nv = binding
    yield


def _slab_to_plain(buf, rows, K, per_row):
    rt, nkt = (rows + 255) // 256, K // 128
    a = buf.reshape(rt, nkt, 256, per_row)
    r = np.arange(256)
    pos = (r & ~63) | ((r & 7) << 3) | ((r >> 3) & 7)
    a = a[:, :, pos, :]
    return a.transpose(0, 2, 1, 3).reshape(rt * 256, nkt * per_row)[:rows]


def _inputs(M, F, dtype, seed):
    dH = synth.gradient_like(M, F, seed, dtype=dtype)
    G = synth.normal(M, F, 2.0, seed + 1, dtype)
    U = synth.normal(M, F, 1.0, seed + 2, dtype)
    return dH, G, U


def _as_torch(a, dtype):
    """oracle hand-over (uint16 bit patterns or float32) -> CPU torch tensor of dtype"""
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).view(torch.bfloat16)
    return torch.from_numpy(a)


@pytest.mark.parametrize("fmt_name", ["NVFP4", "MXFP4"])
@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_fused_swiglu_backward_quantizers_match_the_oracle(fmt_name, dtype):
    fmt = getattr(nv, fmt_name)
    of = ofmt(fmt)
    for M, F, sg, su in ((64, 96, 10, 20), (288, 704, 11, 23), (128, 1024, 5, 5)):
        print(f"[case] swiglu bwd fused {fmt_name} {dtype} M={M} F={F}", flush=True)
        dH, G, U = _inputs(M, F, dtype, 900 + M)
        dG, dU = nv.swiglu_bwd_quantize(dH.cuda(), G.cuda(), U.cuda(), sg, su, fmt)
        torch.cuda.synchronize()
        oG, oU = oracle.swiglu_bwd(dH, G, U)
        for got, ref, seed, what in ((dG, oG, sg, "dG"), (dU, oU, su, "dU")):
            assert_quant_equal(got.rows, oracle.quantize(ref, 1, oracle.SR, seed, of), what + " rows")
            assert_quant_equal(got.cols, oracle.quantize(ref, 0, oracle.SR, seed + 1, of), what + " cols")
        # the form that stores the two results in its first pass: same operands, and the stored tensors are the
        # oracle's hand-over
        sG, sU = torch.empty_like(dH, device="cuda"), torch.empty_like(dH, device="cuda")
        dG2, dU2 = nv.swiglu_bwd_quantize(dH.cuda(), G.cuda(), U.cuda(), sg, su, fmt, store=(sG, sU))
        torch.cuda.synchronize()
        for a, b in ((dG, dG2), (dU, dU2)):
            for x, y in zip((a.codes_rows, a.scales_rows, a.codes_cols, a.scales_cols, a.g), (b.codes_rows, b.scales_rows, b.codes_cols, b.scales_cols, b.g)):
                assert torch.equal(x, y)
        view0 = (lambda t: to_np(t.view(torch.int16)).view(np.uint16)) if dtype == torch.bfloat16 else to_np
        assert np.array_equal(view0(sG), oG) and np.array_equal(view0(sU), oU)
        # the elementwise step alone: the stored tensors are the oracle's hand-over, bit for bit
        tG, tU = nv.swiglu_bwd(dH.cuda(), G.cuda(), U.cuda())
        torch.cuda.synchronize()
        view = (lambda t: to_np(t.view(torch.int16)).view(np.uint16)) if dtype == torch.bfloat16 else to_np
        assert np.array_equal(view(tG), oG) and np.array_equal(view(tU), oU)
    # degenerate: an all-zero upstream gradient (scale 1, zero codes with the sign bits of the products)
    dH, G, U = _inputs(64, 128, dtype, 77)
    dH.zero_()
    dG, dU = nv.swiglu_bwd_quantize(dH.cuda(), G.cuda(), U.cuda(), 1, 2, fmt)
    oG, oU = oracle.swiglu_bwd(dH, G, U)
    assert_quant_equal(dG.rows, oracle.quantize(oG, 1, oracle.SR, 1, of), "zero dG rows")
    assert_quant_equal(dU.cols, oracle.quantize(oU, 0, oracle.SR, 3, of), "zero dU cols")


@pytest.mark.parametrize("fmt_name", ["NVFP4", "MXFP4"])
def test_fused_swiglu_slab_outputs_and_prequantized_backward(fmt_name):
    # the gate/up layers' backward at a size where every GEMM takes slab operands: the fused quantizers write
    # slabs, nvfp4_linear_bwd_dyq consumes them, and dX / dW must equal, bit for bit, nvfp4_linear_bwd on the
    # tensor dG that an elementwise kernel with the same arithmetic would have stored (taken from the oracle)
    fmt = getattr(nv, fmt_name)
    of = ofmt(fmt)
    T, D, F, sg, su = 2944, 2816, 3200, 40, 50   # tokens, model width (K of gate/up), ffn width (N of gate/up)
    print(f"[case] swiglu bwd slabs + dyq {fmt_name}", flush=True)
    dH, G, U = _inputs(T, F, torch.bfloat16, 300)
    X = synth.normal(T, D, 1.0, 303).cuda()
    Wg = synth.normal(F, D, 0.02, 304).cuda()
    takes = lambda m, n, k: bool(nv.lib.nvfp4_gemm_takes_slabs(m, n, k, fmt.c()))
    s_r, s_c = takes(T, D, F), takes(F, D, T)
    assert s_r and s_c
    dGq, dUq = nv.swiglu_bwd_quantize(dH.cuda(), G.cuda(), U.cuda(), sg, su, fmt, slab_rows=s_r, slab_cols=s_c)
    pG, pU = nv.swiglu_bwd_quantize(dH.cuda(), G.cuda(), U.cuda(), sg, su, fmt)
    torch.cuda.synchronize()
    oG, oU = oracle.swiglu_bwd(dH, G, U)
    assert_quant_equal(pG.rows, oracle.quantize(oG, 1, oracle.SR, sg, of), "dG rows")
    assert_quant_equal(pU.cols, oracle.quantize(oU, 0, oracle.SR, su + 1, of), "dU cols")
    assert np.array_equal(_slab_to_plain(to_np(dGq.codes_rows), T, F, 64), to_np(pG.codes_rows))
    assert np.array_equal(_slab_to_plain(to_np(dUq.codes_cols), F, T, 64), to_np(pU.codes_cols))
    assert np.array_equal(_slab_to_plain(to_np(dGq.scales_cols), F, T, 128 // fmt.block), to_np(pG.scales_cols))
    assert np.array_equal(_slab_to_plain(to_np(dUq.scales_rows), T, F, 128 // fmt.block), to_np(pU.scales_rows))
    dG_t = _as_torch(oG, torch.bfloat16).cuda()
    want = nv.linear_bwd(dG_t, X, Wg, sg, fmt, out_dtype=torch.bfloat16)
    for q, what in ((dGq, "slabs"), (pG, "row-major")):
        got = nv.linear_bwd_dyq(q, X, Wg, sg, T, F, D, fmt, out_dtype=torch.bfloat16)
        torch.cuda.synchronize()
        assert torch.equal(got[0], want[0]) and torch.equal(got[1], want[1]), what
    # with the forward call's saved operands and with weight operands quantized once
    saved = torch.empty(nv.linear_saved_bytes(T, F, D, fmt), dtype=torch.uint8, device="cuda")
    wq = nv.quantize_weight(Wg, T, fmt)
    nv.linear_fwd(X, None, fmt, out_dtype=torch.bfloat16, w_operands=wq, N=F, saved=saved, bwd_seed=sg)
    got = nv.linear_bwd_dyq(dGq, None, None, sg, T, F, D, fmt, out_dtype=torch.bfloat16, saved=saved, w_operands=wq)
    torch.cuda.synchronize()
    assert torch.equal(got[0], want[0]) and torch.equal(got[1], want[1])
    # and the products against the oracle on a few sampled outputs
    rng = np.random.default_rng(8)
    ii, kk, jj = rng.integers(0, T, 40), rng.integers(0, D, 40), rng.integers(0, F, 40)
    qdy, qwt = oracle.quantize(oG, 1, oracle.SR, sg, of), oracle.quantize(Wg.cpu(), 0, oracle.RTN, 0, of)
    assert_bf16_gemm_close(to_np(got[0].float())[ii, kk], oracle.gemm_nt_sample(qdy, qwt, ii, kk, of),
                           oracle.gemm_nt_sample(qdy, qwt, ii, kk, of, take_abs=True), "dX")
    qdyt, qxt = oracle.quantize(oG, 0, oracle.SR, sg + 1, of), oracle.quantize(X.cpu(), 0, oracle.SR, sg + 2, of)
    assert_bf16_gemm_close(to_np(got[1].float())[jj, kk], oracle.gemm_nt_sample(qdyt, qxt, jj, kk, of),
                           oracle.gemm_nt_sample(qdyt, qxt, jj, kk, of, take_abs=True), "dW")


def test_prequantized_backward_small_and_single_gemm():
    # row-major operands from nvfp4_quantize_dual, a shape below the slab threshold, dX only and dW only
    M, N, K, seed = 256, 192, 320, 9
    X, W, dY = synth.normal(M, K, 1.0, 1).cuda(), synth.normal(N, K, 0.02, 2).cuda(), synth.gradient_like(M, N, 3).cuda()
    for fmt in (nv.NVFP4, nv.MXFP4):
        print(f"[case] dyq small fmt={fmt}", flush=True)
        (cr, sr, g), (cc, sc, _) = nv.quantize_dual(dY, nv.SR, seed, nv.SR, seed + 1, fmt)
        q = nv.DualOperands(cr, sr, cc, sc, g, 0)
        want = nv.linear_bwd(dY, X, W, seed, fmt)
        got = nv.linear_bwd_dyq(q, X, W, seed, M, N, K, fmt)
        torch.cuda.synchronize()
        assert torch.equal(got[0], want[0]) and torch.equal(got[1], want[1])
        import ctypes as C
        f = fmt.c()
        ws = torch.empty(nv.lib.nvfp4_linear_bwd_workspace_bytes(M, N, K, C.byref(f)), dtype=torch.uint8, device="cuda")
        dx = torch.zeros((M, K), device="cuda")
        cd = q.c()
        rc = nv.lib.nvfp4_linear_bwd_dyq(C.byref(cd), None, W.data_ptr(), None, dx.data_ptr(), None, M, N, K, nv.BF16, nv.F32, C.byref(f), seed,
                                          ws.data_ptr(), ws.numel(), torch.cuda.current_stream().cuda_stream, None, None)
        torch.cuda.synchronize()
        assert rc == nv.OK and torch.equal(dx, want[0])
