"""GPU parity of nvfp4_gemm and the fused linear entries against the fp64 CPU oracle."""
import numpy as np
import pytest
import torch

import oracle
from paper_2505_19115_amd import synth
from gpu_util import assert_bf16_gemm_close, assert_gemm_close, assert_quant_equal, ofmt, to_np

pytestmark = pytest.mark.gpu

nv = None


@pytest.fixture(scope="module", autouse=True)
def _binding():
    global nv
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2505_19115_amd import binding
    nv = binding
    yield


@pytest.fixture
def switches():
    """A test that flips the library's cross-check switches gets them restored afterwards."""
    before = nv.cross_check_switches()
    yield
    nv.cross_check_switches(before)


def dev(q):
    """oracle-side (codes, scales, g) -> device tensors."""
    c, s, g = q
    return (torch.from_numpy(c).cuda(), torch.from_numpy(s).cuda(),
            torch.tensor([g], dtype=torch.float32, device="cuda"))


def random_operand(rng, rows, K, block=16, lo=0x01, hi=0x7F, g=1.0):
    codes = rng.integers(0, 256, (rows, K // 2)).astype(np.uint8)
    scales = rng.integers(lo, hi, (rows, K // block)).astype(np.uint8)
    return codes, scales, g


def check(A, B, fmt, what, out_dtype=torch.float32, tol=None):
    print(f"[case] gemm {what} M={A[0].shape[0]} N={B[0].shape[0]} K={A[0].shape[1] * 2} fmt={fmt}", flush=True)
    Y = nv.gemm(dev(A), dev(B), fmt, out_dtype)
    torch.cuda.synchronize()
    ref = oracle.gemm_nt(A, B, ofmt(fmt))
    ref_abs = oracle.gemm_nt(A, B, ofmt(fmt), take_abs=True)
    if out_dtype == torch.bfloat16:
        # bf16 output: the fp32 result rounded once more (8 significant bits)
        assert np.all(np.abs(to_np(Y.float()) - ref) <= 2.0 ** -8 * np.abs(ref) + 1e-5 * ref_abs), what
    else:
        assert_gemm_close(to_np(Y), ref, ref_abs, what, **({} if tol is None else {"tol": tol}))
    return Y


def test_config1_forward():
    # Y = Q(X) Q(W)^T for X, W fp32 [256, 256] ~ N(0,1), quantized on the GPU
    X = synth.normal(256, 256, 1.0, 1, torch.float32)
    W = synth.normal(256, 256, 1.0, 2, torch.float32)
    qa, qb = nv.quantize(X.cuda(), 1), nv.quantize(W.cuda(), 1)
    A, B = oracle.quantize(X, 1), oracle.quantize(W, 1)
    assert_quant_equal(qa, A, "X")
    assert_quant_equal(qb, B, "W")
    Y = nv.gemm(qa, qb)
    torch.cuda.synchronize()
    assert_gemm_close(to_np(Y), oracle.gemm_nt(A, B), oracle.gemm_nt(A, B, take_abs=True), "config1")
    Yf = nv.linear_fwd(X.cuda(), W.cuda())
    torch.cuda.synchronize()
    assert torch.equal(Y, Yf)


def test_unit_scales_give_exact_integers():
    # all scales 1, g = 1: every partial sum is a multiple of 1/4 below 2^24/4, so fp32
    # accumulation is exact whatever the order and the result must EQUAL the integer product
    rng = np.random.default_rng(0)
    M, N, K = 200, 136, 1184
    A = (rng.integers(0, 256, (M, K // 2)).astype(np.uint8), np.full((M, K // 16), 0x38, np.uint8), 1.0)
    B = (rng.integers(0, 256, (N, K // 2)).astype(np.uint8), np.full((N, K // 16), 0x38, np.uint8), 1.0)
    Y = to_np(nv.gemm(dev(A), dev(B)))
    assert np.array_equal(Y.astype(np.float64), oracle.gemm_nt(A, B))


@pytest.mark.parametrize("shape", [(256, 256, 256), (200, 136, 160), (1, 1, 32), (130, 257, 416), (384, 512, 1024)])
def test_random_codes_and_scales(shape):
    # every scale byte from the smallest subnormal to 448 next to each other, random codes
    M, N, K = shape
    rng = np.random.default_rng(M * 7 + N)
    check(random_operand(rng, M, K, g=0.37), random_operand(rng, N, K, g=2.5e-3), nv.NVFP4, "random")

@pytest.mark.parametrize("shape", [(2900, 3000, 256), (2560, 3330, 512), (4100, 8200, 256), (3000, 2900, 384)],
                         ids=["144 ragged tiles, 2 K tiles", "140 tiles, 4 K tiles", "561 tiles", "3 K tiles"])
def test_large_tile_kernel_ragged_edges(shape):
    # >= 128 tiles of 256 x 256 select the 8-wave kernel: edge tiles (clamped rows, element-wise stores),
    # even and odd numbers of K tiles, more tiles than CUs
    M, N, K = shape
    rng = np.random.default_rng(M + N + K)
    A, B = random_operand(rng, M, K, lo=0x30, hi=0x48, g=0.5), random_operand(rng, N, K, lo=0x30, hi=0x48, g=0.25)
    check(A, B, nv.NVFP4, "large-ragged")
    if K == 256:
        check(A, B, nv.NVFP4, "large-ragged-bf16", out_dtype=torch.bfloat16)


def test_moderate_scales_tight():
    # scales within a few binades (what real tensors give): no cancellation of huge terms
    rng = np.random.default_rng(5)
    check(random_operand(rng, 320, 2048, lo=0x30, hi=0x48), random_operand(rng, 192, 2048, lo=0x30, hi=0x48),
          nv.NVFP4, "moderate")


@pytest.mark.parametrize("block", [32, 64, 128])
def test_wider_blocks(block):
    fmt = nv.Format(block, nv.SCALE_E4M3, 1)
    rng = np.random.default_rng(block)
    check(random_operand(rng, 192, 640, block), random_operand(rng, 160, 640, block), fmt, f"block{block}")
    X = synth.normal(128, 512, 1.0, 7, torch.bfloat16)
    W = synth.normal(256, 512, 0.02, 8, torch.bfloat16)
    check(oracle.quantize(X, 1, 0, 0, ofmt(fmt)), oracle.quantize(W, 1, 0, 0, ofmt(fmt)), fmt, f"block{block}-real")


@pytest.mark.parametrize("block", [64, 128])
@pytest.mark.parametrize("shape", [(256, 256, 128), (200, 136, 384), (1, 1, 128), (130, 257, 640), (520, 300, 1024), (2900, 3000, 256)])
def test_wide_blocks_on_the_fp4_instruction(block, shape, switches):
    # E4M3 scales at blocks of 64 / 128: unit-scale FP4 matrix instructions per block, each block's exact partial sum
    # scaled by sA * sB in binary32 -- against the oracle at 1e-5 (every scale byte from the smallest subnormal to
    # 448), ragged tiles, 1 to 8 K tiles; and against the fp16 route, which must agree to rounding order
    M, N, K = shape
    fmt = nv.Format(block, nv.SCALE_E4M3, 1)
    rng = np.random.default_rng(M + N + K + block)
    A, B = random_operand(rng, M, K, block, g=0.37), random_operand(rng, N, K, block, g=2.5e-3)
    nv.cross_check_switches(nv.SWITCH_FP4_WIDE_BLOCKS)
    Y = check(A, B, fmt, f"fp4-rescale-b{block}")
    Yb = check(A, B, fmt, f"fp4-rescale-b{block}-bf16", out_dtype=torch.bfloat16)
    nv.cross_check_switches(0)
    Y16 = check(A, B, fmt, f"f16-route-b{block}")
    ref_abs = oracle.gemm_nt(A, B, ofmt(fmt), take_abs=True)
    assert np.all(np.abs(to_np(Y).astype(np.float64) - to_np(Y16).astype(np.float64)) <= 2e-5 * ref_abs + 1e-300)
    # unit scales: exact integers on this route too
    U = (A[0], np.full_like(A[1], 0x38), 1.0), (B[0], np.full_like(B[1], 0x38), 1.0)
    nv.cross_check_switches(nv.SWITCH_FP4_WIDE_BLOCKS)
    Yu = to_np(nv.gemm(dev(U[0]), dev(U[1]), fmt))
    assert np.array_equal(Yu.astype(np.float64), oracle.gemm_nt(U[0], U[1], ofmt(fmt)))


def test_bf16_output_and_leading_dimension():
    rng = np.random.default_rng(9)
    A, B = random_operand(rng, 96, 256, lo=0x30, hi=0x40), random_operand(rng, 80, 256, lo=0x30, hi=0x40)
    check(A, B, nv.NVFP4, "bf16-out", out_dtype=torch.bfloat16)
    out = torch.full((96, 128), -1.0, device="cuda")
    nv.gemm(dev(A), dev(B), out=out[:, :80])
    ref = oracle.gemm_nt(A, B)
    assert_gemm_close(to_np(out[:, :80]), ref, oracle.gemm_nt(A, B, take_abs=True), "ldc")
    assert torch.all(out[:, 80:] == -1.0)


def test_7b_shape_sampled():
    # gate projection of the 7B model, tokens = 4096: [4096, 4096] x [11008, 4096]^T; 4000
    # sampled outputs are checked one by one, plus one full output row and column
    M, N, K = 4096, 11008, 4096
    X = synth.normal(M, K, 1.0, 31)
    W = synth.normal(N, K, 0.02, 32)
    A, B = oracle.quantize(X, 1), oracle.quantize(W, 1)
    print("[case] gemm 7B gate sampled", flush=True)
    Y = nv.gemm(dev(A), dev(B))
    torch.cuda.synchronize()
    rng = np.random.default_rng(3)
    ii = np.concatenate([rng.integers(0, M, 4000), np.full(N, 1234), np.arange(M)])
    jj = np.concatenate([rng.integers(0, N, 4000), np.arange(N), np.full(M, 10007)])
    ref = oracle.gemm_nt_sample(A, B, ii, jj)
    ref_abs = oracle.gemm_nt_sample(A, B, ii, jj, take_abs=True)
    assert_gemm_close(to_np(Y)[ii, jj], ref, ref_abs, "7b-gate")


def test_linear_fwd_bwd_against_oracle():
    # Eqs. 4-6 end to end on a small layer; operands are checked bit-exactly first, then the
    # three products by tolerance
    M, N, K = 256, 384, 512
    X = synth.normal(M, K, 1.0, 41)
    W = synth.normal(N, K, 0.02, 42)
    dY = synth.gradient_like(M, N, 43)
    seed = 1000
    Xg, Wg, dYg = X.cuda(), W.cuda(), dY.cuda()
    print("[case] linear fwd/bwd", flush=True)
    Y = nv.linear_fwd(Xg, Wg)
    dX, dW = nv.linear_bwd(dYg, Xg, Wg, seed)
    torch.cuda.synchronize()
    qx, qw = oracle.quantize(X, 1), oracle.quantize(W, 1)
    assert_gemm_close(to_np(Y), oracle.gemm_nt(qx, qw), oracle.gemm_nt(qx, qw, take_abs=True), "Y")
    qdy, qwt = oracle.quantize(dY, 1, oracle.SR, seed), oracle.quantize(W, 0)
    assert_quant_equal(nv.quantize(dYg, 1, nv.SR, seed), qdy, "Q_SR(dY)")
    assert_quant_equal(nv.quantize(Wg, 0), qwt, "Q_RtN(W^T)")
    assert_gemm_close(to_np(dX), oracle.gemm_nt(qdy, qwt), oracle.gemm_nt(qdy, qwt, take_abs=True), "dX")
    qdyt, qxt = oracle.quantize(dY, 0, oracle.SR, seed + 1), oracle.quantize(X, 0, oracle.SR, seed + 2)
    assert_quant_equal(nv.quantize(dYg, 0, nv.SR, seed + 1), qdyt, "Q_SR(dY^T)")
    assert_quant_equal(nv.quantize(Xg, 0, nv.SR, seed + 2), qxt, "Q_SR(X^T)")
    assert_gemm_close(to_np(dW), oracle.gemm_nt(qdyt, qxt), oracle.gemm_nt(qdyt, qxt, take_abs=True), "dW")
    # the oracle's own composition agrees too
    odX, odW = oracle.linear_bwd(dY, X, W, seed)
    assert np.allclose(to_np(dX), odX, rtol=1e-4, atol=1e-9) and np.allclose(to_np(dW), odW, rtol=1e-4, atol=1e-9)


def test_linear_fp32_inputs_bf16_outputs():
    M, N, K = 128, 96, 256
    X = synth.normal(M, K, 1.0, 51, torch.float32)
    W = synth.normal(N, K, 0.05, 52, torch.float32)
    dY = synth.gradient_like(M, N, 53, dtype=torch.float32)
    Y = nv.linear_fwd(X.cuda(), W.cuda(), out_dtype=torch.bfloat16)
    dX, dW = nv.linear_bwd(dY.cuda(), X.cuda(), W.cuda(), 7, out_dtype=torch.bfloat16)
    torch.cuda.synchronize()
    oY = oracle.linear_fwd(X, W)
    odX, odW = oracle.linear_bwd(dY, X, W, 7)
    for got, ref in ((Y, oY), (dX, odX), (dW, odW)):
        assert np.all(np.abs(to_np(got.float()) - ref) <= 2.0 ** -8 * np.abs(ref) + 1e-5 * np.abs(ref).max())


def sample_positions(rng, M, N, n=3000):
    """n random outputs, one full row, one full column, and the last row/column corner tile."""
    ii = np.concatenate([rng.integers(0, M, n), np.full(N, M // 3), np.arange(M), np.full(256, M - 1)])
    jj = np.concatenate([rng.integers(0, N, n), np.arange(N), np.full(M, N - 7), np.arange(N - 256, N)])
    return ii, jj


def check_sampled(Y, A, B, of, what, rng, n=3000):
    """Sampled outputs of a large product against the oracle's fp64 dot products: fp32 outputs to the stated
    1e-5, bf16 outputs to the bf16 rounding of that interval."""
    M, N = A[0].shape[0], B[0].shape[0]
    ii, jj = sample_positions(rng, M, N, n)
    ref = oracle.gemm_nt_sample(A, B, ii, jj, of)
    ref_abs = oracle.gemm_nt_sample(A, B, ii, jj, of, take_abs=True)
    got = to_np(Y.float())[ii, jj]
    if Y.dtype == torch.bfloat16:
        assert_bf16_gemm_close(got, ref, ref_abs, what)
    else:
        assert_gemm_close(got, ref, ref_abs, what)


@pytest.mark.parametrize("out_dtype", [torch.float32, torch.bfloat16], ids=["f32", "bf16"])
@pytest.mark.parametrize("fmt_name", ["NVFP4", "MXFP4"])
@pytest.mark.parametrize("shape", [(4096, 4096, 11008), (11008, 4096, 4096)], ids=["down-or-dX", "dW"])
def test_7b_backward_gemm_shapes_sampled(shape, fmt_name, out_dtype):
    # the other two GEMM shapes of the benchmark step (K = 11008: 86 K tiles; 11008 output rows), the kernels
    # and launch configuration bench.py times, checked on sampled outputs the oracle computes one by one:
    # fp32 output at the stated 1e-5, bf16 output (what the benchmark stores) at the rounding of that interval
    M, N, K = shape
    fmt, of = getattr(nv, fmt_name), getattr(oracle, fmt_name)
    A = oracle.quantize(synth.normal(M, K, 1.0, 81), 1, 0, 0, of)
    B = oracle.quantize(synth.normal(N, K, 0.02, 82), 1, 0, 0, of)
    print(f"[case] gemm {fmt_name} {shape} {out_dtype} sampled", flush=True)
    Y = nv.gemm(dev(A), dev(B), fmt, out_dtype)
    torch.cuda.synchronize()
    check_sampled(Y, A, B, of, f"{fmt_name} {shape}", np.random.default_rng(6))


@pytest.mark.parametrize("fmt_name", ["NVFP4", "MXFP4"])
@pytest.mark.parametrize("layer", [("gate", 11008, 4096), ("down", 4096, 11008)], ids=["gate", "down"])
def test_fused_entries_as_the_benchmark_calls_them(layer, fmt_name):
    # nvfp4_linear_fwd / nvfp4_linear_bwd exactly as bench.py's timed step calls them (bf16 in and out,
    # caller-owned workspaces, operands saved by the forward call, slab hand-over active), each of the three
    # products of Eqs. 4-6 checked on sampled outputs against the oracle's quantization OF THE INPUTS THE CALL
    # RECEIVED (RtN, RtN / SR, RtN / SR, SR) and its fp64 dot products
    import ctypes as C
    name, N, K = layer
    M, seed = 4096, 1000
    fmt, of = getattr(nv, fmt_name), getattr(oracle, fmt_name)
    X, W, dY = synth.normal(M, K, 1.0, 100), synth.normal(N, K, 0.02, 200), synth.gradient_like(M, N, 300)
    Xg, Wg, dYg = X.cuda(), W.cuda(), dY.cuda()
    f = fmt.c()
    wf = torch.empty(nv.lib.nvfp4_linear_fwd_workspace_bytes(M, N, K, C.byref(f)), dtype=torch.uint8, device="cuda")
    wb = torch.empty(nv.lib.nvfp4_linear_bwd_workspace_bytes(M, N, K, C.byref(f)), dtype=torch.uint8, device="cuda")
    saved = torch.empty(nv.linear_saved_bytes(M, N, K, fmt), dtype=torch.uint8, device="cuda")
    Y = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    dX = torch.empty((M, K), dtype=torch.bfloat16, device="cuda")
    dW = torch.empty((N, K), dtype=torch.bfloat16, device="cuda")
    print(f"[case] fused entries, bench configuration, {name} {fmt_name}", flush=True)
    nv.linear_fwd(Xg, Wg, fmt, workspace=wf, out=Y, saved=saved, bwd_seed=seed)
    nv.linear_bwd(dYg, None, None, seed, fmt, workspace=wb, out=(dX, dW), saved=saved, K=K)
    torch.cuda.synchronize()
    rng = np.random.default_rng(17)
    check_sampled(Y, oracle.quantize(X, 1, oracle.RTN, 0, of), oracle.quantize(W, 1, oracle.RTN, 0, of), of, f"{name} Y", rng)
    check_sampled(dX, oracle.quantize(dY, 1, oracle.SR, seed, of), oracle.quantize(W, 0, oracle.RTN, 0, of), of, f"{name} dX", rng)
    check_sampled(dW, oracle.quantize(dY, 0, oracle.SR, seed + 1, of), oracle.quantize(X, 0, oracle.SR, seed + 2, of), of, f"{name} dW", rng)


@pytest.mark.parametrize("layer", [("qkv", 12288, 4096), ("out_proj", 4096, 4096)], ids=["qkv", "out_proj"])
def test_7b_attention_projections_forward_sampled(layer):
    # the two forward linears of the 7B configuration that the MLP tests do not cover (Sec. 5 setup: fused QKV
    # 4096 -> 12288 and the attention output projection 4096 -> 4096), tokens = 4096, RtN, bf16 inputs; fp32
    # output at 1e-5 and bf16 output at the rounding of that interval
    name, N, K = layer
    M = 4096
    X, W = synth.normal(M, K, 1.0, 111), synth.normal(N, K, 0.02, 112)
    A, B = oracle.quantize(X, 1), oracle.quantize(W, 1)
    for out_dtype in (torch.float32, torch.bfloat16):
        print(f"[case] forward linear {name} {out_dtype}", flush=True)
        Y = nv.linear_fwd(X.cuda(), W.cuda(), out_dtype=out_dtype)
        torch.cuda.synchronize()
        check_sampled(Y, A, B, oracle.NVFP4, f"{name} {out_dtype}", np.random.default_rng(23))


def test_gemm_is_deterministic():
    # fixed accumulation order, no atomics: two launches give the same bits, for both matrix-instruction paths
    rng = np.random.default_rng(123)
    for fmt, mk in ((nv.NVFP4, lambda rows: random_operand(rng, rows, 1024)), (nv.MXFP4, lambda rows: mx_operand(rng, rows, 1024))):
        A, B = dev(mk(520)), dev(mk(392))
        print(f"[case] gemm determinism fmt={fmt}", flush=True)
        y0, y1 = nv.gemm(A, B, fmt), nv.gemm(A, B, fmt)
        torch.cuda.synchronize()
        assert torch.equal(y0, y1)


def test_backward_with_scales_handed_over_from_forward():
    # the per-tensor scales of X and W are functions of the tensors alone: the backward call that is
    # given the forward call's {gX, gW} skips two maximum passes and must produce the same bits
    M, N, K = 256, 192, 320
    X = synth.normal(M, K, 1.0, 71).cuda()
    W = synth.normal(N, K, 0.02, 72).cuda()
    dY = synth.gradient_like(M, N, 73).cuda()
    for fmt in (nv.NVFP4, nv.MXFP4):
        print(f"[case] scale hand-over fmt={fmt}", flush=True)
        sc = torch.full((2,), -1.0, device="cuda")
        Y0 = nv.linear_fwd(X, W, fmt)
        Y1 = nv.linear_fwd(X, W, fmt, scales_out=sc)
        assert torch.equal(Y0, Y1)
        if fmt.tensor_scale:
            gx, gw = float(nv.tensor_scale(X)), float(nv.tensor_scale(W))
            assert sc.cpu().tolist() == [gx, gw]
            assert gx == oracle.quantize(X.cpu(), 1)[2] and gw == oracle.quantize(W.cpu(), 1)[2]
        else:
            assert sc.cpu().tolist() == [1.0, 1.0]
        a = nv.linear_bwd(dY, X, W, 5, fmt)
        b = nv.linear_bwd(dY, X, W, 5, fmt, xw_scales=sc)
        torch.cuda.synchronize()
        assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])

@pytest.mark.parametrize("fmtname", ["nvfp4", "mxfp4", "e4m3_b64"])
@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_backward_from_operands_saved_by_forward(fmtname, dtype):
    # the forward call's passes over X and W also write Q_SR(X^T) and Q_RtN(W^T) (Eqs. 5-6 operands);
    # the backward call given that buffer reads neither X nor W and must produce the same bits as
    # the call that quantizes them itself -- and those are checked against the oracle
    fmt = {"nvfp4": nv.NVFP4, "mxfp4": nv.MXFP4, "e4m3_b64": nv.Format(64, nv.SCALE_E4M3, 1)}[fmtname]
    for M, N, K, seed in ((256, 192, 320, 5), (384, 640, 128, 9)):
        print(f"[case] saved operands fmt={fmtname} dtype={dtype} M={M} N={N} K={K}", flush=True)
        X = synth.normal(M, K, 1.0, 81, dtype).cuda()
        W = synth.normal(N, K, 0.02, 82, dtype).cuda()
        dY = synth.gradient_like(M, N, 83, dtype=dtype).cuda()
        saved = torch.empty(nv.linear_saved_bytes(M, N, K, fmt), dtype=torch.uint8, device="cuda")
        Y0 = nv.linear_fwd(X, W, fmt)
        Y1 = nv.linear_fwd(X, W, fmt, saved=saved, bwd_seed=seed)
        assert torch.equal(Y0, Y1)
        a = nv.linear_bwd(dY, X, W, seed, fmt)
        b = nv.linear_bwd(dY, None, None, seed, fmt, saved=saved, K=K)
        torch.cuda.synchronize()
        assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])
        of = ofmt(fmt)
        Xc, Wc, dYc = X.cpu(), W.cpu(), dY.cpu()
        qdy, qwt = oracle.quantize(dYc, 1, oracle.SR, seed, of), oracle.quantize(Wc, 0, oracle.RTN, 0, of)
        assert_gemm_close(to_np(b[0]), oracle.gemm_nt(qdy, qwt, of), oracle.gemm_nt(qdy, qwt, of, take_abs=True), "saved dX")
        qdyt, qxt = oracle.quantize(dYc, 0, oracle.SR, seed + 1, of), oracle.quantize(Xc, 0, oracle.SR, seed + 2, of)
        assert_gemm_close(to_np(b[1]), oracle.gemm_nt(qdyt, qxt, of), oracle.gemm_nt(qdyt, qxt, of, take_abs=True), "saved dW")


@pytest.mark.parametrize("fmtname", ["nvfp4", "mxfp4", "e4m3_b64"])
def test_weight_operands_reused_across_micro_batches(fmtname):
    # W quantized once (nvfp4_quantize_weight) and reused by the forward and backward calls of several micro-batches:
    # Y, dX, dW must equal, bit for bit, what the calls that quantize W themselves give (and those are checked
    # against the oracle here for the small shape); with and without the saved-operand hand-over of X; small shape
    # (row-major operands) and a shape whose three GEMMs all take slab operands
    fmt = {"nvfp4": nv.NVFP4, "mxfp4": nv.MXFP4, "e4m3_b64": nv.Format(64, nv.SCALE_E4M3, 1)}[fmtname]
    of = ofmt(fmt)
    shapes = [(256, 192, 320)] + ([(2944, 3200, 2816)] if fmtname != "e4m3_b64" else [])
    for M, N, K in shapes:
        W = synth.normal(N, K, 0.02, 142).cuda()
        wq = nv.quantize_weight(W, M, fmt)
        for mb in range(2):
            print(f"[case] weight operands reused fmt={fmtname} M={M} N={N} K={K} micro-batch {mb}", flush=True)
            seed = 50 + 3 * mb
            X, dY = synth.normal(M, K, 1.0, 140 + 10 * mb).cuda(), synth.gradient_like(M, N, 141 + 10 * mb).cuda()
            Y0 = nv.linear_fwd(X, W, fmt, out_dtype=torch.bfloat16)
            Y1 = nv.linear_fwd(X, None, fmt, out_dtype=torch.bfloat16, w_operands=wq, N=N)
            a = nv.linear_bwd(dY, X, W, seed, fmt, out_dtype=torch.bfloat16)
            b = nv.linear_bwd(dY, X, None, seed, fmt, out_dtype=torch.bfloat16, w_operands=wq)
            saved = torch.empty(nv.linear_saved_bytes(M, N, K, fmt), dtype=torch.uint8, device="cuda")
            Y2 = nv.linear_fwd(X, None, fmt, out_dtype=torch.bfloat16, w_operands=wq, N=N, saved=saved, bwd_seed=seed)
            c = nv.linear_bwd(dY, None, None, seed, fmt, out_dtype=torch.bfloat16, saved=saved, K=K, w_operands=wq)
            torch.cuda.synchronize()
            assert torch.equal(Y0, Y1) and torch.equal(Y0, Y2)
            assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])
            assert torch.equal(a[0], c[0]) and torch.equal(a[1], c[1])
            # a saved buffer filled by the _wq forward holds no W^T: the plain backward must refuse it
            with pytest.raises(nv.Nvfp4Error) as e:
                nv.linear_bwd(dY, None, None, seed, fmt, saved=saved, K=K)
            assert e.value.code == nv.EINVAL
            if M == 256:
                Xc, Wc, dYc = X.cpu(), W.cpu(), dY.cpu()
                qx, qw = oracle.quantize(Xc, 1, oracle.RTN, 0, of), oracle.quantize(Wc, 1, oracle.RTN, 0, of)
                assert_bf16_gemm_close(to_np(Y1.float()), oracle.gemm_nt(qx, qw, of), oracle.gemm_nt(qx, qw, of, take_abs=True), "wq Y")
                qdy, qwt = oracle.quantize(dYc, 1, oracle.SR, seed, of), oracle.quantize(Wc, 0, oracle.RTN, 0, of)
                assert_bf16_gemm_close(to_np(c[0].float()), oracle.gemm_nt(qdy, qwt, of), oracle.gemm_nt(qdy, qwt, of, take_abs=True), "wq dX")
                qdyt, qxt = oracle.quantize(dYc, 0, oracle.SR, seed + 1, of), oracle.quantize(Xc, 0, oracle.SR, seed + 2, of)
                assert_bf16_gemm_close(to_np(c[1].float()), oracle.gemm_nt(qdyt, qxt, of), oracle.gemm_nt(qdyt, qxt, of, take_abs=True), "wq dW")
        # operands prepared for another micro-batch size are refused
        X = synth.normal(M + 32, K, 1.0, 1).cuda()
        with pytest.raises(nv.Nvfp4Error) as e:
            nv.linear_fwd(X, None, fmt, w_operands=wq, N=N)
        assert e.value.code == nv.EINVAL


def test_saved_buffer_identity_is_checked(switches):
    # the backward call refuses a `saved` buffer that a forward call wrote for another seed, shape, format or
    # cross-check setting (host record of the buffer), and a copy of such a buffer at an address the library has
    # no record of turns dX and dW into NaN through the tag in the buffer's own header
    M, N, K, seed = 256, 384, 512, 21
    X, W, dY = synth.normal(M, K, 1.0, 131).cuda(), synth.normal(N, K, 0.02, 132).cuda(), synth.gradient_like(M, N, 133).cuda()
    fmts = (nv.NVFP4, nv.MXFP4, nv.Format(64, nv.SCALE_E4M3, 1))
    nbytes = max(nv.linear_saved_bytes(M, N, K, fmt) for fmt in fmts)
    # (both buffers allocated once, before any forward call: `moved_buf` is then an address no forward call ever saw)
    saved_buf = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    moved_buf = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    for fmt in fmts:
        print(f"[case] saved tag fmt={fmt}", flush=True)
        saved = saved_buf[:nv.linear_saved_bytes(M, N, K, fmt)]
        nv.linear_fwd(X, W, fmt, saved=saved, bwd_seed=seed)
        good = nv.linear_bwd(dY, None, None, seed, fmt, saved=saved, K=K)
        with pytest.raises(nv.Nvfp4Error) as e:
            nv.linear_bwd(dY, None, None, seed + 1, fmt, saved=saved, K=K)
        assert e.value.code == nv.EINVAL
        other = nv.Format(32, nv.SCALE_E4M3, 1)
        if nv.linear_saved_bytes(M, N, K, other) <= saved.numel():
            with pytest.raises(nv.Nvfp4Error) as e:
                nv.linear_bwd(dY, None, None, seed, other, saved=saved, K=K)
            assert e.value.code == nv.EINVAL
        nv.cross_check_switches(nv.SWITCH_SOFT_CONVERT)
        with pytest.raises(nv.Nvfp4Error) as e:
            nv.linear_bwd(dY, None, None, seed, fmt, saved=saved, K=K)
        assert e.value.code == nv.EINVAL
        nv.cross_check_switches(0)
        moved = moved_buf[:saved.numel()]  # an address no forward call wrote to: only the tag inside the buffer can tell
        moved.copy_(saved)
        again = nv.linear_bwd(dY, None, None, seed, fmt, saved=moved, K=K)
        bad = nv.linear_bwd(dY, None, None, seed + 1, fmt, saved=moved, K=K)
        only_dx = nv.lib.nvfp4_linear_bwd  # (dW = NULL below: the path without the dual quantizer checks the tag too)
        torch.cuda.synchronize()
        assert torch.equal(again[0], good[0]) and torch.equal(again[1], good[1])
        assert torch.isnan(bad[0]).all() and torch.isnan(bad[1]).all()
        import ctypes as C
        f = fmt.c()
        ws = torch.empty(nv.lib.nvfp4_linear_bwd_workspace_bytes(M, N, K, C.byref(f)), dtype=torch.uint8, device="cuda")
        dx = torch.zeros((M, K), device="cuda")
        for sd, want_nan in ((seed, False), (seed + 1, True)):
            rc = only_dx(dY.data_ptr(), None, None, dx.data_ptr(), None, M, N, K, nv.BF16, nv.F32, C.byref(f), sd,
                         ws.data_ptr(), ws.numel(), torch.cuda.current_stream().cuda_stream, None, moved.data_ptr())
            torch.cuda.synchronize()
            assert rc == nv.OK
            assert bool(torch.isnan(dx).all()) == want_nan
            if not want_nan:
                assert torch.equal(dx, good[0])


# ---------------------------------------------------------------- MXFP4 (block 32, E8M0): native FP4 MFMA
def mx_operand(rng, rows, K, lo=112, hi=142):
    codes = rng.integers(0, 256, (rows, K // 2)).astype(np.uint8)
    scales = rng.integers(lo, hi, (rows, K // 32)).astype(np.uint8)
    return codes, scales, 1.0


@pytest.mark.parametrize("shape", [(256, 256, 256), (200, 136, 512), (1, 1, 32), (130, 257, 96), (384, 512, 1024),
                                   (300, 520, 1280), (64, 64, 160),
                                   # K a multiple of 128: the four-stage direct-to-LDS kernel with 1, 2, 3, 4, 5 K tiles
                                   (256, 512, 128), (1, 1, 128), (257, 300, 256), (130, 257, 384), (512, 256, 512),
                                   (260, 252, 640)])
def test_mxfp4_random_codes_and_scales(shape):
    M, N, K = shape
    rng = np.random.default_rng(M + 3 * N + K)
    check(mx_operand(rng, M, K), mx_operand(rng, N, K), nv.MXFP4, "mxfp4-random")


@pytest.mark.parametrize("out_dtype", [torch.float32, torch.bfloat16])
def test_mxfp4_output_paths(out_dtype):
    # full tiles (vector stores), a window of a wider matrix (ldc > N), and an ldc that rules the
    # vector stores out
    rng = np.random.default_rng(91)
    M, N, K = 512, 768, 896
    A, B = mx_operand(rng, M, K, 120, 134), mx_operand(rng, N, K, 120, 134)
    check(A, B, nv.MXFP4, "mxfp4-full-tiles", out_dtype=out_dtype)
    ref, ref_abs = oracle.gemm_nt(A, B, oracle.MXFP4), oracle.gemm_nt(A, B, oracle.MXFP4, take_abs=True)
    tol = {"tol": 2.0 ** -8} if out_dtype == torch.bfloat16 else {}
    for ld in (N + 256, N + 1):
        print(f"[case] mxfp4 gemm window ldc={ld} {out_dtype}", flush=True)
        out = torch.full((M, ld), -1.0, device="cuda", dtype=out_dtype)
        nv.gemm(dev(A), dev(B), nv.MXFP4, out=out[:, :N])
        torch.cuda.synchronize()
        assert_gemm_close(to_np(out[:, :N].float()), ref, ref_abs, f"ldc{ld}", **tol)
        assert bool((out[:, N:] == -1.0).all()), "columns outside the window were written"


def test_mxfp4_unit_scales_exact_and_extreme_scales():
    rng = np.random.default_rng(77)
    M, N, K = 160, 288, 768
    A = (rng.integers(0, 256, (M, K // 2)).astype(np.uint8), np.full((M, K // 32), 127, np.uint8), 1.0)
    B = (rng.integers(0, 256, (N, K // 2)).astype(np.uint8), np.full((N, K // 32), 127, np.uint8), 1.0)
    Y = to_np(nv.gemm(dev(A), dev(B), nv.MXFP4))
    assert np.array_equal(Y.astype(np.float64), oracle.gemm_nt(A, B, oracle.MXFP4))
    # scale bytes far apart (2^-60 .. 2^+60 on one side, the inverse range on the other)
    A2 = (A[0], rng.integers(67, 187, (M, K // 32)).astype(np.uint8), 1.0)
    B2 = (B[0], rng.integers(67, 187, (N, K // 32)).astype(np.uint8), 1.0)
    check(A2, B2, nv.MXFP4, "mxfp4-extreme")
    # zero blocks: byte 0 with zero codes
    A3 = (A[0].copy(), A2[1].copy(), 1.0)
    A3[1][:, ::3] = 0
    for j in range(0, K // 32, 3):
        A3[0][:, j * 16:(j + 1) * 16] = 0
    check(A3, B2, nv.MXFP4, "mxfp4-zero-blocks")


def test_mxfp4_quantized_linear_fwd_bwd():
    M, N, K = 256, 384, 512
    X = synth.normal(M, K, 1.0, 61)
    W = synth.normal(N, K, 0.02, 62)
    dY = synth.gradient_like(M, N, 63)
    fm, of = nv.MXFP4, oracle.MXFP4
    print("[case] mxfp4 linear fwd/bwd", flush=True)
    Y = nv.linear_fwd(X.cuda(), W.cuda(), fm)
    dX, dW = nv.linear_bwd(dY.cuda(), X.cuda(), W.cuda(), 9, fm)
    torch.cuda.synchronize()
    qx, qw = oracle.quantize(X, 1, 0, 0, of), oracle.quantize(W, 1, 0, 0, of)
    assert_quant_equal(nv.quantize(X.cuda(), 1, nv.RTN, 0, fm), qx, "mx Q(X)")
    assert_gemm_close(to_np(Y), oracle.gemm_nt(qx, qw, of), oracle.gemm_nt(qx, qw, of, take_abs=True), "mx Y")
    qdy, qwt = oracle.quantize(dY, 1, oracle.SR, 9, of), oracle.quantize(W, 0, 0, 0, of)
    assert_gemm_close(to_np(dX), oracle.gemm_nt(qdy, qwt, of), oracle.gemm_nt(qdy, qwt, of, take_abs=True), "mx dX")
    qdyt, qxt = oracle.quantize(dY, 0, oracle.SR, 10, of), oracle.quantize(X, 0, oracle.SR, 11, of)
    assert_gemm_close(to_np(dW), oracle.gemm_nt(qdyt, qxt, of), oracle.gemm_nt(qdyt, qxt, of, take_abs=True), "mx dW")


def test_mxfp4_7b_shape_sampled():
    M, N, K = 4096, 11008, 4096
    X = synth.normal(M, K, 1.0, 31)
    W = synth.normal(N, K, 0.02, 32)
    A, B = oracle.quantize(X, 1, 0, 0, oracle.MXFP4), oracle.quantize(W, 1, 0, 0, oracle.MXFP4)
    print("[case] mxfp4 gemm 7B gate sampled", flush=True)
    Y = nv.gemm(dev(A), dev(B), nv.MXFP4)
    torch.cuda.synchronize()
    rng = np.random.default_rng(5)
    ii = np.concatenate([rng.integers(0, M, 4000), np.full(N, 4095), np.arange(M)])
    jj = np.concatenate([rng.integers(0, N, 4000), np.arange(N), np.full(M, 11007)])
    ref = oracle.gemm_nt_sample(A, B, ii, jj, oracle.MXFP4)
    ref_abs = oracle.gemm_nt_sample(A, B, ii, jj, oracle.MXFP4, take_abs=True)
    assert_gemm_close(to_np(Y)[ii, jj], ref, ref_abs, "mx-7b-gate")


def test_fused_calls_replay_from_a_hip_graph():
    # the fused entries launch only kernels on the given stream (no allocation, no memset, no host
    # synchronisation), so a forward + backward pair can be captured once and replayed; every
    # replay is checked against the eager result for the data then in the buffers
    M, N, K = 256, 384, 512
    f = nv.NVFP4.c()
    import ctypes as C
    X = synth.normal(M, K, 1.0, 91).cuda()
    W = synth.normal(N, K, 0.02, 92).cuda()
    dY = synth.gradient_like(M, N, 93).cuda()
    wf = torch.empty(nv.lib.nvfp4_linear_fwd_workspace_bytes(M, N, K, C.byref(f)), dtype=torch.uint8, device="cuda")
    wb = torch.empty(nv.lib.nvfp4_linear_bwd_workspace_bytes(M, N, K, C.byref(f)), dtype=torch.uint8, device="cuda")
    saved = torch.empty(nv.linear_saved_bytes(M, N, K), dtype=torch.uint8, device="cuda")
    Y = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    dX = torch.empty((M, K), dtype=torch.bfloat16, device="cuda")
    dW = torch.empty((N, K), dtype=torch.bfloat16, device="cuda")

    def step():
        nv.linear_fwd(X, W, workspace=wf, out=Y, saved=saved, bwd_seed=17)
        nv.linear_bwd(dY, None, None, seed=17, workspace=wb, out=(dX, dW), saved=saved, K=K)

    step()  # (first launches set kernel attributes: outside the capture)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for it in range(3):
        print(f"[case] graph replay {it}", flush=True)
        X.copy_(synth.normal(M, K, 1.0, 100 + it).cuda())
        dY.copy_(synth.gradient_like(M, N, 200 + it).cuda())
        step()
        torch.cuda.synchronize()
        want = (Y.clone(), dX.clone(), dW.clone())
        for t in (Y, dX, dW):
            t.fill_(-1.0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(Y, want[0]) and torch.equal(dX, want[1]) and torch.equal(dW, want[2])


def test_saved_operand_path_at_the_benchmark_shapes():
    # the launch configuration bench.py times (bf16 in/out, saved operands, dual quantizers) against the
    # plain calls, whose operands and GEMMs the other full-size tests check against the oracle
    M = 4096
    for N, K in ((11008, 4096), (4096, 11008)):
        print(f"[case] saved operands full size N={N} K={K}", flush=True)
        X = synth.normal(M, K, 1.0, 100).cuda()
        W = synth.normal(N, K, 0.02, 200).cuda()
        dY = synth.gradient_like(M, N, 300).cuda()
        saved = torch.empty(nv.linear_saved_bytes(M, N, K), dtype=torch.uint8, device="cuda")
        Y0 = nv.linear_fwd(X, W, out_dtype=torch.bfloat16)
        Y1 = nv.linear_fwd(X, W, out_dtype=torch.bfloat16, saved=saved, bwd_seed=1000)
        a = nv.linear_bwd(dY, X, W, 1000, out_dtype=torch.bfloat16)
        b = nv.linear_bwd(dY, None, None, 1000, out_dtype=torch.bfloat16, saved=saved, K=K)
        torch.cuda.synchronize()
        assert torch.equal(Y0, Y1) and torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])
        del X, W, dY, saved, Y0, Y1, a, b


@pytest.mark.parametrize("fmt_name", ["NVFP4", "MXFP4"])
def test_full_size_outputs_follow_row_permutations(fmt_name):
    # a property that holds at any size and checks EVERY output of the benchmark-shape GEMM: an output
    # element depends on one row of A and one row of B and is accumulated in a fixed order along K, so
    # permuting the rows of A (of B) permutes the rows (columns) of the result bit for bit -- whatever
    # tile, wave and lane a row lands in.  (Sampled outputs of these shapes are checked against the
    # oracle in the tests above.)
    fmt = getattr(nv, fmt_name)
    M, N, K = 4096, 11008, 4096
    X = synth.normal(M, K, 1.0, 100).cuda()
    W = synth.normal(N, K, 0.02, 200).cuda()
    qa, qb = nv.quantize(X, 1, fmt=fmt), nv.quantize(W, 1, fmt=fmt)
    Y = nv.gemm(qa, qb, fmt, torch.bfloat16)
    g = torch.Generator(device="cuda")
    g.manual_seed(5)
    pm, pn = torch.randperm(M, device="cuda", generator=g), torch.randperm(N, device="cuda", generator=g)
    qa2 = (qa[0][pm].contiguous(), qa[1][pm].contiguous(), qa[2])
    qb2 = (qb[0][pn].contiguous(), qb[1][pn].contiguous(), qb[2])
    Y2 = nv.gemm(qa2, qb2, fmt, torch.bfloat16)
    torch.cuda.synchronize()
    assert torch.equal(Y2, Y[pm][:, pn])


@pytest.mark.parametrize("pad", [0, 4, 8])
def test_large_tile_bf16_output_with_padded_rows(pad):
    # the 8-wave kernel's bf16 epilogue writes complete lines through LDS when the output rows are
    # 16-byte aligned (pad 0, 8) and falls back to 8-byte stores otherwise (pad 4); both into a
    # wider buffer whose padding must stay untouched
    M, N, K = 2816, 3072, 256
    rng = np.random.default_rng(77 + pad)
    A, B = random_operand(rng, M, K, lo=0x30, hi=0x48, g=0.5), random_operand(rng, N, K, lo=0x30, hi=0x48, g=0.25)
    for fmt, a, b in ((nv.NVFP4, A, B), (nv.MXFP4, mx_operand(rng, M, 512), mx_operand(rng, N, 512))):  # (K = 512: the direct-to-LDS MXFP4 kernel)
        print(f"[case] padded bf16 output pad={pad} fmt={fmt}", flush=True)
        buf = torch.full((M, N + pad), -3.0, dtype=torch.bfloat16, device="cuda")
        nv.gemm(dev(a), dev(b), fmt, out=buf[:, :N])
        torch.cuda.synchronize()
        ref = oracle.gemm_nt(a, b, ofmt(fmt))
        ref_abs = oracle.gemm_nt(a, b, ofmt(fmt), take_abs=True)
        got = to_np(buf[:, :N].float())
        assert np.all(np.abs(got - ref) <= 2.0 ** -8 * np.abs(ref) + 1e-5 * ref_abs)
        if pad:
            assert torch.all(buf[:, N:] == -3.0)


def test_swiglu_mlp_fwd_bwd_stage_by_stage():
    # The SwiGLU MLP graph of the 7B benchmark configuration at reduced width (tokens 256, d 256, ffn 704):
    # gate and up share X, h = silu(G) * U feeds down, and the backward pass walks the graph in reverse with
    # every operand of Eqs. 5-6 stochastically rounded.  bf16 tensors between the calls and saved operands, as
    # in the timed step.  The elementwise SwiGLU belongs to the caller (plain torch ops on the device here);
    # every library call is checked against the oracle ON THE INPUTS IT ACTUALLY RECEIVED, so a one-ulp bf16
    # difference upstream cannot be mistaken for, or hide, an error downstream.
    T, D, F = 256, 256, 704
    X = synth.normal(T, D, 1.0, 901).cuda()
    Wg, Wu = synth.normal(F, D, 0.02, 902).cuda(), synth.normal(F, D, 0.02, 903).cuda()
    Wd = synth.normal(D, F, 0.02, 904).cuda()
    dY = synth.gradient_like(T, D, 905).cuda()
    bf = torch.bfloat16

    def close_bf16(got, qa, qb, what):
        ref, ref_abs = oracle.gemm_nt(qa, qb), oracle.gemm_nt(qa, qb, take_abs=True)
        assert np.all(np.abs(to_np(got.float()) - ref) <= 2.0 ** -8 * np.abs(ref) + 1e-5 * ref_abs), what

    def fwd(x, w, seed, what):
        print(f"[case] mlp chain fwd {what}", flush=True)
        saved = torch.empty(nv.linear_saved_bytes(x.shape[0], w.shape[0], x.shape[1]), dtype=torch.uint8, device="cuda")
        y = nv.linear_fwd(x, w, out_dtype=bf, saved=saved, bwd_seed=seed)
        torch.cuda.synchronize()
        close_bf16(y, oracle.quantize(x.cpu(), 1), oracle.quantize(w.cpu(), 1), what)
        return y, saved

    def bwd(dy, x, w, seed, saved, what):
        print(f"[case] mlp chain bwd {what}", flush=True)
        dx, dw = nv.linear_bwd(dy, None, None, seed, out_dtype=bf, saved=saved, K=x.shape[1])
        torch.cuda.synchronize()
        dyc, xc, wc = dy.cpu(), x.cpu(), w.cpu()
        close_bf16(dx, oracle.quantize(dyc, 1, oracle.SR, seed), oracle.quantize(wc, 0), what + " dX")
        close_bf16(dw, oracle.quantize(dyc, 0, oracle.SR, seed + 1), oracle.quantize(xc, 0, oracle.SR, seed + 2), what + " dW")
        return dx, dw

    G, sg = fwd(X, Wg, 10, "gate")
    U, su = fwd(X, Wu, 20, "up")
    sig = torch.sigmoid(G.float())
    H = (G.float() * sig * U.float()).to(bf)
    Y, sd = fwd(H, Wd, 30, "down")
    assert Y.shape == (T, D)
    dH, dWd = bwd(dY, H, Wd, 30, sd, "down")
    dG = (dH.float() * U.float() * sig * (1.0 + G.float() * (1.0 - sig))).to(bf)
    dU = (dH.float() * G.float() * sig).to(bf)
    dXg, dWg = bwd(dG, X, Wg, 10, sg, "gate")
    dXu, dWu = bwd(dU, X, Wu, 20, su, "up")
    dX = dXg.float() + dXu.float()
    # sanity of the whole graph against the unquantized fp64 MLP: same direction, moderate relative error
    Xd, Wgd, Wud, Wdd = (t.double().cpu().numpy() for t in (X, Wg, Wu, Wd))
    g, u = Xd @ Wgd.T, Xd @ Wud.T
    s = 1.0 / (1.0 + np.exp(-g))
    dh = dY.double().cpu().numpy() @ Wdd
    dx_ref = (dh * u * s * (1.0 + g * (1.0 - s))) @ Wgd + (dh * g * s) @ Wud
    got = dX.double().cpu().numpy()
    cos = (got * dx_ref).sum() / (np.linalg.norm(got) * np.linalg.norm(dx_ref))
    print(f"[info] mlp chain: cosine of dX with the unquantized fp64 MLP {cos:.4f}", flush=True)
    assert cos > 0.9
    for t in (dWd, dWg, dWu):
        assert torch.isfinite(t.float()).all()


@pytest.mark.parametrize("fmt_name", ["NVFP4", "MXFP4"])
@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_slab_operand_layout_is_invisible(dtype, fmt_name, switches):
    # Between the quantizers and the large-tile GEMM the fused entries keep their packed operands as per-K-tile
    # slabs; NVFP4_PLAIN_OPERANDS=1 keeps them row-major.  Both must give the same bits.  Shape: all three GEMMs
    # of the layer large enough for the slab path, two of the three dimensions not multiples of the 256-row slab.
    M, N, K = 2944, 3200, 2816
    fmt = getattr(nv, fmt_name)
    of = ofmt(fmt)
    print(f"[case] slab layout vs plain M={M} N={N} K={K} {dtype} {fmt_name}", flush=True)
    X = synth.normal(M, K, 1.0, 611, dtype).cuda()
    W = synth.normal(N, K, 0.02, 612, dtype).cuda()
    dY = synth.gradient_like(M, N, 613, dtype=dtype).cuda()
    outs = []
    for plain in ("0", "1"):
        nv.cross_check_switches(nv.SWITCH_PLAIN_OPERANDS if plain == "1" else 0)
        saved = torch.empty(nv.linear_saved_bytes(M, N, K, fmt), dtype=torch.uint8, device="cuda")
        Y = nv.linear_fwd(X, W, fmt, out_dtype=torch.bfloat16, saved=saved, bwd_seed=77)
        dX, dW = nv.linear_bwd(dY, None, None, 77, fmt, out_dtype=torch.bfloat16, saved=saved, K=K)
        torch.cuda.synchronize()
        outs.append((Y, dX, dW))
    for a, b, what in zip(outs[0], outs[1], ("Y", "dX", "dW")):
        assert torch.equal(a, b), what
    # and against the oracle on sampled outputs (rows from the ragged last slabs included)
    rng = np.random.default_rng(5)
    Xc, Wc, dYc = X.cpu(), W.cpu(), dY.cpu()
    ii = np.concatenate([rng.integers(0, M, 24), [M - 1, M - 100, 2816]])
    jj = np.concatenate([rng.integers(0, N, 24), [N - 1, N - 60, 3072]])
    qx, qw = oracle.quantize(Xc, 1, oracle.RTN, 0, of), oracle.quantize(Wc, 1, oracle.RTN, 0, of)
    ref, ref_abs = oracle.gemm_nt_sample(qx, qw, ii, jj, of), oracle.gemm_nt_sample(qx, qw, ii, jj, of, take_abs=True)
    got = to_np(outs[0][0].float())[ii, jj]
    assert np.all(np.abs(got - ref) <= 2.0 ** -8 * np.abs(ref) + 1e-5 * ref_abs)
    kk = rng.integers(0, K, 27)
    qdy, qwt = oracle.quantize(dYc, 1, oracle.SR, 77, of), oracle.quantize(Wc, 0, oracle.RTN, 0, of)
    ref, ref_abs = oracle.gemm_nt_sample(qdy, qwt, ii, kk, of), oracle.gemm_nt_sample(qdy, qwt, ii, kk, of, take_abs=True)
    got = to_np(outs[0][1].float())[ii, kk]
    assert np.all(np.abs(got - ref) <= 2.0 ** -8 * np.abs(ref) + 1e-5 * ref_abs)
    qdyt, qxt = oracle.quantize(dYc, 0, oracle.SR, 78, of), oracle.quantize(Xc, 0, oracle.SR, 79, of)
    ref, ref_abs = oracle.gemm_nt_sample(qdyt, qxt, jj, kk, of), oracle.gemm_nt_sample(qdyt, qxt, jj, kk, of, take_abs=True)
    got = to_np(outs[0][2].float())[jj, kk]
    assert np.all(np.abs(got - ref) <= 2.0 ** -8 * np.abs(ref) + 1e-5 * ref_abs)


def _slab_to_plain(buf, rows, K, per_row):
    """Undo the documented slab layout: [rows/256][K/128] slabs of 256 positions x per_row bytes, tile row r at
    position (r & ~63) | ((r & 7) << 3) | ((r >> 3) & 7)."""
    rt, nkt = (rows + 255) // 256, K // 128
    a = buf.reshape(rt, nkt, 256, per_row)
    r = np.arange(256)
    pos = (r & ~63) | ((r & 7) << 3) | ((r >> 3) & 7)
    a = a[:, :, pos, :]                                  # [rt, kt, r, bytes]
    return a.transpose(0, 2, 1, 3).reshape(rt * 256, nkt * per_row)[:rows]


@pytest.mark.parametrize("fmt_name", ["NVFP4", "MXFP4"])
@pytest.mark.parametrize("rounding", [(0, 0), (0, 1), (1, 1)], ids=["rtn-rtn", "rtn-sr", "sr-sr"])
def test_slab_outputs_of_the_dual_quantizer_and_slab_gemm(rounding, fmt_name):
    # the slab layout as the header documents it: un-permuted on the host it must be the oracle's quantization,
    # and the GEMM must give the same bits from slab operands as from row-major ones
    rows, cols = 2944, 3200   # 11.5 and 12.5 slabs of rows; 23 and 25 K tiles
    rr, rc = rounding
    fmt = getattr(nv, fmt_name)
    x = synth.gradient_like(rows, cols, 71).cuda()
    print(f"[case] slab outputs rows={rows} cols={cols} rounding={rounding} {fmt_name}", flush=True)
    (cr, sr, g), (cc, sc, _) = nv.quantize_dual(x, rr, 11, rc, 12, fmt, slab_rows=True, slab_cols=True)
    (pr, psr, pg), (pc, psc, _) = nv.quantize_dual(x, rr, 11, rc, 12, fmt)
    torch.cuda.synchronize()
    assert cr.numel() == 12 * 25 * 16384 and cc.numel() == 13 * 23 * 16384
    assert np.array_equal(_slab_to_plain(to_np(cr), rows, cols, 64), to_np(pr))
    assert np.array_equal(_slab_to_plain(to_np(cc), cols, rows, 64), to_np(pc))
    per_row = 128 // fmt.block   # scale bytes per row and K tile: 8 (NVFP4) or 4 (MXFP4)
    assert sr.numel() == 12 * 25 * 256 * per_row and sc.numel() == 13 * 23 * 256 * per_row
    assert np.array_equal(_slab_to_plain(to_np(sr), rows, cols, per_row), to_np(psr))
    assert np.array_equal(_slab_to_plain(to_np(sc), cols, rows, per_row), to_np(psc))
    assert float(g) == float(pg)
    xc = x.cpu()
    assert_quant_equal((pr, psr, pg), oracle.quantize(xc, 1, rr, 11, ofmt(fmt)), "rows side")
    assert_quant_equal((pc, psc, pg), oracle.quantize(xc, 0, rc, 12, ofmt(fmt)), "cols side")
    # GEMM: out[rows, rows'] with K = cols from the row-blocked side against itself, and the column-blocked side
    # (operand rows = cols of x, K = rows of x) against itself; mixed slab / plain operands too
    assert nv.lib.nvfp4_gemm_takes_slabs(rows, rows, cols, fmt.c()) == 1
    ref = nv.gemm((pr, psr, pg), (pr, psr, pg), fmt, out_dtype=torch.bfloat16)
    for slabs in ((True, True), (True, False), (False, True)):
        A = (cr, sr, g) if slabs[0] else (pr, psr, pg)
        B = (cr, sr, g) if slabs[1] else (pr, psr, pg)
        got = nv.gemm(A, B, fmt, out_dtype=torch.bfloat16, slabs=slabs, shape=(rows, rows, cols))
        assert torch.equal(got, ref), slabs
    ref = nv.gemm((pc, psc, pg), (pc, psc, pg), fmt)
    got = nv.gemm((cc, sc, g), (cc, sc, g), fmt, slabs=(True, True), shape=(cols, cols, rows))
    assert torch.equal(got, ref)


@pytest.mark.parametrize("fmt_name", ["NVFP4", "MXFP4"])
@pytest.mark.parametrize("shape", [(4096, 4096, 256), (8192, 256, 8192), (2048, 2048, 2048), (4096, 640, 4096)],
                         ids=["fwd-only", "dX-only", "none-for-nvfp4", "mixed"])
def test_slab_layout_chosen_per_operand(shape, fmt_name, switches):
    # shapes where only some of the three GEMMs take slab operands (few output tiles, short K): each operand's
    # layout is decided by its own consumer, and every combination must equal the all-row-major run bit for bit
    M, N, K = shape
    fmt = getattr(nv, fmt_name)
    print(f"[case] per-operand slab choice M={M} N={N} K={K} {fmt_name}", flush=True)
    X = synth.normal(M, K, 1.0, 701).cuda()
    W = synth.normal(N, K, 0.02, 702).cuda()
    dY = synth.gradient_like(M, N, 703).cuda()
    outs = []
    for plain in ("0", "1"):
        nv.cross_check_switches(nv.SWITCH_PLAIN_OPERANDS if plain == "1" else 0)
        saved = torch.empty(nv.linear_saved_bytes(M, N, K, fmt), dtype=torch.uint8, device="cuda")
        Y = nv.linear_fwd(X, W, fmt, out_dtype=torch.bfloat16, saved=saved, bwd_seed=5)
        dX, dW = nv.linear_bwd(dY, None, None, 5, fmt, out_dtype=torch.bfloat16, saved=saved, K=K)
        torch.cuda.synchronize()
        outs.append((Y, dX, dW))
    for a, b, what in zip(outs[0], outs[1], ("Y", "dX", "dW")):
        assert torch.equal(a, b), what
    assert torch.isfinite(outs[0][0].float()).all() and torch.isfinite(outs[0][1].float()).all() and torch.isfinite(outs[0][2].float()).all()
