"""Pins for the oracle's dequantized GEMMs (Eqs. 4-6), CPU only."""
import numpy as np
import pytest

import oracle
from oracle import MXFP4, NVFP4, RTN, SR

GRID = np.array([0, 0.5, 1, 1.5, 2, 3, 4, 6], dtype=np.float64)
E4M3 = np.array([oracle.e4m3_decode(b) for b in range(127)], dtype=np.float64)


def unpack(codes):
    out = np.empty((codes.shape[0], codes.shape[1] * 2), np.uint8)
    out[:, 0::2] = codes & 15
    out[:, 1::2] = codes >> 4
    return out


def np_dequant(codes, scales, g, block=16, table=E4M3):
    """Independent statement of an operand's value, from the format tables."""
    u = unpack(codes)
    return np.where(u & 8, -1.0, 1.0) * GRID[u & 7] * np.repeat(table[scales], block, axis=1) * g


def test_dequantize_matches_format_tables():
    rng = np.random.default_rng(0)
    codes = rng.integers(0, 256, (8, 32)).astype(np.uint8)
    scales = rng.integers(0, 127, (8, 4)).astype(np.uint8)
    assert np.array_equal(oracle.dequantize(codes, scales, 0.375), np_dequant(codes, scales, 0.375))
    sc = rng.integers(100, 150, (8, 2)).astype(np.uint8)
    e8 = np.array([2.0 ** (b - 127) for b in range(255)])
    assert np.array_equal(oracle.dequantize(codes, sc, 1.0, MXFP4), np_dequant(codes, sc, 1.0, 32, e8))


def test_unit_scale_gemm_is_exact_integer_arithmetic():
    # all block scales 1 (byte 0x38), g = 1: every product is a multiple of 1/4 and the sum is
    # exactly an integer GEMM of the doubled element values, divided by 4
    rng = np.random.default_rng(1)
    M, N, K = 24, 40, 96
    ac = rng.integers(0, 256, (M, K // 2)).astype(np.uint8)
    bc = rng.integers(0, 256, (N, K // 2)).astype(np.uint8)
    ones_a = np.full((M, K // 16), 0x38, np.uint8)
    ones_b = np.full((N, K // 16), 0x38, np.uint8)
    two_grid = np.array([0, 1, 2, 3, 4, 6, 8, 12], dtype=np.int64)

    def ints(c):
        u = unpack(c)
        return np.where(u & 8, -1, 1) * two_grid[u & 7]

    want = (ints(ac) @ ints(bc).T).astype(np.float64) / 4.0
    got = oracle.gemm_nt((ac, ones_a, 1.0), (bc, ones_b, 1.0))
    assert np.array_equal(got, want)


def test_tiny_gemm_by_triple_loop():
    rng = np.random.default_rng(2)
    M, N, K = 3, 4, 32
    ac = rng.integers(0, 256, (M, K // 2)).astype(np.uint8)
    bc = rng.integers(0, 256, (N, K // 2)).astype(np.uint8)
    asc = rng.integers(0x20, 0x50, (M, K // 16)).astype(np.uint8)
    bsc = rng.integers(0x20, 0x50, (N, K // 16)).astype(np.uint8)
    ga, gb = 0.75, 1.5
    va, vb = np_dequant(ac, asc, ga), np_dequant(bc, bsc, gb)
    got = oracle.gemm_nt((ac, asc, ga), (bc, bsc, gb))
    for i in range(M):
        for j in range(N):
            acc = 0.0
            for k in range(K):
                acc += va[i, k] * vb[j, k]
            assert got[i, j] == acc


def test_gemm_equals_matmul_of_dequantized_and_is_linear_in_g():
    rng = np.random.default_rng(3)
    X = rng.standard_normal((48, 128)).astype(np.float32)
    W = (rng.standard_normal((64, 128)) * 0.02).astype(np.float32)
    A, B = oracle.quantize(X, 1, RTN), oracle.quantize(W, 1, RTN)
    Y = oracle.gemm_nt(A, B)
    ref = np_dequant(*A) @ np_dequant(*B).T
    Yabs = oracle.gemm_nt(A, B, take_abs=True)
    assert np.all(np.abs(Y - ref) <= 1e-13 * Yabs)  # fp64 summation-order noise only
    Y2 = oracle.gemm_nt((A[0], A[1], A[2] * 4.0), (B[0], B[1], B[2] * 0.5))
    assert np.array_equal(Y2, Y * 2.0)
    # |.| form bounds the signed form
    assert np.all(Yabs >= np.abs(Y)) and np.allclose(Yabs, np.abs(np_dequant(*A)) @ np.abs(np_dequant(*B)).T)


def test_sampled_entries_equal_full_product():
    rng = np.random.default_rng(4)
    X = rng.standard_normal((40, 64)).astype(np.float32)
    W = rng.standard_normal((24, 64)).astype(np.float32)
    A, B = oracle.quantize(X, 1, SR, 1), oracle.quantize(W, 1, RTN)
    full = oracle.gemm_nt(A, B)
    ii = rng.integers(0, 40, 50)
    jj = rng.integers(0, 24, 50)
    assert np.array_equal(oracle.gemm_nt_sample(A, B, ii, jj), full[ii, jj])
    assert np.array_equal(oracle.gemm_nt_sample(A, B, ii, jj, take_abs=True),
                          oracle.gemm_nt(A, B, take_abs=True)[ii, jj])


def test_quantized_linear_tracks_the_unquantized_one():
    # sanity only (the paper prints no number for this): NVFP4 forward stays within ~10 % of the
    # exact product in Frobenius norm for Gaussian data
    rng = np.random.default_rng(5)
    X = rng.standard_normal((64, 512)).astype(np.float32)
    W = (rng.standard_normal((96, 512)) * 0.02).astype(np.float32)
    Y = oracle.linear_fwd(X, W)
    ref = X.astype(np.float64) @ W.astype(np.float64).T
    rel = np.linalg.norm(Y - ref) / np.linalg.norm(ref)
    assert 0.01 < rel < 0.2


def test_backward_and_update_shapes_and_rounding_assignment():
    # Eqs. 5-6: dX = Q_SR(dY) Q_RtN(W) contracted over N; dW = Q_SR(dY)^T Q_SR(X) over M
    rng = np.random.default_rng(6)
    M, N, K = 32, 48, 64
    X = rng.standard_normal((M, K)).astype(np.float32)
    W = (rng.standard_normal((N, K)) * 0.05).astype(np.float32)
    dY = (rng.standard_normal((M, N)) * 1e-3).astype(np.float32)
    dX, dW = oracle.linear_bwd(dY, X, W, seed=10)
    assert dX.shape == (M, K) and dW.shape == (N, K)
    # operand by operand, with the tables
    qdy = oracle.quantize(dY, 1, SR, 10)
    qwt = oracle.quantize(W, 0, RTN)           # [K, N/2]: W^T blocked along N
    assert qwt[0].shape == (K, N // 2)
    assert np.allclose(dX, np_dequant(*qdy) @ np_dequant(*qwt).T, rtol=1e-9, atol=1e-12)
    qdyt = oracle.quantize(dY, 0, SR, 11)      # [N, M/2]
    qxt = oracle.quantize(X, 0, SR, 12)        # [K, M/2]
    assert np.allclose(dW, np_dequant(*qdyt) @ np_dequant(*qxt).T, rtol=1e-9, atol=1e-12)
    # the weight operand of the backward GEMM is deterministic, the gradient operand is not
    dX2, dW2 = oracle.linear_bwd(dY, X, W, seed=20)
    assert not np.array_equal(dX, dX2) and not np.array_equal(dW, dW2)
    # both track the exact gradients
    for got, ref in ((dX, dY.astype(np.float64) @ W), (dW, dY.astype(np.float64).T @ X)):
        assert np.linalg.norm(got - ref) / np.linalg.norm(ref) < 0.3


def test_sr_gradient_estimate_is_unbiased_rtn_is_not():
    # Sec. 4's premise, on the update GEMM: averaging dW over seeds converges to the exact
    # product; the deterministic rounding keeps a fixed error
    rng = np.random.default_rng(7)
    M, N, K = 32, 16, 16
    X = rng.standard_normal((M, K)).astype(np.float32)
    dY = (rng.standard_normal((M, N)) * 1e-3).astype(np.float32)
    ref = dY.astype(np.float64).T @ X
    acc = np.zeros_like(ref)
    S = 200
    for s in range(S):
        acc += oracle.gemm_nt(oracle.quantize(dY, 0, SR, 3 * s + 1), oracle.quantize(X, 0, SR, 3 * s + 2))
    one = oracle.gemm_nt(oracle.quantize(dY, 0, SR, 1), oracle.quantize(X, 0, SR, 2))
    err_mean = np.linalg.norm(acc / S - ref)
    err_one = np.linalg.norm(one - ref)
    assert err_mean < 3.0 * err_one / np.sqrt(S)
