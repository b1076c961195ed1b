"""Helpers shared by the GPU parity tests."""
import numpy as np
import torch

import oracle

GPU_TO_ORACLE_FMT = {}


def ofmt(fmt):
    """binding.Format -> oracle.Format (same three integers, separate modules)."""
    return oracle.Format(fmt.block, fmt.scale, fmt.tensor_scale)


def to_np(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().numpy()


def assert_quant_equal(got, want, what=""):
    """Bit-exact comparison of (codes, scales, g)."""
    gc, gs, gg = to_np(got[0]), to_np(got[1]), float(got[2].item())
    wc, ws, wg = want
    assert gg == wg, f"{what}: tensor scale {gg} != {wg}"
    if not np.array_equal(gs, ws):
        bad = np.argwhere(gs != ws)
        raise AssertionError(f"{what}: {len(bad)} scale bytes differ, first at {bad[0]}: "
                             f"{gs[tuple(bad[0])]:#x} != {ws[tuple(bad[0])]:#x}")
    if not np.array_equal(gc, wc):
        bad = np.argwhere(gc != wc)
        raise AssertionError(f"{what}: {len(bad)} code bytes differ, first at {bad[0]}: "
                             f"{gc[tuple(bad[0])]:#x} != {wc[tuple(bad[0])]:#x}")


REL_TOL = 1e-5  # the stated bar: fp32 accumulation against the fp64 oracle


def assert_gemm_close(Y: np.ndarray, ref: np.ndarray, ref_abs: np.ndarray, what="", tol=REL_TOL):
    """|Y - ref| <= tol * sum_k |a||b| element-wise, and tol in Frobenius norm."""
    Y = Y.astype(np.float64)
    err = np.abs(Y - ref)
    worst = (err / np.maximum(ref_abs, 1e-300)).max() if ref.size else 0.0
    assert np.all(err <= tol * ref_abs + 1e-300), f"{what}: element error {worst:.3e} x sum|a||b|"
    if ref.size:
        fro = np.linalg.norm(Y - ref) / max(np.linalg.norm(ref), 1e-300)
        assert fro <= tol, f"{what}: Frobenius relative error {fro:.3e}"


def _to_bf16_f64(a: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even of fp64 values to bf16, returned as fp64 (through fp32: every value
    used here is far from the fp32 rounding boundaries that could make the double rounding matter)."""
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float64)).to(torch.float32).to(torch.bfloat16).to(torch.float64).numpy()


def assert_bf16_gemm_close(Y: np.ndarray, ref: np.ndarray, ref_abs: np.ndarray, what="", tol=REL_TOL):
    """bf16 output of a GEMM whose fp32 result must lie within tol * sum_k |a||b| of ref: rounding
    to bf16 is monotonic, so the stored value must lie between the bf16 roundings of the two ends
    of that interval (no allowance beyond the one rounding the output format forces)."""
    Y = Y.astype(np.float64)
    slack = tol * ref_abs + 1e-300
    lo, hi = _to_bf16_f64(ref - slack * (1 + 1e-6)), _to_bf16_f64(ref + slack * (1 + 1e-6))
    bad = (Y < lo) | (Y > hi)
    if bad.any():
        t = np.argwhere(bad)[0]
        raise AssertionError(f"{what}: {int(bad.sum())} of {Y.size} bf16 outputs outside [bf16(ref - tol), bf16(ref + tol)], "
                             f"first at {tuple(t)}: got {Y[tuple(t)]!r}, ref {ref[tuple(t)]!r}")
