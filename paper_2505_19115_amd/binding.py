"""ctypes binding of libnvfp4.so: argument marshalling only.

Every function takes torch tensors that already live on the GPU, passes their
device pointers and the current HIP stream to the C ABI declared in
``include/nvfp4.h`` and returns torch tensors it allocated for the outputs.
No arithmetic of the method happens in Python, and there is no fallback: if
the library is missing, importing this module fails.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libnvfp4.so")

RTN, SR = 0, 1
F32, BF16 = 0, 1
SCALE_E4M3, SCALE_E8M0 = 0, 1
PRESET_TSCALE = 1
SLAB_ROWS = 2
SLAB_COLS = 4

OK, EINVAL, ESHAPE, EALIGN, EUNSUPPORTED, EWORKSPACE, EHIP = range(7)


class _DualOperands(C.Structure):
    _fields_ = [("codes_rows", C.c_void_p), ("scales_rows", C.c_void_p), ("codes_cols", C.c_void_p),
                ("scales_cols", C.c_void_p), ("g", C.c_void_p), ("layout", C.c_uint32)]


class _Format(C.Structure):
    _fields_ = [("block", C.c_int32), ("scale", C.c_int32), ("tensor_scale", C.c_int32)]


@dataclass(frozen=True)
class Format:
    block: int = 16
    scale: int = SCALE_E4M3
    tensor_scale: int = 1

    def c(self) -> _Format:
        return _Format(self.block, self.scale, self.tensor_scale)


NVFP4 = Format(16, SCALE_E4M3, 1)
MXFP4 = Format(32, SCALE_E8M0, 0)


class Nvfp4Error(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {lib.nvfp4_status_string(code).decode()} (status {code})")


def _load() -> C.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is not built: run `python -c 'import __graft_entry__ as g; g.build()'`")
    L = C.CDLL(LIB_PATH)
    vp, i64, u64, u32, sz, ci = C.c_void_p, C.c_int64, C.c_uint64, C.c_uint32, C.c_size_t, C.c_int
    fp = C.POINTER(_Format)
    L.nvfp4_status_string.restype = C.c_char_p
    L.nvfp4_status_string.argtypes = [ci]
    L.nvfp4_codes_bytes.restype = sz
    L.nvfp4_codes_bytes.argtypes = [i64, i64]
    L.nvfp4_scales_bytes.restype = sz
    L.nvfp4_scales_bytes.argtypes = [i64, i64, ci, fp]
    L.nvfp4_quantize_workspace_bytes.restype = sz
    L.nvfp4_quantize_workspace_bytes.argtypes = [i64, i64]
    L.nvfp4_linear_fwd_workspace_bytes.restype = sz
    L.nvfp4_linear_fwd_workspace_bytes.argtypes = [i64, i64, i64, fp]
    L.nvfp4_linear_bwd_workspace_bytes.restype = sz
    L.nvfp4_linear_bwd_workspace_bytes.argtypes = [i64, i64, i64, fp]
    L.nvfp4_tensor_scale.restype = ci
    L.nvfp4_tensor_scale.argtypes = [vp, ci, i64, i64, i64, vp, vp, sz, vp]
    L.nvfp4_quantize.restype = ci
    L.nvfp4_quantize.argtypes = [vp, ci, i64, i64, i64, ci, ci, u64, fp, vp, vp, vp, u32, vp, sz, vp]
    L.nvfp4_quantize_static.restype = ci
    L.nvfp4_quantize_static.argtypes = [vp, ci, i64, i64, i64, ci, ci, u64, fp, vp, vp, vp, u32, vp]
    L.nvfp4_cross_check_switches.restype = u32
    L.nvfp4_cross_check_switches.argtypes = [ci, u32]
    L.nvfp4_quantize_dual.restype = ci
    L.nvfp4_quantize_dual.argtypes = [vp, ci, i64, i64, i64, ci, u64, ci, u64, fp, vp, vp, vp, vp, vp, u32, vp, sz, vp]
    L.nvfp4_gemm.restype = ci
    L.nvfp4_gemm.argtypes = [i64, i64, i64, fp, vp, vp, vp, vp, vp, vp, ci, i64, vp]
    L.nvfp4_gemm_slab.restype = ci
    L.nvfp4_gemm_slab.argtypes = [i64, i64, i64, fp, vp, vp, vp, vp, vp, vp, ci, i64, ci, ci, vp]
    L.nvfp4_gemm_takes_slabs.restype = ci
    L.nvfp4_gemm_takes_slabs.argtypes = [i64, i64, i64, fp]
    L.nvfp4_slab_codes_bytes.restype = sz
    L.nvfp4_slab_codes_bytes.argtypes = [i64, i64]
    L.nvfp4_slab_scales_bytes.restype = sz
    L.nvfp4_slab_scales_bytes.argtypes = [i64, i64]
    L.nvfp4_linear_fwd.restype = ci
    L.nvfp4_linear_fwd.argtypes = [vp, vp, vp, i64, i64, i64, ci, ci, fp, vp, sz, vp, vp, vp, u64]
    L.nvfp4_linear_bwd.restype = ci
    L.nvfp4_linear_bwd.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, ci, ci, fp, u64, vp, sz, vp, vp, vp]
    L.nvfp4_linear_fwd_wq.restype = ci
    L.nvfp4_linear_fwd_wq.argtypes = L.nvfp4_linear_fwd.argtypes
    L.nvfp4_linear_bwd_wq.restype = ci
    L.nvfp4_linear_bwd_wq.argtypes = L.nvfp4_linear_bwd.argtypes
    L.nvfp4_weight_operands_bytes.restype = sz
    L.nvfp4_weight_operands_bytes.argtypes = [i64, i64, fp]
    L.nvfp4_quantize_weight.restype = ci
    L.nvfp4_quantize_weight.argtypes = [vp, ci, i64, i64, i64, fp, vp, vp, sz, vp]
    dp = C.POINTER(_DualOperands)
    L.nvfp4_swiglu_bwd_workspace_bytes.restype = sz
    L.nvfp4_swiglu_bwd_workspace_bytes.argtypes = [i64, i64]
    L.nvfp4_swiglu_bwd_quantize.restype = ci
    L.nvfp4_swiglu_bwd_quantize.argtypes = [vp, vp, vp, ci, i64, i64, u64, u64, fp, dp, dp, vp, vp, vp, sz, vp]
    L.nvfp4_linear_bwd_dyq.restype = ci
    L.nvfp4_linear_bwd_dyq.argtypes = [dp, vp, vp, vp, vp, vp, i64, i64, i64, ci, ci, fp, u64, vp, sz, vp, vp, vp]
    L.nvfp4_swiglu_bwd.restype = ci
    L.nvfp4_swiglu_bwd.argtypes = [vp, vp, vp, ci, i64, vp, vp, vp]
    L.nvfp4_host_swiglu_bwd.restype = None
    L.nvfp4_host_swiglu_bwd.argtypes = [vp, vp, vp, i64, vp, vp]
    L.nvfp4_linear_saved_bytes.restype = sz
    L.nvfp4_linear_saved_bytes.argtypes = [i64, i64, i64, fp]
    # host probes
    L.nvfp4_host_e4m3_encode.restype = C.c_uint8
    L.nvfp4_host_e4m3_encode.argtypes = [C.c_float]
    L.nvfp4_host_e4m3_decode.restype = C.c_float
    L.nvfp4_host_e4m3_decode.argtypes = [C.c_uint8]
    L.nvfp4_host_round_rtn.restype = C.c_uint8
    L.nvfp4_host_round_rtn.argtypes = [C.c_float]
    L.nvfp4_host_round_sr.restype = C.c_uint8
    L.nvfp4_host_round_sr.argtypes = [C.c_float, u32]
    L.nvfp4_host_philox4x32_10.restype = None
    L.nvfp4_host_philox4x32_10.argtypes = [vp, vp, vp]
    L.nvfp4_host_sr_bits.restype = u32
    L.nvfp4_host_sr_bits.argtypes = [u64, u64]
    L.nvfp4_host_e8m0_encode.restype = C.c_uint8
    L.nvfp4_host_e8m0_encode.argtypes = [C.c_float]
    L.nvfp4_host_e4m3_encode_n.restype = None
    L.nvfp4_host_e4m3_encode_n.argtypes = [vp, i64, vp]
    L.nvfp4_host_round_rtn_n.restype = None
    L.nvfp4_host_round_rtn_n.argtypes = [vp, i64, vp]
    L.nvfp4_host_round_sr_n.restype = None
    L.nvfp4_host_round_sr_n.argtypes = [vp, vp, i64, vp]
    L.nvfp4_quant_noise_workspace_bytes.restype = C.c_size_t
    L.nvfp4_quant_noise_workspace_bytes.argtypes = [i64, i64, C.c_int]
    L.nvfp4_quant_noise.restype = C.c_int
    L.nvfp4_quant_noise.argtypes = [vp, C.c_int, i64, i64, i64, C.c_int, C.POINTER(_Format), vp, vp, vp, vp, vp,
                                    C.c_size_t, vp]
    L.nvfp4_probe_mfma_rate.restype = C.c_int
    L.nvfp4_probe_mfma_rate.argtypes = [C.c_int, C.c_int, C.c_int, vp, C.c_size_t, C.POINTER(C.c_double), vp]
    return L


lib = _load()

EXPORTS = (
    "nvfp4_status_string", "nvfp4_codes_bytes", "nvfp4_scales_bytes",
    "nvfp4_quantize_workspace_bytes", "nvfp4_linear_fwd_workspace_bytes",
    "nvfp4_linear_bwd_workspace_bytes", "nvfp4_linear_saved_bytes", "nvfp4_tensor_scale", "nvfp4_quantize", "nvfp4_quantize_dual", "nvfp4_gemm",
    "nvfp4_gemm_slab", "nvfp4_gemm_takes_slabs", "nvfp4_slab_codes_bytes", "nvfp4_slab_scales_bytes",
    "nvfp4_linear_fwd", "nvfp4_linear_bwd", "nvfp4_host_e4m3_encode", "nvfp4_host_e4m3_decode",
    "nvfp4_host_round_rtn", "nvfp4_host_round_sr", "nvfp4_host_philox4x32_10",
    "nvfp4_host_sr_bits", "nvfp4_host_e8m0_encode", "nvfp4_host_e4m3_encode_n",
    "nvfp4_host_round_rtn_n", "nvfp4_host_round_sr_n", "nvfp4_probe_mfma_rate",
    "nvfp4_quant_noise_workspace_bytes", "nvfp4_quant_noise", "nvfp4_quantize_static", "nvfp4_cross_check_switches",
    "nvfp4_weight_operands_bytes", "nvfp4_quantize_weight", "nvfp4_linear_fwd_wq", "nvfp4_linear_bwd_wq",
    "nvfp4_swiglu_bwd_workspace_bytes", "nvfp4_swiglu_bwd_quantize", "nvfp4_linear_bwd_dyq", "nvfp4_host_swiglu_bwd", "nvfp4_swiglu_bwd",
)


def _dtype_tag(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def _torch_dtype(tag: int) -> torch.dtype:
    return torch.float32 if tag == F32 else torch.bfloat16


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _check(code: int, where: str) -> None:
    if code != OK:
        raise Nvfp4Error(code, where)


def _require_gpu(*ts: torch.Tensor) -> None:
    for t in ts:
        if t is not None and not t.is_cuda:
            raise ValueError("tensors must live on the GPU")


def tensor_scale(x: torch.Tensor) -> torch.Tensor:
    """nvfp4_tensor_scale: g = max|x| / 2688 as a device fp32[1] tensor."""
    _require_gpu(x)
    assert x.dim() == 2 and x.stride(1) == 1
    g = torch.empty(1, dtype=torch.float32, device=x.device)
    ws = torch.empty(lib.nvfp4_quantize_workspace_bytes(*x.shape), dtype=torch.uint8, device=x.device)
    _check(lib.nvfp4_tensor_scale(x.data_ptr(), _dtype_tag(x), x.shape[0], x.shape[1], x.stride(0),
                                  g.data_ptr(), ws.data_ptr(), ws.numel(), _stream()), "nvfp4_tensor_scale")
    return g


def quantize(x: torch.Tensor, axis: int = 1, rounding: int = RTN, seed: int = 0,
             fmt: Format = NVFP4, tensor_scale: torch.Tensor | None = None, out=None):
    """nvfp4_quantize -> (codes u8 [outer, inner/2], scales u8 [outer, inner/block], g fp32[1]).

    `tensor_scale` presets g (device fp32[1]); it is then used and returned as is.
    `out` = (codes, scales, g) reuses caller-provided output tensors.
    """
    _require_gpu(x, tensor_scale)
    assert x.dim() == 2 and (x.stride(1) == 1 or x.shape[1] <= 1)
    rows, cols = x.shape
    ld = x.stride(0) if rows > 1 else cols
    outer, inner = (rows, cols) if axis == 1 else (cols, rows)
    f = fmt.c()
    if out is None:
        codes = torch.empty((outer, inner // 2), dtype=torch.uint8, device=x.device)
        scales = torch.empty((outer, inner // fmt.block), dtype=torch.uint8, device=x.device)
        g = torch.empty(1, dtype=torch.float32, device=x.device) if tensor_scale is None else tensor_scale
    else:
        codes, scales, g = out
        if tensor_scale is not None:
            g = tensor_scale
    flags = PRESET_TSCALE if tensor_scale is not None else 0
    ws = torch.empty(lib.nvfp4_quantize_workspace_bytes(rows, cols), dtype=torch.uint8, device=x.device)
    _check(lib.nvfp4_quantize(x.data_ptr(), _dtype_tag(x), rows, cols, ld, axis, rounding, seed,
                              C.byref(f), codes.data_ptr(), scales.data_ptr(), g.data_ptr(), flags,
                              ws.data_ptr(), ws.numel(), _stream()), "nvfp4_quantize")
    return codes, scales, g


def quantize_static(x: torch.Tensor, axis: int = 1, rounding: int = RTN, seed: int = 0, fmt: Format = NVFP4,
                    tensor_scale: torch.Tensor | None = None, out=None):
    """nvfp4_quantize_static: nvfp4_quantize on the library's own static scratch (no workspace argument).
    `out` = (codes, scales, g) must be given by a caller that may not allocate; otherwise torch allocates them."""
    _require_gpu(x, tensor_scale)
    assert x.dim() == 2 and (x.stride(1) == 1 or x.shape[1] <= 1)
    rows, cols = x.shape
    ld = x.stride(0) if rows > 1 else cols
    outer, inner = (rows, cols) if axis == 1 else (cols, rows)
    f = fmt.c()
    if out is None:
        codes = torch.empty((outer, inner // 2), dtype=torch.uint8, device=x.device)
        scales = torch.empty((outer, inner // fmt.block), dtype=torch.uint8, device=x.device)
        g = torch.empty(1, dtype=torch.float32, device=x.device) if tensor_scale is None else tensor_scale
    else:
        codes, scales, g = out
        if tensor_scale is not None:
            g = tensor_scale
    flags = PRESET_TSCALE if tensor_scale is not None else 0
    _check(lib.nvfp4_quantize_static(x.data_ptr(), _dtype_tag(x), rows, cols, ld, axis, rounding, seed,
                                     C.byref(f), codes.data_ptr(), scales.data_ptr(), g.data_ptr(), flags,
                                     _stream()), "nvfp4_quantize_static")
    return codes, scales, g


SWITCH_SOFT_CONVERT, SWITCH_PLAIN_OPERANDS, SWITCH_FP4_WIDE_BLOCKS = 1, 2, 4


def cross_check_switches(value: int | None = None) -> int:
    """nvfp4_cross_check_switches: returns the switches in force; with `value` given, replaces them."""
    return lib.nvfp4_cross_check_switches(0 if value is None else 1, 0 if value is None else value)


def slab_scales_bytes(rows: int, K: int, fmt: Format = NVFP4) -> int:
    """Bytes of an operand's scale slabs: nvfp4_slab_scales_bytes is stated for blocks of 16 (8 bytes per row and
    K tile); MXFP4's slabs hold 4 bytes per row and K tile."""
    return lib.nvfp4_slab_scales_bytes(rows, K) * 16 // fmt.block


def quantize_dual(x: torch.Tensor, rounding_rows: int = RTN, seed_rows: int = 0, rounding_cols: int = RTN,
                  seed_cols: int = 0, fmt: Format = NVFP4, tensor_scale: torch.Tensor | None = None, out=None,
                  slab_rows: bool = False, slab_cols: bool = False):
    """nvfp4_quantize_dual -> ((codes [rows, cols/2], scales [rows, cols/block], g),
    (codes [cols, rows/2], scales [cols, rows/block], g)): both orientations, one shared g.

    `out` = (codes_rows, scales_rows, codes_cols, scales_cols, g) reuses caller-provided tensors.
    slab_rows / slab_cols: that side comes back in the slab layout instead (flat byte tensors of
    nvfp4_slab_codes_bytes / slab_scales_bytes), for gemm(..., slabs=...).
    """
    _require_gpu(x, tensor_scale)
    assert x.dim() == 2 and (x.stride(1) == 1 or x.shape[1] <= 1)
    rows, cols = x.shape
    ld = x.stride(0) if rows > 1 else cols
    f = fmt.c()
    if out is None:
        cr = torch.empty((rows, cols // 2), dtype=torch.uint8, device=x.device)
        sr = torch.empty((rows, cols // fmt.block), dtype=torch.uint8, device=x.device)
        cc = torch.empty((cols, rows // 2), dtype=torch.uint8, device=x.device)
        sc = torch.empty((cols, rows // fmt.block), dtype=torch.uint8, device=x.device)
        if slab_rows:
            cr = torch.empty(lib.nvfp4_slab_codes_bytes(rows, cols), dtype=torch.uint8, device=x.device)
            sr = torch.empty(slab_scales_bytes(rows, cols, fmt), dtype=torch.uint8, device=x.device)
        if slab_cols:
            cc = torch.empty(lib.nvfp4_slab_codes_bytes(cols, rows), dtype=torch.uint8, device=x.device)
            sc = torch.empty(slab_scales_bytes(cols, rows, fmt), dtype=torch.uint8, device=x.device)
        g = torch.empty(1, dtype=torch.float32, device=x.device) if tensor_scale is None else tensor_scale
    else:
        cr, sr, cc, sc, g = out
        if tensor_scale is not None:
            g = tensor_scale
    flags = (PRESET_TSCALE if tensor_scale is not None else 0) | (SLAB_ROWS if slab_rows else 0) | (SLAB_COLS if slab_cols else 0)
    ws = torch.empty(lib.nvfp4_quantize_workspace_bytes(rows, cols), dtype=torch.uint8, device=x.device)
    _check(lib.nvfp4_quantize_dual(x.data_ptr(), _dtype_tag(x), rows, cols, ld, rounding_rows, seed_rows, rounding_cols, seed_cols,
                                   C.byref(f), cr.data_ptr(), sr.data_ptr(), cc.data_ptr(), sc.data_ptr(),
                                   g.data_ptr(), flags, ws.data_ptr(), ws.numel(), _stream()), "nvfp4_quantize_dual")
    return (cr, sr, g), (cc, sc, g)


def gemm(A, B, fmt: Format = NVFP4, out_dtype: torch.dtype = torch.float32, out=None, slabs=(False, False),
         shape=None, tensor_scales: torch.Tensor | None = None) -> torch.Tensor:
    """nvfp4_gemm: A = (codes [M,K/2], scales, g[1]), B = (codes [N,K/2], scales, g[1]) -> [M, N].
    slabs = (a, b): that operand is in the slab layout (nvfp4_gemm_slab); then shape = (M, N, K) is required,
    since a flat slab buffer does not carry it."""
    (ac, asc, ga), (bc, bsc, gb) = A, B
    _require_gpu(ac, asc, ga, bc, bsc, gb)
    if shape is None:
        assert not (slabs[0] or slabs[1]), "slab operands: pass shape=(M, N, K)"
        M, N, K = ac.shape[0], bc.shape[0], ac.shape[1] * 2
    else:
        M, N, K = shape
    # {gA, gB} side by side: as given (a caller that keeps them so), else gathered here
    ts = torch.cat([ga.reshape(1), gb.reshape(1)]) if tensor_scales is None else tensor_scales
    if out is None:
        out = torch.empty((M, N), dtype=out_dtype, device=ac.device)
    f = fmt.c()
    _check(lib.nvfp4_gemm_slab(M, N, K, C.byref(f), ac.data_ptr(), asc.data_ptr(), bc.data_ptr(),
                               bsc.data_ptr(), ts.data_ptr(), out.data_ptr(), _dtype_tag(out),
                               out.stride(0), int(bool(slabs[0])), int(bool(slabs[1])), _stream()), "nvfp4_gemm")
    return out


def linear_fwd(X: torch.Tensor, W: torch.Tensor, fmt: Format = NVFP4,
               out_dtype: torch.dtype = torch.float32, workspace: torch.Tensor | None = None,
               out: torch.Tensor | None = None, scales_out: torch.Tensor | None = None,
               saved: torch.Tensor | None = None, bwd_seed: int = 0, w_operands: torch.Tensor | None = None,
               N: int | None = None) -> torch.Tensor:
    """nvfp4_linear_fwd (Eq. 4): Y[M,N] = Q_RtN(X[M,K]) Q_RtN(W[N,K])^T.
    w_operands: what quantize_weight wrote for W (then W may be None, pass N): nvfp4_linear_fwd_wq.
    scales_out: device fp32[2] that receives {gX, gW} for linear_bwd(..., xw_scales=...).
    saved: device u8 buffer of linear_saved_bytes(M, N, K, fmt) that receives Q_SR(X^T), Q_RtN(W^T) and the
    scales for linear_bwd(..., seed=bwd_seed, saved=saved)."""
    _require_gpu(X, *([W] if W is not None else []))
    assert X.is_contiguous() and (W is None or (W.is_contiguous() and X.dtype == W.dtype))
    assert (W is None) != (w_operands is None), "give W or w_operands"
    M, K = X.shape
    N = W.shape[0] if W is not None else N
    f = fmt.c()
    if workspace is None:
        workspace = torch.empty(lib.nvfp4_linear_fwd_workspace_bytes(M, N, K, C.byref(f)),
                                dtype=torch.uint8, device=X.device)
    Y = torch.empty((M, N), dtype=out_dtype, device=X.device) if out is None else out
    entry = lib.nvfp4_linear_fwd if w_operands is None else lib.nvfp4_linear_fwd_wq
    _check(entry(X.data_ptr(), (W if w_operands is None else w_operands).data_ptr(), Y.data_ptr(), M, N, K, _dtype_tag(X),
                 _dtype_tag(Y), C.byref(f), workspace.data_ptr(), workspace.numel(),
                 _stream(), None if scales_out is None else scales_out.data_ptr(),
                 None if saved is None else saved.data_ptr(), bwd_seed),
           "nvfp4_linear_fwd")
    return Y


def linear_bwd(dY: torch.Tensor, X: torch.Tensor, W: torch.Tensor, seed: int, fmt: Format = NVFP4,
               out_dtype: torch.dtype = torch.float32, workspace: torch.Tensor | None = None,
               out=None, xw_scales: torch.Tensor | None = None, saved: torch.Tensor | None = None,
               K: int | None = None, w_operands: torch.Tensor | None = None):
    """nvfp4_linear_bwd (Eqs. 5-6) -> (dX [M,K], dW [N,K]).
    w_operands: what quantize_weight wrote for W (then W is not read): nvfp4_linear_bwd_wq.
    xw_scales: device fp32[2] = {gX, gW} from linear_fwd(..., scales_out=...) for the same X and W.
    saved: what linear_fwd(..., saved=..., bwd_seed=seed) wrote; X and W may then be None (pass K)."""
    _require_gpu(dY, *[t for t in (X, W) if t is not None])
    assert dY.is_contiguous() and (X is None or X.is_contiguous()) and (W is None or W.is_contiguous())
    assert saved is not None or (X is not None and (W is not None or w_operands is not None))
    M, N = dY.shape
    K = K if K is not None else (X.shape[1] if X is not None else W.shape[1])
    f = fmt.c()
    if workspace is None:
        workspace = torch.empty(lib.nvfp4_linear_bwd_workspace_bytes(M, N, K, C.byref(f)),
                                dtype=torch.uint8, device=dY.device)
    if out is None:
        dX = torch.empty((M, K), dtype=out_dtype, device=dY.device)
        dW = torch.empty((N, K), dtype=out_dtype, device=dY.device)
    else:
        dX, dW = out
    entry = lib.nvfp4_linear_bwd if w_operands is None else lib.nvfp4_linear_bwd_wq
    third = w_operands if w_operands is not None else W
    _check(entry(dY.data_ptr(), None if X is None else X.data_ptr(),
                                None if third is None else third.data_ptr(), dX.data_ptr(),
                                dW.data_ptr(), M, N, K, _dtype_tag(dY), _dtype_tag(dX), C.byref(f),
                                seed, workspace.data_ptr(), workspace.numel(), _stream(),
                                None if xw_scales is None else xw_scales.data_ptr(),
                                None if saved is None else saved.data_ptr()),
           "nvfp4_linear_bwd")
    return dX, dW


@dataclass
class DualOperands:
    """A tensor quantized along both axes (nvfp4_dual_operands): rows side, columns side, shared g, layout bits."""
    codes_rows: torch.Tensor
    scales_rows: torch.Tensor
    codes_cols: torch.Tensor
    scales_cols: torch.Tensor
    g: torch.Tensor
    layout: int = 0

    def c(self) -> _DualOperands:
        return _DualOperands(self.codes_rows.data_ptr(), self.scales_rows.data_ptr(), self.codes_cols.data_ptr(),
                             self.scales_cols.data_ptr(), self.g.data_ptr(), self.layout)

    @property
    def rows(self):
        return self.codes_rows, self.scales_rows, self.g

    @property
    def cols(self):
        return self.codes_cols, self.scales_cols, self.g


def empty_dual_operands(rows: int, cols: int, fmt: Format = NVFP4, slab_rows: bool = False, slab_cols: bool = False,
                        device="cuda") -> DualOperands:
    """Output buffers for a [rows, cols] tensor quantized along both axes (row-major, or slabs per side)."""
    u8 = dict(dtype=torch.uint8, device=device)
    cr = torch.empty(lib.nvfp4_slab_codes_bytes(rows, cols), **u8) if slab_rows else torch.empty((rows, cols // 2), **u8)
    cc = torch.empty(lib.nvfp4_slab_codes_bytes(cols, rows), **u8) if slab_cols else torch.empty((cols, rows // 2), **u8)
    sr = torch.empty(slab_scales_bytes(rows, cols, fmt), **u8) if slab_rows else torch.empty((rows, cols // fmt.block), **u8)
    sc = torch.empty(slab_scales_bytes(cols, rows, fmt), **u8) if slab_cols else torch.empty((cols, rows // fmt.block), **u8)
    return DualOperands(cr, sr, cc, sc, torch.empty(1, dtype=torch.float32, device=device),
                        (SLAB_ROWS if slab_rows else 0) | (SLAB_COLS if slab_cols else 0))


def swiglu_bwd_quantize(dH: torch.Tensor, G: torch.Tensor, U: torch.Tensor, seed_gate: int, seed_up: int,
                        fmt: Format = NVFP4, slab_rows: bool = False, slab_cols: bool = False, out=None, store=None):
    """nvfp4_swiglu_bwd_quantize -> (dG, dU) as DualOperands: Q_SR of the SwiGLU backward's two results, both
    orientations each.  `out` = (dG, dU) reuses caller-provided buffers.  `store` = (dG_tensor, dU_tensor) of the
    inputs' shape and dtype: the results are also stored there (and read back by the quantizer passes); None:
    nothing but the operands is written."""
    _require_gpu(dH, G, U)
    assert dH.is_contiguous() and G.is_contiguous() and U.is_contiguous() and dH.shape == G.shape == U.shape
    assert dH.dtype == G.dtype == U.dtype
    M, F = dH.shape
    f = fmt.c()
    dG, dU = out if out is not None else (empty_dual_operands(M, F, fmt, slab_rows, slab_cols, dH.device),
                                          empty_dual_operands(M, F, fmt, slab_rows, slab_cols, dH.device))
    ws = torch.empty(lib.nvfp4_swiglu_bwd_workspace_bytes(M, F), dtype=torch.uint8, device=dH.device)
    cg, cu = dG.c(), dU.c()
    _check(lib.nvfp4_swiglu_bwd_quantize(dH.data_ptr(), G.data_ptr(), U.data_ptr(), _dtype_tag(dH), M, F, seed_gate, seed_up,
                                         C.byref(f), C.byref(cg), C.byref(cu),
                                         None if store is None else store[0].data_ptr(), None if store is None else store[1].data_ptr(),
                                         ws.data_ptr(), ws.numel(), _stream()),
           "nvfp4_swiglu_bwd_quantize")
    return dG, dU


def swiglu_bwd(dH: torch.Tensor, G: torch.Tensor, U: torch.Tensor, out=None):
    """nvfp4_swiglu_bwd -> (dG, dU) tensors of the inputs' dtype (the elementwise step alone)."""
    _require_gpu(dH, G, U)
    assert dH.is_contiguous() and G.is_contiguous() and U.is_contiguous() and dH.shape == G.shape == U.shape
    dG, dU = out if out is not None else (torch.empty_like(dH), torch.empty_like(dH))
    _check(lib.nvfp4_swiglu_bwd(dH.data_ptr(), G.data_ptr(), U.data_ptr(), _dtype_tag(dH), dH.numel(), dG.data_ptr(),
                                dU.data_ptr(), _stream()), "nvfp4_swiglu_bwd")
    return dG, dU


def linear_bwd_dyq(dyq: DualOperands, X, W, seed: int, M: int, N: int, K: int, fmt: Format = NVFP4,
                   in_dtype: torch.dtype = torch.bfloat16, out_dtype: torch.dtype = torch.float32,
                   workspace: torch.Tensor | None = None, out=None, xw_scales: torch.Tensor | None = None,
                   saved: torch.Tensor | None = None, w_operands: torch.Tensor | None = None):
    """nvfp4_linear_bwd_dyq (Eqs. 5-6 on an upstream gradient that is already quantized) -> (dX [M,K], dW [N,K])."""
    f = fmt.c()
    dev = dyq.g.device
    if workspace is None:
        workspace = torch.empty(lib.nvfp4_linear_bwd_workspace_bytes(M, N, K, C.byref(f)), dtype=torch.uint8, device=dev)
    if out is None:
        dX = torch.empty((M, K), dtype=out_dtype, device=dev)
        dW = torch.empty((N, K), dtype=out_dtype, device=dev)
    else:
        dX, dW = out
    cd = dyq.c()
    ptr = lambda t: None if t is None else t.data_ptr()
    _check(lib.nvfp4_linear_bwd_dyq(C.byref(cd), ptr(X), ptr(W), ptr(w_operands), dX.data_ptr(), dW.data_ptr(), M, N, K,
                                    BF16 if in_dtype == torch.bfloat16 else F32, _dtype_tag(dX), C.byref(f), seed,
                                    workspace.data_ptr(), workspace.numel(), _stream(), ptr(xw_scales), ptr(saved)),
           "nvfp4_linear_bwd_dyq")
    return dX, dW


def quantize_weight(W: torch.Tensor, M: int, fmt: Format = NVFP4, out: torch.Tensor | None = None) -> torch.Tensor:
    """nvfp4_quantize_weight: W [N, K] -> the library's weight-operand buffer (u8) for micro-batches of M tokens."""
    _require_gpu(W)
    assert W.dim() == 2 and W.is_contiguous()
    N, K = W.shape
    f = fmt.c()
    if out is None:
        out = torch.empty(lib.nvfp4_weight_operands_bytes(N, K, C.byref(f)), dtype=torch.uint8, device=W.device)
    ws = torch.empty(lib.nvfp4_quantize_workspace_bytes(N, K), dtype=torch.uint8, device=W.device)
    _check(lib.nvfp4_quantize_weight(W.data_ptr(), _dtype_tag(W), M, N, K, C.byref(f), out.data_ptr(), ws.data_ptr(),
                                     ws.numel(), _stream()), "nvfp4_quantize_weight")
    return out


def linear_saved_bytes(M: int, N: int, K: int, fmt: Format = NVFP4) -> int:
    f = fmt.c()
    return lib.nvfp4_linear_saved_bytes(M, N, K, C.byref(f))


MFMA_F16, MFMA_FP4 = 0, 1


def probe_mfma_rate(kind: int, random_operands: bool, iters: int = 20000) -> float:
    """nvfp4_probe_mfma_rate -> sustained TFLOP/s of the matrix instruction on the current device."""
    assert torch.cuda.is_available(), "the probe runs on the GPU"
    cus = torch.cuda.get_device_properties(torch.cuda.current_device()).multi_processor_count
    scratch = torch.empty(cus * 512, dtype=torch.float32, device="cuda")
    out = C.c_double(0.0)
    _check(lib.nvfp4_probe_mfma_rate(kind, int(bool(random_operands)), iters, scratch.data_ptr(),
                                     scratch.numel() * 4, C.byref(out), _stream()), "nvfp4_probe_mfma_rate")
    return out.value


def quant_noise(x: torch.Tensor, q, axis: int = 1, fmt: Format = NVFP4, out: torch.Tensor | None = None,
                workspace: torch.Tensor | None = None) -> torch.Tensor:
    """nvfp4_quant_noise (Sec. 4 monitor): device double[2] = (sum x^2, sum (Q(x) - x)^2) for q = (codes, scales, g)
    as quantize(x, axis, ..., fmt) returned."""
    _require_gpu(x)
    assert x.dim() == 2 and x.stride(1) == 1
    rows, cols = x.shape
    codes, scales, g = q
    f = fmt.c()
    ws = workspace
    if ws is None:
        ws = torch.empty(max(lib.nvfp4_quant_noise_workspace_bytes(rows, cols, axis), 16), dtype=torch.uint8, device=x.device)
    if out is None:
        out = torch.empty(2, dtype=torch.float64, device=x.device)
    _check(lib.nvfp4_quant_noise(x.data_ptr(), _dtype_tag(x), rows, cols, x.stride(0) if rows > 1 else cols, axis,
                                 C.byref(f), codes.data_ptr(), scales.data_ptr(), g.data_ptr(), out.data_ptr(),
                                 ws.data_ptr(), ws.numel(), _stream()), "nvfp4_quant_noise")
    return out
