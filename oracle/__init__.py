"""CPU oracle for the FP4 quantized linear layer -- TEST INFRASTRUCTURE.

Thin ctypes access to ``nvfp4_oracle.c`` (plain C, fp32 scale arithmetic, fp64
GEMM accumulation) plus the composition of its steps into the forward,
backward and update GEMMs of Eqs. 4-6 of the paper.  Nothing in the product
package imports this module; only ``tests/``, the smoke check and the
benchmark's ``cpu_baseline`` leg do.  It shares no code with the HIP library.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "nvfp4_oracle.c")
_LIB = os.path.join(_HERE, "libnvfp4_oracle.so")

RTN, SR = 0, 1
F32, BF16 = 0, 1
SCALE_E4M3, SCALE_E8M0 = 0, 1


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (strict IEEE: no contraction, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
             "-fno-fast-math", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"])
    return _LIB


class _Format(C.Structure):
    _fields_ = [("block", C.c_int32), ("scale_fmt", C.c_int32), ("tensor_scale", C.c_int32)]


@dataclass(frozen=True)
class Format:
    """Block format: NVFP4 = (16, E4M3, tensor scale), MXFP4 = (32, E8M0, none)."""
    block: int = 16
    scale_fmt: int = SCALE_E4M3
    tensor_scale: int = 1

    def c(self) -> _Format:
        return _Format(self.block, self.scale_fmt, self.tensor_scale)


NVFP4 = Format(16, SCALE_E4M3, 1)
MXFP4 = Format(32, SCALE_E8M0, 0)

_lib = None


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(build())
        L.orc_e2m1_decode.restype = C.c_float
        L.orc_e2m1_decode.argtypes = [C.c_uint8]
        L.orc_e4m3_decode.restype = C.c_float
        L.orc_e4m3_decode.argtypes = [C.c_uint8]
        L.orc_e4m3_encode.restype = C.c_uint8
        L.orc_e4m3_encode.argtypes = [C.c_float]
        L.orc_e8m0_decode.restype = C.c_float
        L.orc_e8m0_decode.argtypes = [C.c_uint8]
        L.orc_sr_bits.restype = C.c_uint32
        L.orc_sr_bits.argtypes = [C.c_uint64, C.c_uint64]
        L.orc_round_rtn.restype = C.c_uint8
        L.orc_round_rtn.argtypes = [C.c_float]
        L.orc_round_sr.restype = C.c_uint8
        L.orc_round_sr.argtypes = [C.c_float, C.c_uint32]
        L.orc_tensor_amax.restype = C.c_float
        L.orc_tensor_amax.argtypes = [C.c_void_p, C.c_int, C.c_int64, C.c_int64, C.c_int64]
        L.orc_tensor_scale_from_amax.restype = C.c_float
        L.orc_tensor_scale_from_amax.argtypes = [C.c_float]
        L.orc_quantize.restype = C.c_int
        L.orc_quantize.argtypes = [C.c_void_p, C.c_int, C.c_int64, C.c_int64, C.c_int64, C.c_int,
                                   C.c_int, C.c_uint64, C.POINTER(_Format), C.c_void_p,
                                   C.c_void_p, C.POINTER(C.c_float), C.c_int]
        L.orc_dequantize.restype = None
        L.orc_dequantize.argtypes = [C.c_void_p, C.c_void_p, C.c_float, C.c_int64, C.c_int64,
                                     C.POINTER(_Format), C.c_void_p]
        L.orc_gemm_nt.restype = None
        L.orc_quant_noise.restype = None
        L.orc_quant_noise.argtypes = [C.c_void_p, C.c_int, C.c_int64, C.c_int64, C.c_int64, C.c_int,
                                      C.POINTER(_Format), C.c_void_p, C.c_void_p, C.c_float, C.c_void_p]
        L.orc_gemm_nt.argtypes = [C.c_int64, C.c_int64, C.c_int64, C.POINTER(_Format),
                                  C.c_void_p, C.c_void_p, C.c_float,
                                  C.c_void_p, C.c_void_p, C.c_float, C.c_int, C.c_void_p]
        L.orc_exp_nonpos.restype = C.c_float
        L.orc_exp_nonpos.argtypes = [C.c_float]
        L.orc_swiglu_bwd.restype = None
        L.orc_swiglu_bwd.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int64, C.c_void_p, C.c_void_p]
        L.orc_gemm_nt_sample.restype = None
        L.orc_gemm_nt_sample.argtypes = [C.c_int64, C.c_int64, C.c_int64, C.POINTER(_Format),
                                         C.c_void_p, C.c_void_p, C.c_float,
                                         C.c_void_p, C.c_void_p, C.c_float, C.c_int,
                                         C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p]
        for name in ("orc_e4m3_encode_array", "orc_round_rtn_array"):
            getattr(L, name).restype = None
            getattr(L, name).argtypes = [C.c_void_p, C.c_int64, C.c_void_p]
        L.orc_round_sr_array.restype = None
        L.orc_round_sr_array.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p]
        L.orc_sr_bits_array.restype = None
        L.orc_sr_bits_array.argtypes = [C.c_uint64, C.c_uint64, C.c_int64, C.c_void_p]
        L.orc_philox4x32_10.restype = None
        L.orc_philox4x32_10.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p]
        _lib = L
    return _lib


def _p(a: np.ndarray):
    return a.ctypes.data_as(C.c_void_p)


# ------------------------------------------------------------------ scalars
def e2m1_decode(code: int) -> float:
    return float(lib().orc_e2m1_decode(code))


def e4m3_decode(byte: int) -> float:
    return float(lib().orc_e4m3_decode(byte))


def e4m3_encode(r) -> int | np.ndarray:
    if np.isscalar(r):
        return int(lib().orc_e4m3_encode(float(r)))
    r = np.ascontiguousarray(r, dtype=np.float32)
    out = np.empty(r.shape, np.uint8)
    lib().orc_e4m3_encode_array(_p(r), r.size, _p(out))
    return out


def e8m0_decode(byte: int) -> float:
    return float(lib().orc_e8m0_decode(byte))


def philox4x32_10(ctr, key) -> np.ndarray:
    c = np.asarray(ctr, dtype=np.uint32)
    k = np.asarray(key, dtype=np.uint32)
    out = np.empty(4, np.uint32)
    lib().orc_philox4x32_10(_p(c), _p(k), _p(out))
    return out


def sr_bits(seed: int, e) -> int | np.ndarray:
    if np.isscalar(e):
        return int(lib().orc_sr_bits(seed, int(e)))
    raise TypeError("use sr_bits_range for arrays")


def sr_bits_range(seed: int, e0: int, n: int) -> np.ndarray:
    out = np.empty(n, np.uint32)
    lib().orc_sr_bits_array(seed, e0, n, _p(out))
    return out


def round_rtn(m) -> int | np.ndarray:
    if np.isscalar(m):
        return int(lib().orc_round_rtn(float(m)))
    m = np.ascontiguousarray(m, dtype=np.float32)
    out = np.empty(m.shape, np.uint8)
    lib().orc_round_rtn_array(_p(m), m.size, _p(out))
    return out


def round_sr(m, u16) -> int | np.ndarray:
    if np.isscalar(m):
        return int(lib().orc_round_sr(float(m), int(u16)))
    m = np.ascontiguousarray(m, dtype=np.float32)
    u = np.ascontiguousarray(u16, dtype=np.uint32)
    assert u.shape == m.shape
    out = np.empty(m.shape, np.uint8)
    lib().orc_round_sr_array(_p(m), _p(u), m.size, _p(out))
    return out


def tensor_scale_from_amax(T: float) -> float:
    return float(lib().orc_tensor_scale_from_amax(float(T)))


# ------------------------------------------------------------------ tensors
def _as_input(x):
    """-> (contiguous 2-D numpy array, dtype tag).  fp32 arrays pass through; bf16 arrives as a
    torch.bfloat16 CPU tensor or as a numpy uint16 array holding the bf16 bit patterns."""
    if not isinstance(x, np.ndarray):  # torch tensor
        import torch
        x = x.detach().cpu().contiguous()
        if x.dtype == torch.bfloat16:
            x = x.view(torch.int16).numpy().view(np.uint16)
        elif x.dtype == torch.float32:
            x = x.numpy()
        else:
            raise TypeError(f"unsupported dtype {x.dtype}")
    if x.dtype == np.uint16:
        tag = BF16
    elif x.dtype == np.float32:
        tag = F32
    else:
        raise TypeError(f"unsupported dtype {x.dtype}")
    assert x.ndim == 2
    return np.ascontiguousarray(x), tag


def tensor_amax(x) -> float:
    a, tag = _as_input(x)
    return float(lib().orc_tensor_amax(_p(a), tag, a.shape[0], a.shape[1], a.shape[1]))


def quantize(x, axis: int = 1, rounding: int = RTN, seed: int = 0, fmt: Format = NVFP4,
             g: float | None = None):
    """Q of Eqs. 1-6.  Returns (codes u8 [outer, inner/2], scales u8 [outer, inner/block], g)."""
    a, tag = _as_input(x)
    rows, cols = a.shape
    outer, inner = (rows, cols) if axis == 1 else (cols, rows)
    codes = np.empty((outer, inner // 2), np.uint8)
    scales = np.empty((outer, inner // fmt.block), np.uint8)
    gio = C.c_float(0.0 if g is None else g)
    f = fmt.c()
    rc = lib().orc_quantize(_p(a), tag, rows, cols, cols, axis, rounding, seed, C.byref(f),
                            _p(codes), _p(scales), C.byref(gio), 0 if g is None else 1)
    if rc != 0:
        raise ValueError("shape not representable in this block format")
    return codes, scales, float(gio.value)


def dequantize(codes: np.ndarray, scales: np.ndarray, g: float, fmt: Format = NVFP4) -> np.ndarray:
    """fp64 values [outer, K] of a quantized operand."""
    outer, K = codes.shape[0], codes.shape[1] * 2
    out = np.empty((outer, K), np.float64)
    f = fmt.c()
    lib().orc_dequantize(_p(np.ascontiguousarray(codes)), _p(np.ascontiguousarray(scales)),
                         g, outer, K, C.byref(f), _p(out))
    return out


def quant_noise(x, q, axis: int = 1, fmt: Format = NVFP4):
    """(sum x^2, sum (Q(x) - x)^2) in fp64 for q = (codes, scales, g) as quantize(x, axis, ...) returned
    (Sec. 4: the monitored gradient-to-noise ratio is sqrt of their quotient)."""
    a, tag = _as_input(x)
    rows, cols = a.shape
    codes, scales, g = q
    out = np.zeros(2, np.float64)
    f = fmt.c()
    lib().orc_quant_noise(_p(a), tag, rows, cols, cols, axis, C.byref(f), _p(np.ascontiguousarray(codes)),
                          _p(np.ascontiguousarray(scales)), g, _p(out))
    return float(out[0]), float(out[1])


def gemm_nt(A, B, fmt: Format = NVFP4, take_abs: bool = False) -> np.ndarray:
    """A = (codes [M,K/2], scales, g), B = (codes [N,K/2], scales, g) -> fp64 [M, N]."""
    (ac, asc, ga), (bc, bsc, gb) = A, B
    M, N, K = ac.shape[0], bc.shape[0], ac.shape[1] * 2
    assert bc.shape[1] * 2 == K
    out = np.empty((M, N), np.float64)
    f = fmt.c()
    lib().orc_gemm_nt(M, N, K, C.byref(f), _p(np.ascontiguousarray(ac)),
                      _p(np.ascontiguousarray(asc)), ga, _p(np.ascontiguousarray(bc)),
                      _p(np.ascontiguousarray(bsc)), gb, int(take_abs), _p(out))
    return out


def gemm_nt_sample(A, B, ii, jj, fmt: Format = NVFP4, take_abs: bool = False) -> np.ndarray:
    """out[t] = (A B^T)[ii[t], jj[t]] in fp64, for sampled positions of a large product."""
    (ac, asc, ga), (bc, bsc, gb) = A, B
    M, N, K = ac.shape[0], bc.shape[0], ac.shape[1] * 2
    ii = np.ascontiguousarray(ii, dtype=np.int64)
    jj = np.ascontiguousarray(jj, dtype=np.int64)
    out = np.empty(ii.shape, np.float64)
    f = fmt.c()
    lib().orc_gemm_nt_sample(M, N, K, C.byref(f), _p(np.ascontiguousarray(ac)),
                             _p(np.ascontiguousarray(asc)), ga, _p(np.ascontiguousarray(bc)),
                             _p(np.ascontiguousarray(bsc)), gb, int(take_abs),
                             _p(ii), _p(jj), ii.size, _p(out))
    return out


def exp_nonpos(t: float) -> float:
    """The fixed binary32 evaluation of exp(t), t <= 0, that swiglu_bwd uses."""
    return float(lib().orc_exp_nonpos(float(t)))


def swiglu_bwd(dH, G, U):
    """Elementwise backward of h = silu(g) * u in the fixed binary32 evaluation stated in nvfp4_oracle.c:
    -> (dG, dU) in the element type of the inputs (bf16 as numpy uint16 bit patterns, fp32 as float32), the
    tensors the quantizers of the gate and up layers' backward GEMMs (Eqs. 5-6) then see."""
    (h, tag), (g, tg), (u, tu) = _as_input(dH), _as_input(G), _as_input(U)
    assert tag == tg == tu and h.shape == g.shape == u.shape
    dG, dU = np.empty_like(h), np.empty_like(h)
    lib().orc_swiglu_bwd(_p(h), _p(g), _p(u), tag, h.size, _p(dG), _p(dU))
    return dG, dU


# ------------------------------------------------- the three GEMMs, Eqs. 4-6
# Row-major batch notation: X [M, K] activations, W [N, K] weights, dY [M, N].

def linear_fwd(X, W, fmt: Format = NVFP4):
    """Eq. 4: Y = Q_RtN(X) Q_RtN(W)^T, blocks along K."""
    return gemm_nt(quantize(X, 1, RTN, 0, fmt), quantize(W, 1, RTN, 0, fmt), fmt)


def linear_bwd(dY, X, W, seed: int, fmt: Format = NVFP4):
    """Eq. 5: dX = Q_SR(dY) Q_RtN(W^T)^T with blocks along N (stream seed);
    Eq. 6: dW = Q_SR(dY^T) Q_SR(X^T)^T with blocks along M (streams seed+1, seed+2)."""
    dX = gemm_nt(quantize(dY, 1, SR, seed, fmt), quantize(W, 0, RTN, 0, fmt), fmt)
    dW = gemm_nt(quantize(dY, 0, SR, seed + 1, fmt), quantize(X, 0, SR, seed + 2, fmt), fmt)
    return dX, dW
