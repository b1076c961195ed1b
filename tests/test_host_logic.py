"""CPU-only checks of the HIP library's host side: the shared object loads and exports the
declared C ABI, argument validation returns the documented codes before anything is launched,
and the scalar steps the kernels use (compiled for the host) agree with the oracle."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import oracle
from paper_2505_19115_amd import binding as nv

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _p(a):
    return a.ctypes.data_as(C.c_void_p)


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "nvfp4.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(nvfp4_[a-z0-9_]+)\s*\(", hdr))
    assert len(declared) >= 20
    raw = C.CDLL(nv.LIB_PATH)
    for name in declared:
        assert hasattr(raw, name), name
    assert declared == set(nv.EXPORTS)


def test_sizes():
    f = nv.NVFP4.c()
    assert nv.lib.nvfp4_codes_bytes(8192, 8192) == 8192 * 8192 // 2
    assert nv.lib.nvfp4_scales_bytes(8192, 4096, 1, C.byref(f)) == 8192 * 4096 // 16
    assert nv.lib.nvfp4_scales_bytes(8192, 4096, 0, C.byref(f)) == 4096 * 8192 // 16
    m = nv.MXFP4.c()
    assert nv.lib.nvfp4_scales_bytes(64, 128, 1, C.byref(m)) == 64 * 4
    assert nv.lib.nvfp4_quantize_workspace_bytes(10, 10) >= 4
    fw = nv.lib.nvfp4_linear_fwd_workspace_bytes(4096, 11008, 4096, C.byref(f))
    assert fw >= (4096 + 11008) * 4096 * 9 // 16
    bw = nv.lib.nvfp4_linear_bwd_workspace_bytes(4096, 11008, 4096, C.byref(f))
    assert bw >= 2 * 4096 * 11008 * 9 // 16 + (4096 + 11008) * 4096 * 9 // 16
    assert nv.lib.nvfp4_status_string(0) == b"ok"
    for code in range(1, 7):
        assert len(nv.lib.nvfp4_status_string(code)) > 3


FAKE = 0x10000  # non-null, 16-byte aligned; never dereferenced because validation fails first


def _quant(x=FAKE, dt=nv.BF16, rows=64, cols=64, ld=64, axis=1, rnd=nv.RTN, fmt=nv.NVFP4,
           codes=FAKE, scales=FAKE, ts=FAKE, flags=0, ws=FAKE, ws_bytes=1 << 20):
    f = fmt.c()
    return nv.lib.nvfp4_quantize(x, dt, rows, cols, ld, axis, rnd, 0, C.byref(f), codes, scales, ts,
                                 flags, ws, ws_bytes, None)


def test_quantize_argument_errors():
    assert _quant(x=None) == nv.EINVAL
    assert _quant(codes=None) == nv.EINVAL
    assert _quant(dt=7) == nv.EINVAL
    assert _quant(axis=2) == nv.EINVAL
    assert _quant(rnd=3) == nv.EINVAL
    assert _quant(flags=8) == nv.EINVAL
    assert _quant(rows=-1) == nv.ESHAPE
    assert _quant(cols=72, ld=72) == nv.ESHAPE            # 72 is not a multiple of 16
    assert _quant(rows=24, axis=0) == nv.ESHAPE           # blocked axis is rows
    assert _quant(ld=32) == nv.ESHAPE                     # ld < cols
    assert _quant(x=FAKE + 2) == nv.EALIGN
    assert _quant(ld=68) == nv.EALIGN                     # rows not 16-byte aligned (bf16)
    assert _quant(fmt=nv.Format(8, 0, 1)) == nv.EUNSUPPORTED
    assert _quant(fmt=nv.Format(32, nv.SCALE_E8M0, 1)) == nv.EUNSUPPORTED
    assert _quant(fmt=nv.Format(16, 5, 1)) == nv.EINVAL
    assert _quant(ws=None) == nv.EWORKSPACE
    assert _quant(ws_bytes=2) == nv.EWORKSPACE


def test_quantize_static_argument_errors():
    # the entry that allocates nothing validates like nvfp4_quantize, and refuses a tensor whose partial maxima
    # do not fit its static scratch before it touches any device
    def qs(x=FAKE, rows=64, cols=64, ld=64, axis=1, rnd=nv.RTN, fmt=nv.NVFP4, codes=FAKE, ts=FAKE, flags=0):
        f = fmt.c()
        return nv.lib.nvfp4_quantize_static(x, nv.BF16, rows, cols, ld, axis, rnd, 0, C.byref(f), codes, FAKE, ts, flags, None)
    assert qs(rows=16385, cols=16, ld=24) == nv.EWORKSPACE          # 16385 row spans > 16384 partial maxima
    assert qs(rows=4096, cols=5 * 8192, ld=5 * 8192 + 8) == nv.EWORKSPACE
    assert qs(rows=16385, cols=16, ld=24, flags=nv.PRESET_TSCALE) == nv.EWORKSPACE  # the limit does not depend on flags


def test_weight_operand_argument_errors():
    f = nv.NVFP4.c()
    n = nv.lib.nvfp4_weight_operands_bytes(11008, 4096, C.byref(f))
    assert n >= 2 * 11008 * 4096 * 9 // 16 and n < 2 * 11008 * 4096 * 9 // 16 + (1 << 21)
    assert nv.lib.nvfp4_weight_operands_bytes(0, 4096, C.byref(f)) == 0
    qw = lambda **k: nv.lib.nvfp4_quantize_weight(k.get("W", FAKE), k.get("dt", nv.BF16), k.get("M", 256), k.get("N", 128), k.get("K", 128),
                                                  C.byref(k.get("f", f)), k.get("out", FAKE + 256 - FAKE % 256 if FAKE % 256 else FAKE), k.get("ws", FAKE), k.get("wsb", 1 << 20), None)
    assert qw(W=None) == nv.EINVAL
    assert qw(out=None) == nv.EINVAL
    assert qw(dt=5) == nv.EINVAL
    assert qw(N=72) == nv.ESHAPE          # W^T is blocked along N
    assert qw(K=48) == nv.ESHAPE
    assert qw(M=0) == nv.ESHAPE
    assert qw(out=FAKE + 16) == nv.EALIGN
    assert qw(ws=None) == nv.EWORKSPACE
    assert qw(f=nv.Format(64, nv.SCALE_E8M0, 0).c()) == nv.EUNSUPPORTED
    fw = lambda **k: nv.lib.nvfp4_linear_fwd_wq(FAKE, k.get("wq", FAKE), FAKE, k.get("M", 64), k.get("N", 64), 64, nv.BF16, nv.BF16, C.byref(f),
                                                FAKE, 1 << 30, None, None, None, 0)
    assert fw(wq=None) == nv.EINVAL
    assert fw(N=72) == nv.ESHAPE
    assert fw(wq=FAKE + 16) == nv.EALIGN
    bw = nv.lib.nvfp4_linear_bwd_wq(FAKE, FAKE, None, FAKE, FAKE, 64, 64, 64, nv.BF16, nv.BF16, C.byref(f), 0, FAKE, 1 << 30, None, None, None)
    assert bw == nv.EINVAL


def test_swiglu_backward_scalar_step_equals_the_oracle_bit_for_bit():
    # the kernels' own inline function for the SwiGLU backward (compiled for the host) against the oracle's fixed
    # binary32 evaluation: every bit, over gates from deep saturation to deep saturation, zeros and signed zeros
    rng = np.random.default_rng(3)
    n = 200000
    g = np.concatenate([rng.standard_normal(n // 2) * 4.0, rng.uniform(-120.0, 120.0, n // 2 - 8), [0.0, -0.0, 87.0, -87.0, 88.5, -88.5, 1e-30, -1e-30]]).astype(np.float32)
    u = (rng.standard_normal(n) * 1.5).astype(np.float32)
    h = (rng.standard_normal(n) * 1e-3).astype(np.float32)
    dg, du = np.empty(n, np.float32), np.empty(n, np.float32)
    nv.lib.nvfp4_host_swiglu_bwd(_p(h), _p(g), _p(u), n, _p(dg), _p(du))
    og, ou = oracle.swiglu_bwd(h.reshape(1, n), g.reshape(1, n), u.reshape(1, n))
    assert np.array_equal(dg.view(np.uint32), og.reshape(-1).view(np.uint32))
    assert np.array_equal(du.view(np.uint32), ou.reshape(-1).view(np.uint32))


def test_swiglu_and_dyq_argument_errors():
    f = nv.NVFP4.c()
    ops = nv._DualOperands(FAKE, FAKE, FAKE, FAKE, FAKE, 0)
    sq = lambda **k: nv.lib.nvfp4_swiglu_bwd_quantize(k.get("dH", FAKE), FAKE, k.get("U", FAKE), k.get("dt", nv.BF16), k.get("M", 64), k.get("F", 64), 1, 2,
                                                      C.byref(k.get("f", f)), C.byref(k.get("dG", ops)), C.byref(ops), k.get("sg", None), k.get("su", None), k.get("ws", FAKE), k.get("wsb", 1 << 20), None)
    assert sq(dH=None) == nv.EINVAL
    assert sq(sg=FAKE) == nv.EINVAL                      # the two result tensors come together or not at all
    assert sq(sg=FAKE + 4, su=FAKE) == nv.EALIGN
    assert sq(U=None) == nv.EINVAL
    assert sq(dt=4) == nv.EINVAL
    assert sq(M=72) == nv.ESHAPE
    assert sq(F=24) == nv.ESHAPE
    assert sq(f=nv.Format(64, nv.SCALE_E4M3, 1).c()) == nv.EUNSUPPORTED
    assert sq(ws=None) == nv.EWORKSPACE
    assert sq(wsb=100) == nv.EWORKSPACE
    assert sq(dG=nv._DualOperands(FAKE, FAKE, None, FAKE, FAKE, 0)) == nv.EINVAL
    assert sq(dG=nv._DualOperands(FAKE, FAKE, FAKE, FAKE, FAKE, 8)) == nv.EINVAL
    assert sq(dG=nv._DualOperands(FAKE, FAKE, FAKE, FAKE, FAKE, nv.SLAB_ROWS)) == nv.ESHAPE     # F = 64: no whole K tile
    assert sq(dG=nv._DualOperands(FAKE + 8, FAKE, FAKE, FAKE, FAKE, 0)) == nv.EALIGN
    assert nv.lib.nvfp4_swiglu_bwd_workspace_bytes(4096, 11008) >= 4096
    bq = lambda **k: nv.lib.nvfp4_linear_bwd_dyq(k["dy"] if "dy" in k else C.byref(ops), FAKE, FAKE, None, FAKE, FAKE, 64, k.get("N", 64), 64, nv.BF16, nv.BF16,
                                                  C.byref(f), 0, FAKE, 1 << 30, None, None, None)
    assert bq(dy=None) == nv.EINVAL
    assert bq(dy=C.byref(nv._DualOperands(FAKE, FAKE, FAKE, FAKE, None, 0))) == nv.EINVAL
    assert bq(dy=C.byref(nv._DualOperands(None, FAKE, FAKE, FAKE, FAKE, 0))) == nv.EINVAL
    assert bq(dy=C.byref(nv._DualOperands(FAKE, FAKE, FAKE, FAKE, FAKE, nv.SLAB_ROWS))) == nv.EUNSUPPORTED  # the small GEMM takes no slabs
    assert bq(N=72) == nv.ESHAPE


def test_cross_check_switches_round_trip():
    before = nv.cross_check_switches()
    assert 0 <= before <= 7
    assert nv.cross_check_switches(nv.SWITCH_PLAIN_OPERANDS) == before
    assert nv.cross_check_switches() == nv.SWITCH_PLAIN_OPERANDS
    assert nv.cross_check_switches(0xFFFFFFFF) == nv.SWITCH_PLAIN_OPERANDS and nv.cross_check_switches() == 7
    nv.cross_check_switches(before)
    assert nv.cross_check_switches() == before


def test_quantize_dual_argument_errors():
    def dual(x=FAKE, dt=nv.BF16, rows=64, cols=64, ld=64, rnd=nv.SR, fmt=nv.NVFP4, cr=FAKE, sr=FAKE, cc=FAKE,
             sc=FAKE, ts=FAKE, flags=0, ws=FAKE, ws_bytes=1 << 20, k2=nv.SR):
        f = fmt.c()
        return nv.lib.nvfp4_quantize_dual(x, dt, rows, cols, ld, rnd, 1, k2, 2, C.byref(f), cr, sr, cc, sc, ts, flags,
                                          ws, ws_bytes, None)
    assert dual(x=None) == nv.EINVAL
    assert dual(cc=None) == nv.EINVAL
    assert dual(sr=None) == nv.EINVAL
    assert dual(rnd=2) == nv.EINVAL
    assert dual(k2=5) == nv.EINVAL
    assert dual(flags=8) == nv.EINVAL
    # slab outputs: NVFP4 and MXFP4 only, through the one-pass kernel only, whole K tiles of 128 only
    assert dual(flags=nv.SLAB_ROWS) == nv.ESHAPE                      # cols = 64
    assert dual(flags=nv.SLAB_COLS, cols=128, ld=128) == nv.ESHAPE    # rows = 64
    assert dual(flags=nv.SLAB_ROWS, fmt=nv.Format(32, nv.SCALE_E4M3, 1), rows=128, cols=128, ld=128) == nv.EUNSUPPORTED
    assert dual(flags=nv.SLAB_ROWS, rows=128, cols=128, ld=128, rnd=nv.SR, k2=nv.RTN) == nv.EUNSUPPORTED
    assert dual(rows=72) == nv.ESHAPE                     # both axes are blocked
    assert dual(cols=72, ld=72) == nv.ESHAPE
    assert dual(rows=96, cols=96, ld=96, fmt=nv.Format(64, 0, 1)) == nv.ESHAPE
    assert dual(cr=FAKE + 4) == nv.EALIGN
    assert dual(ws=None) == nv.EWORKSPACE
    assert dual(fmt=nv.Format(16, nv.SCALE_E8M0, 1)) == nv.EUNSUPPORTED
    assert dual(rows=0, cr=None, sr=None, cc=None, sc=None, ws=None, fmt=nv.MXFP4) == nv.OK  # empty: nothing launched


def test_gemm_and_linear_argument_errors():
    f = nv.NVFP4.c()
    g = lambda **k: nv.lib.nvfp4_gemm(k.get("M", 64), k.get("N", 64), k.get("K", 64), C.byref(k.get("f", f)),
                                      k.get("a", FAKE), FAKE, FAKE, FAKE, FAKE, k.get("out", FAKE),
                                      k.get("odt", nv.F32), k.get("ldc", 64), None)
    assert g(a=None) == nv.EINVAL
    assert g(odt=9) == nv.EINVAL
    assert g(K=48) == nv.ESHAPE      # multiple of the block but not of 32
    assert g(K=0) == nv.ESHAPE
    assert g(ldc=8) == nv.ESHAPE
    assert g(out=FAKE + 4) == nv.EALIGN
    assert g(f=nv.Format(64, nv.SCALE_E8M0, 0).c()) == nv.EUNSUPPORTED  # E8M0 GEMM exists for block 32 only
    assert g(M=0) == nv.OK           # empty product: nothing to do, nothing launched
    assert g(K=(1 << 23) + 32) == nv.ESHAPE  # contraction length beyond the kernels' 32-bit tile offsets
    # slab operands: only where the large-tile kernel runs (NVFP4, K % 128 == 0, >= 128 tiles of 256 x 256)
    gs = lambda M, N, K, fmt=nv.NVFP4, a=1, b=0: nv.lib.nvfp4_gemm_slab(M, N, K, C.byref(fmt.c()), FAKE, FAKE, FAKE, FAKE, FAKE, FAKE,
                                                                        nv.F32, N, a, b, None)
    assert gs(64, 64, 128) == nv.EUNSUPPORTED
    assert gs(4096, 4096, 192) == nv.EUNSUPPORTED
    assert gs(4096, 4096, 256, nv.MXFP4) == nv.EUNSUPPORTED      # MXFP4: the direct-to-LDS kernel needs K >= 512
    assert gs(4096, 4096, 4096, nv.Format(32, nv.SCALE_E4M3, 1)) == nv.EUNSUPPORTED
    takes = lambda M, N, K, fmt=nv.NVFP4: nv.lib.nvfp4_gemm_takes_slabs(M, N, K, C.byref(fmt.c()))
    assert takes(4096, 11008, 4096) == 1 and takes(2944, 3200, 2816) == 1
    assert takes(2048, 2048, 4096) == 0 and takes(4096, 4096, 4096 + 64) == 0
    assert takes(4096, 4096, 4096, nv.MXFP4) == 1 and takes(64, 64, 512, nv.MXFP4) == 1 and takes(64, 64, 384, nv.MXFP4) == 0
    # slab buffers: rows padded to whole slabs of 256
    assert nv.lib.nvfp4_slab_codes_bytes(256, 128) == 16384 and nv.lib.nvfp4_slab_scales_bytes(256, 128) == 2048
    assert nv.lib.nvfp4_slab_codes_bytes(257, 256) == 2 * 2 * 16384 and nv.lib.nvfp4_slab_scales_bytes(1, 128) == 2048
    assert nv.lib.nvfp4_slab_codes_bytes(0, 128) == 0
    # (MXFP4: 4 scale bytes per row and K tile, half of what the query states)
    assert nv.slab_scales_bytes(257, 256, nv.MXFP4) == 2 * 2 * 1024 and nv.slab_scales_bytes(257, 256) == 2 * 2 * 2048
    fw = lambda **k: nv.lib.nvfp4_linear_fwd(k.get("X", FAKE), FAKE, FAKE, k.get("M", 64), 64, k.get("K", 64), nv.BF16,
                                             nv.F32, C.byref(f), k.get("ws", FAKE), k.get("wsb", 1 << 30), None, None,
                                             k.get("saved"), 0)
    assert fw(X=None) == nv.EINVAL
    assert fw(K=40) == nv.ESHAPE
    assert fw(ws=None) == nv.EWORKSPACE
    assert fw(wsb=16) == nv.EWORKSPACE
    assert fw(M=48, saved=FAKE) == nv.ESHAPE     # X^T is blocked along M for the backward call
    assert fw(saved=FAKE + 16) == nv.EALIGN
    assert nv.linear_saved_bytes(4096, 11008, 4096) >= 4096 * (4096 + 11008) * 9 // 16
    bw = lambda **k: nv.lib.nvfp4_linear_bwd(k.get("dY", FAKE), FAKE, FAKE, FAKE, FAKE, k.get("M", 64), 64, 64,
                                             nv.BF16, nv.F32, C.byref(f), 0, FAKE, k.get("wsb", 1 << 30), None, None,
                                             k.get("saved"))
    assert bw(dY=None) == nv.EINVAL
    assert bw(M=48) == nv.ESHAPE     # the update GEMM contracts over M
    assert bw(wsb=16) == nv.EWORKSPACE
    assert bw(saved=FAKE + 16) == nv.EALIGN


# ---------------------------------------------------------------- scalar steps vs the oracle
def test_host_e4m3_encode_matches_oracle():
    hi = int(np.float32(500.0).view(np.uint32))
    x = np.arange(0, hi, 211, dtype=np.uint32).view(np.float32)
    grid = np.array([oracle.e4m3_decode(b) for b in range(127)], dtype=np.float32)
    mids = ((grid[:-1].astype(np.float64) + grid[1:]) / 2).astype(np.float32)
    sp = np.concatenate([grid, mids])
    sp = np.concatenate([sp, np.nextafter(sp, np.float32(1e9)), np.nextafter(sp, np.float32(-1))])
    x = np.ascontiguousarray(np.concatenate([x, sp[sp >= 0], np.float32([1e4, 3e38])]))
    got = np.empty(x.size, np.uint8)
    nv.lib.nvfp4_host_e4m3_encode_n(_p(x), x.size, _p(got))
    assert np.array_equal(got, oracle.e4m3_encode(x))
    for b in range(127):
        assert nv.lib.nvfp4_host_e4m3_decode(b) == oracle.e4m3_decode(b)


def test_host_round_rtn_matches_oracle_on_every_float_in_range():
    # every binary32 pattern in [2^-3, 6]; below 2^-3 a strided sample (all map to code 0)
    lo, hi = int(np.float32(0.125).view(np.uint32)), int(np.float32(6.0).view(np.uint32))
    for a in range(lo, hi + 1, 1 << 22):
        x = np.arange(a, min(a + (1 << 22), hi + 1), dtype=np.uint32).view(np.float32)
        got = np.empty(x.size, np.uint8)
        nv.lib.nvfp4_host_round_rtn_n(_p(x), x.size, _p(got))
        assert np.array_equal(got, oracle.round_rtn(x))
    x = np.arange(0, lo, 4099, dtype=np.uint32).view(np.float32)
    got = np.empty(x.size, np.uint8)
    nv.lib.nvfp4_host_round_rtn_n(_p(x), x.size, _p(got))
    assert np.array_equal(got, oracle.round_rtn(x)) and got.max() == 0


def test_host_round_sr_matches_oracle():
    rng = np.random.default_rng(0)
    hi = int(np.float32(6.0).view(np.uint32))
    # random magnitudes x random draws, plus every draw for magnitudes around each threshold
    m = rng.integers(0, hi + 1, 4_000_000, dtype=np.uint32).view(np.float32)
    u = rng.integers(0, 65536, m.size, dtype=np.uint32)
    got = np.empty(m.size, np.uint8)
    nv.lib.nvfp4_host_round_sr_n(_p(m), _p(u), m.size, _p(got))
    assert np.array_equal(got, oracle.round_sr(m, u))
    uu = np.arange(65536, dtype=np.uint32)
    for mv in [0.0, 1e-30, 0.1, 0.25, 0.4999999, 0.5, 0.75, 1.0, 1.2, 1.9999999, 2.0, 2.4, 3.0, 3.999999, 4.0, 5.0,
               5.9999995, 6.0, 2.0 ** -17 * 0.5, 0.5 + 2.0 ** -18, 4 + 2.0 ** -16,
               # exact ties between the position and a centred draw, one per binade of the grid
               0.5 * 100.5 / 65536, 0.5 + 0.5 * 7.5 / 65536, 1.5 + 0.5 * 65535.5 / 65536, 2 + 100.5 / 65536,
               3 + 0.5 / 65536, 4 + 2 * 32767.5 / 65536]:
        mm = np.full(65536, mv, np.float32)
        nv.lib.nvfp4_host_round_sr_n(_p(mm), _p(uu), 65536, _p(got[:65536]))
        assert np.array_equal(got[:65536], oracle.round_sr(mm, uu)), mv


def test_host_philox_and_sr_bits(golden_dir):
    for ln in open(os.path.join(golden_dir, "philox4x32_10_kat.txt")):
        if ln.startswith("#") or not ln.strip():
            continue
        w = [int(t, 16) for t in ln.split()]
        c, k, out = np.array(w[0:4], np.uint32), np.array(w[4:6], np.uint32), np.empty(4, np.uint32)
        nv.lib.nvfp4_host_philox4x32_10(_p(c), _p(k), _p(out))
        assert [int(v) for v in out] == w[6:10]
    seed = 0xFEDCBA9876543210
    for e0 in (0, 8 * 12345, (1 << 36) + 24):
        want = oracle.sr_bits_range(seed, e0, 64)
        assert [nv.lib.nvfp4_host_sr_bits(seed, e0 + t) for t in range(64)] == [int(v) for v in want]


def test_host_e8m0_matches_oracle_rule():
    rng = np.random.default_rng(1)
    a = np.abs(rng.standard_normal(2000).astype(np.float32)) * np.float32(10) ** rng.integers(-30, 30, 2000).astype(np.float32)
    a = np.concatenate([a, np.float32([1e-45, 1e-40, 2.0 ** -126, 2.0 ** -127, 1.0, 6.0, 7.99, 8.0, 3e38])]).astype(np.float32)
    for v in a:
        x = np.zeros((1, 32), np.float32)
        x[0, 0] = v
        want = oracle.quantize(x, 1, oracle.RTN, 0, oracle.MXFP4)[1][0, 0]
        assert nv.lib.nvfp4_host_e8m0_encode(float(v)) == want, v
