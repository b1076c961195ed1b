"""GPU parity of nvfp4_quantize / nvfp4_tensor_scale against the CPU oracle: codes, scale bytes
and the tensor scale must be bit-identical on the same seeded inputs."""
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2505_19115_amd import synth
from gpu_util import assert_quant_equal, ofmt, to_np

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


def run_both(x_cpu, axis, rounding, seed, fmt, preset=None, what=""):
    print(f"[case] {what} shape={tuple(x_cpu.shape)} dtype={x_cpu.dtype} axis={axis} rounding={rounding} "
          f"seed={seed} fmt={fmt}", flush=True)
    x = x_cpu.cuda()
    ts = None if preset is None else torch.tensor([preset], dtype=torch.float32, device="cuda")
    got = nv.quantize(x, axis, rounding, seed, fmt, tensor_scale=ts)
    torch.cuda.synchronize()
    want = oracle.quantize(x_cpu, axis, rounding, seed, ofmt(fmt), g=preset)
    assert_quant_equal(got, want, what)
    return got


FORMATS = {
    "nvfp4": lambda: nv.NVFP4,
    "mxfp4": lambda: nv.MXFP4,
    "e4m3_b32": lambda: nv.Format(32, nv.SCALE_E4M3, 1),
    "e4m3_b64": lambda: nv.Format(64, nv.SCALE_E4M3, 1),
    "e4m3_b128": lambda: nv.Format(128, nv.SCALE_E4M3, 1),
}


def test_config1_fp32_256():
    # X, W fp32 [256, 256] ~ N(0,1): row-blocked RtN as the forward GEMM consumes them
    for seed in (1, 2):
        x = synth.normal(256, 256, 1.0, seed, torch.float32)
        run_both(x, 1, nv.RTN, 0, nv.NVFP4, what="config1")
        run_both(x, 0, nv.RTN, 0, nv.NVFP4, what="config1-cols")
        run_both(x, 1, nv.SR, 5, nv.NVFP4, what="config1-sr")
        run_both(x, 0, nv.SR, 5, nv.NVFP4, what="config1-cols-sr")


@pytest.mark.parametrize("fmt", list(FORMATS))
@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
@pytest.mark.parametrize("axis", [1, 0])
@pytest.mark.parametrize("rounding", [0, 1])
def test_all_formats_ragged_tiles(fmt, dtype, axis, rounding):
    # several workgroup tiles in both directions plus ragged tails: 384 rows = 3 row tiles of
    # 128; 1152 columns = 2.25 column tiles of 512 (bf16) and 4.5 of 256 (fp32)
    f = FORMATS[fmt]()
    x = synth.student_t_outliers(384, 1152, seed=11, dtype=dtype)
    run_both(x, axis, rounding, 1234, f, what=f"{fmt}")


@pytest.mark.parametrize("axis", [1, 0])
@pytest.mark.parametrize("rounding", [0, 1])
def test_ragged_rows_and_leading_dimension(axis, rounding):
    # rows = 16 * 19 (one block short of the 32-row lane tile), cols = 16 * 65; the tensor is a
    # window of a wider one, so rows are not contiguous
    big = synth.student_t_outliers(304, 1200, seed=12, dtype=torch.bfloat16)
    xg = big.cuda()[:, 8:8 + 1040]
    x_cpu = big[:, 8:8 + 1040].contiguous()
    print(f"[case] window axis={axis} rounding={rounding}", flush=True)
    got = nv.quantize(xg, axis, rounding, 77, nv.NVFP4)
    want = oracle.quantize(x_cpu, axis, rounding, 77)
    assert_quant_equal(got, want, "window")


@pytest.mark.parametrize("rounding", [0, 1])
def test_columns_not_multiple_of_8(rounding):
    # axis 0 only needs the row count to be a multiple of the block; 1003 columns leave a
    # 3-column tail and misalign the 8-element random-number groups from row to row
    big = synth.normal(160, 1008, 1.0, 13, torch.bfloat16)
    xg = big.cuda()[:, :1003]
    x_cpu = big[:, :1003].contiguous()
    print(f"[case] cols=1003 rounding={rounding}", flush=True)
    got = nv.quantize(xg, 0, rounding, 99, nv.NVFP4)
    want = oracle.quantize(x_cpu, 0, rounding, 99)
    assert_quant_equal(got, want, "cols1003")
    big32 = synth.normal(48, 1004, 1.0, 14, torch.float32)
    got = nv.quantize(big32.cuda()[:, :1001], 0, rounding, 5, nv.NVFP4)
    assert_quant_equal(got, oracle.quantize(big32[:, :1001].contiguous(), 0, rounding, 5), "cols1001-f32")


def test_software_rounding_path_equals_hardware_convert(switches):
    x = synth.student_t_outliers(256, 1024, seed=15, dtype=torch.bfloat16)
    hw = run_both(x, 1, nv.RTN, 0, nv.NVFP4, what="hw")
    hw0 = run_both(x, 0, nv.RTN, 0, nv.NVFP4, what="hw-cols")
    nv.cross_check_switches(nv.SWITCH_SOFT_CONVERT)
    sw = run_both(x, 1, nv.RTN, 0, nv.NVFP4, what="soft")
    sw0 = run_both(x, 0, nv.RTN, 0, nv.NVFP4, what="soft-cols")
    assert torch.equal(hw[0], sw[0]) and torch.equal(hw0[0], sw0[0])


def test_software_sr_path_equals_hardware_sr_convert(switches):
    # the integer formulation of the SR rule and the hardware SR convert fed with seed words built from the
    # same draws: both against the oracle, rows and columns, aligned and unaligned widths, and the
    # dual-orientation entry (one fused kernel vs its two-kernel fallback)
    x = synth.student_t_outliers(288, 1024, seed=16, dtype=torch.bfloat16)
    xu = synth.normal(64, 1004, 1.0, 17, torch.float32)   # its first 1001 columns: rows stay 16-byte aligned
    res = {}
    for mode in ("hw", "soft"):
        if mode == "soft":
            nv.cross_check_switches(nv.SWITCH_SOFT_CONVERT)
        res[mode] = [run_both(x, 1, nv.SR, 3, nv.NVFP4, what=mode + "-rows"),
                     run_both(x, 0, nv.SR, 4, nv.NVFP4, what=mode + "-cols"),
                     run_both(x, 0, nv.SR, 4, nv.MXFP4, what=mode + "-cols-mx"),
                     nv.quantize(xu.cuda()[:, :1001], 0, nv.SR, 5, nv.NVFP4)]
        assert_quant_equal(res[mode][3], oracle.quantize(xu[:, :1001].contiguous(), 0, oracle.SR, 5), mode + "-cols-unaligned")
        qr, qc = nv.quantize_dual(x.cuda(), nv.RTN, 0, nv.SR, 6, nv.NVFP4)
        torch.cuda.synchronize()
        assert_quant_equal(qr, oracle.quantize(x, 1, oracle.RTN, 0), mode + " dual rows")
        assert_quant_equal(qc, oracle.quantize(x, 0, oracle.SR, 6), mode + " dual cols")
    for a, b in zip(res["hw"], res["soft"]):
        assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])


def _blocks_with_leader(values, leader):
    """Rows of 1024 = 64 blocks, each block [leader, 15 values]."""
    n = (values.size + 14) // 15
    n = (n + 63) // 64 * 64
    v = np.concatenate([values, np.zeros(n * 15 - values.size, np.float32)])
    x = np.empty((n, 16), np.float32)
    x[:, 0] = leader
    x[:, 1:] = v.reshape(n, 15)
    return torch.from_numpy(x.reshape(-1, 1024))


def test_every_fp32_value_rounds_like_the_oracle():
    # blocks [6, v1 .. v15] with g preset to 1 have scale exactly 1, so the element codes are
    # the rounding of the raw values: every binary32 pattern from 2^-3 to 6 (alternating sign)
    # plus a strided sample of the smaller ones
    lo, hi = int(np.float32(0.125).view(np.uint32)), int(np.float32(6.0).view(np.uint32))
    v = np.concatenate([np.arange(lo, hi + 1, dtype=np.uint32),
                        np.arange(0, lo, 8191, dtype=np.uint32)]).view(np.float32).copy()
    v[1::2] *= -1
    x = _blocks_with_leader(v, 6.0)
    for rounding, seed in ((nv.RTN, 0), (nv.SR, 3)):
        run_both(x, 1, rounding, seed, nv.NVFP4, preset=1.0, what="sweep")
    # saturation: with g = 2^-10 every block scale saturates at 448 (d = 0.4375) and most
    # scaled values exceed 6
    w = np.arange(lo, int(np.float32(1e6).view(np.uint32)), 1021, dtype=np.uint32).view(np.float32).copy()
    w[::2] *= -1
    xs = _blocks_with_leader(w, 1e6)
    for rounding, seed in ((nv.RTN, 0), (nv.SR, 4)):
        run_both(xs, 1, rounding, seed, nv.NVFP4, preset=2.0 ** -10, what="saturate")


def test_every_scale_value_encodes_like_the_oracle():
    # g = fl(1/6) makes 6 g round to exactly 1, so the scale byte is E4M3(block maximum)
    g = float(np.float32(1.0) / np.float32(6.0))
    assert np.float32(6.0) * np.float32(g) == np.float32(1.0)
    hi = int(np.float32(520.0).view(np.uint32))
    a = np.arange(0, hi, 67, dtype=np.uint32).view(np.float32)
    n = (a.size // 64) * 64
    x = np.zeros((n, 16), np.float32)
    x[:, 5] = a[:n]
    x[::2, 5] *= -1
    x[:, 9] = a[:n] * np.float32(0.37)
    xt = torch.from_numpy(x.reshape(-1, 1024))
    run_both(xt, 1, nv.RTN, 0, nv.NVFP4, preset=g, what="scale-sweep")
    run_both(xt, 1, nv.SR, 8, nv.NVFP4, preset=g, what="scale-sweep-sr")


def test_degenerate_inputs():
    z = torch.zeros(32, 64, dtype=torch.bfloat16)
    z[3, 7] = -0.0
    for axis in (0, 1):
        got = run_both(z, axis, nv.SR, 1, nv.NVFP4, what="zeros")
        assert float(got[2].item()) == 1.0
    one = torch.zeros(16, 16, dtype=torch.float32)
    one[2, 3] = -3.0e-41  # subnormal maximum: the tensor scale hits its floor
    run_both(one, 1, nv.RTN, 0, nv.NVFP4, what="subnormal")
    run_both(one, 0, nv.RTN, 0, nv.NVFP4, what="subnormal-cols")
    huge = synth.normal(32, 32, 1.0, 3, torch.float32) * 1e30
    run_both(huge, 1, nv.RTN, 0, nv.NVFP4, what="huge")
    run_both(huge, 0, nv.SR, 2, nv.MXFP4, what="huge-mx")
    tiny = synth.normal(32, 64, 1.0, 4, torch.float32) * 1e-38
    run_both(tiny, 1, nv.SR, 2, nv.MXFP4, what="tiny-mx")
    # preset scale far too small: everything saturates
    x = synth.normal(64, 64, 1.0, 5, torch.bfloat16)
    run_both(x, 1, nv.RTN, 0, nv.NVFP4, preset=1e-6, what="preset-small")
    run_both(x, 0, nv.SR, 6, nv.NVFP4, preset=10.0, what="preset-large")
    # empty tensor: nothing written, scale 1
    e = torch.empty(0, 64, dtype=torch.bfloat16, device="cuda")
    c, s, g = nv.quantize(e, 1, nv.RTN, 0, nv.NVFP4)
    torch.cuda.synchronize()
    assert c.numel() == 0 and float(g.item()) == 1.0
    # empty and strided with many rows: no maximum kernel may run (there is nothing for it to cover)
    e2 = torch.empty(3000, 8, dtype=torch.bfloat16, device="cuda")[:, :0]
    guard = torch.full((1 << 16,), 7, dtype=torch.uint8, device="cuda")
    ws = guard[:nv.lib.nvfp4_quantize_workspace_bytes(3000, 0)]
    import ctypes as C
    f = nv.NVFP4.c()
    g2 = torch.zeros(1, device="cuda")
    for entry in (nv.lib.nvfp4_quantize,):
        rc = entry(e2.data_ptr(), nv.BF16, 3000, 0, 8, 1, nv.RTN, 0, C.byref(f), None, None, g2.data_ptr(), 0,
                   ws.data_ptr(), ws.numel(), torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        assert rc == nv.OK and float(g2) == 1.0
    assert bool((guard[ws.numel():] == 7).all()), "wrote past the workspace"
    assert float(nv.tensor_scale(e2)) == 1.0


def test_tensor_scale_entry_and_determinism():
    x = synth.student_t_outliers(1024, 2048, seed=21)
    xg = x.cuda()
    g = nv.tensor_scale(xg)
    assert float(g.item()) == oracle.tensor_scale_from_amax(oracle.tensor_amax(x))
    win = xg[:, 16:16 + 1000]
    assert float(nv.tensor_scale(win).item()) == oracle.tensor_scale_from_amax(
        oracle.tensor_amax(x[:, 16:16 + 1000].contiguous()))
    a = nv.quantize(xg, 0, nv.SR, 42)
    b = nv.quantize(xg, 0, nv.SR, 42)
    c = nv.quantize(xg, 0, nv.SR, 43)
    assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])
    assert not torch.equal(a[0], c[0]) and torch.equal(a[1], c[1])


_SWEEP_TENSOR = {}


@pytest.mark.parametrize("axis", [1, 0])
@pytest.mark.parametrize("rounding,seed", [(0, 0)] + [(1, s) for s in range(8)],
                         ids=["rtn"] + [f"sr-seed{s}" for s in range(8)])
def test_full_size_quantizer_sweep_tensor(axis, rounding, seed):
    # the quantizer sweep in full: bf16 [8192, 8192], Student-t(3) * 0.02 with 0.1 % outliers x100, along rows
    # and down columns, RtN and stochastic rounding with seeds 0..7 -- all 18 runs compared element by element
    if "x" not in _SWEEP_TENSOR:
        _SWEEP_TENSOR["x"] = synth.student_t_outliers(8192, 8192, seed=100)
    run_both(_SWEEP_TENSOR["x"], axis, rounding, seed, nv.NVFP4, what="config2")


@pytest.mark.parametrize("what,shape,axis,rounding,fmt", [
    ("dY rows SR (dX operand)", (4096, 11008), 1, 1, "NVFP4"),
    ("dY columns SR (dW operand)", (4096, 11008), 0, 1, "NVFP4"),
    ("W columns RtN (W^T operand)", (11008, 4096), 0, 0, "NVFP4"),
    ("X columns SR, MXFP4", (4096, 4096), 0, 1, "MXFP4"),
])
def test_full_size_7b_backward_operands(what, shape, axis, rounding, fmt):
    # the tensors the benchmark step quantizes for its backward GEMMs, element by element
    rows, cols = shape
    x = synth.gradient_like(rows, cols, 300) if what.startswith("dY") else synth.normal(rows, cols, 0.02, 200)
    run_both(x, axis, rounding, 1000, getattr(nv, fmt), what=what)


@pytest.mark.parametrize("axis", [1, 0])
def test_sr_exact_ties_between_draw_and_position(axis):
    # every element sits exactly where its own draw ties with its position between the grid
    # neighbours (65536 t = u + 1/2), offset by -1, 0 or +1 draws, in every binade of the grid;
    # one 6.0 per block and a preset tensor scale of 1 make the block multiplier exactly 1
    rows, cols, seed = 96, 128, 11
    u = oracle.sr_bits_range(seed, 0, rows * cols).astype(np.float64).reshape(rows, cols)
    rng = np.random.default_rng(4)
    lo_step = np.array([(0.0, 0.5), (0.5, 0.5), (1.0, 0.5), (1.5, 0.5), (2.0, 1.0), (3.0, 1.0), (4.0, 2.0)])
    pick = lo_step[rng.integers(0, len(lo_step), (rows, cols))]
    off = rng.integers(-1, 2, (rows, cols))
    pos = np.clip(u + off, 0, 65535) + 0.5
    x = pick[..., 0] + pick[..., 1] * pos / 65536
    x *= rng.choice([-1.0, 1.0], (rows, cols))
    if axis == 1:
        x[:, ::16] = 6.0
    else:
        x[::16, :] = 6.0
    x32 = x.astype(np.float32)
    assert np.array_equal(x32.astype(np.float64), x)
    got = run_both(torch.from_numpy(x32), axis, nv.SR, seed, nv.NVFP4, preset=1.0, what="sr-ties")
    assert np.all(to_np(got[1]) == 0x38)  # every block scale is 1.0


@pytest.mark.parametrize("fmt", list(FORMATS))
@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
@pytest.mark.parametrize("rounding", ["rtn-rtn", "sr-sr", "rtn-sr", "sr-rtn"])
def test_dual_orientation_matches_oracle(fmt, dtype, rounding):
    # Eqs. 5-6 use dY blocked along N and along M: one pass must give exactly the two
    # single-orientation results (blocks 16/32 run fused, 64/128 as two kernels); sizes span
    # several 128 x 256 tiles with ragged last tiles in both directions
    f = FORMATS[fmt]()
    B = f.block
    rr, rc = {"rtn-rtn": (0, 0), "sr-sr": (1, 1), "rtn-sr": (0, 1), "sr-rtn": (1, 0)}[rounding]
    for rows, cols, preset in ((2 * B, 2 * B, None), (128 + 3 * B, 512 + 5 * B, None), (384, 256, 0.37)):
        x = synth.student_t_outliers(rows, cols, 40 + rows, dtype=dtype)
        print(f"[case] dual {fmt} {dtype} rounding={rounding} shape=({rows},{cols}) preset={preset}", flush=True)
        ts = None if preset is None else torch.tensor([preset], dtype=torch.float32, device="cuda")
        qr, qc = nv.quantize_dual(x.cuda(), rr, 21, rc, 22, f, tensor_scale=ts)
        torch.cuda.synchronize()
        assert_quant_equal(qr, oracle.quantize(x, 1, rr, 21, ofmt(f), g=preset), "dual rows")
        assert_quant_equal(qc, oracle.quantize(x, 0, rc, 22, ofmt(f), g=preset), "dual cols")


def test_dual_orientation_strided_and_full_size():
    # a strided view (ld > cols), and the 7B gradient shape checked against the single-orientation kernels
    base = synth.student_t_outliers(160, 400, 9)
    x = base[:, 16:16 + 368]
    xg = base.cuda()[:, 16:16 + 368]
    qr, qc = nv.quantize_dual(xg, nv.SR, 5, nv.SR, 6, nv.NVFP4)
    torch.cuda.synchronize()
    xc = x.contiguous()
    assert_quant_equal(qr, oracle.quantize(xc, 1, nv.SR, 5, oracle.NVFP4), "dual strided rows")
    assert_quant_equal(qc, oracle.quantize(xc, 0, nv.SR, 6, oracle.NVFP4), "dual strided cols")
    dY = synth.gradient_like(4096, 11008, 77).cuda()
    for f in (nv.NVFP4, nv.MXFP4):
        g = nv.tensor_scale(dY) if f.tensor_scale else None
        qr, qc = nv.quantize_dual(dY, nv.SR, 1, nv.SR, 2, f, tensor_scale=g)
        r1 = nv.quantize(dY, 1, nv.SR, 1, f, tensor_scale=g)
        c1 = nv.quantize(dY, 0, nv.SR, 2, f, tensor_scale=g)
        torch.cuda.synchronize()
        for a, b in ((qr, r1), (qc, c1)):
            assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1]) and torch.equal(a[2], b[2])
