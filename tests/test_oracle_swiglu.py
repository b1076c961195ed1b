"""Pins of the oracle's SwiGLU backward (the elementwise step between the down layer's input gradient and the
gate/up layers' backward GEMMs): the fixed binary32 evaluation against the mathematics -- the exponential against
a library fp64 exp, dG and dU against finite differences of h = silu(g) u and against the closed form in fp64,
special values, and the rounding to the hand-over type."""
import numpy as np
import torch

import oracle
from paper_2505_19115_amd import synth


def _bf16_to_f64(a: np.ndarray) -> np.ndarray:
    return (a.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def _silu_u(g, u):
    return g / (1.0 + np.exp(-g)) * u


def test_exponential_matches_a_library_exp_to_three_ulp():
    ts = np.concatenate([np.linspace(0.0, -87.0, 20001), -np.random.default_rng(0).random(5000) * 20.0, [-0.0, -1e-30, -86.999]])
    got = np.array([oracle.exp_nonpos(t) for t in ts.astype(np.float32)], dtype=np.float64)
    ref = np.exp(ts.astype(np.float32).astype(np.float64))
    ulp = np.spacing(ref.astype(np.float32)).astype(np.float64)
    assert np.all(np.abs(got - ref) <= 3.0 * ulp), float((np.abs(got - ref) / ulp).max())
    assert oracle.exp_nonpos(0.0) == 1.0
    # below the clamp the value stays at exp(-87): a normal number, so every later operation is exact-safe
    assert oracle.exp_nonpos(-500.0) == oracle.exp_nonpos(-87.0) > 2.0 ** -126


def test_fp32_results_match_the_closed_form_and_finite_differences():
    rng = np.random.default_rng(1)
    n = 4096
    g = (rng.standard_normal((1, n)) * 3.0).astype(np.float32)
    u = rng.standard_normal((1, n)).astype(np.float32)
    h = (rng.standard_normal((1, n)) * 1e-3).astype(np.float32)
    dG, dU = oracle.swiglu_bwd(h, g, u)
    g64, u64, h64 = g.astype(np.float64), u.astype(np.float64), h.astype(np.float64)
    sig = 1.0 / (1.0 + np.exp(-g64))
    dG_ref = h64 * u64 * sig * (1.0 + g64 * (1.0 - sig))
    dU_ref = h64 * g64 * sig
    # each result is a product of a few rounded binary32 factors: a handful of ulp
    assert np.all(np.abs(dG - dG_ref) <= 4e-6 * np.abs(h64 * u64) * (1.0 + np.abs(g64)))
    assert np.all(np.abs(dU - dU_ref) <= 2e-6 * np.abs(h64 * g64) + 1e-300)
    # the same through central differences of h = silu(g) u (independent of the derivative formulas)
    eps = 1e-5
    fd_g = h64 * (_silu_u(g64 + eps, u64) - _silu_u(g64 - eps, u64)) / (2 * eps)
    fd_u = h64 * (_silu_u(g64, u64 + eps) - _silu_u(g64, u64 - eps)) / (2 * eps)
    assert np.all(np.abs(dG - fd_g) <= 1e-5 * np.abs(h64) * (1.0 + np.abs(u64)) * (1.0 + np.abs(g64)))
    assert np.all(np.abs(dU - fd_u) <= 1e-5 * np.abs(h64) * (1.0 + np.abs(g64)))


def test_special_values_and_symmetries():
    z = np.zeros((1, 4), np.float32)
    h = np.array([[1.0, -2.0, 0.5, 3.0]], np.float32)
    u = np.array([[2.0, 4.0, -8.0, 0.25]], np.float32)
    dG, dU = oracle.swiglu_bwd(h, z, u)
    assert np.array_equal(dG, h * u * 0.5) and np.array_equal(dU, z)          # sigma(0) = 1/2 exactly, silu(0) = 0
    big = np.array([[30.0, -30.0, 100.0, -100.0]], np.float32)
    dG, dU = oracle.swiglu_bwd(h, big, u)
    assert np.allclose(dG[0, 0], h[0, 0] * u[0, 0], rtol=1e-6) and np.allclose(dU[0, 0], h[0, 0] * 30.0, rtol=1e-6)
    assert abs(dG[0, 1]) < 1e-10 and abs(dU[0, 1]) < 1e-10                    # saturated negative gate: no gradient
    assert np.isfinite(dG).all() and np.isfinite(dU).all()
    assert dG[0, 2] == np.float32(h[0, 2] * u[0, 2]) and abs(dG[0, 3]) < 1e-30
    # dG is odd in dH and in u, dU is odd in dH and does not see u
    dG2, dU2 = oracle.swiglu_bwd(-h, big, u)
    assert np.array_equal(dG2, -dG) and np.array_equal(dU2, -dU)
    dG3, dU3 = oracle.swiglu_bwd(h, big, -u)
    assert np.array_equal(dG3, -dG) and np.array_equal(dU3, dU)
    # sigma(g) + sigma(-g) = 1 through dU = dH g sigma(g): dU(g) - dU(-g) = dH g (to rounding)
    g = np.array([[0.3, 1.7, 4.0, 9.0]], np.float32)
    one = np.ones_like(g)
    a, b = oracle.swiglu_bwd(one, g, one)[1], oracle.swiglu_bwd(one, -g, one)[1]
    assert np.allclose(a - b, g, rtol=3e-7, atol=0)


def test_bf16_hand_over_is_one_rounding_of_the_fp32_value():
    dH = synth.gradient_like(64, 96, 5)
    G, U = synth.normal(64, 96, 2.0, 6), synth.normal(64, 96, 1.0, 7)
    dG, dU = oracle.swiglu_bwd(dH, G, U)
    assert dG.dtype == np.uint16 and dG.shape == (64, 96)
    f32 = lambda t: t.float().numpy()
    rG, rU = oracle.swiglu_bwd(f32(dH), f32(G), f32(U))   # the same values before the final rounding
    want = lambda r: torch.from_numpy(r).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(dG, want(rG)) and np.array_equal(dU, want(rU))   # an independent bf16 cast
    # and the quantizer accepts the hand-over as it is
    codes, scales, g = oracle.quantize(dG, 1, oracle.SR, 3)
    assert codes.shape == (64, 48) and g > 0
    assert np.float32(np.abs(_bf16_to_f64(dG)).max()) / np.float32(2688.0) == np.float32(g)
