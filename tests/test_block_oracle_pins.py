"""Pins for the decoder-block oracle (silu, gated MLP epilogue, residual add, binary16 rounding).

Everything here runs on the CPU and checks oracle/ptqtp_block_oracle.c against things that
are not itself: closed forms and identities of silu, a library sigmoid, a library silu on the
dense reconstruction of a whole gated MLP, numpy's own binary16 rounding.
"""
import math

import numpy as np
import pytest
import scipy.special
import torch

import oracle
import workloads


def test_silu_closed_forms():
    assert oracle.silu(0.0) == 0.0
    # silu(z) - silu(-z) = z because sigmoid(z) + sigmoid(-z) = 1
    for z in (1e-3, 0.5, 1.0, 2.75, 11.0, 30.0):
        assert oracle.silu(z) - oracle.silu(-z) == pytest.approx(z, rel=1e-15)
    # large |z|: silu(z) -> z (1 - e^-z), silu(-z) -> -z e^-z
    assert oracle.silu(40.0) == pytest.approx(40.0 * (1 - math.exp(-40.0)), rel=1e-15)
    assert oracle.silu(-40.0) == pytest.approx(-40.0 * math.exp(-40.0), rel=1e-12)
    # silu(1) = 1 / (1 + 1/e)
    assert oracle.silu(1.0) == pytest.approx(1.0 / (1.0 + 1.0 / math.e), rel=1e-15)


def test_silu_minimum_and_slope_bound():
    # the minimum solves 1 + e^-z (1 + z) = 0  ->  z* = -1.27846454..., silu(z*) = -0.27846454...  (silu(z*) = z* + 1)
    zs = np.linspace(-1.3, -1.25, 50001)
    vals = np.array([oracle.silu(z) for z in zs])
    i = int(vals.argmin())
    assert zs[i] == pytest.approx(-1.2784645, abs=2e-6)
    assert vals[i] == pytest.approx(-1.2784645427610738 + 1.0, abs=1e-11)      # silu(z*) = z* + 1 at the stationary point
    # numerical slope never exceeds the Lipschitz constant the error bounds use
    z = np.linspace(-20, 20, 400001)
    v = np.array([oracle.silu(t) for t in z])
    slope = np.abs(np.diff(v) / np.diff(z))
    assert slope.max() < oracle.SILU_LIPSCHITZ and slope.max() > 1.0997


def test_silu_against_library_sigmoid():
    rng = np.random.default_rng(5)
    z = np.concatenate([rng.normal(0, 3, 2000), [-700.0, -30.0, 30.0, 700.0]])
    ref = z * scipy.special.expit(z)
    got = np.array([oracle.silu(t) for t in z])
    np.testing.assert_allclose(got, ref, rtol=4e-16, atol=1e-300)


def test_swiglu_order_and_hand_case():
    # gate columns first, up columns second; one hand-computed row
    y = np.array([[0.0, 1.0, -2.0, 5.0, 3.0, 7.0]])
    h = oracle.swiglu(y, 3)
    expect = [0.0 * 5.0, (1.0 / (1.0 + math.exp(-1.0))) * 3.0, (-2.0 / (1.0 + math.exp(2.0))) * 7.0]
    np.testing.assert_allclose(h[0], expect, rtol=1e-15)
    # swapping the halves is a different function
    assert not np.allclose(oracle.swiglu(y[:, [3, 4, 5, 0, 1, 2]], 3), h)
    with pytest.raises(oracle.OracleError):
        oracle.swiglu(np.zeros((1, 5)), 3)


def test_gated_mlp_against_library_on_dense_weights():
    # mlp(x) = W_down (silu(W_gate x) * W_up x) with every W rebuilt densely and library ops in float64
    I, H, M = 96, 256, 3
    gu = workloads.make_linear(2 * I, H, 91, 1)
    dn = workloads.make_linear(H, I + 32, 91, 2)     # K of down = 128 (one group)
    x = workloads.make_x(M, H, 91, 3)
    st = oracle.stage(gu, x, "swiglu")
    Wgu = torch.from_numpy(oracle.reconstruct_dense(gu["T1"], gu["T2"], gu["a1"], gu["a2"]))
    xt = torch.from_numpy(x.astype(np.float64))
    g = xt @ Wgu[:I].T
    u = xt @ Wgu[I:].T
    h_ref = torch.nn.functional.silu(g) * u
    np.testing.assert_allclose(st["out"], h_ref.numpy(), rtol=1e-12, atol=1e-15)
    # feed the binary16 rounding of h to down, add the residual
    h16 = np.zeros((M, I + 32), np.float16)
    h16[:, :I] = oracle.round_half(st["out"]).astype(np.float16)
    res = workloads.make_x(M, H, 91, 4)
    st2 = oracle.stage(dn, h16, "none", residual=res)
    Wd = torch.from_numpy(oracle.reconstruct_dense(dn["T1"], dn["T2"], dn["a1"], dn["a2"]))
    ref2 = torch.from_numpy(h16.astype(np.float64)) @ Wd.T + torch.from_numpy(res.astype(np.float64))
    np.testing.assert_allclose(st2["out"], ref2.numpy(), rtol=1e-12, atol=1e-15)


def test_stage_error_bound_covers_perturbed_linear():
    # move every entry of the linear's result by +-tau*B: the epilogue's result moves by at most tau*E + tau^2*E2
    I, H, M = 64, 128, 2
    gu = workloads.make_linear(2 * I, H, 92, 1)
    x = workloads.make_x(M, H, 92, 2)
    st = oracle.stage(gu, x, "swiglu")
    y, B = oracle.forward(gu["T1"], gu["T2"], gu["a1"], gu["a2"], x)
    rng = np.random.default_rng(6)
    tau = 2e-3
    for _ in range(20):
        yp = y + tau * B * rng.choice([-1.0, 1.0], size=y.shape)
        hp = oracle.swiglu(yp, I)
        assert np.all(np.abs(hp - st["out"]) <= tau * st["err"] + tau * tau * st["err2"] + 1e-18)


def test_residual_add_and_shapes():
    y = np.array([[1.5, -2.25, 1e-8]])
    r = np.array([[0.5, 2.25, 1.0]], dtype=np.float16)
    np.testing.assert_array_equal(oracle.residual_add(y, r), [[2.0, 0.0, 1.0 + 1e-8]])
    with pytest.raises(oracle.OracleError):
        oracle.residual_add(y, r[:, :2])


def test_round_half_against_numpy():
    rng = np.random.default_rng(7)
    v = np.concatenate([rng.normal(0, 1, 4000), rng.normal(0, 1e-6, 2000), rng.normal(0, 3e4, 2000),
                        [0.0, -0.0, 65504.0, 65519.9, 65520.0, -65520.0, 2.0 ** -24, 2.0 ** -25, 3 * 2.0 ** -25,
                         1.0 + 2.0 ** -11, 1.0 + 3 * 2.0 ** -11, 6.1e-5, 5.96e-8]])
    with np.errstate(over="ignore"):
        ref = v.astype(np.float16).astype(np.float64)
    got = oracle.round_half(v)
    np.testing.assert_array_equal(got, ref)
    # exact halves round to even
    assert oracle.round_half(np.array([1.0 + 2.0 ** -11]))[0] == 1.0
    assert oracle.round_half(np.array([1.0 + 3 * 2.0 ** -11]))[0] == 1.0 + 2.0 ** -9


def test_forward_fused_pins():
    # (a) within 2^-11 of the L1 bound of the unfused layer, and not identical to it on general scales
    lin = workloads.make_linear(96, 512, 93, 1)
    x = workloads.make_x(5, 512, 93, 2)
    y, B = oracle.forward(lin["T1"], lin["T2"], lin["a1"], lin["a2"], x)
    yf, Bf = oracle.forward_fused(lin["T1"], lin["T2"], lin["a1"], lin["a2"], x)
    assert np.all(np.abs(yf - y) <= 2.0 ** -11 * B * (1 + 1e-12))
    assert np.abs(yf - y).max() > 0
    # (b) scales whose sums are binary16 numbers: rounding changes nothing
    lin2, x2 = workloads.integer_exact_case(48, 384, 3, 93, 3)
    y2, _ = oracle.forward(lin2["T1"], lin2["T2"], lin2["a1"], lin2["a2"], x2)
    y2f, _ = oracle.forward_fused(lin2["T1"], lin2["T2"], lin2["a1"], lin2["a2"], x2)
    np.testing.assert_array_equal(y2f, y2)
    # (c) one plane empty: the other plane's products are binary16 already
    lin3 = dict(lin); lin3["T2"] = np.zeros_like(lin["T2"])
    y3, _ = oracle.forward(lin3["T1"], lin3["T2"], lin3["a1"], lin3["a2"], x)
    y3f, _ = oracle.forward_fused(lin3["T1"], lin3["T2"], lin3["a1"], lin3["a2"], x)
    np.testing.assert_allclose(y3f, y3, rtol=1e-13, atol=1e-15)
    # (d) against numpy's own rounding of the dense weight and a float64 matmul, entry by entry
    W = oracle.reconstruct_dense(lin["T1"], lin["T2"], lin["a1"], lin["a2"])
    ref = x.astype(np.float64) @ W.astype(np.float16).astype(np.float64).T
    np.testing.assert_allclose(yf, ref, rtol=1e-13, atol=1e-15)
