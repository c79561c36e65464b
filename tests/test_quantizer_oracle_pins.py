"""Pins for the quantizer oracle (CPU).  The quantizer is an iteration with integer decisions, so it
is pinned by what the paper and the mathematics fix: the closed form of the first ridge solve, the
normal equations at every step, per-element optimality over the nine candidates (with the stated
tie order), the monotone trit step, exact invariances (power-of-two scaling, permutation inside a
group), exactly representable inputs, and numpy's binary16 rounding for the stored scales.
Paper: Sec. "Dual Trit-planes Approximation", "Progressive Optimization", both algorithm listings,
appendix "Implementation Details" and "Computational Complexity"."""
from fractions import Fraction

import numpy as np
import pytest

import oracle

G = 128


def _w(n=6, k=512, seed=0, scale=0.02):
    return (np.random.default_rng(seed).standard_normal((n, k)) * scale).astype(np.float16)


def _err(W, q, a1="a1_f64", a2="a2_f64", group=G):
    What = oracle.reconstruct_dense(q["T1"], q["T2"], q[a1], q[a2], group=group)
    return np.linalg.norm(W.astype(np.float64) - What)


def test_zero_iterations_is_the_initialisation():
    W = _w()
    W[0, 3] = 0.0
    W[1, 7] = -0.0
    q = oracle.quantize(W, max_iters=0)
    s = np.where(W.astype(np.float64) < 0, -1, 1)            # sign(W) with 0 -> +1
    assert np.array_equal(q["T1"], s) and np.array_equal(q["T2"], s)
    assert np.all(q["a1_f64"] == 1) and np.all(q["a2_f64"] == 1) and np.all(q["lam"] == 1e-8)
    assert q["iters"] == 0


def test_first_solve_closed_form():
    # identical planes: A = [[G+l, G], [G, G+l]], b = [sum|w|, sum|w|]  =>  alpha1 = alpha2 = sum|w| / (2G + l)
    # kappa = ||A||_F ||A^-1||_F >= 1e6 at l = 1e-8, so l is raised once (before the solve) to l*sqrt(kappa/1e6)
    W = _w(4, 256, 1)
    q = oracle.quantize(W, max_iters=1, eps=0.0)
    l0 = 1e-8
    A = np.array([[G + l0, G], [G, G + l0]])
    # ||A^-1||_F = ||A||_F / |det A| for a 2x2 matrix; det written out to avoid cancellation in the check itself
    kappa = (np.linalg.norm(A) ** 2) / (2 * G * l0 + l0 * l0)
    assert kappa >= 1e6
    l1 = min(1.0, l0 * np.sqrt(kappa / 1e6))
    # kappa comes out of a cancelling determinant (as in the algorithm): good to ~1e-6 in binary64
    assert np.allclose(q["lam"], l1, rtol=1e-5)
    sabs = np.abs(W.astype(np.float64)).reshape(4, 2, G).sum(-1)
    lam = q["lam"].astype(np.float64)
    assert np.allclose(q["a1_f64"], sabs / (2 * G + lam), rtol=1e-5)
    assert np.array_equal(q["a1_f64"], q["a2_f64"])
    assert np.allclose(q["a1_f64"] + q["a2_f64"], sabs / G, rtol=1e-5)                       # mean |w|


@pytest.mark.parametrize("t", [2, 3, 7, 20])
def test_alpha_solves_the_ridge_normal_equations(t):
    W = _w(8, 384, 2)
    prev = oracle.quantize(W, max_iters=t - 1, eps=0.0)
    cur = oracle.quantize(W, max_iters=t, eps=0.0)
    w = W.astype(np.float64).reshape(8, 3, G)
    t1 = prev["T1"].astype(np.float64).reshape(8, 3, G)
    t2 = prev["T2"].astype(np.float64).reshape(8, 3, G)
    for n in range(8):
        for g in range(3):
            S = np.stack([t1[n, g], t2[n, g]], axis=1)
            lam = float(cur["lam"][n, g])
            A = S.T @ S + lam * np.eye(2)
            ref = np.linalg.solve(A, S.T @ w[n, g])
            got = np.array([cur["a1_f64"][n, g], cur["a2_f64"][n, g]], dtype=np.float64)
            cond = np.linalg.cond(A)
            assert np.allclose(got, ref, rtol=0, atol=1e-15 * cond * np.abs(ref).max() + 1e-18), (n, g, cond)
            # lambda only ever grows, never past 1, and only moves when the system is ill-conditioned
            assert float(prev["lam"][n, g]) <= lam <= 1.0


def test_every_trit_pair_is_the_first_minimum_of_the_nine_candidates():
    W = _w(5, 256, 3)
    q = oracle.quantize(W, max_iters=9, eps=0.0)
    order = [(c1, c2) for c1 in (-1, 0, 1) for c2 in (-1, 0, 1)]
    for n in range(5):
        for j in range(256):
            a1 = Fraction(float(q["a1_f64"][n, j // G]))
            a2 = Fraction(float(q["a2_f64"][n, j // G]))
            w = Fraction(float(W[n, j]))
            errs = [(w - a1 * c1 - a2 * c2) ** 2 for c1, c2 in order]
            chosen = (int(q["T1"][n, j]), int(q["T2"][n, j]))
            e_chosen = errs[order.index(chosen)]
            best = min(errs)
            # exact optimum up to binary64 rounding of the three operations that form the error
            assert e_chosen <= best + Fraction(1, 10 ** 14) * (best + w * w + Fraction(1, 10 ** 20))


def test_tie_break_order_on_exact_ties():
    # alpha1 == alpha2 after the first solve, so every value is hit by several pairs: the first one in the
    # order c1 = -1,0,1 (outer), c2 = -1,0,1 (inner) must win.  w = +-a or 0 exactly after a power-of-two setup:
    # G = 4, |w| = 1 everywhere => alpha1 = alpha2 = 4/(8+l) ~ 0.5; candidates 2a=1 -> (1,1); -1 -> (-1,-1)
    W = np.array([[1, -1, 1, 1]], dtype=np.float16)
    q = oracle.quantize(W, group=4, max_iters=1, eps=0.0)
    assert q["T1"].tolist() == [[1, -1, 1, 1]] and q["T2"].tolist() == [[1, -1, 1, 1]]
    # |w| in {1, 0.5-ish}: with w = (2,2,2,1): alpha = 7/(8+l) ~ 0.875 each; 1 is nearest to a (0.875): first pair with
    # value +a is (0, 1); 2 is nearest to 2a = 1.75: (1, 1)
    W = np.array([[2, 2, 2, 1]], dtype=np.float16)
    q = oracle.quantize(W, group=4, max_iters=1, eps=0.0)
    assert q["T1"].tolist() == [[1, 1, 1, 0]] and q["T2"].tolist() == [[1, 1, 1, 1]]
    # a value nearest to 0: first pair with value 0 when alpha1 == alpha2 is (-1, +1)
    W = np.array([[2, 2, 2, 0.25]], dtype=np.float16)
    q = oracle.quantize(W, group=4, max_iters=1, eps=0.0)
    assert q["T1"][0, 3] == -1 and q["T2"][0, 3] == 1


def test_trit_step_never_increases_the_error():
    W = _w(6, 512, 4)
    for t in (1, 2, 5, 12):
        prev = oracle.quantize(W, max_iters=t - 1, eps=0.0)
        cur = oracle.quantize(W, max_iters=t, eps=0.0)
        mixed = {"T1": prev["T1"], "T2": prev["T2"], "a1_f64": cur["a1_f64"], "a2_f64": cur["a2_f64"]}
        assert _err(W, cur) <= _err(W, mixed) * (1 + 1e-6)


def test_converges_and_beats_sign_quantisation():
    W = _w(16, 1024, 5)
    q = oracle.quantize(W)                       # eps = 1e-4, T_max = 50 (the paper's settings)
    assert 1 <= q["iters"] <= 50
    again = oracle.quantize(W, max_iters=q["iters"], eps=0.0)
    assert np.array_equal(q["T1"], again["T1"]) and np.array_equal(q["a1_f64"], again["a1_f64"])
    wn = np.linalg.norm(W.astype(np.float64))
    assert _err(W, q) / wn < 0.25
    # best single sign plane with one scale per group (binary quantisation): relative error ~0.6 on Gaussian weights
    w = W.astype(np.float64).reshape(16, 8, G)
    binq = np.sign(w) * np.abs(w).mean(-1, keepdims=True)
    assert _err(W, q) < 0.5 * np.linalg.norm(w - binq)
    # stored scales are the binary16 rounding of the iteration's scales
    assert np.array_equal(q["a1"], q["a1_f64"].astype(np.float16))
    assert np.array_equal(q["a2"], q["a2_f64"].astype(np.float16))


def test_exactly_ternary_rows_are_recovered():
    # w in {-c, 0, +c}: after convergence the reconstruction is exact up to the ridge shrinkage
    r = np.random.default_rng(6)
    c = np.float16(0.0625)
    W = (r.integers(-1, 2, size=(4, 256)) * c).astype(np.float16)
    q = oracle.quantize(W, max_iters=50, eps=0.0)
    What = oracle.reconstruct_dense(q["T1"], q["T2"], q["a1_f64"], q["a2_f64"])
    assert np.abs(What - W.astype(np.float64)).max() < 2e-3 * float(c)


def test_power_of_two_scaling_is_exact():
    W = _w(4, 256, 7)
    q1 = oracle.quantize(W, max_iters=15, eps=0.0)
    q2 = oracle.quantize((W * np.float16(8)).astype(np.float16), max_iters=15, eps=0.0)
    assert np.array_equal(q1["T1"], q2["T1"]) and np.array_equal(q1["T2"], q2["T2"])
    assert np.array_equal(q1["a1_f64"] * 8.0, q2["a1_f64"])
    assert np.array_equal(q1["a2_f64"] * 8.0, q2["a2_f64"])


def test_permutation_inside_a_group_permutes_the_trits():
    W = _w(3, 256, 8)
    perm = np.random.default_rng(8).permutation(G)
    Wp = W.copy()
    Wp[:, :G] = W[:, :G][:, perm]
    q1 = oracle.quantize(W, max_iters=12, eps=0.0)
    q2 = oracle.quantize(Wp, max_iters=12, eps=0.0)
    assert np.array_equal(q1["a1_f64"], q2["a1_f64"]) and np.array_equal(q1["a2_f64"], q2["a2_f64"])
    assert np.array_equal(q1["T1"][:, :G][:, perm], q2["T1"][:, :G])
    assert np.array_equal(q1["T2"][:, G:], q2["T2"][:, G:])


def test_units_are_independent_and_convergence_is_global():
    W = _w(4, 256, 9)
    q = oracle.quantize(W, max_iters=6, eps=0.0)
    sub = oracle.quantize(W[1:2, G:], max_iters=6, eps=0.0)
    assert np.array_equal(sub["T1"], q["T1"][1:2, G:]) and np.array_equal(sub["a2_f64"], q["a2_f64"][1:2, 1:])
    # the stopping rule looks at the Frobenius norm of the change of ALL scales of the matrix
    a = oracle.quantize(W, eps=1e-4)["iters"]
    b = oracle.quantize(np.concatenate([W, _w(4, 256, 10)]), eps=1e-4)["iters"]
    c = oracle.quantize(_w(4, 256, 10), eps=1e-4)["iters"]
    assert b >= max(a, c)


def test_stopping_rule_is_the_norm_not_its_square():
    # alpha after t iterations, for every t, from restarts with max_iters = t (the iteration is deterministic): the
    # stopping iteration for a given eps then follows from the Frobenius norms of the changes alone
    W = _w(4, 256, 12)
    alphas = []
    for t in range(0, 13):
        q = oracle.quantize(W, max_iters=t, eps=0.0)
        alphas.append(np.concatenate([q["a1_f64"].ravel(), q["a2_f64"].ravel()]))
    deltas = np.array([np.sqrt(np.sum((alphas[t] - alphas[t - 1]) ** 2)) for t in range(1, 13)])   # change made by iteration t
    t_star = 5
    assert deltas[t_star - 1] < deltas[t_star - 2] < 1.0            # still shrinking there, and below 1 (so d*d < d)
    eps = float(np.sqrt(deltas[t_star - 1] * deltas[t_star - 2]))  # between the changes of iterations t*-1 and t*
    by_norm = 1 + int(np.argmax(deltas < eps))
    by_square = 1 + int(np.argmax(deltas ** 2 < eps))
    assert by_norm == t_star and by_square < by_norm                # the two rules really differ on this input
    assert oracle.quantize(W, max_iters=50, eps=eps)["iters"] == by_norm


def test_lambda_is_capped_at_one():
    # lambda_max = 1 (hyper-parameters of the experiments; second listing).  With groups of 128 the cap is out of reach
    # (the update has the fixed point 2G / 1e6), so the pin uses ONE unit of G = 2^20 equal weights: T1 = T2 = +1 is
    # then a fixed point of the trit search (alpha1 + alpha2 = c reproduces every entry), A = [[G + l, G], [G, G + l]]
    # stays as singular as l allows, and l follows l <- l * sqrt(kappa / 1e6) from 1e-8 up: 1.4e-4, 1.7e-2, 0.19, 0.63,
    # then 1.15 -> capped.  The recurrence is rebuilt here with numpy's inverse and norms.
    big = 1 << 20
    c = np.float16(0.25)
    W = np.full((1, big), c, dtype=np.float16)
    lam, seen = 1e-8, []
    for _ in range(8):
        A = np.array([[big + lam, big], [big, big + lam]], dtype=np.float64)
        kappa = np.linalg.norm(A) * np.linalg.norm(np.linalg.inv(A))
        if not kappa < 1e6:
            lam = min(1.0, lam * np.sqrt(kappa / 1e6))
        seen.append(lam)
    assert seen[3] < 1.0 and seen[4] == 1.0 and seen[-1] == 1.0        # the cap is what stops the growth
    for t in (1, 2, 4, 5, 8):
        q = oracle.quantize(W, group=big, max_iters=t, eps=0.0)
        assert q["iters"] == t
        # the cancelling determinant limits kappa, hence lambda below the cap, to ~1e-6 relative
        assert abs(q["lam"][0, 0] - seen[t - 1]) <= 1e-5 * seen[t - 1]
        if t >= 5:
            assert q["lam"][0, 0] == 1.0
        assert np.all(q["T1"] == 1) and np.all(q["T2"] == 1)
        alpha = float(c) * big / (2.0 * big + q["lam"][0, 0])              # closed form of the ridge solve on this unit
        assert abs(q["a1_f64"][0, 0] - alpha) <= 1e-9 * alpha and abs(q["a2_f64"][0, 0] - alpha) <= 1e-9 * alpha


def test_double_to_half_rounding_matches_numpy():
    r = np.random.default_rng(11)
    h = np.arange(0, 0x7c00, dtype=np.uint16).view(np.float16).astype(np.float64)      # every finite binary16 value
    mid = (h[:-1] + h[1:]) / 2                                                          # every exact tie
    vals = np.concatenate([
        r.standard_normal(20000) * 0.05, r.standard_normal(5000) * 1e-6, h, -h, mid, -mid,
        np.nextafter(mid, np.inf), np.nextafter(mid, -np.inf),
        np.array([0.0, -0.0, 65504.0, 65519.999, 65520.0, 1e9, -1e9, 6.1e-5, 5.96e-8, 2.98e-8, 2.99e-8, 1e-9, 1e-30,
                  1.0009765625, 1.00048828125, 1.001464843750,
                  1.00048828125 + 2.0 ** -40, 1.00048828125 - 2.0 ** -40])])     # would break under double rounding
    got = np.array([oracle.double_to_half_bits(float(v)) for v in vals], dtype=np.uint16)
    with np.errstate(over="ignore"):
        ref = vals.astype(np.float16).view(np.uint16)
    assert np.array_equal(got, ref)


def test_rejects_bad_shapes():
    with pytest.raises(oracle.OracleError):
        oracle.quantize(_w(2, 200))
    with pytest.raises(TypeError):
        oracle.quantize(_w(2, 256).astype(np.float32))
