"""Pins for the CPU oracle's CG (Alg. 2), line search (Alg. 3) and SSN loop (Alg. 1); no GPU."""
import numpy as np
import pytest

from oracle.oracle import Problem
from paper_1802_09113_amd import synth
from tests.test_oracle_hessian import explicit_hessian


def tiny(n=400, p=5, C=3, lam=1e-2, seed=21):
    g = np.random.default_rng(seed)
    X = g.standard_normal((n, p))
    Wt = g.standard_normal((p, C))
    labels = np.argmax(X @ Wt + g.gumbel(size=(n, C)), axis=1).astype(np.int32)
    return Problem(labels, C, lam, X=X), X, labels, g


def test_cg_converges_to_newton_direction_on_tiny_spd_system():
    pr, X, labels, g = tiny()
    W = 0.3 * g.standard_normal((pr.p, pr.K))
    S = np.sort(g.choice(pr.n, 100, replace=False)).astype(np.int32)
    grad, _ = pr.gradient(W)
    H = explicit_hessian(X, W, S, pr.lam, 1.0 / S.size)
    exact = -np.linalg.solve(H, grad.reshape(-1)).reshape(pr.p, pr.K)
    out = pr.cg(W, S, grad, theta=1e-14, T=4 * pr.d)
    assert np.linalg.norm(out["p"] - exact) <= 1e-10 * np.linalg.norm(exact)
    # textbook CG in exact arithmetic ends within d products; allow rounding slack
    assert out["iters"] <= 2 * pr.d


def test_cg_reported_residual_matches_returned_iterate_and_trace():
    pr, X, labels, g = tiny(seed=22)
    W = 0.3 * g.standard_normal((pr.p, pr.K))
    S = np.sort(g.choice(pr.n, 60, replace=False)).astype(np.int32)
    grad, _ = pr.gradient(W)
    H = explicit_hessian(X, W, S, pr.lam, 1.0 / S.size)
    gn = np.linalg.norm(grad)
    for T in (1, 2, 3, 5):
        out = pr.cg(W, S, grad, theta=1e-30, T=T)
        assert out["iters"] == T
        res = np.linalg.norm(H @ out["p"].reshape(-1) + grad.reshape(-1)) / gn
        assert res == pytest.approx(out["rel_res"], rel=1e-9)
        assert out["rel_res"] <= 1.0 + 1e-15
        assert out["rel_res"] == pytest.approx(out["rnorm"].min() / gn if out["rnorm"].min() <= gn else 1.0, rel=1e-12)
    # first step: alpha_0 = g.g / g.H.g and r_1 = -g - alpha_0 H(-g)
    a0 = (grad.reshape(-1) @ grad.reshape(-1)) / (grad.reshape(-1) @ H @ grad.reshape(-1))
    out = pr.cg(W, S, grad, theta=1e-30, T=1)
    assert out["alpha"][0] == pytest.approx(a0, rel=1e-12)
    r1 = -grad.reshape(-1) + a0 * (H @ grad.reshape(-1))
    assert out["rnorm"][0] == pytest.approx(np.linalg.norm(r1), rel=1e-10)


def test_cg_second_iterate_is_the_two_dimensional_krylov_minimiser():
    # CG's k-th iterate minimises the quadratic over span{g, Hg, ...}: check k = 2 by a 2x2 solve.
    pr, X, labels, g = tiny(seed=23)
    W = 0.2 * g.standard_normal((pr.p, pr.K))
    S = np.arange(0, pr.n, 3, dtype=np.int32)
    grad, _ = pr.gradient(W)
    H = explicit_hessian(X, W, S, pr.lam, 1.0 / S.size)
    gv = grad.reshape(-1)
    B = np.stack([gv, H @ gv], axis=1)
    coef = np.linalg.solve(B.T @ H @ B, -B.T @ gv)
    x2 = B @ coef
    out = pr.cg(W, S, grad, theta=1e-30, T=2)
    # the returned p_best is p_2 as long as ||r_2|| <= ||r_1|| <= ||r_0||, true for this well-conditioned case
    assert np.all(np.diff(np.concatenate([[np.linalg.norm(gv)], out["rnorm"]])) <= 0)
    assert np.linalg.norm(out["p"].reshape(-1) - x2) <= 1e-9 * np.linalg.norm(x2)


def test_cg_stops_on_theta_and_handles_zero_budget_and_zero_gradient():
    pr, X, labels, g = tiny(seed=24)
    W = 0.1 * g.standard_normal((pr.p, pr.K))
    S = np.arange(pr.n, dtype=np.int32)
    grad, _ = pr.gradient(W)
    out = pr.cg(W, S, grad, theta=0.5, T=50)
    assert out["flags"] & 1 and out["iters"] < 50
    assert out["rnorm"][-1] <= 0.5 * np.linalg.norm(grad)
    assert np.all(out["rnorm"][:-1] > 0.5 * np.linalg.norm(grad))
    # T = 0: nothing is multiplied, p_best stays at its initial value s_0 = -g
    out0 = pr.cg(W, S, grad, theta=1e-4, T=0)
    assert out0["iters"] == 0
    np.testing.assert_array_equal(out0["p"], -grad)
    outz = pr.cg(W, S, np.zeros_like(grad), theta=1e-4, T=5)
    assert outz["iters"] == 0 and np.all(outz["p"] == 0)


def test_linesearch_returns_first_power_of_rho_that_satisfies_armijo():
    pr, X, labels, g = tiny(seed=25)
    W = 0.5 * g.standard_normal((pr.p, pr.K))
    grad, f = pr.gradient(W)
    beta, rho = 1e-4, 0.5
    for stretch in (1.0, 30.0, 500.0):
        P = -stretch * grad / pr.lam * 0.05      # a descent direction, too long for large stretch
        out = pr.linesearch(W, P, grad, f, beta=beta, rho=rho, imax=40)
        j = out["n_eval"] - 1
        assert out["ok"] == 1
        assert out["alpha"] == rho ** j
        slope = np.sum(P * grad)
        assert slope < 0
        assert out["f_new"] == pytest.approx(pr.objective(W + out["alpha"] * P), rel=1e-15)
        assert out["f_new"] <= f + out["alpha"] * beta * slope
        for i in range(j):                        # every earlier trial must have failed
            a = rho ** i
            assert pr.objective(W + a * P) > f + a * beta * slope
    assert j > 0                                   # the longest direction really needed back-tracking


def test_linesearch_gives_up_after_imax_reductions():
    pr, X, labels, g = tiny(seed=26)
    W = 0.5 * g.standard_normal((pr.p, pr.K))
    grad, f = pr.gradient(W)
    out = pr.linesearch(W, grad, grad, f, beta=1e-4, rho=0.5, imax=3)      # ascent direction: never accepted
    # trials at alpha = 1, rho, ..., rho^(imax+1); the exit test i > imax sits after the Armijo test
    assert out["ok"] == 0 and out["n_eval"] == 3 + 2
    assert out["alpha"] == 0.5 ** 4


def test_ssn_decreases_objective_and_reaches_the_optimum_with_full_hessian():
    d = synth.make(0, n=1000)
    pr = Problem(d["labels"], d["C"], d["lam"], X=d["X"])
    iters = 12
    S_all = np.tile(np.arange(pr.n, dtype=np.int32), (iters, 1))            # full Newton
    W, log, done = pr.ssn(np.zeros((pr.p, pr.K)), S_all, eps=0.0, theta=1e-10, T=10 * pr.d)
    assert done == iters
    f = log[:, 0]
    assert f[0] == pytest.approx(np.log(pr.C), rel=1e-13)
    assert np.all(np.diff(f) <= 1e-15)
    G, _ = pr.gradient(W)
    assert np.linalg.norm(G) < 1e-10
    assert np.all(log[:, 4] == 1.0)               # Newton steps with exact solves take alpha = 1 here


def test_ssn_subsampled_schedule_and_eps_stop():
    d = synth.make(0)
    pr = Problem(d["labels"], d["C"], d["lam"], X=d["X"])
    S_all = synth.sample_schedule(pr.n, d["nS"], d["iters"])
    assert S_all.shape == (10, 100) and np.all(np.diff(S_all, axis=1) > 0)
    W, log, done = pr.ssn(np.zeros((pr.p, pr.K)), S_all, theta=1e-4, T=10)
    assert done == 10
    assert np.all(np.diff(log[:, 0]) < 0)
    assert np.all(np.abs(log[:, 5]) >= 1) and np.all(log[:, 2] <= 10)
    # replay the first iteration by hand from the pinned parts
    G0, f0 = pr.gradient(np.zeros((pr.p, pr.K)))
    cg = pr.cg(np.zeros((pr.p, pr.K)), S_all[0], G0, 1e-4, 10)
    ls = pr.linesearch(np.zeros((pr.p, pr.K)), cg["p"], G0, f0)
    W1 = ls["alpha"] * cg["p"]
    assert log[1, 0] == pytest.approx(pr.objective(W1), rel=1e-14)
    assert log[0, 4] == ls["alpha"] and log[0, 2] == cg["iters"]
    # a huge eps stops before the first update
    W2, log2, done2 = pr.ssn(np.zeros((pr.p, pr.K)), S_all, eps=1e9)
    assert done2 == 0 and np.all(W2 == 0)


def _krylov_iterates(H, gv, T):
    """p_1..p_T of CG on H p = -g without CG's recurrences: p_k minimises the quadratic over the Krylov space
    span{g, Hg, .., H^(k-1) g}, built here with an orthonormal basis (Gram-Schmidt, twice) and a dense solve."""
    Q = np.zeros((gv.size, 0))
    v = gv.copy()
    out = []
    for _ in range(T):
        for _ in range(2):
            v = v - Q @ (Q.T @ v)
        Q = np.concatenate([Q, (v / np.linalg.norm(v))[:, None]], axis=1)
        y = np.linalg.solve(Q.T @ H @ Q, -Q.T @ gv)
        out.append(Q @ y)
        v = H @ Q[:, -1]
    return out


@pytest.mark.parametrize("seed", [31, 37, 43, 47])
def test_cg_keeps_the_iterate_of_smallest_residual_when_the_residual_rises(seed):
    """Best-iterate memory of Alg. 2 on ill-conditioned systems whose residual norm goes up and down: for every
    budget T the direction returned is the p_k (k <= T) of smallest ||H p_k + g||, not the last one, and it is
    the start value s_0 = -g while no iterate has a residual at most ||g||."""
    g = np.random.default_rng(seed)
    n, p, C = 60, 6, 3
    X = g.standard_normal((n, p)) * np.array([0.2, 0.5, 1.0, 2.0, 5.0, 10.0])
    Wt = g.standard_normal((p, C))
    labels = np.argmax(X @ Wt + g.gumbel(size=(n, C)), axis=1).astype(np.int32)
    pr = Problem(labels, C, 1e-3, X=X)
    W = 0.3 * g.standard_normal((p, C - 1))
    S = np.sort(g.choice(n, 40, replace=False)).astype(np.int32)
    grad, _ = pr.gradient(W)
    gv = grad.reshape(-1)
    gn = np.linalg.norm(gv)
    H = explicit_hessian(X, W, S, pr.lam, 1.0 / S.size)
    Tmax = 8
    iterates = _krylov_iterates(H, gv, Tmax)
    res = np.array([np.linalg.norm(H @ pk + gv) for pk in iterates])
    full = pr.cg(W, S, grad, theta=1e-30, T=Tmax)
    # the residual norms of the oracle's trace are those of the Krylov minimisers, and they do rise
    np.testing.assert_allclose(full["rnorm"], res, rtol=1e-6)
    assert np.any(np.diff(np.concatenate([[gn], res])) > 0)
    saw_not_last = saw_start = False
    for T in range(1, Tmax + 1):
        out = pr.cg(W, S, grad, theta=1e-30, T=T)
        assert out["iters"] == T
        best = int(np.argmin(res[:T]))
        pv = out["p"].reshape(-1)
        if res[best] <= gn:
            assert np.linalg.norm(pv - iterates[best]) <= 1e-6 * np.linalg.norm(iterates[best])
            assert out["rel_res"] == pytest.approx(res[best] / gn, rel=1e-6)
            if best != T - 1:
                saw_not_last = True
                assert np.linalg.norm(pv - iterates[T - 1]) > 1e-3 * np.linalg.norm(iterates[T - 1])
        else:
            saw_start = True
            np.testing.assert_array_equal(out["p"], -grad)
            assert out["rel_res"] == 1.0
    assert saw_not_last
    if seed in (31, 43):
        assert saw_start          # the first residual of these systems is larger than ||g||
