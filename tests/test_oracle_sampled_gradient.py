"""Pins for the CPU oracle's sub-sampled gradient, eq. (2a), and the SSN loop that uses it (no GPU).

Fixed by mathematics, written here independently with numpy:
  the gradient of a sample's objective by central finite differences,
  the all-rows sample (any order) = the full gradient of eq. (6),
  the one-row closed form a_i (p_i - y_i)^T,
  additivity over concatenated multiset samples,
  the paper's sum scaling n/|S| against the mean scaling 1/|S|,
  and, for the loop, that a gradient sample of all rows reproduces the full-gradient iteration.
"""
import numpy as np
import pytest

from oracle.oracle import Problem


def small_problem(n=240, p=6, C=4, lam=1e-2, seed=3, scale="mean"):
    g = np.random.default_rng(seed)
    X = g.standard_normal((n, p))
    labels = g.integers(0, C, size=n).astype(np.int32)
    return Problem(labels, C, lam, X=X, scale=scale), X, labels, g


def naive_sample_objective(X, labels, W, lam, S, factor):
    Z = X[S].astype(np.longdouble) @ W.astype(np.longdouble)
    K = W.shape[1]
    lab = labels[S]
    lse = np.log1p(np.exp(Z).sum(axis=1))
    lin = np.where(lab < K, Z[np.arange(S.size), np.minimum(lab, K - 1)], 0.0)
    return float(factor * (lse - lin).sum() + 0.5 * lam * (W.astype(np.longdouble) ** 2).sum())


@pytest.mark.parametrize("scale", ["mean", "sum"])
def test_sampled_objective_and_finite_differences(scale):
    pr, X, labels, g = small_problem(scale=scale)
    W = 0.3 * g.standard_normal((pr.p, pr.K))
    S = g.integers(0, pr.n, size=50).astype(np.int32)          # a multiset
    factor = (pr.n / S.size) if scale == "sum" else 1.0 / S.size
    G, fS = pr.gradient_sampled(W, S)
    assert fS == pytest.approx(naive_sample_objective(X, labels, W, pr.lam, S, factor), rel=1e-13)
    h = 1e-6
    for (j, c) in [(0, 0), (2, 1), (5, 2), (3, 0)]:
        E = np.zeros_like(W)
        E[j, c] = h
        fd = (naive_sample_objective(X, labels, W + E, pr.lam, S, factor)
              - naive_sample_objective(X, labels, W - E, pr.lam, S, factor)) / (2 * h)
        assert G[j, c] == pytest.approx(fd, rel=2e-7, abs=1e-9)


@pytest.mark.parametrize("scale", ["mean", "sum"])
def test_all_rows_in_any_order_is_the_full_gradient(scale):
    pr, X, labels, g = small_problem(scale=scale)
    W = 0.2 * g.standard_normal((pr.p, pr.K))
    G_full, f_full = pr.gradient(W)
    S = g.permutation(pr.n).astype(np.int32)
    G, fS = pr.gradient_sampled(W, S)
    np.testing.assert_allclose(G, G_full, rtol=1e-13, atol=1e-15)
    assert fS == pytest.approx(f_full, rel=1e-14)


def test_one_row_closed_form():
    pr, X, labels, g = small_problem()
    W = 0.5 * g.standard_normal((pr.p, pr.K))
    for i in (0, 17, 239):
        z = X[i] @ W
        e = np.exp(np.append(z, 0.0))
        prob = (e / e.sum())[: pr.K]
        y = np.zeros(pr.K)
        if labels[i] < pr.K:
            y[labels[i]] = 1.0
        expect = np.outer(X[i], prob - y) + pr.lam * W                 # mean scaling, |S| = 1
        G, _ = pr.gradient_sampled(W, np.array([i], dtype=np.int32))
        np.testing.assert_allclose(G, expect, rtol=1e-12, atol=1e-14)


def test_additivity_over_concatenated_multisets_and_sum_scaling():
    pr, X, labels, g = small_problem()
    prs = Problem(labels, pr.C, pr.lam, X=X, scale="sum")
    W = 0.4 * g.standard_normal((pr.p, pr.K))
    S1 = g.integers(0, pr.n, size=30).astype(np.int32)
    S2 = g.integers(0, pr.n, size=70).astype(np.int32)
    S12 = np.concatenate([S1, S2])
    G1, _ = pr.gradient_sampled(W, S1)
    G2, _ = pr.gradient_sampled(W, S2)
    G12, _ = pr.gradient_sampled(W, S12)
    lamW = pr.lam * W
    np.testing.assert_allclose(100 * (G12 - lamW), 30 * (G1 - lamW) + 70 * (G2 - lamW), rtol=1e-12, atol=1e-13)
    Gs, _ = prs.gradient_sampled(W, S12)                              # eq. (2a): factor n/|S| instead of 1/|S|
    np.testing.assert_allclose(Gs - lamW, pr.n * (G12 - lamW), rtol=1e-12, atol=1e-13)


def test_loop_with_an_all_rows_gradient_sample_is_the_full_gradient_loop():
    pr, X, labels, g = small_problem(n=200, p=5, C=3, lam=1e-3)
    iters, nS = 4, 40
    S_all = np.stack([g.choice(pr.n, nS, replace=False) for _ in range(iters)]).astype(np.int32)
    Sg_all = np.tile(np.arange(pr.n, dtype=np.int32), (iters, 1))
    W0 = np.zeros((pr.p, pr.K))
    Wa, la, da = pr.ssn(W0, S_all)
    Wb, lb, db = pr.ssn_sg(W0, Sg_all, S_all)
    assert da == db == iters
    np.testing.assert_allclose(Wb, Wa, rtol=1e-9, atol=1e-12)
    np.testing.assert_allclose(lb[:, 0], la[:, 0], rtol=1e-12)          # F carried over = F recomputed
    assert list(lb[:, 2]) == list(la[:, 2]) and list(lb[:, 4]) == list(la[:, 4])


def test_loop_with_a_true_gradient_sample_decreases_the_full_objective():
    pr, X, labels, g = small_problem(n=400, p=5, C=3, lam=1e-3)
    iters = 5
    S_all = np.stack([g.choice(pr.n, 40, replace=False) for _ in range(iters)]).astype(np.int32)
    Sg_all = np.stack([g.choice(pr.n, 200, replace=False) for _ in range(iters)]).astype(np.int32)
    W, log, done = pr.ssn_sg(np.zeros((pr.p, pr.K)), Sg_all, S_all)
    assert done == iters
    assert log[0, 0] == pytest.approx(np.log(pr.C), rel=1e-14)
    f_end = pr.objective(W)
    assert f_end < log[0, 0]
    assert np.all(np.diff(np.append(log[:, 0], f_end)) <= 1e-12)        # Armijo on the full objective
