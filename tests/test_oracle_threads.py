"""The OpenMP build of the oracle (same source, -fopenmp: one contiguous chunk of rows per thread, per-thread sums
added in thread order) is pinned to the plain single-thread build, which the other oracle tests pin to the paper."""
import numpy as np
import pytest

from oracle import oracle
from oracle.oracle import Problem
from paper_1802_09113_amd import synth


def _pair(cfg, n):
    d = synth.make(cfg, n=n, p=20011 if cfg == 4 else None)      # the sparse shape with fewer columns: seconds, not minutes
    kw = dict(X=d["X"]) if d["layout"] == "dense" else dict(csr=(d["rowptr"], d["colidx"], d["vals"]), p=d["p"])
    return d, Problem(d["labels"], d["C"], d["lam"], **kw), Problem(d["labels"], d["C"], d["lam"], threads=True, **kw)


def _close(a, b):
    a, b = np.asarray(a, dtype=np.float64), np.asarray(b, dtype=np.float64)
    return np.max(np.abs(a - b)) <= 4e-16 * max(np.max(np.abs(b)), 1e-300)


@pytest.mark.parametrize("cfg,n", [(0, 2003), (1, 1501), (3, 4999), (4, 203)])
def test_threaded_build_equals_the_single_thread_build(cfg, n, monkeypatch):
    assert oracle.threads_of(False) == 1 and oracle.threads_of(True) >= 1
    d, one, many = _pair(cfg, n)
    W = synth.probe(one.p, one.K, sub=1, scale=0.2)
    V = synth.probe(one.p, one.K, sub=2)
    assert _close([many.objective(W)], [one.objective(W)])
    (Ga, fa), (Gb, fb) = many.gradient(W), one.gradient(W)
    assert _close(Ga, Gb) and _close([fa], [fb])
    for nS in (3, 157):                      # fewer rows than threads; rows that do not divide evenly
        S = synth.sample_rows(n, nS)
        S[0] = S[1]                          # a repeated row
        assert _close(many.hessvec(W, S, V), one.hessvec(W, S, V))
        (Ga, fa), (Gb, fb) = many.gradient_sampled(W, S), one.gradient_sampled(W, S)
        assert _close(Ga, Gb) and _close([fa], [fb])
    S = synth.sample_rows(n, 100)
    ca, cb = many.cg(W, S, Gb, 1e-6, 12), one.cg(W, S, Gb, 1e-6, 12)
    assert ca["iters"] == cb["iters"] and ca["flags"] == cb["flags"]
    np.testing.assert_allclose(ca["alpha"], cb["alpha"], rtol=1e-11)
    np.testing.assert_allclose(ca["p"], cb["p"], rtol=0, atol=1e-11 * np.max(np.abs(cb["p"])))
    S_all = synth.sample_schedule(n, 100, 3)
    Wa, la, _ = many.ssn(np.zeros_like(W), S_all)
    Wb, lb, _ = one.ssn(np.zeros_like(W), S_all)
    # iterations amplify the last-bit differences of the products (a sampled Hessian of rank far below d is
    # ill-conditioned): the elementary functions above agree to the last bits, the loops to a looser bound
    np.testing.assert_allclose(la[:, 0], lb[:, 0], rtol=1e-6)           # objective per iteration
    np.testing.assert_array_equal(la[:, [2, 4, 5]], lb[:, [2, 4, 5]])   # CG products, step length, trials: decisions
    np.testing.assert_allclose(la[:, [1, 3]], lb[:, [1, 3]], rtol=1e-4) # gradient norm, CG relative residual
    np.testing.assert_allclose(Wa, Wb, rtol=0, atol=1e-5 * np.max(np.abs(Wb)))
