"""GPU parity at the full workload sizes, in the launch configuration bench.py times (same entry points,
same grid choices): objective, gradient and the sub-sampled Hessian-vector product against the complete
oracle result, plus properties that hold at any size (symmetry, positive definiteness, W = 0 value)."""
import numpy as np
import pytest
import torch

from paper_1802_09113_amd import synth
from tests.gpu_util import TOL, Pair, rel_err, rel_scalar

pytestmark = pytest.mark.gpu

F64, F32 = torch.float64, torch.float32


def _check(cfg, dtypes, grad=True, all_rows=False, cg=False):
    print(f"[gen] full-size workload {cfg}", flush=True)
    d = synth.make(cfg)
    S = synth.sample_rows(d["n"], d["nS"])
    for dtype in dtypes:
        pair = Pair(d, dtype)
        tol = TOL[dtype]
        Wh, Wd = pair.block(synth.probe(pair.p, pair.K, sub=1, scale=0.05))
        Vh, Vd = pair.block(synth.probe(pair.p, pair.K, sub=2))
        Uh, Ud = pair.block(synth.probe(pair.p, pair.K, sub=3))
        print(f"[case] full cfg={cfg} dtype={dtype} n={pair.n} p={pair.p}", flush=True)
        Zh, Zd = pair.block(np.zeros((pair.p, pair.K)))
        f0 = pair.gpu.ssn_objective(Zd)
        assert rel_scalar(f0, np.log(pair.C)) <= tol                     # closed form at W = 0
        f = pair.gpu.ssn_objective(Wd)
        assert rel_scalar(f, pair.oracle.objective(Wh)) <= tol
        if grad:
            G, f2 = pair.gpu.ssn_gradient(Wd)
            torch.cuda.synchronize()
            G_ref, f_ref = pair.oracle.gradient(Wh)
            assert rel_scalar(f2, f_ref) <= tol
            assert rel_err(pair.host(G), G_ref) <= tol
        pair.gpu.ssn_hess_prepare(Wd, pair.idx(S))
        HV = pair.gpu.ssn_hess_apply(Vd)
        HU = pair.gpu.ssn_hess_apply(Ud)
        torch.cuda.synchronize()
        assert rel_err(pair.host(HV), pair.oracle.hessvec(Wh, S, Vh)) <= tol
        hv, hu = pair.host(HV), pair.host(HU)
        a, b = float(np.sum(Uh * hv)), float(np.sum(Vh * hu))
        assert abs(a - b) <= 10 * tol * max(abs(a), abs(b))              # <U, H V> = <V, H U>
        assert np.sum(Vh * hv) >= pair.oracle.lam * np.sum(Vh * Vh) * (1 - 10 * tol)
        pred, acc = pair.gpu.ssn_predict(Wd, want_pred=False)
        assert abs(acc - pair.oracle.accuracy(Wh)) <= (0.0 if dtype == F64 else 1e-3)
        if cg and dtype == F64:
            # Alg. 2 on the full-size sample, followed product by product
            print(f"[case] full cfg={cfg}: CG trajectory", flush=True)
            Gh, Gd = pair.block(G_ref)
            ref = pair.oracle.cg(Wh, S, Gh, 1e-4, d["T"])
            out = pair.gpu.ssn_cg(Gd, 1e-4, d["T"])
            torch.cuda.synchronize()
            assert out["iters"] == ref["iters"] and out["flags"] == ref["flags"]
            np.testing.assert_allclose(out["alpha"], ref["alpha"], rtol=1e-8)
            np.testing.assert_allclose(out["rnorm"], ref["rnorm"], rtol=1e-8)
            np.testing.assert_allclose(out["sHs"], ref["sHs"], rtol=1e-8)
            assert rel_err(pair.host(out["p"]), ref["p"]) <= 1e-8
        if all_rows:
            # the FullNewton shape: prepare and product on every row (the many-row-block forms of both kernels)
            Sall = np.arange(pair.n, dtype=np.int32)
            pair.gpu.ssn_hess_prepare(Wd, pair.idx(Sall))
            HVa = pair.gpu.ssn_hess_apply(Vd)
            torch.cuda.synchronize()
            assert rel_err(pair.host(HVa), pair.oracle.hessvec(Wh, Sall, Vh)) <= tol
        pair.close()


def test_image_like_full():
    _check(1, [F64, F32], all_rows=True)


def test_tall_narrow_full():
    _check(3, [F64, F32], all_rows=True)


def test_wide_full():
    _check(2, [F32, F64], all_rows=True, cg=True)


def test_sparse_full():
    _check(4, [F64, F32], all_rows=True, cg=True)


@pytest.mark.parametrize("p,reps", [(512, 1000), (3072, 170)], ids=["one_pass", "two_kernel"])
def test_matrices_of_more_than_2_to_the_31_elements(p, reps):
    """Maximum sizes: element offsets into X beyond 32 bits.  The big matrix is a block of m rows repeated `reps`
    times (built on the device), so with the mean scaling f, grad f and the accuracy equal the block's, which the
    oracle computes, and a product on sampled rows near the end equals the product on the same rows of the block."""
    from paper_1802_09113_amd.binding import Context
    from oracle.oracle import Problem

    g = np.random.default_rng(31 + p)
    m, C, lam = 4400 + 7, 5, 1e-3
    K = C - 1
    Xb = (g.standard_normal((m, p)) * (g.random((m, p)) < 0.4)).astype(np.float32)
    lab_b = g.integers(0, C, size=m).astype(np.int32)
    n = m * reps
    assert n * p > 2 ** 31
    print(f"[case] big matrix n={n} p={p} ({n * p * 4 / 2 ** 30:.1f} GiB)", flush=True)
    X = torch.from_numpy(Xb).cuda().repeat(reps, 1)
    labels = torch.from_numpy(lab_b).cuda().repeat(reps)
    W = (0.1 * g.standard_normal((p, K))).astype(np.float32)
    V = g.standard_normal((p, K)).astype(np.float32)
    Wd, Vd = torch.from_numpy(W).cuda(), torch.from_numpy(V).cuda()
    big = Context(labels, C, lam, X=X)
    small = Problem(lab_b, C, lam, X=Xb.astype(np.float64))
    tol = TOL[F32]
    f = big.ssn_objective(Wd)
    G, f2 = big.ssn_gradient(Wd)
    torch.cuda.synchronize()
    G_ref, f_ref = small.gradient(W.astype(np.float64))
    assert rel_scalar(f, f_ref) <= tol and rel_scalar(f2, f_ref) <= tol
    assert rel_err(G.double().cpu().numpy(), G_ref) <= tol
    # rows of the last repetitions: their offsets into X do not fit 32 bits
    Sb = g.integers(0, m, size=300).astype(np.int64)
    S = (Sb + m * (reps - 1 - (np.arange(300) % 3))).astype(np.int32)
    assert int(S.min()) * p > 2 ** 31
    HV = big.ssn_hessvec(Wd, torch.from_numpy(S).cuda(), Vd)
    _, acc = big.ssn_predict(Wd, want_pred=False)
    torch.cuda.synchronize()
    assert rel_err(HV.double().cpu().numpy(), small.hessvec(W.astype(np.float64), Sb.astype(np.int32), V.astype(np.float64))) <= tol
    assert abs(acc - small.accuracy(W.astype(np.float64))) <= 1e-3
    big.close()
