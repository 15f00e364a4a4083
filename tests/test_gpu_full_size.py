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


def _check(cfg, dtypes, grad=True):
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
        pair.close()


def test_image_like_full():
    _check(1, [F64, F32])


def test_tall_narrow_full():
    _check(3, [F64, F32])


def test_wide_full():
    _check(2, [F32, F64])


def test_sparse_full():
    _check(4, [F64, F32])
