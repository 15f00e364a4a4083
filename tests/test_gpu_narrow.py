"""GPU parity of the vector-unit kernel for long passes over narrow dense matrices (an even number of at most 64
features, at most ten weight columns; Table 1's Covertype- and Drive-Diagnostics-like shapes).  By default it serves
gradient and product passes of 16384 rows and more; SSN_NARROW_PATH=on makes it serve every pass the shape allows, so
that the oracle can check it on sizes it finishes in seconds, and =off keeps the matrix-core kernels (the two are
compared as well)."""
import os

import numpy as np
import pytest
import torch

from tests.gpu_util import TOL, Pair, rel_err, rel_scalar

pytestmark = pytest.mark.gpu

F64, F32 = torch.float64, torch.float32
DTYPES = [F64, F32]


@pytest.fixture
def narrow_on():
    old = os.environ.get("SSN_NARROW_PATH")
    os.environ["SSN_NARROW_PATH"] = "on"
    yield
    if old is None:
        del os.environ["SSN_NARROW_PATH"]
    else:
        os.environ["SSN_NARROW_PATH"] = old


def _problem(n, p, C, seed, margin_scale=1.0):
    g = np.random.default_rng(seed)
    X = g.standard_normal((n, p)) * (g.random((n, p)) < 0.6)
    W_true = g.standard_normal((p, C))
    labels = np.argmax(X @ W_true + g.gumbel(size=(n, C)), axis=1).astype(np.int32)
    return dict(layout="dense", X=X * margin_scale, labels=labels, C=C, p=p, n=n, lam=1e-3), g


# (n, p, C): several 64-row blocks with a ragged tail, one block, fewer rows than one block, the widest and the
# narrowest shapes, every count of weight columns from 1 to 10
SHAPES = [(1003, 54, 7), (777, 48, 11), (64, 64, 3), (37, 2, 2), (200, 8, 5), (4099, 62, 10), (650, 30, 4), (129, 10, 6),
          (300, 16, 8), (500, 22, 9), (1000, 40, 10)]


@pytest.mark.parametrize("dtype", DTYPES, ids=["f64", "f32"])
@pytest.mark.parametrize("n,p,C", SHAPES)
def test_narrow_kernel_against_the_oracle(narrow_on, n, p, C, dtype):
    d, g = _problem(n, p, C, seed=n + p + C)
    pair = Pair(d, dtype)
    tol = TOL[dtype]
    Wh, Wd = pair.block(0.3 * g.standard_normal((p, C - 1)))
    Vh, Vd = pair.block(g.standard_normal((p, C - 1)))
    print(f"[case] narrow n={n} p={p} C={C} dtype={dtype}", flush=True)
    f = pair.gpu.ssn_objective(Wd)
    G, f2 = pair.gpu.ssn_gradient(Wd)
    torch.cuda.synchronize()
    G_ref, f_ref = pair.oracle.gradient(Wh)
    assert rel_scalar(f, f_ref) <= tol, (f, f_ref)
    assert rel_scalar(f2, f_ref) <= tol, (f2, f_ref)
    assert rel_err(pair.host(G), G_ref) <= tol, rel_err(pair.host(G), G_ref)
    # products: on all rows, on a sample with repeats that is not sorted, on a single row
    for S in (np.arange(n, dtype=np.int32), g.integers(0, n, size=max(3, n // 3)).astype(np.int32), np.array([n - 1], dtype=np.int32)):
        print(f"[case] narrow product nS={S.size}", flush=True)
        HV = pair.gpu.ssn_hessvec(Wd, pair.idx(S), Vd)
        torch.cuda.synchronize()
        ref = pair.oracle.hessvec(Wh, S, Vh)
        assert rel_err(pair.host(HV), ref) <= tol, rel_err(pair.host(HV), ref)
    # sub-sampled gradient of eq. (2a) on a multiset
    S = g.integers(0, n, size=max(5, n // 2)).astype(np.int32)
    Gs, fs = pair.gpu.ssn_gradient_sampled(Wd, pair.idx(S))
    torch.cuda.synchronize()
    Gs_ref, fs_ref = pair.oracle.gradient_sampled(Wh, S)
    assert rel_err(pair.host(Gs), Gs_ref) <= tol
    assert rel_scalar(fs, fs_ref) <= tol
    pair.close()


@pytest.mark.parametrize("dtype", DTYPES, ids=["f64", "f32"])
def test_narrow_kernel_padded_rows_and_weights(narrow_on, dtype):
    # leading dimensions beyond p and K, and rows that start at an address aligned to the element only
    n, p, C = 901, 54, 7
    d, g = _problem(n, p, C, seed=5)
    for kw in (dict(ldx=61, ldw=9), dict(xoff=1), dict(ldx=56, ldw=16)):
        pair = Pair(d, dtype, **kw)
        tol = TOL[dtype]
        Wh, Wd = pair.block(0.3 * g.standard_normal((p, C - 1)))
        Vh, Vd = pair.block(g.standard_normal((p, C - 1)))
        print(f"[case] narrow layout {kw} dtype={dtype}", flush=True)
        G, f = pair.gpu.ssn_gradient(Wd)
        S = g.integers(0, n, size=400).astype(np.int32)
        HV = pair.gpu.ssn_hessvec(Wd, pair.idx(S), Vd)
        torch.cuda.synchronize()
        G_ref, f_ref = pair.oracle.gradient(Wh)
        assert rel_scalar(f, f_ref) <= tol
        assert rel_err(pair.host(G), G_ref) <= tol
        assert rel_err(pair.host(HV), pair.oracle.hessvec(Wh, S, Vh)) <= tol
        pair.close()


@pytest.mark.parametrize("dtype", DTYPES, ids=["f64", "f32"])
def test_narrow_kernel_large_margins_stay_finite(narrow_on, dtype):
    # margins of several hundred in both directions: the stable log-sum-exp of eqs. (8), (9), (14)-(17)
    n, p, C = 260, 6, 4
    d, g = _problem(n, p, C, seed=9, margin_scale=300.0)
    pair = Pair(d, dtype)
    Wh, Wd = pair.block(g.standard_normal((p, C - 1)))
    G, f = pair.gpu.ssn_gradient(Wd)
    torch.cuda.synchronize()
    G_ref, f_ref = pair.oracle.gradient(Wh)
    assert np.isfinite(f) and np.all(np.isfinite(pair.host(G)))
    assert rel_scalar(f, f_ref) <= TOL[dtype]
    assert rel_err(pair.host(G), G_ref) <= TOL[dtype]
    pair.close()


@pytest.mark.parametrize("dtype", DTYPES, ids=["f64", "f32"])
def test_narrow_kernel_takes_over_on_long_passes_and_agrees_with_the_matrix_core_kernel(dtype):
    # 70000 rows: above the size from which the vector-unit kernel serves by itself; the same calls with the path
    # switched off go through the matrix-core kernel.  Both are compared with the oracle on the gradient (every row
    # counts in it) and with each other on a product over all rows.
    n, p, C = 70000, 54, 7
    d, g = _problem(n, p, C, seed=21)
    Wn = 0.3 * g.standard_normal((p, C - 1))
    Vn = g.standard_normal((p, C - 1))
    out = {}
    old = os.environ.get("SSN_NARROW_PATH")
    try:
        for mode in ("default", "off"):
            if mode == "off":
                os.environ["SSN_NARROW_PATH"] = "off"
            else:
                os.environ.pop("SSN_NARROW_PATH", None)
            pair = Pair(d, dtype)
            Wh, Wd = pair.block(Wn)
            Vh, Vd = pair.block(Vn)
            print(f"[case] narrow takeover mode={mode} dtype={dtype}", flush=True)
            G, f = pair.gpu.ssn_gradient(Wd)
            HV = pair.gpu.ssn_hessvec(Wd, pair.idx(np.arange(n, dtype=np.int32)), Vd)
            torch.cuda.synchronize()
            out[mode] = (f, pair.host(G), pair.host(HV))
            if mode == "default":
                G_ref, f_ref = pair.oracle.gradient(Wh)
                HV_ref = pair.oracle.hessvec(Wh, np.arange(n), Vh)
            pair.close()
    finally:
        if old is None:
            os.environ.pop("SSN_NARROW_PATH", None)
        else:
            os.environ["SSN_NARROW_PATH"] = old
    tol = TOL[dtype]
    for mode in ("default", "off"):
        f, G, HV = out[mode]
        assert rel_scalar(f, f_ref) <= tol
        assert rel_err(G, G_ref) <= tol
        assert rel_err(HV, HV_ref) <= tol
    # the two kernels sum in different orders: equal to rounding, not bit for bit
    assert rel_err(out["default"][1], out["off"][1]) <= tol


@pytest.mark.parametrize("dtype", DTYPES, ids=["f64", "f32"])
def test_cg_and_the_ssn_loop_through_the_narrow_kernel(narrow_on, dtype):
    # Alg. 2 followed product by product (the kernel leaves the curvature sums of z_i . u_i that CG reads, and obeys the
    # loop's stop flag), then Alg. 1 over a fixed schedule with full gradients and with sub-sampled ones, every gradient,
    # product and trial objective going through the vector-unit kernel
    from paper_1802_09113_amd import synth
    n, p, C = 3001, 54, 7
    d, g = _problem(n, p, C, seed=33)
    pair = Pair(d, dtype)
    Wh, Wd = pair.block(0.1 * g.standard_normal((p, C - 1)))
    nS = 600
    S = synth.sample_rows(n, nS)
    G_ref, _ = pair.oracle.gradient(Wh)
    Gh, Gd = pair.block(G_ref)
    pair.gpu.ssn_hess_prepare(Wd, pair.idx(S))
    ttol = 1e-8 if dtype == F64 else 5e-3
    for theta, T in [(1e-4, 10), (0.3, 10), (1e-30, 3)]:
        print(f"[case] narrow cg dtype={dtype} theta={theta} T={T}", flush=True)
        ref = pair.oracle.cg(Wh, S, Gh, theta, T)
        out = pair.gpu.ssn_cg(Gd, theta, T)
        torch.cuda.synchronize()
        assert out["iters"] == ref["iters"] and out["flags"] == ref["flags"]
        np.testing.assert_allclose(out["alpha"], ref["alpha"], rtol=ttol)
        np.testing.assert_allclose(out["rnorm"], ref["rnorm"], rtol=ttol)
        np.testing.assert_allclose(out["sHs"], ref["sHs"], rtol=ttol)
        assert rel_err(pair.host(out["p"]), ref["p"]) <= ttol
    iters = 6
    S_all = synth.sample_schedule(n, nS, iters)
    W0 = 0.01 * g.standard_normal((p, C - 1))
    for sub_sampled in (False, True):
        print(f"[case] narrow ssn dtype={dtype} sub-sampled gradient={sub_sampled}", flush=True)
        W0h, W0d = pair.block(W0)
        kw = {}
        if sub_sampled:
            Sg_all = np.stack([synth.sample_rows(n, n // 5, seed=900 + it) for it in range(iters)]).astype(np.int32)
            Wref, log_ref, done_ref = pair.oracle.ssn_sg(W0h, Sg_all, S_all, theta=1e-4, T=10)
            kw["Sg_all"] = torch.from_numpy(Sg_all).cuda()
        else:
            Wref, log_ref, done_ref = pair.oracle.ssn(W0h, S_all, theta=1e-4, T=10)
        recs, done = pair.gpu.ssn_solve(W0d, torch.from_numpy(S_all).cuda(), theta=1e-4, T=10, **kw)
        torch.cuda.synchronize()
        assert done == done_ref
        np.testing.assert_allclose(np.array([r["f"] for r in recs]), log_ref[:done, 0], rtol=1e-8 if dtype == F64 else 1e-3)
        assert [r["cg_iters"] for r in recs] == [int(x) for x in log_ref[:done, 2]]
        assert [r["alpha"] for r in recs] == list(log_ref[:done, 4])
        assert rel_err(pair.host(W0d), Wref) <= (1e-6 if dtype == F64 else 2e-2)
    pair.close()
