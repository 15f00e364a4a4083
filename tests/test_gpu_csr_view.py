"""The column-sorted view of a CSR sample, built two ways: filtered out of the whole matrix's view (the default) and
by the sorting construction (SSN_CSR_VIEW=sort, also the fallback for very uneven row lengths).  Both feed the same
product kernels; every result is compared with the oracle and the two constructions with each other."""
import os

import numpy as np
import pytest
import torch

from paper_1802_09113_amd import synth
from tests.gpu_util import TOL, Pair, rel_err, rel_scalar, workload

pytestmark = pytest.mark.gpu

F64, F32 = torch.float64, torch.float32


def _with_view(kind, fn):
    old = os.environ.get("SSN_CSR_VIEW")
    os.environ["SSN_CSR_VIEW"] = kind
    try:
        return fn()
    finally:
        if old is None:
            del os.environ["SSN_CSR_VIEW"]
        else:
            os.environ["SSN_CSR_VIEW"] = old


def _samples(n, g):
    """Sorted without repeats, unsorted, with repeats, one row, all rows."""
    base = np.sort(g.choice(n, size=min(n, 150), replace=False)).astype(np.int32)
    return {
        "sorted": base,
        "unsorted": g.permutation(base).astype(np.int32),
        "repeats": np.concatenate([base[:40], base[:40][::-1], base[10:15]]).astype(np.int32),
        "one_row": base[:1].copy(),
        "all_rows": np.arange(n, dtype=np.int32),
    }


@pytest.mark.parametrize("dtype", [F64, F32], ids=["f64", "f32"])
@pytest.mark.parametrize("cfg,n", [(4, 403), (6, 20011)])
def test_products_on_both_constructions(cfg, n, dtype):
    # workload 4: 450 entries in every row (a 150-row sample has 67 500 entries: prefix sums over several tiles);
    # workload 6: 20 011 rows, so the prefix sum over the rows' multiplicities takes the tiled path as well
    d = workload(cfg, n)
    pair = Pair(d, dtype)
    g = np.random.default_rng(31)
    Wh, Wd = pair.block(synth.probe(pair.p, pair.K, sub=1, scale=0.1))
    Vh, Vd = pair.block(synth.probe(pair.p, pair.K, sub=2, scale=1.0))
    tol = TOL[dtype]
    for name, S in _samples(n, g).items():
        print(f"[case] csr view cfg={cfg} dtype={dtype} sample={name} nS={S.size}", flush=True)
        Sd = pair.idx(S)
        ref_hv = pair.oracle.hessvec(Wh, S, Vh)
        ref_g, ref_f = pair.oracle.gradient_sampled(Wh, S)
        got = {}
        for kind in ("filter", "sort"):
            def run():
                hv = pair.gpu.ssn_hessvec(Wd, Sd, Vd)
                gs, fs = pair.gpu.ssn_gradient_sampled(Wd, Sd)
                torch.cuda.synchronize()
                return pair.host(hv), pair.host(gs), fs
            got[kind] = _with_view(kind, run)
            hv, gs, fs = got[kind]
            assert rel_err(hv, ref_hv) <= tol, (kind, name)
            assert rel_err(gs, ref_g) <= tol, (kind, name)
            assert rel_scalar(fs, ref_f) <= tol, (kind, name)
        # the two constructions order the entries of a column differently only for unsorted samples or repeats
        same = 1e-13 if dtype == F64 else 1e-5
        assert rel_err(got["filter"][0], got["sort"][0]) <= same
        assert rel_err(got["filter"][1], got["sort"][1]) <= same
        if name == "sorted":
            np.testing.assert_array_equal(got["filter"][0], got["sort"][0])
            np.testing.assert_array_equal(got["filter"][1], got["sort"][1])
    pair.close()


def test_cg_on_both_constructions():
    n = 403
    d = workload(4, n)
    pair = Pair(d, F64)
    g = np.random.default_rng(32)
    Wh, Wd = pair.block(synth.probe(pair.p, pair.K, sub=1, scale=0.1))
    G_ref, _ = pair.oracle.gradient(Wh)
    Gh, Gd = pair.block(G_ref)
    for name, S in _samples(n, g).items():
        if name == "all_rows":
            continue
        ref = pair.oracle.cg(Wh, S, Gh, 1e-4, 8)
        for kind in ("filter", "sort"):
            print(f"[case] csr view cg sample={name} construction={kind}", flush=True)
            def run():
                pair.gpu.ssn_hess_prepare(Wd, pair.idx(S))
                out = pair.gpu.ssn_cg(Gd, 1e-4, 8)
                torch.cuda.synchronize()
                return out
            out = _with_view(kind, run)
            assert out["iters"] == ref["iters"] and out["flags"] == ref["flags"]
            np.testing.assert_allclose(out["alpha"], ref["alpha"], rtol=1e-8)
            np.testing.assert_allclose(out["rnorm"], ref["rnorm"], rtol=1e-8)
            assert rel_err(pair.host(out["p"]), ref["p"]) <= 1e-8
    pair.close()


def _uneven_csr(n, p, C, seed, long_row_len):
    """Rows of about ten entries, some empty, and one row of long_row_len entries."""
    g = np.random.default_rng(seed)
    rowptr = np.zeros(n + 1, dtype=np.int64)
    cols, vals = [], []
    for i in range(n):
        k = long_row_len if i == 7 else (0 if i % 13 == 0 else int(g.integers(1, 20)))
        c = np.sort(g.choice(p, size=k, replace=False))
        cols.append(c)
        vals.append(g.standard_normal(k))
        rowptr[i + 1] = rowptr[i] + k
    labels = g.integers(0, C, size=n).astype(np.int32)
    return dict(layout="csr", rowptr=rowptr, colidx=np.concatenate(cols).astype(np.int32), vals=np.concatenate(vals),
                labels=labels, C=C, p=p, n=n, lam=1e-3)


@pytest.mark.parametrize("long_row_len", [60, 2500], ids=["within_the_bound", "falls_back_to_the_sort"])
def test_uneven_row_lengths(long_row_len):
    # the filtering construction sizes its buffers by (rows sampled) x (longest row); a row 250 times the average makes
    # that bound useless and the library sorts instead.  Either way the results are the oracle's.
    n, p, C = 500, 3000, 5
    d = _uneven_csr(n, p, C, 41, long_row_len)
    pair = Pair(d, F64)
    Wh, Wd = pair.block(synth.probe(p, C - 1, sub=1, scale=0.3))
    Vh, Vd = pair.block(synth.probe(p, C - 1, sub=2, scale=1.0))
    for S in (np.array([7, 0, 13, 26, 100, 7], dtype=np.int32), np.array([0, 13, 26], dtype=np.int32),
              np.arange(0, n, 3, dtype=np.int32)):
        hv = pair.gpu.ssn_hessvec(Wd, pair.idx(S), Vd)
        gs, fs = pair.gpu.ssn_gradient_sampled(Wd, pair.idx(S))
        torch.cuda.synchronize()
        assert rel_err(pair.host(hv), pair.oracle.hessvec(Wh, S, Vh)) <= 1e-10
        ref_g, ref_f = pair.oracle.gradient_sampled(Wh, S)
        assert rel_err(pair.host(gs), ref_g) <= 1e-10
        assert rel_scalar(fs, ref_f) <= 1e-10
    pair.close()


@pytest.mark.parametrize("dtype", [F64, F32], ids=["f64", "f32"])
@pytest.mark.parametrize("C", [4, 20, 33], ids=["K3", "K19", "K32"])
def test_workgroup_per_row_passes_on_rows_of_every_length(C, dtype):
    # Sampled passes over a CSR matrix with long rows on average (128 stored entries and more) give every row to a
    # workgroup whose four waves share its entries.  Rows here are empty, shorter than one round of the four waves
    # (so that some waves get nothing), ragged, and long; the sample repeats rows and is not sorted.
    n, p = 600, 5000
    g = np.random.default_rng(100 + C)
    counts = g.integers(300, 700, size=n)
    counts[::7] = 0
    counts[1::7] = g.integers(1, 6, size=counts[1::7].size)
    counts[2::7] = g.integers(60, 70, size=counts[2::7].size)
    rowptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(counts, out=rowptr[1:])
    nnz = int(rowptr[-1])
    assert nnz // n >= 128
    colidx = np.concatenate([np.sort(g.choice(p, size=k, replace=False)) for k in counts]).astype(np.int32)
    vals = g.standard_normal(nnz) / 20.0
    labels = g.integers(0, C, size=n).astype(np.int32)
    d = dict(layout="csr", rowptr=rowptr, colidx=colidx, vals=vals, labels=labels, C=C, K=C - 1, p=p, n=n, lam=1e-3, nnz=nnz)
    pair = Pair(d, dtype)
    tol = TOL[dtype]
    Wh, Wd = pair.block(0.3 * g.standard_normal((p, C - 1)))
    Vh, Vd = pair.block(g.standard_normal((p, C - 1)))
    for name, S in (("multiset", g.integers(0, n, size=250).astype(np.int32)), ("all rows", np.arange(n, dtype=np.int32)),
                    ("short rows only", np.array([0, 1, 8, 7, 1, 2], dtype=np.int32))):
        print(f"[case] workgroup per row C={C} dtype={dtype} sample={name}", flush=True)
        HV = pair.gpu.ssn_hessvec(Wd, pair.idx(S), Vd)
        torch.cuda.synchronize()
        assert rel_err(pair.host(HV), pair.oracle.hessvec(Wh, S, Vh)) <= tol
    S = g.integers(0, n, size=300).astype(np.int32)
    Gh, Gd = pair.block(pair.oracle.gradient(Wh)[0])
    pair.gpu.ssn_hess_prepare(Wd, pair.idx(S))
    ref = pair.oracle.cg(Wh, S, Gh, 1e-4, 5)
    out = pair.gpu.ssn_cg(Gd, 1e-4, 5)
    torch.cuda.synchronize()
    assert out["iters"] == ref["iters"]
    np.testing.assert_allclose(out["alpha"], ref["alpha"], rtol=1e-8 if dtype == F64 else 5e-3)
    assert rel_err(pair.host(out["p"]), ref["p"]) <= (1e-8 if dtype == F64 else 5e-3)
    pair.close()
