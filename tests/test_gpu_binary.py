"""The binary problem (C = 2; Appendix A.1: plain logistic regression) on the GPU against the oracle: the dense
matrix-vector kernels that serve K = 1 (every mode, aligned and unaligned rows, padded leading dimensions, tails),
the CSR path with a single weight column, CG, Alg. 1 over a fixed schedule with held-out accuracy, and the entry
point that allocates nothing.  Workloads 5 and 6 are shaped like the two binary data sets of Table 1."""
import numpy as np
import pytest
import torch

from paper_1802_09113_amd import binding, synth
from tests.gpu_util import TOL, Pair, oracle_sensitivity, rel_err, rel_scalar, workload

pytestmark = pytest.mark.gpu

F64, F32 = torch.float64, torch.float32
DTYPES = [F64, F32]
# The samples here have far fewer rows than the matrices have columns, so with the workloads' lambda = 1e-4 the
# sampled Hessians are ill-conditioned and ten CG products amplify last-bit differences (fp32 runs leave the
# oracle's trajectory after six or seven products).  The step-by-step comparisons use lambda = 1e-2; the
# full-size test keeps the workload's own value.
LAM = 1e-2


def _check_calls(pair, n, nS, dtype, path=None):
    tol = TOL[dtype]
    if path is not None:
        assert pair.gpu.ssn_dense_path() == path
    for sub, scale in [(0, 0.0), (1, 0.3)]:
        Wh, Wd = pair.block(synth.probe(pair.p, pair.K, sub=sub, scale=scale))
        f_ref = pair.oracle.objective(Wh)
        G_ref, _ = pair.oracle.gradient(Wh)
        f = pair.gpu.ssn_objective(Wd)
        G, f2 = pair.gpu.ssn_gradient(Wd)
        torch.cuda.synchronize()
        assert rel_scalar(f, f_ref) <= tol and rel_scalar(f2, f_ref) <= tol
        assert rel_err(pair.host(G), G_ref) <= tol
    Vh, Vd = pair.block(synth.probe(pair.p, pair.K, sub=2))
    S = synth.sample_rows(n, nS)
    S[:2] = S[2]                                       # a repeated row
    HV = pair.gpu.ssn_hessvec(Wd, pair.idx(S), Vd)
    Gs, fs = pair.gpu.ssn_gradient_sampled(Wd, pair.idx(S))
    torch.cuda.synchronize()
    assert rel_err(pair.host(HV), pair.oracle.hessvec(Wh, S, Vh)) <= tol
    Gs_ref, fs_ref = pair.oracle.gradient_sampled(Wh, S)
    assert rel_err(pair.host(Gs), Gs_ref) <= tol and rel_scalar(fs, fs_ref) <= tol
    pred, acc = pair.gpu.ssn_predict(Wd)
    ref_pred = pair.oracle.predict(Wh)
    flips = int(np.count_nonzero(pred.cpu().numpy() != ref_pred))
    assert flips <= (0 if dtype == F64 else max(1, n // 500))
    assert abs(acc - pair.oracle.accuracy(Wh)) <= (0.0 if dtype == F64 else 2e-3)
    Gh, Gd = pair.block(G_ref)
    ref = pair.oracle.cg(Wh, S, Gh, 1e-4, 10)
    out = pair.gpu.ssn_cg(Gd, 1e-4, 10)
    torch.cuda.synchronize()
    if dtype == F64:
        assert out["iters"] == ref["iters"] and out["flags"] == ref["flags"]
        np.testing.assert_allclose(out["alpha"], ref["alpha"], rtol=1e-8)
        np.testing.assert_allclose(out["rnorm"], ref["rnorm"], rtol=1e-8)
        assert rel_err(pair.host(out["p"]), ref["p"]) <= 1e-8
    else:
        # CG with fp32 vectors loses the oracle's trajectory after six or seven products on these systems (rows far
        # fewer than columns): the first products are followed step by step, the direction is judged by the
        # residual it really has, measured with the oracle's product
        k = min(5, ref["iters"], out["iters"])
        np.testing.assert_allclose(out["alpha"][:k], ref["alpha"][:k], rtol=5e-3)
        np.testing.assert_allclose(out["rnorm"][:k], ref["rnorm"][:k], rtol=5e-3)
        true_res = np.linalg.norm(pair.oracle.hessvec(Wh, S, pair.host(out["p"])) + Gh) / np.linalg.norm(Gh)
        assert true_res <= 1.5 * ref["rel_res"] + 1e-3


@pytest.mark.parametrize("dtype", DTYPES, ids=["f64", "f32"])
@pytest.mark.parametrize("p,ldx,xoff", [(5000, None, 0), (1301, None, 0), (1301, 1312, 0), (1301, None, 1), (129, None, 0),
                                        (127, None, 0)],
                         ids=["gisette_width", "odd_width", "padded_rows", "element_aligned", "just_wide_enough", "narrow"])
def test_dense_binary_calls(p, ldx, xoff, dtype):
    n = 1003
    d = synth.make(5, n=n, p=p)
    pair = Pair(d, dtype, ldx=ldx, xoff=xoff, lam=LAM)
    print(f"[case] dense binary p={p} ldx={ldx} xoff={xoff} dtype={dtype}", flush=True)
    _check_calls(pair, n, 120, dtype, path=3 if p >= 128 else None)
    pair.close()


@pytest.mark.parametrize("dtype", DTYPES, ids=["f64", "f32"])
def test_sparse_binary_calls(dtype):
    n = 3001
    d = workload(6, n)
    pair = Pair(d, dtype, lam=LAM)
    print(f"[case] sparse binary n={n} dtype={dtype}", flush=True)
    _check_calls(pair, n, 150, dtype)
    pair.close()


@pytest.mark.parametrize("dtype", DTYPES, ids=["f64", "f32"])
@pytest.mark.parametrize("cfg,n,p,nS", [(5, 2003, 600, 1000), (6, 3001, None, 1500)], ids=["dense", "sparse"])
def test_binary_fixed_schedule_with_held_out_accuracy(cfg, n, p, nS, dtype):
    # samples with more rows than (touched) columns: the sampled systems are well-conditioned, CG reaches its
    # tolerance, and the iteration does not amplify rounding differences from one step to the next
    d = synth.make(cfg, n=n, p=p)
    test = synth.make(cfg, n=n, p=p, part="test")
    pair, tpair = Pair(d, dtype, lam=LAM), Pair(test, dtype, lam=LAM)
    iters = 4        # these runs converge within five or six steps; at convergence the Armijo test compares equal numbers
    S_all = synth.sample_schedule(n, nS, iters)
    W0h, W0d = pair.block(synth.probe(pair.p, pair.K, sub=7, scale=0.01))
    print(f"[case] binary schedule cfg={cfg} dtype={dtype}", flush=True)
    Wref, log_ref, done_ref = pair.oracle.ssn(W0h, S_all, theta=1e-4, T=d["T"])
    recs, done = pair.gpu.ssn_solve(W0d, torch.from_numpy(S_all).cuda(), theta=1e-4, T=d["T"], test=tpair.gpu)
    torch.cuda.synchronize()
    assert done == done_ref == iters
    f64 = dtype == F64
    # even these systems amplify last-bit differences by eight orders of magnitude within ten CG products (the
    # oracle's direction moves by 3e-7 when the gradient is perturbed by 1e-15), so the comparison is as sharp as
    # the oracle's own sensitivity to perturbations of the size of the library's rounding allows
    f_own, w_own, same_steps = oracle_sensitivity(pair, d, W0h, S_all, d["T"], 1e-14 if f64 else 1e-6)
    f_dev = np.abs(np.array([r["f"] for r in recs]) / log_ref[:, 0] - 1.0)
    print(f"[info] own sensitivity f {f_own.max():.2e} W {w_own:.2e}; library f {f_dev.max():.2e}", flush=True)
    assert np.all(f_dev <= (1e-10 if f64 else 1e-4) + 100.0 * f_own)
    assert rel_err(pair.host(W0d), Wref) <= (1e-9 if f64 else 1e-3) + 100.0 * w_own
    if same_steps:
        assert [r["alpha"] for r in recs] == list(log_ref[:, 4])
    assert all(abs(r["cg_iters"] - int(x)) <= (0 if f64 else 1) for r, x in zip(recs, log_ref[:, 2]))
    acc_ref = tpair.oracle.accuracy(Wref)
    assert abs(recs[-1]["test_acc"] - acc_ref) <= 1e-3
    assert acc_ref > 0.6                                 # these labels are learnable
    pair.close()
    tpair.close()


@pytest.mark.parametrize("dtype", DTYPES, ids=["f64", "f32"])
def test_dense_binary_at_full_size_and_without_allocations(dtype):
    # the 6000 x 5000 shape of Table 1 in the launch configuration the benchmark times, and the same product
    # through the entry point that allocates nothing
    d = synth.make(5)
    pair = Pair(d, dtype)
    tol = TOL[dtype]
    n = d["n"]
    Wh, Wd = pair.block(synth.probe(pair.p, pair.K, sub=1, scale=0.2))
    Vh, Vd = pair.block(synth.probe(pair.p, pair.K, sub=2))
    print(f"[case] dense binary full size dtype={dtype}", flush=True)
    G, f = pair.gpu.ssn_gradient(Wd)
    torch.cuda.synchronize()
    G_ref, f_ref = pair.oracle.gradient(Wh)
    assert rel_scalar(f, f_ref) <= tol and rel_err(pair.host(G), G_ref) <= tol
    for S in (synth.sample_rows(n, d["nS"]), np.arange(n, dtype=np.int32)):
        HV = pair.gpu.ssn_hessvec(Wd, pair.idx(S), Vd)
        torch.cuda.synchronize()
        ref = pair.oracle.hessvec(Wh, S, Vh)
        assert rel_err(pair.host(HV), ref) <= tol
        nd = np.float64 if dtype == F64 else np.float32
        X = torch.from_numpy(d["X"].astype(nd)).cuda()
        desc, keep = binding.make_desc(torch.from_numpy(d["labels"]).cuda(), d["C"], d["lam"], X=X)
        HV2 = torch.full_like(Vd, float("nan"))
        st = binding.ssn_hessvec_static(desc, Wd, pair.idx(S), Vd, HV2)
        torch.cuda.synchronize()
        assert st == binding.SSN_OK and rel_err(pair.host(HV2), ref) <= tol
    pair.close()


@pytest.mark.parametrize("dtype", DTYPES, ids=["f64", "f32"])
def test_sparse_binary_with_more_rows_per_wave_than_lanes(dtype):
    # The one-weight-column CSR rows kernel parks a row's margin in a lane and does the per-row work when 64 rows are
    # parked or the wave runs out of rows.  The launch never has more than 16 waves per compute unit, so only a matrix
    # of more than a million rows fills a wave's lanes: 1.2 M rows of zero to four entries (empty rows included).
    n, p = 1_200_000, 40
    g = np.random.default_rng(7)
    counts = g.integers(0, 5, size=n)
    rowptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(counts, out=rowptr[1:])
    nnz = int(rowptr[-1])
    colidx = g.integers(0, p, size=nnz).astype(np.int32)
    # distinct, ascending columns inside a row: offsets 0..4 times 8 plus a per-entry draw below 8
    within = np.arange(nnz) - np.repeat(rowptr[:-1], counts)
    colidx = (within * 8 + colidx % 8).astype(np.int32)
    vals = g.standard_normal(nnz)
    w_true = g.standard_normal(p)
    scores = np.zeros(n)
    np.add.at(scores, np.repeat(np.arange(n), counts), vals * w_true[colidx])
    labels = (scores + g.logistic(size=n) < 0).astype(np.int32)
    d = dict(layout="csr", rowptr=rowptr, colidx=colidx, vals=vals, labels=labels, C=2, K=1, p=p, n=n, lam=1e-3, nnz=nnz)
    pair = Pair(d, dtype)
    tol = TOL[dtype]
    Wh, Wd = pair.block(0.5 * g.standard_normal((p, 1)))
    Vh, Vd = pair.block(g.standard_normal((p, 1)))
    print(f"[case] sparse binary, 1.2 M short rows dtype={dtype}", flush=True)
    f = pair.gpu.ssn_objective(Wd)
    G, f2 = pair.gpu.ssn_gradient(Wd)
    S = np.arange(n, dtype=np.int32)
    HV = pair.gpu.ssn_hessvec(Wd, pair.idx(S), Vd)
    pred, acc = pair.gpu.ssn_predict(Wd)
    torch.cuda.synchronize()
    G_ref, f_ref = pair.oracle.gradient(Wh)
    assert rel_scalar(f, f_ref) <= tol and rel_scalar(f2, f_ref) <= tol
    assert rel_err(pair.host(G), G_ref) <= tol
    assert rel_err(pair.host(HV), pair.oracle.hessvec(Wh, S, Vh)) <= tol
    assert abs(acc - pair.oracle.accuracy(Wh)) <= (1e-12 if dtype == F64 else 2e-3)
    pair.close()


@pytest.mark.parametrize("dtype", DTYPES, ids=["f64", "f32"])
def test_sparse_binary_columns_that_end_where_a_wave_of_pieces_ends(dtype):
    # The column-sorted product with one weight column cuts the sorted entries into pieces of at most 64 and adds the
    # pieces of a column with a lane per piece, 64 pieces per wave.  Here the pieces fall exactly on those edges:
    # column 0 has 64 x 64 entries (the 64 pieces of the first wave and nothing else), column 1 one entry in every row
    # (192 pieces: three whole waves, followed from the wave where it starts to a step that finds no piece of it),
    # then a column of a single entry, one of 100 (two pieces) and one of 64 (one whole piece).
    n, p = 12288, 7
    rows = [np.arange(4096), np.arange(n), np.array([5]), np.arange(200, 300), np.arange(1000, 1064)]
    cols = [0, 1, 2, 4, 6]                               # columns 3 and 5 stay empty
    g = np.random.default_rng(11)
    r = np.concatenate(rows)
    c = np.concatenate([np.full(len(x), k) for x, k in zip(rows, cols)])
    order = np.lexsort((c, r))
    r, c = r[order], c[order].astype(np.int32)
    vals = g.standard_normal(r.size)
    rowptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(np.bincount(r, minlength=n), out=rowptr[1:])
    labels = g.integers(0, 2, size=n).astype(np.int32)
    d = dict(layout="csr", rowptr=rowptr, colidx=c, vals=vals, labels=labels, C=2, K=1, p=p, n=n, lam=1e-3, nnz=int(r.size))
    pair = Pair(d, dtype)
    tol = TOL[dtype]
    Wh, Wd = pair.block(0.5 * g.standard_normal((p, 1)))
    Vh, Vd = pair.block(g.standard_normal((p, 1)))
    print(f"[case] sparse binary, columns on the edges of waves of pieces dtype={dtype}", flush=True)
    G, f = pair.gpu.ssn_gradient(Wd)
    torch.cuda.synchronize()
    G_ref, f_ref = pair.oracle.gradient(Wh)
    assert rel_scalar(f, f_ref) <= tol and rel_err(pair.host(G), G_ref) <= tol
    # all rows; the first 4096 rows (column 1 then has exactly the pieces of one wave, behind column 0's); a multiset
    for S in (np.arange(n, dtype=np.int32), np.arange(4096, dtype=np.int32), g.integers(0, n, size=5000).astype(np.int32)):
        HV = pair.gpu.ssn_hessvec(Wd, pair.idx(S), Vd)
        torch.cuda.synchronize()
        assert rel_err(pair.host(HV), pair.oracle.hessvec(Wh, S, Vh)) <= tol
    pair.close()


@pytest.mark.parametrize("dtype", DTYPES, ids=["f64", "f32"])
def test_sparse_binary_full_passes_with_a_lane_per_entry_on_odd_row_lengths(dtype):
    # Full passes over a CSR matrix with one weight column take the stored entries in aligned windows of 64, a lane per
    # entry, and find each entry's row among the 63 rows that follow the window's first.  Here most rows have no entry
    # or one (far more than 63 rows end inside a window: the rows are looked up in the row pointers instead), a few
    # have hundreds (one row runs through several windows), the last rows are empty, and one row ends exactly where
    # a window ends.
    n, p = 50_000, 300
    g = np.random.default_rng(19)
    counts = g.integers(0, 2, size=n)
    counts[::997] = g.integers(150, 300, size=counts[::997].size)
    counts[5] = 64 + (-int(counts[:5].sum())) % 64       # row 5 ends where a window ends
    counts[-40:] = 0
    rowptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(counts, out=rowptr[1:])
    assert rowptr[6] % 64 == 0 and counts[5] > 0
    nnz = int(rowptr[-1])
    colidx = np.concatenate([np.sort(g.choice(p, size=k, replace=False)) for k in counts if k]).astype(np.int32)
    vals = g.standard_normal(nnz)
    labels = g.integers(0, 2, size=n).astype(np.int32)
    d = dict(layout="csr", rowptr=rowptr, colidx=colidx, vals=vals, labels=labels, C=2, K=1, p=p, n=n, lam=1e-3, nnz=nnz)
    pair = Pair(d, dtype)
    tol = TOL[dtype]
    for scale in (0.0, 0.7):
        Wh, Wd = pair.block(scale * g.standard_normal((p, 1)))
        print(f"[case] sparse binary, lane per entry, odd row lengths dtype={dtype} scale={scale}", flush=True)
        f = pair.gpu.ssn_objective(Wd)
        G, f2 = pair.gpu.ssn_gradient(Wd)
        pred, acc = pair.gpu.ssn_predict(Wd)
        torch.cuda.synchronize()
        G_ref, f_ref = pair.oracle.gradient(Wh)
        assert rel_scalar(f, f_ref) <= tol and rel_scalar(f2, f_ref) <= tol
        assert rel_err(pair.host(G), G_ref) <= tol
        flips = int(np.count_nonzero(pred.cpu().numpy() != pair.oracle.predict(Wh)))
        assert flips <= (0 if dtype == F64 else n // 500)
    pair.close()


@pytest.mark.parametrize("dtype", DTYPES, ids=["f64", "f32"])
@pytest.mark.parametrize("counts", [[1], [0, 0, 0], [3, 0, 2], [1] * 70, [0] * 5 + [130] + [0] * 3, [64, 64, 1]],
                         ids=["one_entry", "no_entries", "three_rows", "seventy_rows", "one_long_row", "whole_windows"])
def test_sparse_binary_tiny_matrices(counts, dtype):
    # degenerate shapes of the one-weight-column CSR kernels: a single stored entry, none at all, fewer entries than
    # one window of 64, a last window that is not full, one row that is longer than two windows between empty rows,
    # rows that fill windows exactly
    counts = np.array(counts, dtype=np.int64)
    n, p = counts.size, 140
    g = np.random.default_rng(int(counts.sum()) + n)
    rowptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(counts, out=rowptr[1:])
    nnz = int(rowptr[-1])
    colidx = (np.concatenate([np.sort(g.choice(p, size=k, replace=False)) for k in counts]).astype(np.int32)
              if nnz else np.zeros(0, dtype=np.int32))
    vals = g.standard_normal(nnz)
    labels = g.integers(0, 2, size=n).astype(np.int32)
    d = dict(layout="csr", rowptr=rowptr, colidx=colidx, vals=vals, labels=labels, C=2, K=1, p=p, n=n, lam=1e-2, nnz=nnz)
    pair = Pair(d, dtype)
    tol = TOL[dtype]
    Wh, Wd = pair.block(0.5 * g.standard_normal((p, 1)))
    Vh, Vd = pair.block(g.standard_normal((p, 1)))
    print(f"[case] sparse binary tiny counts={counts.tolist()[:8]} dtype={dtype}", flush=True)
    f = pair.gpu.ssn_objective(Wd)
    G, f2 = pair.gpu.ssn_gradient(Wd)
    S = np.arange(n, dtype=np.int32)
    HV = pair.gpu.ssn_hessvec(Wd, pair.idx(S), Vd)
    pred, acc = pair.gpu.ssn_predict(Wd)
    torch.cuda.synchronize()
    G_ref, f_ref = pair.oracle.gradient(Wh)
    assert rel_scalar(f, f_ref) <= tol and rel_scalar(f2, f_ref) <= tol
    assert rel_err(pair.host(G), G_ref) <= tol
    assert rel_err(pair.host(HV), pair.oracle.hessvec(Wh, S, Vh)) <= tol
    assert np.array_equal(pred.cpu().numpy(), pair.oracle.predict(Wh)) or dtype == F32
    pair.close()
