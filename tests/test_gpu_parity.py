"""GPU parity: the HIP library (through its C ABI) against the CPU oracle, element by element, on the
same seeded inputs.  Tolerances: fp64 1e-10, fp32 1e-4 relative (norm-wise for blocks)."""
import numpy as np
import pytest
import torch

from paper_1802_09113_amd import synth
from tests.gpu_util import TOL, Pair, rel_err, rel_scalar, workload

pytestmark = pytest.mark.gpu

F64, F32 = torch.float64, torch.float32

# (config index, reduced n) -- sizes the oracle finishes in seconds, several tiles plus a ragged tail
CASES = [(0, 2000), (1, 3001), (2, 1003), (3, 5003), (4, 403)]
DTYPES = [F64, F32]


def _weights(pair, sub, scale):
    return pair.block(synth.probe(pair.p, pair.K, sub=sub, scale=scale))


@pytest.fixture(scope="module")
def data_cache():
    cache = {}

    def get(cfg, n):
        if (cfg, n) not in cache:
            print(f"[gen] cfg={cfg} n={n}", flush=True)
            cache[(cfg, n)] = workload(cfg, n)
        return cache[(cfg, n)]

    return get


@pytest.mark.parametrize("dtype", DTYPES, ids=["f64", "f32"])
@pytest.mark.parametrize("cfg,n", CASES)
def test_objective_and_gradient(data_cache, cfg, n, dtype):
    pair = Pair(data_cache(cfg, n), dtype)
    tol = TOL[dtype]
    for sub, scale in [(0, 0.0), (1, 0.1), (2, 1.0)]:
        Wh, Wd = _weights(pair, sub, scale)
        print(f"[case] obj/grad cfg={cfg} n={n} dtype={dtype} scale={scale}", flush=True)
        f_ref = pair.oracle.objective(Wh)
        G_ref, _ = pair.oracle.gradient(Wh)
        f = pair.gpu.ssn_objective(Wd)
        G, f2 = pair.gpu.ssn_gradient(Wd)
        torch.cuda.synchronize()
        assert rel_scalar(f, f_ref) <= tol, (f, f_ref)
        assert rel_scalar(f2, f_ref) <= tol
        assert rel_err(pair.host(G), G_ref) <= tol, rel_err(pair.host(G), G_ref)
    pair.close()


@pytest.mark.parametrize("dtype", DTYPES, ids=["f64", "f32"])
@pytest.mark.parametrize("cfg,n", CASES)
def test_hessvec(data_cache, cfg, n, dtype):
    d = data_cache(cfg, n)
    pair = Pair(d, dtype)
    tol = TOL[dtype]
    S = synth.sample_rows(n, d["nS"])
    Sd = pair.idx(S)
    for sub, scale in [(0, 0.0), (1, 0.1)]:
        Wh, Wd = _weights(pair, sub, scale)
        print(f"[case] hessvec cfg={cfg} n={n} dtype={dtype} scale={scale} nS={S.size}", flush=True)
        pair.gpu.ssn_hess_prepare(Wd, Sd)
        for vs in (7, 8):
            Vh, Vd = _weights(pair, vs, 1.0)
            HV = pair.gpu.ssn_hess_apply(Vd)
            torch.cuda.synchronize()
            ref = pair.oracle.hessvec(Wh, S, Vh)
            assert rel_err(pair.host(HV), ref) <= tol, rel_err(pair.host(HV), ref)
        # the combined entry point gives the same block
        HV2 = pair.gpu.ssn_hessvec(Wd, Sd, Vd)
        torch.cuda.synchronize()
        assert rel_err(pair.host(HV2), ref) <= tol
    pair.close()


@pytest.mark.parametrize("dtype", DTYPES, ids=["f64", "f32"])
@pytest.mark.parametrize("cfg,n", CASES)
def test_sampled_gradient(data_cache, cfg, n, dtype):
    # eq. (2a): 20 % of the rows without replacement, and a multiset with repeats
    d = data_cache(cfg, n)
    pair = Pair(d, dtype)
    tol = TOL[dtype]
    rng = np.random.default_rng(11)
    samples = [synth.sample_rows(n, max(1, n // 5), seed=77), rng.integers(0, n, size=max(3, n // 7)).astype(np.int32)]
    Wh, Wd = _weights(pair, 1, 0.1)
    for S in samples:
        print(f"[case] sampled gradient cfg={cfg} n={n} dtype={dtype} nS={S.size}", flush=True)
        G, fS = pair.gpu.ssn_gradient_sampled(Wd, pair.idx(S))
        torch.cuda.synchronize()
        G_ref, f_ref = pair.oracle.gradient_sampled(Wh, S)
        assert rel_err(pair.host(G), G_ref) <= tol, rel_err(pair.host(G), G_ref)
        assert rel_scalar(fS, f_ref) <= tol
    # the Hessian sample prepared before a sampled gradient stays usable after it
    Sh = synth.sample_rows(n, d["nS"])
    Vh, Vd = _weights(pair, 7, 1.0)
    pair.gpu.ssn_hess_prepare(Wd, pair.idx(Sh))
    pair.gpu.ssn_gradient_sampled(Wd, pair.idx(samples[0]), want_f=False)
    HV = pair.gpu.ssn_hess_apply(Vd)
    torch.cuda.synchronize()
    assert rel_err(pair.host(HV), pair.oracle.hessvec(Wh, Sh, Vh)) <= tol
    pair.close()


@pytest.mark.parametrize("dtype", DTYPES, ids=["f64", "f32"])
def test_hessvec_multiset_sample_and_single_row(data_cache, dtype):
    d = data_cache(0, 2000)
    pair = Pair(d, dtype)
    Wh, Wd = _weights(pair, 1, 0.3)
    Vh, Vd = _weights(pair, 2, 1.0)
    for S in ([5], [3, 3, 3, 1999, 0, 7, 7], list(range(2000)) + [11] * 37, [1999, 5, 1000]):
        S = np.array(S, dtype=np.int32)
        print(f"[case] multiset nS={S.size} dtype={dtype}", flush=True)
        HV = pair.gpu.ssn_hessvec(Wd, pair.idx(S), Vd)
        torch.cuda.synchronize()
        ref = pair.oracle.hessvec(Wh, S, Vh)
        assert rel_err(pair.host(HV), ref) <= TOL[dtype]
    pair.close()


@pytest.mark.parametrize("dtype", DTYPES, ids=["f64", "f32"])
def test_hessvec_sample_of_several_row_blocks_per_workgroup(data_cache, dtype):
    # 6000 sample rows = 375 row blocks, more than one per workgroup of the one-pass kernel (whose
    # one-block-per-workgroup variant serves the smaller samples of the other tests)
    d = data_cache(1, 5000)
    pair = Pair(d, dtype)
    rng = np.random.default_rng(5)
    S = np.concatenate([rng.permutation(5000), rng.permutation(5000)[:1000]]).astype(np.int32)
    Wh, Wd = _weights(pair, 1, 0.1)
    Vh, Vd = _weights(pair, 2, 1.0)
    print(f"[case] several blocks per workgroup nS={S.size} dtype={dtype}", flush=True)
    HV = pair.gpu.ssn_hessvec(Wd, pair.idx(S), Vd)
    torch.cuda.synchronize()
    ref = pair.oracle.hessvec(Wh, S, Vh)
    assert rel_err(pair.host(HV), ref) <= TOL[dtype]
    pair.close()


@pytest.mark.parametrize("dtype", DTYPES, ids=["f64", "f32"])
def test_wide_matrix_with_many_row_blocks(data_cache, dtype):
    # 9001 rows of the 3072-feature workload: more row blocks than the chip has places for workgroups of 8 or 16
    # waves, so four waves share a row block, with a ragged last block
    d = data_cache(2, 9001)
    pair = Pair(d, dtype)
    tol = TOL[dtype]
    Wh, Wd = _weights(pair, 1, 0.1)
    print(f"[case] wide many blocks dtype={dtype}", flush=True)
    f = pair.gpu.ssn_objective(Wd)
    G, f2 = pair.gpu.ssn_gradient(Wd)
    torch.cuda.synchronize()
    G_ref, f_ref = pair.oracle.gradient(Wh)
    assert rel_scalar(f, f_ref) <= tol and rel_scalar(f2, f_ref) <= tol
    assert rel_err(pair.host(G), G_ref) <= tol
    S = np.arange(9001, dtype=np.int32)[::-1].copy()                 # all rows, reversed: 563 blocks in the product too
    Vh, Vd = _weights(pair, 2, 1.0)
    HV = pair.gpu.ssn_hessvec(Wd, pair.idx(S), Vd)
    torch.cuda.synchronize()
    assert rel_err(pair.host(HV), pair.oracle.hessvec(Wh, S, Vh)) <= tol
    _, acc = pair.gpu.ssn_predict(Wd)
    assert abs(acc - pair.oracle.accuracy(Wh)) <= (1e-12 if dtype == F64 else 2e-3)
    pair.close()


@pytest.mark.parametrize("dtype", DTYPES, ids=["f64", "f32"])
@pytest.mark.parametrize("scale", ["mean", "sum"])
def test_scaling_modes_and_padded_leading_dimensions(data_cache, scale, dtype):
    d = data_cache(0, 2000)
    # ldw > K, ldx > p and an ldx that breaks 16-byte row alignment (scalar-load kernel variant)
    for ldw, ldx in [(None, None), (5, 64), (2, 51), (3, 53)]:
        pair = Pair(d, dtype, scale=scale, ldw=ldw, ldx=ldx)
        print(f"[case] scale={scale} ldw={ldw} ldx={ldx} dtype={dtype}", flush=True)
        Wh, Wd = _weights(pair, 3, 0.2)
        Vh, Vd = _weights(pair, 4, 1.0)
        S = synth.sample_rows(2000, 100, it=3)
        f = pair.gpu.ssn_objective(Wd)
        G, _ = pair.gpu.ssn_gradient(Wd)
        HV = pair.gpu.ssn_hessvec(Wd, pair.idx(S), Vd)
        torch.cuda.synchronize()
        tol = TOL[dtype]
        assert rel_scalar(f, pair.oracle.objective(Wh)) <= tol
        assert rel_err(pair.host(G), pair.oracle.gradient(Wh)[0]) <= tol
        assert rel_err(pair.host(HV), pair.oracle.hessvec(Wh, S, Vh)) <= tol
        pair.close()


@pytest.mark.parametrize("dtype", DTYPES, ids=["f64", "f32"])
@pytest.mark.parametrize("p,C", [(300, 17), (200, 4), (416, 9), (1000, 6), (90, 3), (70, 12)])
def test_one_pass_kernel_shapes_between_the_workloads(p, C, dtype):
    # the register footprints the workloads do not reach: four waves per workgroup (200-416 features; two workgroups
    # share a compute unit where their LDS allows, which 16 class columns do not), the widest eight-wave shape
    # (1000 features), and the single-wave shapes of 57-104 features
    g = np.random.default_rng(p + C)
    n = 9000 + 7
    X = g.standard_normal((n, p)) * (g.random((n, p)) < 0.5)
    labels = g.integers(0, C, size=n).astype(np.int32)
    d = dict(layout="dense", X=X, labels=labels, C=C, p=p, n=n, lam=1e-3)
    pair = Pair(d, dtype)
    assert pair.gpu.ssn_dense_path() == 2
    Wh, Wd = pair.block(0.1 * g.standard_normal((p, C - 1)))
    Vh, Vd = pair.block(g.standard_normal((p, C - 1)))
    S = g.integers(0, n, size=450).astype(np.int32)
    print(f"[case] one-pass shape p={p} C={C} dtype={dtype}", flush=True)
    f = pair.gpu.ssn_objective(Wd)
    G, f2 = pair.gpu.ssn_gradient(Wd)
    HV = pair.gpu.ssn_hessvec(Wd, pair.idx(S), Vd)
    HVall = pair.gpu.ssn_hessvec(Wd, pair.idx(np.arange(n, dtype=np.int32)), Vd)
    _, acc = pair.gpu.ssn_predict(Wd)
    torch.cuda.synchronize()
    tol = TOL[dtype]
    G_ref, f_ref = pair.oracle.gradient(Wh)
    assert rel_scalar(f, f_ref) <= tol and rel_scalar(f2, f_ref) <= tol
    assert rel_err(pair.host(G), G_ref) <= tol
    assert rel_err(pair.host(HV), pair.oracle.hessvec(Wh, S, Vh)) <= tol
    assert rel_err(pair.host(HVall), pair.oracle.hessvec(Wh, np.arange(n), Vh)) <= tol
    assert abs(acc - pair.oracle.accuracy(Wh)) <= (1e-12 if dtype == F64 else 2e-3)
    pair.close()


@pytest.mark.parametrize("dtype", DTYPES, ids=["f64", "f32"])
def test_medium_width_matrix_two_row_blocks_per_trip(dtype):
    # 1200 features: too wide for the one-pass kernel, narrower than the 2048 from which a workgroup shares a row
    # block on full passes; 8211 rows are 514 row blocks (one ragged), so the wave-per-block kernel runs in its
    # two-blocks-per-trip form
    g = np.random.default_rng(1200)
    n, p, C = 8211, 1200, 6
    X = g.standard_normal((n, p)) * (g.random((n, p)) < 0.3)
    labels = g.integers(0, C, size=n).astype(np.int32)
    d = dict(layout="dense", X=X, labels=labels, C=C, p=p, n=n, lam=1e-3)
    pair = Pair(d, dtype)
    assert pair.gpu.ssn_dense_path() == 1
    Wh, Wd = pair.block(0.05 * g.standard_normal((p, C - 1)))
    Vh, Vd = pair.block(g.standard_normal((p, C - 1)))
    S = g.integers(0, n, size=700).astype(np.int32)
    print(f"[case] medium width dtype={dtype}", flush=True)
    f = pair.gpu.ssn_objective(Wd)
    G, f2 = pair.gpu.ssn_gradient(Wd)
    HV = pair.gpu.ssn_hessvec(Wd, pair.idx(S), Vd)
    torch.cuda.synchronize()
    tol = TOL[dtype]
    G_ref, f_ref = pair.oracle.gradient(Wh)
    assert rel_scalar(f, f_ref) <= tol and rel_scalar(f2, f_ref) <= tol
    assert rel_err(pair.host(G), G_ref) <= tol
    assert rel_err(pair.host(HV), pair.oracle.hessvec(Wh, S, Vh)) <= tol
    pair.close()


@pytest.mark.parametrize("dtype", DTYPES, ids=["f64", "f32"])
@pytest.mark.parametrize("xoff", [0, 1, 3])
def test_rows_aligned_to_their_element_only(data_cache, xoff, dtype):
    # 54 features: fp32 rows of 216 bytes; with xoff the matrix itself starts 4 / 8 (12 / 24) bytes into its allocation, and
    # the allocation ends with the last row (whole-vector loads of that row's end must not leave it)
    d = data_cache(3, 1003)
    pair = Pair(d, dtype, xoff=xoff)
    print(f"[case] element-aligned rows xoff={xoff} dtype={dtype}", flush=True)
    Wh, Wd = _weights(pair, 3, 0.2)
    Vh, Vd = _weights(pair, 4, 1.0)
    S = np.concatenate([synth.sample_rows(1003, 60, it=2), np.array([1002, 1002, 0], dtype=np.int32)])   # the last row, twice
    f = pair.gpu.ssn_objective(Wd)
    G, fg = pair.gpu.ssn_gradient(Wd)
    HV = pair.gpu.ssn_hessvec(Wd, pair.idx(S), Vd)
    _, acc = pair.gpu.ssn_predict(Wd)
    torch.cuda.synchronize()
    tol = TOL[dtype]
    assert rel_scalar(f, pair.oracle.objective(Wh)) <= tol
    assert rel_scalar(fg, pair.oracle.objective(Wh)) <= tol
    assert rel_err(pair.host(G), pair.oracle.gradient(Wh)[0]) <= tol
    assert rel_err(pair.host(HV), pair.oracle.hessvec(Wh, S, Vh)) <= tol
    assert abs(acc - pair.oracle.accuracy(Wh)) <= (1e-12 if dtype == F64 else 2e-3)
    pair.close()


@pytest.mark.parametrize("dtype", DTYPES, ids=["f64", "f32"])
@pytest.mark.parametrize("p", [45, 54])
@pytest.mark.parametrize("C", [2, 17, 18, 33])
def test_class_counts_across_mfma_tile_boundaries(C, p, dtype):
    # more than 16 weight columns go to the two-kernel path, whose loads follow the rows' alignment: 45 features are
    # element-aligned rows (scalar loads), 54 fp32 features 8-byte aligned ones (two-element loads)
    g = np.random.default_rng(C)
    n = 777
    X = g.standard_normal((n, p))
    labels = g.integers(0, C, size=n).astype(np.int32)
    d = dict(layout="dense", X=X, labels=labels, C=C, p=p, n=n, lam=1e-3)
    pair = Pair(d, dtype)
    Wh, Wd = pair.block(0.3 * g.standard_normal((p, C - 1)))
    Vh, Vd = pair.block(g.standard_normal((p, C - 1)))
    S = np.sort(g.choice(n, 100, replace=False)).astype(np.int32)
    print(f"[case] C={C} p={p} dtype={dtype}", flush=True)
    f = pair.gpu.ssn_objective(Wd)
    G, _ = pair.gpu.ssn_gradient(Wd)
    HV = pair.gpu.ssn_hessvec(Wd, pair.idx(S), Vd)
    pred, acc = pair.gpu.ssn_predict(Wd)
    torch.cuda.synchronize()
    tol = TOL[dtype]
    assert rel_scalar(f, pair.oracle.objective(Wh)) <= tol
    assert rel_err(pair.host(G), pair.oracle.gradient(Wh)[0]) <= tol
    assert rel_err(pair.host(HV), pair.oracle.hessvec(Wh, S, Vh)) <= tol
    if dtype == F64:
        np.testing.assert_array_equal(pred.cpu().numpy(), pair.oracle.predict(Wh))
    pair.close()


@pytest.mark.parametrize("dtype", DTYPES, ids=["f64", "f32"])
def test_degenerate_shapes(dtype):
    g = np.random.default_rng(77)
    for n, p, C in [(1, 1, 2), (1, 3, 3), (15, 2, 4), (17, 5, 2), (16, 64, 3), (33, 65, 5)]:
        X = g.standard_normal((n, p))
        labels = g.integers(0, C, size=n).astype(np.int32)
        d = dict(layout="dense", X=X, labels=labels, C=C, p=p, n=n, lam=1e-2)
        pair = Pair(d, dtype)
        Wh, Wd = pair.block(g.standard_normal((p, C - 1)))
        Vh, Vd = pair.block(g.standard_normal((p, C - 1)))
        S = g.integers(0, n, size=max(1, n // 2)).astype(np.int32)
        print(f"[case] degenerate n={n} p={p} C={C} dtype={dtype}", flush=True)
        f = pair.gpu.ssn_objective(Wd)
        G, _ = pair.gpu.ssn_gradient(Wd)
        HV = pair.gpu.ssn_hessvec(Wd, pair.idx(S), Vd)
        torch.cuda.synchronize()
        tol = TOL[dtype]
        assert rel_scalar(f, pair.oracle.objective(Wh)) <= tol
        assert rel_err(pair.host(G), pair.oracle.gradient(Wh)[0]) <= tol
        assert rel_err(pair.host(HV), pair.oracle.hessvec(Wh, S, Vh)) <= tol
        pair.close()


def test_csr_with_empty_rows_and_large_margins():
    g = np.random.default_rng(5)
    n, p, C = 300, 1000, 6
    dense = g.standard_normal((n, p)) * (g.random((n, p)) < 0.02)
    dense[[0, 17, 299]] = 0.0
    rowptr = np.zeros(n + 1, dtype=np.int64)
    cols, vals = [], []
    for i in range(n):
        nz = np.nonzero(dense[i])[0]
        cols.append(nz)
        vals.append(dense[i, nz])
        rowptr[i + 1] = rowptr[i] + nz.size
    labels = g.integers(0, C, size=n).astype(np.int32)
    d = dict(layout="csr", rowptr=rowptr, colidx=np.concatenate(cols).astype(np.int32), vals=np.concatenate(vals),
             labels=labels, C=C, p=p, n=n, lam=1e-3)
    pair = Pair(d, F64)
    Wh, Wd = pair.block(200.0 * g.standard_normal((p, C - 1)))      # margins of several hundred
    Vh, Vd = pair.block(g.standard_normal((p, C - 1)))
    S = np.array([0, 17, 5, 5, 299, 100], dtype=np.int32)
    f = pair.gpu.ssn_objective(Wd)
    G, _ = pair.gpu.ssn_gradient(Wd)
    HV = pair.gpu.ssn_hessvec(Wd, pair.idx(S), Vd)
    torch.cuda.synchronize()
    assert np.isfinite(f)
    assert rel_scalar(f, pair.oracle.objective(Wh)) <= 1e-10
    assert rel_err(pair.host(G), pair.oracle.gradient(Wh)[0]) <= 1e-10
    assert rel_err(pair.host(HV), pair.oracle.hessvec(Wh, S, Vh)) <= 1e-10
    pair.close()


@pytest.mark.parametrize("dtype", DTYPES, ids=["f64", "f32"])
def test_dense_large_margins_stay_finite(dtype):
    X = np.array([[800.0, 0.0], [-800.0, 0.0], [0.0, 800.0], [0.0, -800.0]] * 5)
    labels = np.array([0, 0, 1, 2] * 5, dtype=np.int32)
    d = dict(layout="dense", X=X, labels=labels, C=3, p=2, n=20, lam=0.0)
    pair = Pair(d, dtype, scale="sum")
    Wh, Wd = pair.block(np.eye(2))
    f = pair.gpu.ssn_objective(Wd)
    G, _ = pair.gpu.ssn_gradient(Wd)
    torch.cuda.synchronize()
    assert np.isfinite(f) and torch.isfinite(G[:, :2]).all()
    assert rel_scalar(f, pair.oracle.objective(Wh)) <= TOL[dtype]
    assert rel_err(pair.host(G), pair.oracle.gradient(Wh)[0]) <= TOL[dtype]
    pair.close()


@pytest.mark.parametrize("dtype", DTYPES, ids=["f64", "f32"])
@pytest.mark.parametrize("cfg,n", [(0, 2000), (1, 3001), (4, 403)])
def test_predict_and_accuracy(data_cache, cfg, n, dtype):
    pair = Pair(data_cache(cfg, n), dtype)
    Wh, Wd = _weights(pair, 5, 1.0)
    pred, acc = pair.gpu.ssn_predict(Wd)
    torch.cuda.synchronize()
    ref = pair.oracle.predict(Wh)
    got = pred.cpu().numpy()
    if dtype == F64:
        np.testing.assert_array_equal(got, ref)
        assert acc == pair.oracle.accuracy(Wh)
    else:
        # fp32 margins decide the argmax in fp32: allow flips only where the top two margins nearly tie
        assert np.mean(got != ref) <= 2e-3
        assert abs(acc - pair.oracle.accuracy(Wh)) <= 1e-3
    assert acc == pytest.approx(float(np.mean(got == pair.labels)), abs=1e-12)
    pair.close()


@pytest.mark.parametrize("dtype", DTYPES, ids=["f64", "f32"])
@pytest.mark.parametrize("C", [34, 40, 65])
def test_csr_with_more_than_32_weight_columns(C, dtype):
    # the CSR kernels split a wave's lanes into (stored entry, class) groups of K lanes: with K in (32, 64] a
    # wave holds a single group with spare lanes.  Objective, gradient, sampled gradient, product, CG, accuracy.
    from tests.test_gpu_solvers import _small_csr
    n, p = 700, 900
    d = _small_csr(n, p, C, seed=100 + C, empty_rows={5, 699})
    pair = Pair(d, dtype)
    tol = TOL[dtype]
    Wh, Wd = pair.block(synth.probe(p, C - 1, sub=1, scale=0.3))
    Vh, Vd = pair.block(synth.probe(p, C - 1, sub=2))
    print(f"[case] csr C={C} dtype={dtype}", flush=True)
    G, f = pair.gpu.ssn_gradient(Wd)
    torch.cuda.synchronize()
    G_ref, f_ref = pair.oracle.gradient(Wh)
    assert rel_scalar(f, f_ref) <= tol and rel_scalar(pair.gpu.ssn_objective(Wd), f_ref) <= tol
    assert rel_err(pair.host(G), G_ref) <= tol
    S = synth.sample_rows(n, 120)
    S[:3] = S[3]                                     # a repeated row
    HV = pair.gpu.ssn_hessvec(Wd, pair.idx(S), Vd)
    Gs, fs = pair.gpu.ssn_gradient_sampled(Wd, pair.idx(S))
    torch.cuda.synchronize()
    assert rel_err(pair.host(HV), pair.oracle.hessvec(Wh, S, Vh)) <= tol
    Gs_ref, fs_ref = pair.oracle.gradient_sampled(Wh, S)
    assert rel_err(pair.host(Gs), Gs_ref) <= tol and rel_scalar(fs, fs_ref) <= tol
    Gh, Gd = pair.block(G_ref)
    ref = pair.oracle.cg(Wh, S, Gh, 1e-4, 8)
    out = pair.gpu.ssn_cg(Gd, 1e-4, 8)
    torch.cuda.synchronize()
    ttol = 1e-8 if dtype == F64 else 5e-3
    assert out["iters"] == ref["iters"]
    np.testing.assert_allclose(out["alpha"], ref["alpha"], rtol=ttol)
    assert rel_err(pair.host(out["p"]), ref["p"]) <= ttol
    _, acc = pair.gpu.ssn_predict(Wd, want_pred=False)
    assert abs(acc - pair.oracle.accuracy(Wh)) <= (0.0 if dtype == F64 else 2e-3)
    pair.close()


@pytest.mark.parametrize("C", [2, 4, 20], ids=["K1", "K3", "K19"])
@pytest.mark.parametrize("dtype", DTYPES, ids=["f64", "f32"])
def test_csr_columns_at_the_piece_and_run_boundaries_of_the_transposed_product(C, dtype):
    """The transposed product cuts every column into pieces of 64 entries and, on views of more than 2048 rows, adds
    the pieces of a column in runs that end at every 16th piece: columns of exactly 64 / 65, 1023 / 1024 / 1025 and
    2048 entries, one present in every row, and cheap ones in between so that the long columns start at different
    places of the piece list.  Gradient over all rows (runs) and a product on a sample of 1500 rows (no runs)."""
    g = np.random.default_rng(77 + C)
    n, p = 4100, 40
    counts = {0: n, 3: 64, 4: 65, 7: 1023, 8: 1024, 9: 1025, 15: 2048, 16: 1, 21: 130, 22: 2049, 30: 63, 39: 1040}
    member = np.zeros((n, p), dtype=bool)
    for j in range(p):
        k = counts.get(j, int(g.integers(1, 40)))
        member[g.choice(n, size=k, replace=False), j] = True
    rowptr = np.zeros(n + 1, dtype=np.int64)
    cols, vals = [], []
    for i in range(n):
        nz = np.nonzero(member[i])[0]
        cols.append(nz)
        vals.append(g.standard_normal(nz.size))
        rowptr[i + 1] = rowptr[i] + nz.size
    d = dict(layout="csr", rowptr=rowptr, colidx=np.concatenate(cols).astype(np.int32), vals=np.concatenate(vals),
             labels=g.integers(0, C, size=n).astype(np.int32), C=C, p=p, n=n, lam=1e-3)
    print(f"[case] csr run boundaries C={C} dtype={dtype}", flush=True)
    pair = Pair(d, dtype)
    Wh, Wd = pair.block(0.3 * g.standard_normal((p, C - 1)))
    Vh, Vd = pair.block(g.standard_normal((p, C - 1)))
    S = np.sort(g.choice(n, size=1500, replace=False)).astype(np.int32)
    G, f = pair.gpu.ssn_gradient(Wd)
    HV = pair.gpu.ssn_hessvec(Wd, pair.idx(S), Vd)
    HVall = pair.gpu.ssn_hessvec(Wd, pair.idx(np.arange(n, dtype=np.int32)), Vd)
    torch.cuda.synchronize()
    tol = TOL[dtype]
    Go, fo = pair.oracle.gradient(Wh)
    assert rel_scalar(f, fo) <= tol
    assert rel_err(pair.host(G), Go) <= tol
    assert rel_err(pair.host(HV), pair.oracle.hessvec(Wh, S, Vh)) <= tol
    assert rel_err(pair.host(HVall), pair.oracle.hessvec(Wh, np.arange(n, dtype=np.int32), Vh)) <= tol
    pair.close()


@pytest.mark.parametrize("C", [2, 4, 20, 41], ids=["K1", "K3", "K19", "K40"])
@pytest.mark.parametrize("dtype", DTYPES, ids=["f64", "f32"])
def test_csr_row_lengths_around_the_rounds_of_the_rows_kernel(C, dtype):
    """A wave of the CSR rows kernel takes 64 / K stored entries per step and eight steps per round, the last round
    with lanes switched off: rows whose lengths sit at and next to the multiples of a step and of a round for
    K = 1, 3, 19 and 40 (64, 21, 3 and 1 entries per step), empty rows included."""
    g = np.random.default_rng(310 + C)
    p = 1300
    lengths = [0, 1, 2, 3, 4, 7, 8, 9, 20, 21, 22, 23, 24, 25, 26, 47, 48, 49, 63, 64, 65, 127, 128, 129, 167, 168, 169, 170,
               335, 336, 337, 511, 512, 513, 514, 575, 576, 577, 1023, 1024, 1025, 1300, 0, 5]
    n = len(lengths)
    rowptr = np.zeros(n + 1, dtype=np.int64)
    cols, vals = [], []
    for i, L in enumerate(lengths):
        nz = np.sort(g.choice(p, size=L, replace=False))
        cols.append(nz)
        vals.append(g.standard_normal(L))
        rowptr[i + 1] = rowptr[i] + L
    d = dict(layout="csr", rowptr=rowptr, colidx=np.concatenate(cols).astype(np.int32), vals=np.concatenate(vals),
             labels=g.integers(0, C, size=n).astype(np.int32), C=C, p=p, n=n, lam=1e-3)
    print(f"[case] csr row lengths C={C} dtype={dtype}", flush=True)
    pair = Pair(d, dtype)
    Wh, Wd = pair.block(0.1 * g.standard_normal((p, C - 1)))
    Vh, Vd = pair.block(g.standard_normal((p, C - 1)))
    S = np.arange(n, dtype=np.int32)
    f = pair.gpu.ssn_objective(Wd)
    G, _ = pair.gpu.ssn_gradient(Wd)
    HV = pair.gpu.ssn_hessvec(Wd, pair.idx(S), Vd)
    torch.cuda.synchronize()
    tol = TOL[dtype]
    assert rel_scalar(f, pair.oracle.objective(Wh)) <= tol
    assert rel_err(pair.host(G), pair.oracle.gradient(Wh)[0]) <= tol
    assert rel_err(pair.host(HV), pair.oracle.hessvec(Wh, S, Vh)) <= tol
    pair.close()


@pytest.mark.parametrize("p,C", [(1040, 10), (1536, 17), (2084, 10), (3080, 5)], ids=["p1040", "p1536-K16", "p2084", "p3080"])
@pytest.mark.parametrize("dtype", DTYPES, ids=["f64", "f32"])
def test_sampled_product_on_feature_slices(p, C, dtype):
    """Samples of few row blocks of a wide matrix: the margins are computed per (row block, feature slice) by waves
    that keep the loads of their next feature group in flight, and the transposed product adds the slices up.
    Widths that leave a wave with no, one, two or three feature groups and an incomplete last one; samples of one
    row, of a ragged last block, and of enough blocks that only two slices are taken."""
    g = np.random.default_rng(p + C)
    n = 2600
    X = g.standard_normal((n, p)) * (g.random((n, p)) < 0.5)
    d = dict(layout="dense", X=X, labels=g.integers(0, C, size=n).astype(np.int32), C=C, p=p, n=n, lam=1e-3)
    pair = Pair(d, dtype)
    Wh, Wd = pair.block(0.05 * g.standard_normal((p, C - 1)))
    Vh, Vd = pair.block(g.standard_normal((p, C - 1)))
    tol = TOL[dtype]
    seen = set()
    for nS in (1, 17, 500, 1001, 2600):
        S = np.sort(g.choice(n, size=nS, replace=False)).astype(np.int32)
        print(f"[case] sliced sampled product p={p} C={C} nS={nS} dtype={dtype}", flush=True)
        HV = pair.gpu.ssn_hessvec(Wd, pair.idx(S), Vd)
        torch.cuda.synchronize()
        seen.add(pair.gpu.ssn_sampled_slices())
        assert rel_err(pair.host(HV), pair.oracle.hessvec(Wh, S, Vh)) <= tol
    assert max(seen) >= 2, "the sliced path did not run"
    pair.close()
