"""Pins for the CPU oracle's unit-column-norm preprocessing of Sec. 4 (no GPU): against numpy written out,
the invariant it exists for (every non-zero column ends with 2-norm 1), zero columns, and the
agreement of the dense and the CSR form on the same matrix."""
import numpy as np

from oracle.oracle import normalize_columns


def test_dense_against_numpy_and_unit_norms():
    g = np.random.default_rng(5)
    X = g.standard_normal((200, 9)) * g.uniform(0.1, 30.0, size=9)
    X[:, 4] = 0.0                                            # a column without entries stays as it is
    Xs, norms = normalize_columns(X=X)
    expect = np.sqrt((X.astype(np.longdouble) ** 2).sum(axis=0)).astype(np.float64)
    np.testing.assert_allclose(norms, expect, rtol=1e-15)
    assert norms[4] == 0.0 and np.all(Xs[:, 4] == 0.0)
    nz = norms > 0
    np.testing.assert_allclose(Xs[:, nz], X[:, nz] / norms[nz], rtol=1e-15)
    np.testing.assert_allclose(np.linalg.norm(Xs[:, nz], axis=0), 1.0, rtol=1e-14)
    assert np.array_equal(X[:, 0], X[:, 0])                 # the input is not touched (a copy is scaled)


def test_csr_agrees_with_dense():
    g = np.random.default_rng(6)
    n, p = 150, 40
    X = g.standard_normal((n, p)) * (g.random((n, p)) < 0.15)
    X[:, 7] = 0.0
    rowptr = np.zeros(n + 1, dtype=np.int64)
    cols, vals = [], []
    for i in range(n):
        j = np.nonzero(X[i])[0]
        cols.append(j.astype(np.int32))
        vals.append(X[i, j])
        rowptr[i + 1] = rowptr[i] + j.size
    colidx, v = np.concatenate(cols), np.concatenate(vals)
    vs, norms_s = normalize_columns(csr=(rowptr, colidx, v), p=p)
    Xd, norms_d = normalize_columns(X=X)
    np.testing.assert_allclose(norms_s, norms_d, rtol=1e-15)
    dense_from_sparse = np.zeros_like(X)
    for i in range(n):
        dense_from_sparse[i, colidx[rowptr[i]:rowptr[i + 1]]] = vs[rowptr[i]:rowptr[i + 1]]
    np.testing.assert_allclose(dense_from_sparse, Xd, rtol=1e-15)
    assert norms_s[7] == 0.0
