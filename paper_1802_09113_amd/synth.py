"""Seeded synthetic inputs shaped like the paper's workloads (Table 1 of the paper).

The real datasets (Covertype, MNIST, CIFAR-10, Newsgroups20, ...) are not
available; these generators stand in for them.  Everything is drawn from
numpy's counter-based Philox generator keyed by (seed, stream), so the same
arrays come out on every machine.  This module only produces inputs (data
matrix, labels, index sets, probe directions); it contains none of the
optimiser's arithmetic and is used by both the GPU tests/benchmark and the CPU
oracle's tests.

Workloads (index = position in the benchmark's config list):
  0 tiny dense        2000 x 50      C=3   N(0,1)
  1 image-like dense  60000 x 784    C=10  U[0,1) with ~80% exact zeros
  2 wide dense        50000 x 3072   C=10  U[0,1), rows mean-centred
  3 tall-narrow dense 581012 x 54    C=7   10 N(0,1) columns + 44 Bernoulli(0.05) columns, skewed class prior
  4 sparse CSR        20000 x 1355191 C=20 ~450 nnz/row, Zipf(1.1) column ids, lognormal values, unit-norm rows
Binary workloads (C = 2) shaped like the two binary data sets of Table 1 (not in the benchmark's config list):
  5 binary dense      6000 x 5000    C=2   ~13% non-zeros U[0,1) (Gisette-shaped)
  6 binary sparse CSR 65078 x 20958  C=2   ~57 nnz/row, recipe of workload 4 (Real-Sim-shaped)
"""
import numpy as np

SEED = 20180209

# stream ids
_ST_X, _ST_WTRUE, _ST_LABEL, _ST_SAMPLE, _ST_TEST, _ST_PROBE = 0, 1, 2, 3, 4, 5

CONFIGS = [
    dict(name="tiny_dense", n=2000, p=50, C=3, lam=1e-3, frac=0.05, T=10, iters=10, layout="dense"),
    dict(name="image_like", n=60000, p=784, C=10, lam=1e-4, frac=0.05, T=10, iters=30, layout="dense"),
    dict(name="wide", n=50000, p=3072, C=10, lam=1e-4, frac=0.05, T=10, iters=10, layout="dense"),
    dict(name="tall_narrow", n=581012, p=54, C=7, lam=1e-5, frac=0.01, T=10, iters=10, layout="dense"),
    dict(name="sparse_csr", n=20000, p=1355191, C=20, lam=1e-4, frac=0.05, T=10, iters=10, layout="csr",
         nnz_row=450),
    dict(name="binary_dense", n=6000, p=5000, C=2, lam=1e-4, frac=0.05, T=10, iters=10, layout="dense"),
    dict(name="binary_sparse_csr", n=65078, p=20958, C=2, lam=1e-4, frac=0.05, T=10, iters=10, layout="csr", nnz_row=57),
]


def rng(seed, stream, sub=0):
    return np.random.Generator(np.random.Philox(key=[(int(seed) << 8) + int(stream), int(sub)]))


def _categorical(scores, g):
    """One draw per row from softmax(scores) by the Gumbel-max trick."""
    u = g.random(scores.shape)
    gumbel = -np.log(-np.log(np.clip(u, 1e-300, 1.0 - 1e-16)))
    return np.argmax(scores + gumbel, axis=1).astype(np.int32)


def _dense_rows(cfg_idx, n, p, g):
    if cfg_idx == 0:
        return g.standard_normal((n, p))
    if cfg_idx == 1:
        X = g.random((n, p))
        X *= (g.random((n, p)) < 0.2)
        return X
    if cfg_idx == 2:
        X = g.random((n, p))
        X -= X.mean(axis=1, keepdims=True)
        return X
    if cfg_idx == 3:
        X = np.empty((n, p))
        X[:, :10] = g.standard_normal((n, 10))
        X[:, 10:] = (g.random((n, p - 10)) < 0.05).astype(np.float64)
        return X
    if cfg_idx == 5:
        X = g.random((n, p))
        X *= (g.random((n, p)) < 0.13)
        return X
    raise ValueError(cfg_idx)


def _zipf_cdf(p, a=1.1):
    w = 1.0 / np.arange(1, p + 1, dtype=np.float64) ** a
    c = np.cumsum(w)
    return c / c[-1]


def _sparse_rows(n, p, nnz_row, g, cdf):
    """CSR rows: nnz_row distinct Zipf(1.1) column ids (sorted), lognormal values, unit L2 norm."""
    k = min(nnz_row, p)
    rowptr = np.arange(n + 1, dtype=np.int64) * k
    colidx = np.empty(n * k, dtype=np.int32)
    vals = np.empty(n * k, dtype=np.float64)
    for i in range(n):
        # draw column ids one after another until k distinct ones have been seen
        seq = np.empty(0, dtype=np.int64)
        uniq, first = seq, seq
        while uniq.size < k and seq.size < 10 * nnz_row:
            m = max(2 * (k - uniq.size), 64)
            cand = np.minimum(np.searchsorted(cdf, g.random(m), side="left"), p - 1)
            seq = np.concatenate([seq, cand])
            uniq, first = np.unique(seq, return_index=True)
        if uniq.size >= k:
            have = np.sort(uniq[np.argsort(first, kind="stable")[:k]])
        else:                                  # draw cap reached (only for tiny p): top up in index order
            rest = np.setdiff1d(np.arange(p), uniq)[: k - uniq.size]
            have = np.sort(np.concatenate([uniq, rest]))
        v = np.exp(g.standard_normal(k))
        v /= np.sqrt(np.sum(v * v))
        colidx[i * k:(i + 1) * k] = have
        vals[i * k:(i + 1) * k] = v
    return rowptr, colidx, vals


def _csr_times_dense(rowptr, colidx, vals, M):
    n = rowptr.shape[0] - 1
    out = np.zeros((n, M.shape[1]))
    k = int(rowptr[1] - rowptr[0]) if n else 0
    # all rows have the same number of stored entries: one gather + reshape
    prod = vals[:, None] * M[colidx]
    return prod.reshape(n, k, M.shape[1]).sum(axis=1) if n else out


def make(cfg_idx, n=None, p=None, seed=SEED, part="train"):
    """Generate workload `cfg_idx`; `n` / `p` override the size (parity tests use reduced n).

    part="train" or "test" (held-out rows from the same model, max(1000, n/10) of them by default).
    Returns a dict: name, layout, n, p, C, K, lam, nS, T, iters, labels (int32), and either
    X (fp64, n x p) or rowptr (int64) / colidx (int32) / vals (fp64).
    """
    cfg = dict(CONFIGS[cfg_idx])
    full_n = cfg["n"]
    n_train = int(n) if n is not None else full_n
    p = int(p) if p is not None else cfg["p"]
    C = cfg["C"]
    if part == "train":
        rows, gx, gl = n_train, rng(seed, _ST_X, cfg_idx), rng(seed, _ST_LABEL, cfg_idx)
    else:
        rows = max(1000, n_train // 10)
        gx, gl = rng(seed, _ST_TEST, cfg_idx), rng(seed, _ST_TEST, 100 + cfg_idx)
    gw = rng(seed, _ST_WTRUE, cfg_idx)
    out = dict(name=cfg["name"], layout=cfg["layout"], n=rows, p=p, C=C, K=C - 1, lam=cfg["lam"],
               nS=max(1, int(round(cfg["frac"] * n_train))), T=cfg["T"], iters=cfg["iters"])
    if cfg["layout"] == "dense":
        X = _dense_rows(cfg_idx, rows, p, gx)
        W_true = gw.standard_normal((p, C))
        if cfg_idx == 0:
            scores = X @ W_true
        elif cfg_idx in (1, 2):
            scores = X @ W_true / np.sqrt(p)
        elif cfg_idx == 5:
            scores = X @ W_true * (4.0 / np.sqrt(0.13 * p / 3.0))        # score spread of about 4: learnable labels
        else:
            prior = np.array([36, 49, 6, 0.5, 1.6, 3, 3.5])
            scores = X @ (0.5 * W_true) + np.log(prior / prior.sum())
        out["X"] = X
    else:
        cdf = _zipf_cdf(p)
        rowptr, colidx, vals = _sparse_rows(rows, p, cfg["nnz_row"], gx, cdf)
        W_true = gw.standard_normal((p, C)) * (gw.random((p, C)) < 0.1)
        scores = _csr_times_dense(rowptr, colidx, vals, W_true)
        sd = scores.std()
        scores *= 2.0 / (sd if sd > 0 else 1.0)
        out.update(rowptr=rowptr, colidx=colidx, vals=vals, nnz=int(rowptr[-1]))
    out["labels"] = _categorical(scores, gl)
    return out


def sample_rows(n, nS, seed=SEED, it=0, replace=False):
    """Hessian sample for SSN iteration `it`: nS row ids, uniform, sorted ascending."""
    g = rng(seed, _ST_SAMPLE, it)
    if replace:
        s = g.integers(0, n, size=nS)
    else:
        s = g.choice(n, size=nS, replace=False)
    return np.sort(s).astype(np.int32)


def sample_schedule(n, nS, iters, seed=SEED):
    return np.stack([sample_rows(n, nS, seed, it) for it in range(iters)])


def probe(p, K, seed=SEED, sub=0, scale=1.0):
    """A p x K block of N(0, scale^2) numbers (probe directions V, non-zero weights W)."""
    return scale * rng(seed, _ST_PROBE, sub).standard_normal((p, K))
