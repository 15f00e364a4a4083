"""ctypes front-end of the CPU oracle (oracle/ssn_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and by
the cpu_baseline leg of bench.py.  The product package never imports it and it
never imports the product package.

All arrays are fp64 / int32 numpy arrays on the host.  W, V, G, HV are p-by-K
row-major (K = C-1).  A problem is dense (X: n-by-p) or CSR (rowptr int64,
colidx int32, vals fp64).
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ssn_oracle.c")
_LIB = os.path.join(_HERE, "libssn_oracle.so")
_LIB_OMP = os.path.join(_HERE, "libssn_oracle_omp.so")      # the same source with -fopenmp (row loops on all cores)
CFLAGS = ["-O2", "-std=c99", "-fPIC", "-shared"]

_c_double_p = ctypes.POINTER(ctypes.c_double)
_c_int32_p = ctypes.POINTER(ctypes.c_int32)
_c_int64_p = ctypes.POINTER(ctypes.c_int64)


class _Problem(ctypes.Structure):
    _fields_ = [
        ("n", ctypes.c_int64), ("p", ctypes.c_int64),
        ("C", ctypes.c_int32), ("scale_sum", ctypes.c_int32),
        ("lam", ctypes.c_double),
        ("X", ctypes.c_void_p), ("ldx", ctypes.c_int64),
        ("rowptr", ctypes.c_void_p), ("colidx", ctypes.c_void_p), ("vals", ctypes.c_void_p),
        ("labels", ctypes.c_void_p),
    ]


def build(force=False):
    """Compile the oracle with gcc -O2 (no fast-math) into oracle/libssn_oracle.so, and once more with -fopenmp
    into oracle/libssn_oracle_omp.so."""
    for lib, extra in ((_LIB, []), (_LIB_OMP, ["-fopenmp"])):
        if force or not os.path.exists(lib) or os.path.getmtime(lib) < os.path.getmtime(_SRC):
            subprocess.check_call(["gcc"] + CFLAGS + extra + ["-o", lib, _SRC, "-lm"])
    # the sanitizer driver, here without sanitizers (tests/test_oracle_sanitizers.py builds it with them)
    drv = os.path.join(_HERE, "sanitize_check.c")
    exe = os.path.join(_HERE, "sanitize_check")
    if force or not os.path.exists(exe) or os.path.getmtime(exe) < max(os.path.getmtime(_SRC), os.path.getmtime(drv)):
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-o", exe, _SRC, drv, "-lm"])
    return _LIB


_libs = {}


def _load(threads=False):
    """threads=False: the plain single-thread build; True: the OpenMP build of the same source."""
    if threads not in _libs:
        build()
        lib = ctypes.CDLL(_LIB_OMP if threads else _LIB)
        lib.orc_objective.restype = ctypes.c_double
        lib.orc_accuracy.restype = ctypes.c_double
        lib.orc_cg.restype = ctypes.c_int
        lib.orc_linesearch.restype = ctypes.c_int
        lib.orc_ssn.restype = ctypes.c_int
        lib.orc_ssn_sg.restype = ctypes.c_int
        lib.orc_threads.restype = ctypes.c_int
        _libs[threads] = lib
    return _libs[threads]


def threads_of(threads):
    """Threads the row loops of that build use (1 for the plain build)."""
    return int(_load(threads).orc_threads())


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _ptr(a):
    return a.ctypes.data_as(ctypes.c_void_p)


class Problem:
    """Holds the data of one logistic-regression problem for the oracle."""

    def __init__(self, labels, C, lam, X=None, csr=None, p=None, scale="mean", threads=False):
        self.threads = bool(threads)
        self.labels = np.ascontiguousarray(labels, dtype=np.int32)
        self.n = int(self.labels.shape[0])
        self.C = int(C)
        self.K = self.C - 1
        self.lam = float(lam)
        self.scale = scale
        st = _Problem()
        st.n, st.C, st.lam = self.n, self.C, self.lam
        st.scale_sum = {"mean": 0, "sum": 1}[scale]
        if X is not None:
            self.X = _f64(X)
            assert self.X.shape[0] == self.n
            self.p = int(self.X.shape[1])
            st.X, st.ldx = _ptr(self.X), self.p
        else:
            rowptr, colidx, vals = csr
            self.rowptr = np.ascontiguousarray(rowptr, dtype=np.int64)
            self.colidx = np.ascontiguousarray(colidx, dtype=np.int32)
            self.vals = _f64(vals)
            self.p = int(p)
            st.X, st.ldx = None, 0
            st.rowptr, st.colidx, st.vals = _ptr(self.rowptr), _ptr(self.colidx), _ptr(self.vals)
        st.p = self.p
        st.labels = _ptr(self.labels)
        self._st = st
        self.d = self.p * self.K

    def _ref(self):
        return ctypes.byref(self._st)

    def _w(self, W):
        W = _f64(W)
        assert W.shape == (self.p, self.K), (W.shape, (self.p, self.K))
        return W

    # ---- eq. (5), Alg. 5 -------------------------------------------------
    def objective(self, W):
        W = self._w(W)
        return float(_load(self.threads).orc_objective(self._ref(), _ptr(W)))

    def row_parts(self, W):
        """maxPart, sumExpPart, linearPart, logPart of Alg. 5 (eqs. 14-17), one value per row."""
        W = self._w(W)
        out = [np.empty(self.n) for _ in range(4)]
        _load(self.threads).orc_row_parts(self._ref(), _ptr(W), *[_ptr(o) for o in out])
        return tuple(out)

    # ---- eq. (6), Alg. 6 -------------------------------------------------
    def gradient(self, W):
        W = self._w(W)
        G = np.empty_like(W)
        f = ctypes.c_double()
        _load(self.threads).orc_gradient(self._ref(), _ptr(W), _ptr(G), ctypes.byref(f))
        return G, f.value

    # ---- eq. (2a): sub-sampled gradient ----------------------------------
    def gradient_sampled(self, W, S):
        """Returns (G, f_S): gradient and objective of the sample S (a multiset of rows)."""
        W = self._w(W)
        S = np.ascontiguousarray(S, dtype=np.int32)
        assert S.size > 0 and S.min() >= 0 and S.max() < self.n
        G = np.empty_like(W)
        f = ctypes.c_double()
        _load(self.threads).orc_gradient_sampled(self._ref(), _ptr(W), _ptr(S), ctypes.c_int64(S.shape[0]), _ptr(G), ctypes.byref(f))
        return G, f.value

    # ---- eqs. (10)-(13), Alg. 7/8 ---------------------------------------
    def sample_probs(self, W, S):
        W = self._w(W)
        S = np.ascontiguousarray(S, dtype=np.int32)
        P = np.empty((S.shape[0], self.K))
        _load(self.threads).orc_sample_probs(self._ref(), _ptr(W), _ptr(S), ctypes.c_int64(S.shape[0]), _ptr(P))
        return P

    def hessvec(self, W, S, V):
        W, V = self._w(W), self._w(V)
        S = np.ascontiguousarray(S, dtype=np.int32)
        assert S.size > 0 and S.min() >= 0 and S.max() < self.n
        HV = np.empty_like(W)
        _load(self.threads).orc_hessvec(self._ref(), _ptr(W), _ptr(S), ctypes.c_int64(S.shape[0]), _ptr(V), _ptr(HV))
        return HV

    # ---- classification rule --------------------------------------------
    def predict(self, W):
        W = self._w(W)
        pred = np.empty(self.n, dtype=np.int32)
        _load(self.threads).orc_predict(self._ref(), _ptr(W), _ptr(pred))
        return pred

    def accuracy(self, W):
        W = self._w(W)
        return float(_load(self.threads).orc_accuracy(self._ref(), _ptr(W)))

    # ---- Alg. 2 ------------------------------------------------------------
    def cg(self, W, S, g, theta, T):
        """Returns dict(p, iters, rel_res, flags, alpha[k], rnorm[k], sHs[k])."""
        W, g = self._w(W), self._w(g)
        S = np.ascontiguousarray(S, dtype=np.int32)
        p_best = np.empty_like(W)
        rel = ctypes.c_double()
        flags = ctypes.c_int32()
        trace = np.zeros((max(T, 1), 3))
        it = _load(self.threads).orc_cg(self._ref(), _ptr(W), _ptr(S), ctypes.c_int64(S.shape[0]), _ptr(g),
                            ctypes.c_double(theta), ctypes.c_int(T), _ptr(p_best),
                            ctypes.byref(rel), ctypes.byref(flags), _ptr(trace))
        return dict(p=p_best, iters=int(it), rel_res=rel.value, flags=flags.value,
                    alpha=trace[:it, 0].copy(), rnorm=trace[:it, 1].copy(), sHs=trace[:it, 2].copy())

    # ---- Alg. 3 ------------------------------------------------------------
    def linesearch(self, W, P, g, fW, beta=1e-4, rho=0.5, imax=10):
        W, P, g = self._w(W), self._w(P), self._w(g)
        alpha, fnew = ctypes.c_double(), ctypes.c_double()
        ok = ctypes.c_int32()
        ev = _load(self.threads).orc_linesearch(self._ref(), _ptr(W), _ptr(P), _ptr(g), ctypes.c_double(fW),
                                    ctypes.c_double(beta), ctypes.c_double(rho), ctypes.c_int(imax),
                                    ctypes.byref(alpha), ctypes.byref(fnew), ctypes.byref(ok))
        return dict(alpha=alpha.value, f_new=fnew.value, n_eval=int(ev), ok=int(ok.value))

    # ---- Alg. 1 ------------------------------------------------------------
    def ssn(self, W0, S_all, eps=0.0, theta=1e-4, T=10, beta=1e-4, rho=0.5, imax=10):
        """S_all: (iters, nS) int32.  Returns (W_final, log[iters, 6], iterations done)."""
        W = self._w(W0).copy()
        S_all = np.ascontiguousarray(S_all, dtype=np.int32)
        iters, nS = S_all.shape
        log = np.zeros((iters, 6))
        done = _load(self.threads).orc_ssn(self._ref(), _ptr(W), ctypes.c_int(iters), _ptr(S_all), ctypes.c_int64(nS),
                               ctypes.c_double(eps), ctypes.c_double(theta), ctypes.c_int(T),
                               ctypes.c_double(beta), ctypes.c_double(rho), ctypes.c_int(imax), _ptr(log))
        return W, log, int(done)

    def ssn_sg(self, W0, Sg_all, S_all, eps=0.0, theta=1e-4, T=10, beta=1e-4, rho=0.5, imax=10):
        """Alg. 1 with sub-sampled gradient (Sg_all: (iters, nSg)) and Hessian (S_all: (iters, nS))."""
        W = self._w(W0).copy()
        Sg_all = np.ascontiguousarray(Sg_all, dtype=np.int32)
        S_all = np.ascontiguousarray(S_all, dtype=np.int32)
        iters, nS = S_all.shape
        assert Sg_all.shape[0] == iters
        log = np.zeros((iters, 6))
        done = _load(self.threads).orc_ssn_sg(self._ref(), _ptr(W), ctypes.c_int(iters), _ptr(Sg_all), ctypes.c_int64(Sg_all.shape[1]),
                                  _ptr(S_all), ctypes.c_int64(nS), ctypes.c_double(eps), ctypes.c_double(theta),
                                  ctypes.c_int(T), ctypes.c_double(beta), ctypes.c_double(rho), ctypes.c_int(imax),
                                  _ptr(log))
        return W, log, int(done)


def normalize_columns(X=None, csr=None, p=None):
    """Sec. 4 preprocessing on a copy: returns (scaled X or scaled CSR values, column norms before scaling)."""
    lib = _load()
    if X is not None:
        Xc = _f64(X).copy()
        n, p = Xc.shape
        norms = np.empty(p)
        lib.orc_normalize_columns(ctypes.c_int64(n), ctypes.c_int64(p), _ptr(Xc), ctypes.c_int64(p), None, None, None,
                                  _ptr(norms))
        return Xc, norms
    rowptr, colidx, vals = csr
    rowptr = np.ascontiguousarray(rowptr, dtype=np.int64)
    colidx = np.ascontiguousarray(colidx, dtype=np.int32)
    vc = _f64(vals).copy()
    norms = np.empty(int(p))
    lib.orc_normalize_columns(ctypes.c_int64(rowptr.shape[0] - 1), ctypes.c_int64(int(p)), None, ctypes.c_int64(0),
                              _ptr(rowptr), _ptr(colidx), _ptr(vc), _ptr(norms))
    return vc, norms
