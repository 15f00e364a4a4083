"""Thin ctypes binding of libssn_hip.so (C ABI in include/ssn.h).

Argument marshalling only: torch tensors supply device pointers and the current HIP stream, every
step of the method runs inside the library's kernels.  There is no fallback: if the library has not
been built (python -m paper_1802_09113_amd.build) importing this module's `lib()` raises.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libssn_hip.so")

SSN_F32, SSN_F64 = 0, 1
SSN_DENSE_ROWMAJOR, SSN_CSR = 0, 1
SSN_SCALE_MEAN, SSN_SCALE_SUM = 0, 1
SSN_OK = 0
SSN_SOLVE_NO_LOOKAHEAD = 1
SSN_SOLVE_NO_PHASE_TIMES = 2
SSN_SOLVE_NO_MARGIN_CACHE = 4
SSN_E_INVALID_ARG, SSN_E_BAD_LABEL, SSN_E_BAD_INDEX, SSN_E_NOT_PREPARED = -1, -2, -3, -4
SSN_E_ALLOC, SSN_E_HIP, SSN_E_NONFINITE, SSN_E_UNSUPPORTED, SSN_E_TOO_LARGE = -5, -6, -7, -8, -9
SSN_STATIC_WORKSPACE_BYTES = 48 << 20

EXPORTS = [
    "ssn_strerror", "ssn_last_error", "ssn_create", "ssn_destroy", "ssn_set_stream", "ssn_objective",
    "ssn_gradient", "ssn_gradient_sampled", "ssn_hess_prepare", "ssn_hess_apply", "ssn_hessvec", "ssn_cg", "ssn_linesearch",
    "ssn_predict", "ssn_solve", "ssn_axpy", "ssn_normalize_columns", "ssn_objective_dev", "ssn_gradient_dev",
    "ssn_accuracy", "ssn_vec_to_rowmajor", "ssn_rowmajor_to_vec", "ssn_hessvec_static",
]
BENCH_EXPORTS = ["ssn_time_kernel", "ssn_dense_path", "ssn_sampled_slices"]          # include/ssn_bench.h


class ssn_desc(ctypes.Structure):
    _fields_ = [
        ("n", ctypes.c_int64), ("p", ctypes.c_int64),
        ("C", ctypes.c_int32), ("dtype", ctypes.c_int32), ("layout", ctypes.c_int32), ("scale", ctypes.c_int32),
        ("lam", ctypes.c_double),
        ("X", ctypes.c_void_p), ("ldx", ctypes.c_int64),
        ("rowptr", ctypes.c_void_p), ("colidx", ctypes.c_void_p), ("vals", ctypes.c_void_p), ("nnz", ctypes.c_int64),
        ("labels", ctypes.c_void_p),
        ("ldw", ctypes.c_int64),
        ("stream", ctypes.c_void_p),
    ]


class ssn_cg_info(ctypes.Structure):
    _fields_ = [("iters", ctypes.c_int32), ("flags", ctypes.c_int32), ("rel_res", ctypes.c_double),
                ("gnorm", ctypes.c_double)]


class ssn_params(ctypes.Structure):
    _fields_ = [
        ("iters", ctypes.c_int32), ("T", ctypes.c_int32), ("imax", ctypes.c_int32), ("flags", ctypes.c_int32),
        ("nS", ctypes.c_int64),
        ("eps", ctypes.c_double), ("theta", ctypes.c_double), ("beta", ctypes.c_double), ("rho", ctypes.c_double),
        ("S_all", ctypes.c_void_p), ("test", ctypes.c_void_p),
        ("Sg_all", ctypes.c_void_p), ("nSg", ctypes.c_int64),
    ]


class ssn_iter_record(ctypes.Structure):
    _fields_ = [
        ("f", ctypes.c_double), ("gnorm", ctypes.c_double), ("cg_rel_res", ctypes.c_double), ("alpha", ctypes.c_double),
        ("test_acc", ctypes.c_double),
        ("ms_grad", ctypes.c_double), ("ms_prepare", ctypes.c_double), ("ms_cg", ctypes.c_double),
        ("ms_linesearch", ctypes.c_double), ("ms_update", ctypes.c_double),
        ("cg_iters", ctypes.c_int32), ("ls_evals", ctypes.c_int32), ("ls_ok", ctypes.c_int32), ("reserved", ctypes.c_int32),
    ]


_lib = None


def lib():
    """Load the HIP library; fails loudly when it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_1802_09113_amd.build`")
        L = ctypes.CDLL(LIB_PATH)
        L.ssn_strerror.restype = ctypes.c_char_p
        L.ssn_strerror.argtypes = [ctypes.c_int]
        L.ssn_last_error.restype = ctypes.c_char_p
        L.ssn_last_error.argtypes = [ctypes.c_void_p]
        vp, dp, ip = ctypes.c_void_p, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int32)
        L.ssn_create.argtypes = [ctypes.POINTER(vp), ctypes.POINTER(ssn_desc)]
        L.ssn_destroy.argtypes = [vp]
        L.ssn_set_stream.argtypes = [vp, vp]
        L.ssn_objective.argtypes = [vp, vp, dp]
        L.ssn_gradient.argtypes = [vp, vp, vp, dp]
        L.ssn_gradient_sampled.argtypes = [vp, vp, vp, ctypes.c_int64, vp, dp]
        L.ssn_hess_prepare.argtypes = [vp, vp, vp, ctypes.c_int64]
        L.ssn_hess_apply.argtypes = [vp, vp, vp]
        L.ssn_hessvec.argtypes = [vp, vp, vp, ctypes.c_int64, vp, vp]
        L.ssn_cg.argtypes = [vp, vp, ctypes.c_double, ctypes.c_int32, vp, ctypes.POINTER(ssn_cg_info), dp]
        L.ssn_linesearch.argtypes = [vp, vp, vp, vp, ctypes.c_double, ctypes.c_double, ctypes.c_double, ctypes.c_int32,
                                     dp, dp, ip, ip]
        L.ssn_predict.argtypes = [vp, vp, vp, dp]
        L.ssn_solve.argtypes = [vp, vp, ctypes.POINTER(ssn_params), ctypes.POINTER(ssn_iter_record), ctypes.c_int32, ip]
        L.ssn_axpy.argtypes = [vp, ctypes.c_double, vp, vp]
        L.ssn_time_kernel.argtypes = [vp, ctypes.c_int32, vp, ctypes.c_int32, dp]
        L.ssn_dense_path.argtypes = [vp]
        L.ssn_sampled_slices.argtypes = [vp]
        L.ssn_normalize_columns.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int64, ctypes.c_int64, vp, ctypes.c_int64,
                                            vp, vp, vp, ctypes.c_int64, vp, vp]
        L.ssn_objective_dev.argtypes = [vp, vp, vp]
        L.ssn_gradient_dev.argtypes = [vp, vp, vp, vp]
        L.ssn_accuracy.argtypes = [vp, ctypes.POINTER(ssn_desc), vp, dp]
        L.ssn_vec_to_rowmajor.argtypes = [vp, vp, vp]
        L.ssn_rowmajor_to_vec.argtypes = [vp, vp, vp]
        L.ssn_hessvec_static.argtypes = [ctypes.POINTER(ssn_desc), vp, vp, ctypes.c_int64, vp, vp]
        for name in EXPORTS + BENCH_EXPORTS:
            fn = getattr(L, name)
            if fn.restype is not ctypes.c_char_p:
                fn.restype = ctypes.c_int
        _lib = L
    return _lib


def ssn_normalize_columns(X=None, csr=None, p=None):
    """Unit-column-norm preprocessing of Sec. 4, in place on device tensors: X (n x p, row-major, float32 / float64)
    or csr = (rowptr int32, colidx int32, vals).  Returns the column norms before scaling (float64, device)."""
    if X is not None:
        assert X.is_cuda and X.dim() == 2 and X.stride(1) == 1
        n, p = X.shape
        norms = torch.empty(p, dtype=torch.float64, device=X.device)
        dt = 0 if X.dtype == torch.float32 else 1
        st = lib().ssn_normalize_columns(0, dt, n, p, _ptr(X), X.stride(0), None, None, None, 0, _ptr(norms), None)
    else:
        rowptr, colidx, vals = csr
        assert rowptr.is_cuda and rowptr.dtype == torch.int32 and colidx.dtype == torch.int32
        n = rowptr.shape[0] - 1
        norms = torch.empty(int(p), dtype=torch.float64, device=vals.device)
        dt = 0 if vals.dtype == torch.float32 else 1
        st = lib().ssn_normalize_columns(1, dt, n, int(p), None, 0, _ptr(rowptr), _ptr(colidx), _ptr(vals), vals.shape[0],
                                         _ptr(norms), None)
    if st != 0:
        raise SsnError(st, "ssn_normalize_columns")
    return norms


class SsnError(RuntimeError):
    def __init__(self, status, detail=""):
        self.status = status
        name = lib().ssn_strerror(status).decode()
        super().__init__(f"ssn status {status} ({name}) {detail}")


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr()) if t is not None else None


def make_desc(labels, C, lam, X=None, csr=None, p=None, scale="mean", ldw=None, stream=None):
    """An ssn_desc for device tensors (and the list of tensors it borrows, to be kept alive by the caller)."""
    assert labels.is_cuda and labels.dtype == torch.int32
    keep = [labels]
    d = ssn_desc()
    d.n, d.C, d.lam = labels.shape[0], C, lam
    d.scale = {"mean": SSN_SCALE_MEAN, "sum": SSN_SCALE_SUM}[scale]
    d.labels = labels.data_ptr()
    if X is not None:
        assert X.is_cuda and X.dim() == 2 and X.stride(1) == 1
        d.layout, d.X, d.ldx, d.p = SSN_DENSE_ROWMAJOR, X.data_ptr(), X.stride(0), X.shape[1]
        tdtype = X.dtype
        keep.append(X)
    else:
        rowptr, colidx, vals = csr
        assert rowptr.dtype == torch.int32 and colidx.dtype == torch.int32
        d.layout, d.p, d.nnz = SSN_CSR, p, vals.shape[0]
        d.rowptr, d.colidx, d.vals = rowptr.data_ptr(), colidx.data_ptr(), vals.data_ptr()
        tdtype = vals.dtype
        keep += [rowptr, colidx, vals]
    d.dtype = {torch.float32: SSN_F32, torch.float64: SSN_F64}[tdtype]
    d.ldw = int(ldw) if ldw is not None else int(C) - 1
    if stream is None:
        stream = torch.cuda.current_stream().cuda_stream
    d.stream = stream
    return d, keep


def ssn_hessvec_static(desc, W, S, V, HV):
    """The product of Context.ssn_hessvec without a context and without any allocation: desc from make_desc,
    W, V, HV p x ldw device blocks, S int32 device indices.  Returns the status (0 = ok)."""
    assert S.is_cuda and S.dtype == torch.int32 and S.is_contiguous()
    return lib().ssn_hessvec_static(ctypes.byref(desc), _ptr(W), _ptr(S), S.shape[0], _ptr(V), _ptr(HV))


class Context:
    """One data set resident on the GPU.  Methods carry the names of the C entry points."""

    def __init__(self, labels, C, lam, X=None, csr=None, p=None, scale="mean", ldw=None, stream=None):
        d, self._keep = make_desc(labels, C, lam, X=X, csr=csr, p=p, scale=scale, ldw=ldw, stream=stream)
        self.tdtype = X.dtype if X is not None else csr[2].dtype
        self.n, self.p, self.C, self.K = int(d.n), int(d.p), int(C), int(C) - 1
        self.ldw = int(d.ldw)
        self.device = labels.device
        self._h = ctypes.c_void_p()
        st = lib().ssn_create(ctypes.byref(self._h), ctypes.byref(d))
        if st != SSN_OK:
            self._h = None
            raise SsnError(st, "in ssn_create")

    def close(self):
        if getattr(self, "_h", None):
            lib().ssn_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, st):
        if st != SSN_OK:
            raise SsnError(st, lib().ssn_last_error(self._h).decode())

    def ssn_set_stream(self, stream):
        """stream: a hipStream_t handle as an integer (e.g. torch.cuda.Stream().cuda_stream), or None for the default."""
        self._check(lib().ssn_set_stream(self._h, ctypes.c_void_p(stream) if stream else None))

    def new_block(self):
        """An uninitialised p x ldw block of the context's dtype."""
        return torch.empty((self.p, self.ldw), dtype=self.tdtype, device=self.device)

    def _blk(self, t):
        assert t.is_cuda and t.dtype == self.tdtype and t.shape[0] == self.p and t.stride(0) == self.ldw and t.stride(1) == 1
        return _ptr(t)

    def ssn_objective(self, W):
        f = ctypes.c_double()
        self._check(lib().ssn_objective(self._h, self._blk(W), ctypes.byref(f)))
        return f.value

    def ssn_gradient(self, W, G=None, want_f=True):
        G = self.new_block() if G is None else G
        f = ctypes.c_double()
        self._check(lib().ssn_gradient(self._h, self._blk(W), self._blk(G), ctypes.byref(f) if want_f else None))
        return G, (f.value if want_f else None)

    def ssn_objective_dev(self, W, f_dev):
        """f_dev: a one-element float64 device tensor that receives f(W); nothing is read back."""
        assert f_dev.is_cuda and f_dev.dtype == torch.float64
        self._check(lib().ssn_objective_dev(self._h, self._blk(W), _ptr(f_dev)))

    def ssn_gradient_dev(self, W, G, f_dev):
        assert f_dev.is_cuda and f_dev.dtype == torch.float64
        self._check(lib().ssn_gradient_dev(self._h, self._blk(W), self._blk(G), _ptr(f_dev)))

    def ssn_accuracy(self, test_desc, W):
        acc = ctypes.c_double()
        self._check(lib().ssn_accuracy(self._h, ctypes.byref(test_desc), self._blk(W), ctypes.byref(acc)))
        return acc.value

    def ssn_vec_to_rowmajor(self, vec, block=None):
        assert vec.is_cuda and vec.dtype == self.tdtype and vec.is_contiguous() and vec.numel() == self.p * self.K
        block = self.new_block() if block is None else block
        self._check(lib().ssn_vec_to_rowmajor(self._h, _ptr(vec), self._blk(block)))
        return block

    def ssn_rowmajor_to_vec(self, block, vec=None):
        vec = torch.empty(self.p * self.K, dtype=self.tdtype, device=self.device) if vec is None else vec
        assert vec.is_cuda and vec.dtype == self.tdtype and vec.is_contiguous() and vec.numel() == self.p * self.K
        self._check(lib().ssn_rowmajor_to_vec(self._h, self._blk(block), _ptr(vec)))
        return vec

    def ssn_gradient_sampled(self, W, S, G=None, want_f=True):
        assert S.is_cuda and S.dtype == torch.int32 and S.is_contiguous()
        G = self.new_block() if G is None else G
        f = ctypes.c_double()
        self._check(lib().ssn_gradient_sampled(self._h, self._blk(W), _ptr(S), S.shape[0], self._blk(G),
                                               ctypes.byref(f) if want_f else None))
        return G, (f.value if want_f else None)

    def ssn_hess_prepare(self, W, S):
        assert S.is_cuda and S.dtype == torch.int32 and S.is_contiguous()
        self._S = S
        self._check(lib().ssn_hess_prepare(self._h, self._blk(W), _ptr(S), S.shape[0]))

    def ssn_hess_apply(self, V, HV=None):
        HV = self.new_block() if HV is None else HV
        self._check(lib().ssn_hess_apply(self._h, self._blk(V), self._blk(HV)))
        return HV

    def ssn_hessvec(self, W, S, V, HV=None):
        assert S.is_cuda and S.dtype == torch.int32 and S.is_contiguous()
        self._S = S
        HV = self.new_block() if HV is None else HV
        self._check(lib().ssn_hessvec(self._h, self._blk(W), _ptr(S), S.shape[0], self._blk(V), self._blk(HV)))
        return HV

    def ssn_cg(self, G, theta, T, P=None, want_trace=True):
        P = self.new_block() if P is None else P
        info = ssn_cg_info()
        tr = (ctypes.c_double * (3 * max(T, 1)))()
        self._check(lib().ssn_cg(self._h, self._blk(G), theta, T, self._blk(P), ctypes.byref(info),
                                 tr if want_trace else None))
        it = info.iters
        out = dict(p=P, iters=it, flags=info.flags, rel_res=info.rel_res, gnorm=info.gnorm)
        if want_trace:
            out.update(alpha=[tr[3 * k] for k in range(it)], rnorm=[tr[3 * k + 1] for k in range(it)],
                       sHs=[tr[3 * k + 2] for k in range(it)])
        return out

    def ssn_linesearch(self, W, P, G, fW, beta=1e-4, rho=0.5, imax=10):
        a, fn = ctypes.c_double(), ctypes.c_double()
        ne, ok = ctypes.c_int32(), ctypes.c_int32()
        self._check(lib().ssn_linesearch(self._h, self._blk(W), self._blk(P), self._blk(G), fW, beta, rho, imax,
                                         ctypes.byref(a), ctypes.byref(fn), ctypes.byref(ne), ctypes.byref(ok)))
        return dict(alpha=a.value, f_new=fn.value, n_eval=ne.value, ok=ok.value)

    def ssn_predict(self, W, want_pred=True):
        pred = torch.empty(self.n, dtype=torch.int32, device=self.device) if want_pred else None
        acc = ctypes.c_double()
        self._check(lib().ssn_predict(self._h, self._blk(W), _ptr(pred), ctypes.byref(acc)))
        return pred, acc.value

    def ssn_axpy(self, alpha, P, W):
        self._check(lib().ssn_axpy(self._h, alpha, self._blk(P), self._blk(W)))

    def ssn_dense_path(self):
        return lib().ssn_dense_path(self._h)

    def ssn_sampled_slices(self):
        return lib().ssn_sampled_slices(self._h)

    def ssn_time_kernel(self, which, M, reps):
        ms = ctypes.c_double()
        self._check(lib().ssn_time_kernel(self._h, which, self._blk(M), reps, ctypes.byref(ms)))
        return ms.value

    def ssn_solve(self, W, S_all, eps=0.0, theta=1e-4, T=10, beta=1e-4, rho=0.5, imax=10, test=None, Sg_all=None,
                  lookahead=True, phase_times=True, margin_cache=True):
        """S_all: (iters, nS) int32 device tensor; Sg_all (optional): (iters, nSg) gradient samples.  W is updated
        in place; returns (records, iterations done).  lookahead=False sets SSN_SOLVE_NO_LOOKAHEAD,
        phase_times=False SSN_SOLVE_NO_PHASE_TIMES."""
        assert S_all.is_cuda and S_all.dtype == torch.int32 and S_all.is_contiguous() and S_all.dim() == 2
        pr = ssn_params()
        if Sg_all is not None:
            assert Sg_all.is_cuda and Sg_all.dtype == torch.int32 and Sg_all.is_contiguous() and Sg_all.dim() == 2
            assert Sg_all.shape[0] == S_all.shape[0]
            pr.Sg_all, pr.nSg = Sg_all.data_ptr(), Sg_all.shape[1]
        pr.iters, pr.nS = S_all.shape
        pr.T, pr.imax, pr.eps, pr.theta, pr.beta, pr.rho = T, imax, eps, theta, beta, rho
        pr.S_all = S_all.data_ptr()
        pr.flags = ((0 if lookahead else SSN_SOLVE_NO_LOOKAHEAD) | (0 if phase_times else SSN_SOLVE_NO_PHASE_TIMES)
                    | (0 if margin_cache else SSN_SOLVE_NO_MARGIN_CACHE))
        pr.test = test._h if test is not None else None
        log = (ssn_iter_record * max(int(pr.iters), 1))()
        done = ctypes.c_int32()
        self._check(lib().ssn_solve(self._h, self._blk(W), ctypes.byref(pr), log, int(pr.iters), ctypes.byref(done)))
        fields = [f[0] for f in ssn_iter_record._fields_ if f[0] != "reserved"]
        nrec = min(done.value + 1, int(pr.iters))
        return [{k: getattr(log[i], k) for k in fields} for i in range(nrec)], done.value
