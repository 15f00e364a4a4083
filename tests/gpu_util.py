"""Helpers of the GPU parity tests: build one workload for both sides (oracle on the host, HIP library on
the device) from the shared seeded generators, and the error measures used in the comparisons."""
import numpy as np
import torch

from oracle.oracle import Problem
from paper_1802_09113_amd import synth
from paper_1802_09113_amd.binding import Context

TOL = {torch.float64: 1e-10, torch.float32: 1e-4}      # relative, stated by the benchmark spec


def np_dtype(dt):
    return np.float64 if dt == torch.float64 else np.float32


def rel_err(a, b):
    """The larger of the norm-wise error ||a - b|| / ||b|| and the element-wise one max|a - b| / max|b|: a block
    passes a tolerance only if no single entry is off by more than that fraction of the largest entry."""
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    normwise = float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))
    elementwise = float(np.max(np.abs(a - b)) / max(np.max(np.abs(b)), 1e-300)) if a.size else 0.0
    return max(normwise, elementwise)


def rel_scalar(a, b):
    return abs(a - b) / max(abs(b), 1e-300)


class Pair:
    """One workload on both sides.  For fp32 the oracle reads the fp32-rounded data widened to fp64."""

    def __init__(self, data, dtype, scale="mean", ldw=None, ldx=None, lam=None, dev="cuda", xoff=0):
        self.dtype = dtype
        nd = np_dtype(dtype)
        self.C, self.K = data["C"], data["C"] - 1
        self.p, self.n = data["p"], data["n"]
        lam = data["lam"] if lam is None else lam
        labels = data["labels"]
        self.labels = labels
        self.dev = dev
        lab_d = torch.from_numpy(labels).to(dev)
        if data["layout"] == "dense":
            Xr = data["X"].astype(nd)
            self.oracle = Problem(labels, self.C, lam, X=Xr.astype(np.float64), scale=scale)
            if xoff:
                # rows packed tightly behind `xoff` elements of a flat allocation that ends with the last row: the
                # matrix starts at an address aligned to its element only
                flat = torch.full((xoff + self.n * self.p,), float("nan"), dtype=dtype, device=dev)
                Xd = flat[xoff:].view(self.n, self.p)
                Xd.copy_(torch.from_numpy(Xr).to(dev))
            elif ldx is None:
                Xd = torch.from_numpy(Xr).to(dev)
            else:
                buf = torch.full((self.n, ldx), float("nan"), dtype=dtype, device=dev)
                buf[:, : self.p] = torch.from_numpy(Xr).to(dev)
                Xd = buf[:, : self.p]
            self.gpu = Context(lab_d, self.C, lam, X=Xd, scale=scale, ldw=ldw)
        else:
            vals = data["vals"].astype(nd)
            self.oracle = Problem(labels, self.C, lam, csr=(data["rowptr"], data["colidx"], vals.astype(np.float64)),
                                  p=self.p, scale=scale)
            rp = torch.from_numpy(data["rowptr"].astype(np.int32)).to(dev)
            ci = torch.from_numpy(data["colidx"]).to(dev)
            vd = torch.from_numpy(vals).to(dev)
            self.gpu = Context(lab_d, self.C, lam, csr=(rp, ci, vd), p=self.p, scale=scale, ldw=ldw)
        self.ldw = self.gpu.ldw

    def block(self, host):
        """host p x K array -> (rounded host fp64 copy for the oracle, device p x ldw block)."""
        r = np.asarray(host).astype(np_dtype(self.dtype))
        t = torch.full((self.p, self.ldw), float("nan"), dtype=self.dtype, device=self.dev)
        t[:, : self.K] = torch.from_numpy(r).to(self.dev)
        return r.astype(np.float64), t

    def host(self, t):
        return t[:, : self.K].double().cpu().numpy()

    def idx(self, S):
        return torch.from_numpy(np.ascontiguousarray(S, dtype=np.int32)).to(self.dev)

    def close(self):
        self.gpu.close()


def workload(cfg, n, **kw):
    return synth.make(cfg, n=n, **kw)


def oracle_sensitivity(pair, data, W0h, S_all, T, rel_noise, theta=1e-4):
    """How far the oracle's SSN run moves when the data are perturbed by relative noise of size rel_noise (1e-14:
    what a different order of summation in fp64 amounts to; 1e-6: fp32 products): the running maximum of the
    relative deviation of the objective per iteration, and the relative deviation of the final iterate.  The
    Krylov process behind Alg. 2 can amplify such perturbations by many orders of magnitude, so an end-to-end
    comparison is only as sharp as this figure."""
    o = pair.oracle
    g = np.random.default_rng(5)
    if data["layout"] == "dense":
        base = Problem(data["labels"], o.C, o.lam, X=o.X, threads=True)
        pert = Problem(data["labels"], o.C, o.lam, X=o.X * (1.0 + rel_noise * g.standard_normal(o.X.shape)), threads=True)
    else:
        base = Problem(data["labels"], o.C, o.lam, csr=(o.rowptr, o.colidx, o.vals), p=o.p, threads=True)
        pert = Problem(data["labels"], o.C, o.lam, p=o.p, threads=True,
                       csr=(o.rowptr, o.colidx, o.vals * (1.0 + rel_noise * g.standard_normal(o.vals.shape))))
    Wa, la, _ = base.ssn(W0h, S_all, theta=theta, T=T)
    Wb, lb, _ = pert.ssn(W0h, S_all, theta=theta, T=T)
    f_dev = np.maximum.accumulate(np.abs(lb[:, 0] / la[:, 0] - 1.0))
    return f_dev, rel_err(Wb, Wa), np.array_equal(la[:, 4], lb[:, 4])
