"""GPU parity of the unit-column-norm preprocessing of Sec. 4 against the CPU oracle."""
import numpy as np
import pytest
import torch

from oracle import oracle
from paper_1802_09113_amd import binding, synth

pytestmark = pytest.mark.gpu
F64, F32 = torch.float64, torch.float32
TOL = {F64: 1e-12, F32: 1e-5}


@pytest.mark.parametrize("dtype", [F64, F32], ids=["f64", "f32"])
def test_dense_columns(dtype):
    g = np.random.default_rng(8)
    n, p, ldx = 3001, 301, 304                                    # several row chunks, a ragged column tile, padded rows
    X = g.standard_normal((n, p)) * g.uniform(0.01, 50.0, size=p)
    X[:, 17] = 0.0
    Xr = X.astype(np.float32 if dtype == F32 else np.float64)
    buf = torch.full((n, ldx), float("nan"), dtype=dtype, device="cuda")
    buf[:, :p] = torch.from_numpy(Xr).cuda()
    Xd = buf[:, :p]
    print(f"[case] normalize dense dtype={dtype}", flush=True)
    norms = binding.ssn_normalize_columns(X=Xd)
    torch.cuda.synchronize()
    X_ref, n_ref = oracle.normalize_columns(X=Xr.astype(np.float64))
    np.testing.assert_allclose(norms.cpu().numpy(), n_ref, rtol=TOL[dtype])
    got = Xd.cpu().numpy().astype(np.float64)
    assert np.linalg.norm(got - X_ref) <= TOL[dtype] * np.linalg.norm(X_ref)
    assert np.all(got[:, 17] == 0.0) and norms[17].item() == 0.0
    assert torch.isnan(buf[:, p:]).all()                          # the padding is not touched


@pytest.mark.parametrize("dtype", [F64, F32], ids=["f64", "f32"])
def test_csr_columns_and_determinism(dtype):
    d = synth.make(4, n=403)
    nd = np.float32 if dtype == F32 else np.float64
    vals = d["vals"].astype(nd)
    rp = torch.from_numpy(d["rowptr"].astype(np.int32)).cuda()
    ci = torch.from_numpy(d["colidx"]).cuda()
    print(f"[case] normalize csr dtype={dtype} nnz={vals.size}", flush=True)
    runs = []
    for _ in range(2):
        vd = torch.from_numpy(vals).cuda()
        norms = binding.ssn_normalize_columns(csr=(rp, ci, vd), p=d["p"])
        torch.cuda.synchronize()
        runs.append((vd.clone(), norms.clone()))
    assert torch.equal(runs[0][0], runs[1][0]) and torch.equal(runs[0][1], runs[1][1])
    v_ref, n_ref = oracle.normalize_columns(csr=(d["rowptr"], d["colidx"], vals.astype(np.float64)), p=d["p"])
    np.testing.assert_allclose(runs[0][1].cpu().numpy(), n_ref, rtol=TOL[dtype], atol=0.0)
    got = runs[0][0].cpu().numpy().astype(np.float64)
    assert np.linalg.norm(got - v_ref) <= TOL[dtype] * np.linalg.norm(v_ref)


def test_bad_arguments():
    X = torch.zeros((4, 3), dtype=F64, device="cuda")
    nrm = torch.zeros(3, dtype=F64, device="cuda")
    L = binding.lib()
    assert L.ssn_normalize_columns(0, 1, 4, 3, None, 3, None, None, None, 0, binding._ptr(nrm), None) == binding.SSN_E_INVALID_ARG
    assert L.ssn_normalize_columns(0, 1, 4, 3, binding._ptr(X), 2, None, None, None, 0, binding._ptr(nrm), None) == binding.SSN_E_INVALID_ARG
    assert L.ssn_normalize_columns(0, 7, 4, 3, binding._ptr(X), 3, None, None, None, 0, binding._ptr(nrm), None) == binding.SSN_E_INVALID_ARG
    assert L.ssn_normalize_columns(1, 1, 4, 3, None, 0, None, None, None, 0, binding._ptr(nrm), None) == binding.SSN_E_INVALID_ARG
