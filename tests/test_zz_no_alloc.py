"""The product entry point that allocates nothing (ssn_hessvec_static) against ssn_hessvec on a created context:
two calls in a row, the second on a smaller input, every call checked; sizes beyond its fixed workspace and
layouts it does not serve are refused with their status."""
import numpy as np
import pytest
import torch

from paper_1802_09113_amd import binding, synth
from tests.gpu_util import TOL, Pair, rel_err, workload

pytestmark = pytest.mark.gpu

F64, F32 = torch.float64, torch.float32


def _one_call(cfg, n, nS, dtype, sub):
    d = workload(cfg, n)
    pair = Pair(d, dtype)
    nd = np.float64 if dtype == F64 else np.float32
    X = torch.from_numpy(d["X"].astype(nd)).cuda()
    lab = torch.from_numpy(d["labels"]).cuda()
    desc, keep = binding.make_desc(lab, d["C"], d["lam"], X=X)
    Wh, Wd = pair.block(synth.probe(pair.p, pair.K, sub=sub, scale=0.1))
    Vh, Vd = pair.block(synth.probe(pair.p, pair.K, sub=sub + 1))
    S = synth.sample_rows(n, nS, it=sub)
    Sd = pair.idx(S)
    print(f"[case] static product cfg={cfg} n={n} nS={nS} dtype={dtype}", flush=True)
    HV = torch.full_like(Vd, float("nan"))
    st = binding.ssn_hessvec_static(desc, Wd, Sd, Vd, HV)
    assert st == binding.SSN_OK, st
    ref = pair.gpu.ssn_hessvec(Wd, Sd, Vd)
    torch.cuda.synchronize()
    assert rel_err(pair.host(HV), pair.host(ref)) <= TOL[dtype]
    assert rel_err(pair.host(HV), pair.oracle.hessvec(Wh, S, Vh)) <= TOL[dtype]
    pair.close()


@pytest.mark.parametrize("dtype", [F64, F32], ids=["f64", "f32"])
def test_two_calls_in_a_row_the_second_smaller(dtype):
    # the one-pass path (784 features), then a smaller problem on the same workspace, which still holds the
    # first call's partial sums and probabilities
    _one_call(1, 3001, 1500, dtype, sub=1)
    _one_call(1, 1003, 50, dtype, sub=3)
    # the two-kernel path (3072 features) and a narrow matrix, again larger then smaller
    _one_call(2, 1003, 400, dtype, sub=5)
    _one_call(3, 5003, 77, dtype, sub=7)


def test_refuses_what_it_cannot_serve():
    d = workload(2, 1003)
    X = torch.from_numpy(d["X"]).cuda()
    lab = torch.from_numpy(d["labels"]).cuda()
    desc, keep = binding.make_desc(lab, d["C"], d["lam"], X=X)
    K = d["C"] - 1
    W = torch.zeros((d["p"], K), dtype=F64, device="cuda")
    V = torch.ones_like(W)
    HV = torch.empty_like(W)
    # a multiset sample long enough for its probabilities and partial sums to outgrow the fixed workspace
    nS = binding.SSN_STATIC_WORKSPACE_BYTES // (16 * 8) + 16
    S = torch.zeros(nS, dtype=torch.int32, device="cuda")
    assert binding.ssn_hessvec_static(desc, W, S, V, HV) == binding.SSN_E_TOO_LARGE
    assert binding.ssn_hessvec_static(desc, W, S[:10], V, V) == binding.SSN_E_INVALID_ARG      # aliased output
    desc.layout = binding.SSN_CSR
    assert binding.ssn_hessvec_static(desc, W, S[:10], V, HV) == binding.SSN_E_UNSUPPORTED
    torch.cuda.synchronize()
