"""GPU tests of the boundary's remaining calls: the device-scalar forms of objective and gradient, the accuracy
of held-out rows described by an ssn_desc, and the conversion between the paper's stacked d-vector and the
p x K blocks of this library (checked through the explicit Hessian of eq. (7a)/(7b) in the paper's ordering)."""
import numpy as np
import pytest
import torch

from paper_1802_09113_amd import binding, synth
from tests.gpu_util import TOL, Pair, rel_err, rel_scalar, workload
from tests.test_oracle_hessian import explicit_hessian

pytestmark = pytest.mark.gpu

F64, F32 = torch.float64, torch.float32


@pytest.mark.parametrize("dtype", [F64, F32], ids=["f64", "f32"])
@pytest.mark.parametrize("cfg,n", [(0, 2000), (1, 3001), (2, 1003), (4, 403)])
def test_objective_and_gradient_with_the_scalar_left_on_the_device(cfg, n, dtype):
    pair = Pair(workload(cfg, n), dtype)
    tol = TOL[dtype]
    Wh, Wd = pair.block(synth.probe(pair.p, pair.K, sub=1, scale=0.1))
    print(f"[case] device scalars cfg={cfg} dtype={dtype}", flush=True)
    f_ref = pair.oracle.objective(Wh)
    G_ref, _ = pair.oracle.gradient(Wh)
    fd = torch.full((2,), float("nan"), dtype=torch.float64, device="cuda")
    pair.gpu.ssn_objective_dev(Wd, fd[0:1])
    G = pair.gpu.new_block()
    pair.gpu.ssn_gradient_dev(Wd, G, fd[1:2])
    torch.cuda.synchronize()
    f_obj, f_grad = fd.cpu().tolist()
    assert rel_scalar(f_obj, f_ref) <= tol and rel_scalar(f_grad, f_ref) <= tol
    assert rel_err(pair.host(G), G_ref) <= tol
    # the same kernels as the host-scalar calls: the same bits
    assert f_obj == pair.gpu.ssn_objective(Wd)
    G2, f2 = pair.gpu.ssn_gradient(Wd)
    torch.cuda.synchronize()
    assert f_grad == f2 and torch.equal(G[:, : pair.K], G2[:, : pair.K])
    pair.close()


@pytest.mark.parametrize("dtype", [F64, F32], ids=["f64", "f32"])
@pytest.mark.parametrize("cfg,n", [(0, 2000), (3, 5003), (4, 403)])
def test_accuracy_of_held_out_rows(cfg, n, dtype):
    pair = Pair(workload(cfg, n), dtype)
    test = workload(cfg, n, part="test")
    tpair = Pair(test, dtype)
    Wh, Wd = pair.block(synth.probe(pair.p, pair.K, sub=4, scale=0.5))
    nd = np.float64 if dtype == F64 else np.float32
    lab = torch.from_numpy(test["labels"]).cuda()
    if test["layout"] == "dense":
        desc, keep = binding.make_desc(lab, test["C"], 0.0, X=torch.from_numpy(test["X"].astype(nd)).cuda())
    else:
        csr = (torch.from_numpy(test["rowptr"].astype(np.int32)).cuda(), torch.from_numpy(test["colidx"]).cuda(),
               torch.from_numpy(test["vals"].astype(nd)).cuda())
        desc, keep = binding.make_desc(lab, test["C"], 0.0, csr=csr, p=test["p"])
    print(f"[case] accuracy cfg={cfg} dtype={dtype} rows={test['n']}", flush=True)
    acc = pair.gpu.ssn_accuracy(desc, Wd)
    assert abs(acc - tpair.oracle.accuracy(Wh)) <= (0.0 if dtype == F64 else 1e-3)
    assert acc == tpair.gpu.ssn_predict(Wd, want_pred=False)[1]
    # a description the context cannot serve is refused, a bad label is reported as at ssn_create
    desc.C = test["C"] + 1
    with pytest.raises(binding.SsnError) as e:
        pair.gpu.ssn_accuracy(desc, Wd)
    assert e.value.status == binding.SSN_E_INVALID_ARG
    desc.C = test["C"]
    lab[3] = test["C"]
    with pytest.raises(binding.SsnError) as e:
        pair.gpu.ssn_accuracy(desc, Wd)
    assert e.value.status == binding.SSN_E_BAD_LABEL
    pair.close()
    tpair.close()


@pytest.mark.parametrize("ldw", [None, 8], ids=["packed", "padded_blocks"])
def test_stacked_vector_ordering_against_the_explicit_hessian(ldw):
    # x = [x_1; ...; x_K] (Sec. 3.3): with the Hessian of eq. (7a)/(7b) assembled in THAT ordering (block (c, b)
    # of size p x p), H vec(V) must equal the library's product converted from its p x K block to the stacked vector
    g = np.random.default_rng(77)
    n, p, C = 300, 7, 4
    K = C - 1
    X = g.standard_normal((n, p))
    labels = g.integers(0, C, size=n).astype(np.int32)
    d = dict(layout="dense", X=X, labels=labels, n=n, p=p, C=C, K=K, lam=1e-2)
    pair = Pair(d, F64, ldw=ldw)
    Wh, Wd = pair.block(0.5 * g.standard_normal((p, K)))
    S = np.sort(g.choice(n, 60, replace=False)).astype(np.int32)
    H = explicit_hessian(X, Wh, S, 1e-2, 1.0 / S.size)               # index (j, c) -> j*K + c
    perm = np.array([j * K + c for c in range(K) for j in range(p)])  # stacked index c*p + j -> block index
    H_stacked = H[np.ix_(perm, perm)]
    v = g.standard_normal(p * K)                                      # a direction in the paper's ordering
    vd = torch.from_numpy(v).cuda()
    Vd = pair.gpu.ssn_vec_to_rowmajor(vd)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(pair.host(Vd), v.reshape(K, p).T)
    HV = pair.gpu.ssn_hessvec(Wd, pair.idx(S), Vd)
    hv = pair.gpu.ssn_rowmajor_to_vec(HV)
    torch.cuda.synchronize()
    assert rel_err(hv.cpu().numpy(), H_stacked @ v) <= 1e-10
    # there and back again
    back = pair.gpu.ssn_rowmajor_to_vec(Vd)
    torch.cuda.synchronize()
    assert torch.equal(back, vd)
    pair.close()
