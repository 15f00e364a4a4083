"""The build's own report of what every kernel needs (paper_1802_09113_amd/kernel_resources.json, written by
build.py from the compiler's resource remarks): no kernel of this library may use scratch memory.  A kernel
that does pays ~14 us per launch on MI355X, more than a whole sampled Hessian-vector product, and a few
spilled registers or a struct kept on the stack are enough to make it one."""
import json
import os

import pytest

from paper_1802_09113_amd import build

pytestmark = pytest.mark.skipif(not os.path.exists(build.RESOURCES),
                                reason="kernel_resources.json is written by the build; not built here")


def _kernels():
    with open(build.RESOURCES) as fh:
        rep = json.load(fh)
    return {(src, name): res for src, kernels in rep.items() for name, res in kernels.items()}


def test_report_covers_the_hot_kernels():
    names = " ".join(name for _, name in _kernels())
    for must in ("dense_fused_kernel", "dense_rows_kernel", "dense_xtu_kernel", "finalize_cg_kernel", "csr_rows_kernel",
                 "csc_piece_kernel", "cg_step2_kernel"):
        assert must in names


def test_no_kernel_of_the_library_uses_scratch_memory():
    own = {k: v for k, v in _kernels().items() if "_ZN3ssn" in k[1]}       # hipCUB's sort kernels are not ours
    assert len(own) > 100
    offenders = {name: res["scratch"] for (_, name), res in own.items() if res.get("scratch", 0) != 0}
    assert not offenders, f"kernels using scratch memory (bytes per lane): {offenders}"
