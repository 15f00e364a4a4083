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


def test_single_wave_one_pass_kernels_fit_the_residency_their_grid_assumes():
    """The launcher gives a compute unit 12 single-wave workgroups of the margin-only modes (three per SIMD: at
    most 512 / 3 registers, allocated in eights) and 8 of the modes with a transposed product (two per SIMD)."""
    import re
    seen = 0
    for (_, name), res in _kernels().items():
        m = re.match(r"_ZN3ssn18dense_fused_kernelI[df]Li(\d+)ELi\d+ELi\d+ELi1ELb0EE", name)
        if not m:
            continue
        seen += 1
        margins_only = int(m.group(1)) in (0, 2, 4)          # objective, prepare, predict
        assert res["vgprs"] <= (168 if margins_only else 256), (name, res)
    assert seen >= 20
