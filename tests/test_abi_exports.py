"""The C-ABI library loads on a machine without a GPU and exports every symbol include/*.h declares."""
import ctypes
import os
import re

from paper_1802_09113_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols(header=None):
    names = ["ssn.h", "ssn_bench.h"] if header is None else [header]
    out = set()
    for name in names:
        text = open(os.path.join(ROOT, "include", name)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        out |= set(re.findall(r"\b(ssn_[a-z_0-9]+)\s*\(", text))
    return sorted(out)


def test_header_and_binding_agree():
    assert declared_symbols("ssn.h") == sorted(binding.EXPORTS)
    assert declared_symbols("ssn_bench.h") == sorted(binding.BENCH_EXPORTS)
    assert sorted(os.listdir(os.path.join(ROOT, "include"))) == ["ssn.h", "ssn_bench.h"]


def test_library_exports_every_declared_symbol():
    assert os.path.exists(binding.LIB_PATH), "build first: python -m paper_1802_09113_amd.build"
    L = ctypes.CDLL(binding.LIB_PATH)
    for name in declared_symbols():
        assert hasattr(L, name), name


def test_status_strings_and_null_arguments_without_a_gpu():
    L = binding.lib()
    assert L.ssn_strerror(0) == b"ok"
    for code in range(-9, 0):
        assert L.ssn_strerror(code) not in (b"ok", b"unknown status")
    assert L.ssn_strerror(-99) == b"unknown status"
    # argument checks come before any device work
    assert L.ssn_create(None, None) == binding.SSN_E_INVALID_ARG
    h = ctypes.c_void_p()
    d = binding.ssn_desc()
    assert L.ssn_create(ctypes.byref(h), ctypes.byref(d)) == binding.SSN_E_INVALID_ARG
    assert L.ssn_destroy(None) == binding.SSN_E_INVALID_ARG
    assert L.ssn_objective(None, None, None) == binding.SSN_E_INVALID_ARG
    assert L.ssn_objective_dev(None, None, None) == binding.SSN_E_INVALID_ARG
    assert L.ssn_accuracy(None, None, None, None) == binding.SSN_E_INVALID_ARG
    assert L.ssn_vec_to_rowmajor(None, None, None) == binding.SSN_E_INVALID_ARG
    # the entry point without allocations checks its description before it touches the device
    assert L.ssn_hessvec_static(None, None, None, 0, None, None) == binding.SSN_E_INVALID_ARG
    d.n, d.p, d.C, d.layout, d.ldw = 10, 4, 3, binding.SSN_CSR, 2
    one = ctypes.c_void_p(16)
    assert L.ssn_hessvec_static(ctypes.byref(d), one, one, 1, one, ctypes.c_void_p(32)) == binding.SSN_E_UNSUPPORTED
