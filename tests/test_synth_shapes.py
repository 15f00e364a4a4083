"""The synthetic workloads against the shapes the paper lists (Sec. 4, Table 1; fixture in tests/golden/)."""
import os

from paper_1802_09113_amd import synth

HERE = os.path.dirname(os.path.abspath(__file__))


def _table1():
    rows = {}
    with open(os.path.join(HERE, "golden", "table1_datasets.txt")) as fh:
        for line in fh:
            if line.startswith("#") or not line.strip():
                continue
            name, n, n_test, p, C, L = line.split()
            rows[name] = dict(n=int(n), n_test=int(n_test), p=int(p), C=int(C), L=float(L))
    return rows


def _cfg(name):
    return next(c for c in synth.CONFIGS if c["name"] == name)


def test_table1_fixture_is_complete():
    t = _table1()
    assert len(t) == 7
    assert sum(1 for r in t.values() if r["C"] == 2) == 2          # the two binary problems
    assert all(r["n"] > 0 and r["p"] > 0 and r["L"] > 0 for r in t.values())


def test_workload_shapes_follow_table1():
    t = _table1()
    wide = _cfg("wide")                                              # CIFAR-10's training set, as listed
    assert (wide["n"], wide["p"], wide["C"]) == (t["CIFAR-10"]["n"], t["CIFAR-10"]["p"], t["CIFAR-10"]["C"])
    tall = _cfg("tall_narrow")                                       # all of Covertype's rows (train + test)
    assert tall["n"] == t["Covertype"]["n"] + t["Covertype"]["n_test"]
    assert (tall["p"], tall["C"]) == (t["Covertype"]["p"], t["Covertype"]["C"])
    img = _cfg("image_like")                                         # MNIST's pixels (the table counts one more column)
    assert img["C"] == t["MNIST"]["C"] and img["p"] == t["MNIST"]["p"] - 1
    sp = _cfg("sparse_csr")                                          # a 20-class text problem with far more columns than rows
    assert sp["C"] == t["Newsgroups20"]["C"] and sp["layout"] == "csr" and sp["p"] > sp["n"]


def test_generated_arrays_have_the_configured_shapes():
    d = synth.make(0)
    assert d["X"].shape == (d["n"], d["p"]) and d["labels"].shape == (d["n"],)
    assert d["labels"].min() >= 0 and d["labels"].max() < d["C"] and d["K"] == d["C"] - 1
    s = synth.make(4, n=300)
    assert s["rowptr"].shape == (301,) and s["rowptr"][-1] == len(s["colidx"]) == len(s["vals"])
    assert s["colidx"].min() >= 0 and s["colidx"].max() < s["p"]
