"""CPU-side checks of the C ABI: the library loads, exports every symbol the header declares,
and its host-only entry points (sizes, budget, payload layout, status text) agree with the
oracle's formulas.  No GPU needed."""
import os
import re

import numpy as np
import pytest

from oracle import pipeline, solver
from paper_2210_17357_amd import binding as B
from paper_2210_17357_amd import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(B.LIB_PATH):
        from paper_2210_17357_amd import build
        build.build()
    return B.lib()


def test_exports_match_header(lib):
    header = open(os.path.join(ROOT, "include", "lgreco.h")).read()
    declared = set(re.findall(r"\b(lgreco_[a-z_]+)\s*\(", header))
    assert declared == set(B.EXPORTS)
    for name in declared:
        assert getattr(lib, name) is not None


def test_struct_layouts_match_header(tmp_path):
    """Size and field offsets of the binding's structures against what a C compiler makes of the
    header (no numbers typed in here)."""
    import ctypes as C
    import subprocess
    structs = {"lgreco_layer_t": B.Layer, "lgreco_cand_t": B.Cand, "lgreco_config_t": B.Config}
    lines = ['#include <stdio.h>', '#include <stddef.h>', '#include "lgreco.h"', 'int main(void) {']
    for cname, cls in structs.items():
        lines.append('printf("%s %%zu\\n", sizeof(%s));' % (cname, cname))
        for field, _ in cls._fields_:
            lines.append('printf("%s.%s %%zu\\n", offsetof(%s, %s));' % (cname, field, cname, field))
    lines += ['return 0;', '}']
    src = tmp_path / "layout.c"
    src.write_text("\n".join(lines))
    exe = tmp_path / "layout"
    include = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include")
    subprocess.run(["gcc", "-I", include, str(src), "-o", str(exe)], check=True)
    out = dict(line.split() for line in subprocess.run([str(exe)], check=True, capture_output=True,
                                                       text=True).stdout.splitlines())
    for cname, cls in structs.items():
        assert int(out[cname]) == C.sizeof(cls), cname
        for field, _ in cls._fields_:
            assert int(out["%s.%s" % (cname, field)]) == getattr(cls, field).offset, (cname, field)


@pytest.mark.parametrize("name", W.WORKLOADS)
def test_sizes_match_oracle_formulas(lib, name):
    w = W.workload(name)
    total, offs, numels, rows, cols, tix, raw = W.layout(w)
    layers = B.layer_table(offs, numels, rows, cols)
    ctab = B.cand_table(list(w.candidates))
    got = B.sizes(layers, ctab, w.bucket)
    assert np.array_equal(got, pipeline.sizes_table(numels, rows, cols, list(w.candidates), w.bucket))


def test_emax_and_layout_and_errors(lib):
    errors = np.random.default_rng(0).random((9, 4))
    assert B.emax(errors, 2) == solver.e_max_uniform(errors, 2)
    layers = B.layer_table([0, 1000, 5000], [1000, 4000, 130], [0, 40, 0], [0, 100, 0])
    cands = B.cand_table([(B.QUANT, 3), (B.TOPK, 0.01), (B.LOWRANK, 4)])
    off = B.payload_layout(layers, cands, np.array([0, 2, 1], np.int32))
    s = B.sizes(B.layer_table([0, 1000, 5000], [1000, 4000, 130], [0, 40, 0], [0, 100, 0]),
                B.cand_table([(B.QUANT, 3), (B.TOPK, 0.01)]))
    assert off[0] == 0 and off[1] == (s[0, 0] + 15) // 16 * 16
    assert off[2] == off[1] + (4 * 140 * 4 + 15) // 16 * 16 and off[3] == off[2] + 16
    with pytest.raises(B.LgrecoError):         # low rank on a tensor without a matrix view
        B.payload_layout(layers, cands, np.array([2, 2, 1], np.int32))
    with pytest.raises(B.LgrecoError):         # choice out of range
        B.payload_layout(layers, cands, np.array([0, 3, 1], np.int32))
    for bad in ([(B.QUANT, 0)], [(B.QUANT, 9)], [(B.QUANT, 2.5)], [(B.TOPK, 0.0)], [(B.TOPK, 1.5)], [(7, 1.0)]):
        with pytest.raises(B.LgrecoError):
            B.sizes(layers, B.cand_table(bad))
    with pytest.raises(B.LgrecoError):
        B.emax(errors, 4)
    assert "budget" in B.strerror(B.EINFEASIBLE) and B.strerror(0) == "ok"


def test_product_package_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2210_17357_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert not re.search(r"^\s*(from|import)\s+oracle\b", text, re.M), f
                assert "oracle/" not in text and "oracle." not in text, f
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith(".py"):
            assert "paper_2210_17357_amd" not in open(os.path.join(ROOT, "oracle", f)).read(), f


def test_candidate_range_rule(lib):
    """Section "Experimental setup", "Parameter ranges": [D/2, 2D] step 1 for bits and ranks,
    [D/10, 10D] step D/10 for densities; the default is inside with room on both sides."""
    cands, d = B.candidate_range(W.QUANT, 4)
    assert [p for _, p in cands] == [2, 3, 4, 5, 6, 7, 8] and cands[d][1] == 4
    assert tuple(cands) == W.workload("c1_resnet18_quant").candidates          # the configs' bit range
    cands, d = B.candidate_range(W.LOWRANK, 32, r_max=64)
    assert [p for _, p in cands] == list(range(16, 65)) and cands[d][1] == 32 and len(cands) == 49
    cands, d = B.candidate_range(W.LOWRANK, 4)
    assert [p for _, p in cands] == [2, 3, 4, 5, 6, 7, 8] and cands[d][1] == 4
    cands, d = B.candidate_range(W.TOPK, 0.01)
    assert len(cands) == 100 and d == 9 and cands[d][1] == 0.01
    assert cands[0][1] == pytest.approx(0.001) and cands[-1][1] == pytest.approx(0.1)
    assert all(b[1] > a[1] for a, b in zip(cands, cands[1:]))
    cands, d = B.candidate_range(W.TOPK, 0.5)                                  # clipped at density 1
    assert cands[-1][1] == pytest.approx(1.0) and len(cands) == 20 and cands[d][1] == 0.5
    for bad in ((W.QUANT, 9), (W.QUANT, 2.5), (W.TOPK, 0.0), (W.TOPK, 1.5), (7, 1)):
        with pytest.raises(B.LgrecoError):
            B.candidate_range(*bad)
