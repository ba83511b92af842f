"""The HBM traffic figures of the benchmark line are not typed in anywhere: bench.py reads them from
the rocprofv3 summaries under profiles/.  These tests hold the two together: the summaries parse,
every section they name is one bench.py prices, the sections that dominate each workload are
there, and the measured bytes of the profile passes (whose algorithmic bytes are known without a
GPU: one read of the gradient and the error feedback and one write of their sum into the error
feedback buffer, 12 bytes per element in the one call the summaries are taken on) are within the
range a streaming pass can have."""
import os
import re

import pytest

import bench
from paper_2210_17357_amd import workloads as W

PROFILES = os.path.join(os.path.dirname(os.path.abspath(bench.__file__)), "profiles")
DOMINANT = {
    "c1_resnet18_quant": ("profile/quant_profile", "compress/quant_compress"),
    "c2_resnet50_topk": ("profile/topk_collect",),
    "c3_transformer_lm_lowrank": ("compress/lowrank_ef",),
    "c4_gpt2_medium_mixed": ("profile/quant_profile_topk_collect", "compress/quant_compress"),
}


def _rows(workload):
    path = os.path.join(PROFILES, workload + "_kernels_hbm.md")
    assert os.path.exists(path), path
    rows = []
    for line in open(path):
        cells = [c.strip() for c in line.strip().strip("|").split("|")]
        if len(cells) == 9 and cells[0] not in ("kernel", "---"):
            rows.append(cells)
    return rows


@pytest.mark.parametrize("workload", sorted(DOMINANT))
def test_summary_parses_and_names_only_priced_sections(workload):
    rows = _rows(workload)
    assert len(rows) >= 5
    named = {r[-1] for r in rows if r[-1] != "-"}
    assert named <= set(bench.STREAMING_SECTIONS) | set(bench.CONTRACTION_SECTIONS), named
    traffic = bench.measured_traffic(workload)
    assert set(traffic) == named
    for sec in DOMINANT[workload]:
        assert sec in traffic and traffic[sec] > 0, sec
    # the parser's figure is the two MB columns of the row, nothing else
    for r in rows:
        if r[-1] != "-":
            assert traffic[r[-1]] == pytest.approx((float(r[6]) + float(r[7])) * 1e6, rel=1e-12)
            # calibrated columns against the raw counters of the same row (KiB; reads count double)
            assert float(r[6]) == pytest.approx(float(r[4]) * 2 * 1024 / 1e6, rel=1e-3, abs=0.06)
            assert float(r[7]) == pytest.approx(float(r[5]) * 1024 / 1e6, rel=1e-3, abs=0.06)


@pytest.mark.parametrize("workload", ["c1_resnet18_quant", "c2_resnet50_topk", "c4_gpt2_medium_mixed"])
def test_profile_pass_traffic_against_its_algorithmic_bytes(workload):
    w = W.workload(workload)
    n = sum(int(__import__("numpy").prod(s)) for s in w.shapes)
    traffic = bench.measured_traffic(workload)
    sec = next(s for s in DOMINANT[workload] if s.startswith("profile/"))
    # never below what must be read (written lines may still sit in the L2 when the dispatch ends,
    # which shows on the small workloads); a pass that re-reads more than a sixth of its input, or
    # writes that much on the side, has a problem worth a look before the number is quoted
    assert 0.995 * 8.0 * n <= traffic[sec] <= 1.17 * 12.0 * n, (sec, traffic[sec] / (12.0 * n))


def test_every_summary_states_its_commands():
    for name in os.listdir(PROFILES):
        text = open(os.path.join(PROFILES, name)).read()
        cmds = re.findall(r"^rocprofv3 .*$", text, flags=re.M)
        assert cmds, name
        for c in cmds:
            assert "-- python3 bench.py" in c, (name, c)
