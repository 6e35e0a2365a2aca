"""Checks of the closed forms the paper prints (Section 3.2.1) against its own worked
examples, stored in tests/golden/paper_footprints.txt."""
import os

from paper_1910_10032_amd.footprint import graph_decode_bytes, paper_fst_bytes, paper_state_bytes


def _golden():
    vals = {}
    with open(os.path.join(os.path.dirname(__file__), "golden", "paper_footprints.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                k, v = line.split()
                vals[k] = float(v)
    return vals


def test_state_footprint_worked_examples():
    g = _golden()
    edge = paper_state_bytes(int(g["state_edge_alpha"]), int(g["state_edge_channels"]), int(g["state_edge_lanes"]))
    assert edge == 6_081_024
    assert round(edge / 2**20, 1) == g["state_edge_printed_MB"]          # the paper's MB is 2^20 bytes
    dc = paper_state_bytes(int(g["state_dc_alpha"]), int(g["state_dc_channels"]), int(g["state_dc_lanes"]))
    assert round(dc / 2**30, 1) == g["state_dc_printed_GB"]


def test_headline_ratios_follow_from_table_2():
    g = _golden()
    assert round(g["aspire_other_gpu_this_work"] / g["aspire_other_cpu_lattice"], -1) == g["printed_speedup_vs_cpu"]
    assert int(g["libri_clean_gpu_this_work"] / g["libri_clean_prior_gpu"] // 10 * 10) == g["printed_speedup_vs_prior_gpu"]


def test_graph_bytes_relation_to_eq1():
    q, e, ee = 8_000_000, 23_000_000, 20_000_000
    assert paper_fst_bytes(q, e, ee) == 12 * q + 8 * e + 4 * ee
    assert graph_decode_bytes(q, e) - paper_fst_bytes(q, e, ee) == 4 * (e - ee)
