"""The approximate max-active mode (the paper's histogram cut, Section 4.1) against the exact mode.
It is not the CPU checker's result where max-active binds, so it is checked by what must hold
between the two modes: identical results where max-active never binds (and then bit-exact
against the checker); where it binds, at least max_active and only slightly more tokens kept,
every state's cost no higher than in the exact mode while the two still start a frame from the
same tokens, a best path that is never worse, and the same bytes for every lane size and frame
form (the cut depends on integer counts only)."""
import numpy as np
import pytest

import oracle
import synth
from gpu_compare import compare_channel, sorted_tokens

pytestmark = pytest.mark.gpu
F32 = np.float32


def decode(B, torch, g, rows, beam, lbeam, alpha, **kw):
    dec = B.WfstDecoder(B.WfstGraph(g), beam, lbeam, alpha, num_channels=1, max_lanes=1, max_frames=len(rows), **kw)
    dec.init_channels([0])
    dec.advance([0], [torch.from_numpy(rows).cuda()])
    torch.cuda.synchronize()
    return dec


def test_identical_to_the_exact_mode_where_max_active_does_not_bind():
    import torch
    from paper_1910_10032_amd import binding as B
    c = synth.configs()[0]                              # ~500 tokens per frame, max_active 2000
    g = synth.make_graph(c.graph)
    rows = c.loglikes(0, 0, 120)
    dec = decode(B, torch, g, rows, c.beam, c.lattice_beam, c.max_active, lattice_capacity=1 << 20, approximate=True)
    od = oracle.OracleDecoder(oracle.OracleGraph(g), c.beam, c.lattice_beam, c.max_active)
    od.advance(rows)
    assert od.max_tokens_pre_prune <= c.max_active
    compare_channel(dec, 0, od, label="approximate, not binding")


def test_histogram_cut_against_the_exact_selection():
    import torch
    from paper_1910_10032_amd import binding as B
    c = synth.configs()[1]                              # ~26 000 tokens within the beam, 7000 kept
    g = synth.make_graph(c.graph)
    T = 40
    rows = c.loglikes(0, 0, T)
    caps = dict(token_capacity=1 << 16, lattice_capacity=1 << 22)
    exact = decode(B, torch, g, rows, c.beam, c.lattice_beam, c.max_active, **caps)
    runs = [decode(B, torch, g, rows, c.beam, c.lattice_beam, c.max_active, approximate=True, lane_threads=nt, frame_form=ff, **caps)
            for nt, ff in ((1024, 0), (512, 0), (256, 1))]
    approx = runs[0]
    assert exact.stats(0)["status"] == 0 and all(r.stats(0)["status"] == 0 for r in runs)
    binding = 0
    same_start = True                                   # both modes started this frame from the same tokens
    for f in range(T + 1):
        es, ec, ea = sorted_tokens(exact.tokens(0, f))
        as_, ac, aa = sorted_tokens(approx.tokens(0, f))
        for r in runs[1:]:                              # deterministic: every lane size and frame form gives the same bytes
            rs, rc, ra = sorted_tokens(r.tokens(0, f))
            assert np.array_equal(rs, as_) and np.array_equal(rc.view(np.uint32), ac.view(np.uint32)) and np.array_equal(ra, aa)
        if len(es) == c.max_active:                     # the limit was reached in the exact mode
            binding += 1
            assert c.max_active <= len(as_) <= c.max_active + c.max_active // 10, (f, len(as_))
        assert ac.min() <= ec.min()                     # the best token is never worse
        if same_start:
            # a superset of the exact frame: every exact token is there, at the same cost
            pos = np.searchsorted(as_, es)
            assert (pos < len(as_)).all() and np.array_equal(as_[pos], es), f
            assert np.array_equal(ac[pos].view(np.uint32), ec.view(np.uint32)), f
        same_start = same_start and len(as_) == len(es)
    assert binding >= T // 2
    assert approx.stats(0)["max_tokens"] > c.max_active == exact.stats(0)["max_tokens"]
    for use_final in (True, False):
        assert approx.best_path(0, use_final)["total_cost"] <= exact.best_path(0, use_final)["total_cost"]
    # the approximate lattice contains the exact mode's best path arcs' frames (it is a lattice of a wider search)
    assert approx.stats(0)["lattice_arcs"] >= exact.stats(0)["lattice_arcs"]
