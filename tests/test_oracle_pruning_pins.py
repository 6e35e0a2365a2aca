"""Pins for the pruning rules of the CPU checker (oracle/): the beam filter of the emitting
step, the lattice-record filter (completeness, effective cutoff, lattice beam), the
tie-break of the best path's end state and the arc count when max-active binds.

Each expected value here comes from something other than the code under test: hand-written
token sets on tiny integer graphs, the unlimited-beam decode (itself pinned by brute force
over all paths), or a frame step written out in Python on top of the stand-alone closure
routine (pinned against a library shortest-path routine).

Rules pinned: candidates above best + beam are dropped and one exactly at it is kept
(Section 3.3, first paragraph; Fig. 1 "Set Beam"); the adaptive beam after max-active is the
cost of the last kept token (Fig. 1, Section 4.1); every arc into a kept token within the
effective cutoff and the lattice beam is recorded with its extra cost (Section 3.4).
"""
import numpy as np
import pytest

import oracle
from helpers import arc_sources, canonical_rank, graph_from_arcs, random_graph

F32 = np.float32
NO_ARC = 0xFFFFFFFF
INF = float("inf")
BIG_ALPHA = 2**31 - 1


def okey(x):
    b = int(np.array([x], F32).view(np.uint32)[0])
    return (~b & 0xFFFFFFFF) if (b & 0x80000000) else (b | 0x80000000)


def emitting_candidates(g, st, co, row):
    """[(x, arc)] for every emitting arc out of the tokens (st, co), x in fp32."""
    out = []
    for s, c in zip(st.tolist(), co):
        for a in range(g.row_offsets[s], g.row_offsets[s + 1]):
            if g.ilabel[a] != 0:
                out.append((F32(F32(F32(c) + g.weight[a]) - row[g.ilabel[a] - 1]), a))
    return out


# ---- (a) beam filter ---------------------------------------------------------------------

def test_beam_filter_hand_written_integer_case():
    """Start state 0, one frame.  Candidates 1, 3, 4, 5 with beam 3: best 1, cutoff 4, so the
    candidate exactly at 4 stays and the one at 5 goes; the epsilon arc out of the kept state 3
    (cost 4 + 0) stays at the cutoff, the one with weight 1 (cost 5) is dropped."""
    arcs = [(0, 1, 1, 0, 1.0), (0, 2, 1, 0, 3.0), (0, 3, 1, 0, 4.0), (0, 4, 1, 0, 5.0),
            (3, 5, 0, 0, 0.0), (3, 6, 0, 0, 1.0), (4, 7, 0, 0, 0.0)]
    g = graph_from_arcs(8, arcs, 1)
    ll = np.zeros((1, 1), F32)
    d = oracle.OracleDecoder(oracle.OracleGraph(g), 3.0, 10.0, BIG_ALPHA)
    d.advance(ll)
    st, co, ia = d.tokens(1)
    assert st.tolist() == [1, 2, 3, 5]
    assert co.tolist() == [1.0, 3.0, 4.0, 4.0]
    assert ia.tolist() == [0, 1, 2, 4]
    # one beam narrower: the candidate at 4 is now a step above the cutoff 3
    d = oracle.OracleDecoder(oracle.OracleGraph(g), 2.0, 10.0, BIG_ALPHA)
    d.advance(ll)
    st, co, _ = d.tokens(1)
    assert st.tolist() == [1, 2] and co.tolist() == [1.0, 3.0]


def _side_by_side_with_unlimited_beam(seed, integer):
    """Side by side with the unlimited-beam decode: while both start a frame from the same
    tokens, the finite-beam frame must hold exactly the unlimited frame's tokens whose cost is
    <= (minimum emitting candidate + beam), with the same costs and incoming arcs.  Returns the
    number of frames in which something was pruned and of tokens seen exactly at the cutoff."""
    rng = np.random.default_rng(900 + seed)
    g = random_graph(rng, num_states=40, n_emit_per_state=(2, 4), eps_prob=0.05, num_pdfs=6, wmax=4,
                     integer=integer)
    T = 10
    ll = (-rng.integers(0, 4, size=(T, 6)).astype(F32)) if integer else rng.normal(-3, 1.5, size=(T, 6)).astype(F32)
    beam = 3.0 if integer else 2.75
    og = oracle.OracleGraph(g)
    fin = oracle.OracleDecoder(og, beam, 50.0, BIG_ALPHA)
    unl = oracle.OracleDecoder(og, INF, 50.0, BIG_ALPHA)
    # frame 0: the start token at cost 0, cutoff 0 + beam for its closure
    fs, fc, fa = fin.tokens()
    us, uc, ua = unl.tokens()
    keep = uc <= F32(beam)
    assert np.array_equal(fs, us[keep]) and np.array_equal(fc, uc[keep]) and np.array_equal(fa, ua[keep])
    pruned_frames = int(not keep.all())
    at_cutoff = int((uc == F32(beam)).sum())
    for t in range(T):
        ps, pc, _ = fin.tokens()
        us, uc, _ = unl.tokens()
        if not (np.array_equal(ps, us) and np.array_equal(pc, uc)):
            break                                  # the two have diverged: nothing more to compare
        best = min(x for x, _ in emitting_candidates(g, ps, pc, ll[t]))
        cutoff = F32(best + F32(beam))
        fin.advance(ll[t:t + 1])
        unl.advance(ll[t:t + 1])
        fs, fc, fa = fin.tokens()
        us, uc, ua = unl.tokens()
        keep = uc <= cutoff
        assert np.array_equal(fs, us[keep]) and np.array_equal(fc, uc[keep]) and np.array_equal(fa, ua[keep])
        pruned_frames += int(not keep.all())
        at_cutoff += int((uc == cutoff).sum())
    return pruned_frames, at_cutoff


@pytest.mark.parametrize("integer", [False, True])
@pytest.mark.parametrize("seed", range(8))
def test_finite_beam_keeps_exactly_the_unlimited_tokens_within_best_plus_beam(seed, integer):
    pruned_frames, _ = _side_by_side_with_unlimited_beam(seed, integer)
    assert pruned_frames >= 1


def test_finite_beam_keeps_tokens_exactly_at_the_cutoff():
    # integer costs: over these seeds several tokens sit exactly at best + beam, and are kept
    assert sum(_side_by_side_with_unlimited_beam(seed, True)[1] for seed in range(8)) >= 3


# ---- one frame written out in Python on top of the stand-alone closure --------------------

def python_frame(g, og, prev, row, beam, alpha):
    """prev: (st, co) of the previous frame.  Returns (V, kept, cutoff, cutoff_eff): V and kept
    are dicts state -> cost before / after max-active."""
    cands = emitting_candidates(g, prev[0], prev[1], row)
    best = min(x for x, _ in cands)
    cutoff = F32(best + F32(beam))
    rank = canonical_rank(g)
    U = {}
    for x, a in cands:
        if x <= cutoff:
            d = int(g.nextstate[a])
            k = (okey(x), int(rank[a]))
            if d not in U or k < U[d][0]:
                U[d] = (k, x, a)
    us = np.array(sorted(U), np.int32)
    st, co, _ = og.closure(us, np.array([U[s][1] for s in us.tolist()], F32),
                           np.array([U[s][2] for s in us.tolist()], np.uint32), float(cutoff))
    V = dict(zip(st.tolist(), co))
    if len(V) <= alpha:
        return V, dict(V), cutoff, cutoff
    keys = np.array([okey(c) for c in co], np.uint64)
    order = np.lexsort((st, keys))[:alpha]
    kept = {int(st[i]): co[i] for i in order}
    return V, kept, cutoff, co[order[-1]]


def python_lattice_records(g, prev, row, kept, cutoff_eff, lbeam):
    """Every arc into a kept token within the effective cutoff and the lattice beam."""
    recs = {}
    src = arc_sources(g)
    for x, a in emitting_candidates(g, prev[0], prev[1], row):
        d = int(g.nextstate[a])
        if d in kept and x <= cutoff_eff and F32(x - kept[d]) <= lbeam:
            recs[a] = F32(x - kept[d])
    for a in np.nonzero(g.ilabel == 0)[0].tolist():
        s, d = int(src[a]), int(g.nextstate[a])
        if s in kept and d in kept:
            x = F32(kept[s] + g.weight[a])
            if x <= cutoff_eff and F32(x - kept[d]) <= lbeam:
                recs[a] = F32(x - kept[d])
    return recs


# ---- (b) lattice records: set equality, effective cutoff, lattice beam --------------------

@pytest.mark.parametrize("integer", [False, True])
@pytest.mark.parametrize("seed", range(6))
def test_lattice_records_are_exactly_the_qualifying_arcs(seed, integer):
    rng = np.random.default_rng(1000 + seed)
    g = random_graph(rng, num_states=45, n_emit_per_state=(3, 5), eps_prob=0.05, num_pdfs=6, wmax=4,
                     integer=integer)
    T = 10
    ll = (-rng.integers(0, 4, size=(T, 6)).astype(F32)) if integer else rng.normal(-3, 1.5, size=(T, 6)).astype(F32)
    beam, lbeam, alpha = (6.0, 2.0, 12) if integer else (6.5, 2.25, 12)
    og = oracle.OracleGraph(g)
    d = oracle.OracleDecoder(og, beam, lbeam, alpha)
    binding = discriminating = at_lbeam = 0
    for t in range(T):
        ps, pc, _ = d.tokens()
        V, kept, cutoff, cutoff_eff = python_frame(g, og, (ps, pc), ll[t], beam, alpha)
        d.advance(ll[t:t + 1])
        st, co, _ = d.tokens()
        assert st.tolist() == sorted(kept) and [kept[s] for s in st.tolist()] == co.tolist()
        assert d.last_cutoff == cutoff_eff
        want = python_lattice_records(g, (ps, pc), ll[t], kept, cutoff_eff, lbeam)
        fr, ar, ex = d.lattice(from_frame=t + 1)
        assert np.all(fr == t + 1)
        assert ar.tolist() == sorted(want)
        assert ex.tolist() == [want[a] for a in ar.tolist()]
        if len(V) > alpha:
            binding += 1
            assert cutoff_eff < cutoff or integer
            # with the plain cutoff in place of the effective one the set would be larger
            discriminating += int(len(python_lattice_records(g, (ps, pc), ll[t], kept, cutoff, lbeam)) > len(want))
        at_lbeam += int(sum(1 for e in want.values() if e == F32(lbeam)))
    assert binding >= 3 and discriminating >= 1
    if integer:
        assert at_lbeam >= 1                       # an extra cost exactly at the lattice beam was recorded


def test_lattice_filter_hand_written_integer_case():
    """Two frames of a tiny integer graph with max-active 2 and lattice beam 1.
    Frame 1 candidates: 0->1 (1), 0->2 (2), 0->3 (3), 0->1 again (2), 0->2 again (4); beam 5 keeps
    all; max-active 2 keeps states 1 (1) and 2 (2), the effective cutoff is 2.  Recorded: arc 0
    (extra 0), arc 3 (into state 1 at cost 2, extra 1 = the lattice beam), arc 1 (extra 0); arc 4
    (into state 2 at cost 4) is above the effective cutoff although within the beam."""
    arcs = [(0, 1, 1, 0, 1.0), (0, 2, 1, 0, 2.0), (0, 3, 1, 0, 3.0), (0, 1, 1, 0, 2.0), (0, 2, 1, 0, 4.0)]
    g = graph_from_arcs(4, arcs, 1)
    d = oracle.OracleDecoder(oracle.OracleGraph(g), 5.0, 1.0, 2)
    d.advance(np.zeros((1, 1), F32))
    st, co, ia = d.tokens(1)
    assert st.tolist() == [1, 2] and co.tolist() == [1.0, 2.0] and ia.tolist() == [0, 1]
    assert d.last_cutoff == 2.0
    fr, ar, ex = d.lattice(from_frame=1)
    assert ar.tolist() == [0, 1, 3] and ex.tolist() == [0.0, 0.0, 1.0]
    # lattice beam 2 and no max-active: arc 4 (extra 2) joins, and so does state 3's arc 2
    d = oracle.OracleDecoder(oracle.OracleGraph(g), 5.0, 2.0, BIG_ALPHA)
    d.advance(np.zeros((1, 1), F32))
    fr, ar, ex = d.lattice(from_frame=1)
    assert ar.tolist() == [0, 1, 2, 3, 4] and ex.tolist() == [0.0, 0.0, 0.0, 1.0, 2.0]


# ---- (c) best path: ties between end states go to the smaller state id --------------------

def test_best_path_tie_goes_to_the_smaller_state_id():
    # the arc into the larger state comes first, so "first found" and "smaller state" differ
    arcs = [(0, 2, 1, 7, 1.0), (0, 1, 1, 5, 1.0), (0, 3, 1, 9, 2.0)]
    g = graph_from_arcs(4, arcs, 1)
    ll = np.zeros((1, 1), F32)
    bp = oracle.OracleDecoder(oracle.OracleGraph(g), 10.0, 10.0, BIG_ALPHA)
    bp.advance(ll)
    for use_final in (False, True):                # no final state: both fall back to plain cost
        r = bp.best_path(use_final)
        assert r["arcs"].tolist() == [1] and r["words"].tolist() == [5] and r["total_cost"] == 1.0
        assert not r["reached_final"]
    # finals: totals 1 + 3 = 2 + 2 = 4 on states 2 and 3, state 1 is not final
    g = graph_from_arcs(4, arcs, 1, finals={2: 3.0, 3: 2.0})
    d = oracle.OracleDecoder(oracle.OracleGraph(g), 10.0, 10.0, BIG_ALPHA)
    d.advance(ll)
    r = d.best_path(True)
    assert r["reached_final"] and r["arcs"].tolist() == [0] and r["words"].tolist() == [7] and r["total_cost"] == 4.0
    r = d.best_path(False)
    assert r["arcs"].tolist() == [1] and r["total_cost"] == 1.0
    # same totals with the roles of the states swapped: still the smaller state id
    g = graph_from_arcs(4, [(0, 3, 1, 9, 1.0), (0, 2, 1, 7, 2.0)], 1, finals={2: 2.0, 3: 3.0})
    d = oracle.OracleDecoder(oracle.OracleGraph(g), 10.0, 10.0, BIG_ALPHA)
    d.advance(ll)
    r = d.best_path(True)
    assert r["arcs"].tolist() == [1] and r["words"].tolist() == [7] and r["total_cost"] == 4.0


def test_best_path_end_state_is_the_lexicographic_minimum():
    """Integer costs, many ties: the path must end in min (cost [+ final], state id)."""
    tied = 0
    for seed in range(10):
        rng = np.random.default_rng(1100 + seed)
        g = random_graph(rng, num_states=25, n_emit_per_state=(2, 4), eps_prob=0.04, num_pdfs=4, wmax=1,
                         integer=True, n_final=10)
        g.final_cost[np.isfinite(g.final_cost)] = rng.integers(0, 2, size=int(np.isfinite(g.final_cost).sum())).astype(F32)
        ll = -rng.integers(0, 2, size=(6, 4)).astype(F32)
        d = oracle.OracleDecoder(oracle.OracleGraph(g), 3.0, 3.0, BIG_ALPHA)
        d.advance(ll)
        st, co, _ = d.tokens()
        for use_final in (False, True):
            tot = sorted((F32(c + g.final_cost[s]) if use_final else c, s) for s, c in zip(st.tolist(), co)
                         if not use_final or np.isfinite(g.final_cost[s]))
            tied += int(len(tot) >= 2 and tot[0][0] == tot[1][0])
            want_cost, want_state = tot[0]
            r = d.best_path(use_final)
            assert r["total_cost"] == want_cost
            assert int(g.nextstate[r["arcs"][-1]]) == want_state
    assert tied >= 6                               # the minimum was tied in most of the cases


# ---- (d) arcs_expanded when max-active binds ----------------------------------------------

@pytest.mark.parametrize("seed", range(4))
def test_arcs_expanded_counts_epsilon_degrees_before_the_max_active_cut(seed):
    rng = np.random.default_rng(1200 + seed)
    g = random_graph(rng, num_states=45, n_emit_per_state=(3, 5), eps_prob=0.06, num_pdfs=6, wmax=4)
    T = 10
    ll = rng.normal(-3, 1.5, size=(T, 6)).astype(F32)
    beam, alpha = 6.0, 10
    og = oracle.OracleGraph(g)
    d = oracle.OracleDecoder(og, beam, 2.0, alpha)
    src = arc_sources(g)
    n_emit = np.bincount(src[g.ilabel != 0], minlength=g.num_states)
    n_eps = np.bincount(src[g.ilabel == 0], minlength=g.num_states)
    st0, _, _ = d.tokens(0)
    total = int(n_eps[st0].sum())                  # frame 0: the start state's closure, nothing cut
    assert len(st0) <= alpha
    differs = 0
    for t in range(T):
        ps, pc, _ = d.tokens()
        V, kept, _, _ = python_frame(g, og, (ps, pc), ll[t], beam, alpha)
        total += int(n_emit[ps].sum()) + int(n_eps[np.array(sorted(V), np.int64)].sum())
        differs += int(n_eps[np.array(sorted(V), np.int64)].sum() != n_eps[np.array(sorted(kept), np.int64)].sum())
        d.advance(ll[t:t + 1])
        assert d.arcs_expanded == total
    assert differs >= 1                            # counting after the cut would give another number
    assert d.max_tokens_pre_prune > alpha and d.max_tokens == alpha


# ---- back-pointers that loop ---------------------------------------------------------------

def test_best_path_on_a_zero_weight_epsilon_cycle_ends_with_an_error():
    """Start state 3, emitting arc 3 -> 1, epsilon arcs 1 -> 2 and 2 -> 1 of weight zero.  Around the
    cycle all candidates tie; the tie goes to the smaller arc rank, and the arcs of states 1 and 2
    rank below the arc of state 3: tokens 1 and 2 point at each other.  The trace must stop with an
    error instead of running for ever (the decoding library refuses to load such a graph)."""
    arcs = [(1, 2, 0, 0, 0.0), (2, 1, 0, 0, 0.0), (3, 1, 1, 0, 1.0)]
    g = graph_from_arcs(4, arcs, 1, start=3)
    d = oracle.OracleDecoder(oracle.OracleGraph(g), 5.0, 5.0, BIG_ALPHA)
    d.advance(np.zeros((1, 1), F32))
    st, co, ia = d.tokens(1)
    assert st.tolist() == [1, 2] and co.tolist() == [1.0, 1.0] and ia.tolist() == [1, 0]
    with pytest.raises(RuntimeError):
        d.best_path(False)
