"""Pins for the CPU checker (oracle/): each test ties it to something other than itself —
brute force over all paths, a library shortest-path routine, dense min-plus products in
numpy, closed forms, sort-and-truncate in numpy, and structural invariants.

The decoding rules being pinned are the paper's per-frame order of operations (Section 3,
first paragraph), its expand / adaptive beam / contract stages (Section 3.3, Fig. 1), the
non-emitting iterations run to convergence (Section 3.3) and the lattice preprocessing
(Section 3.4).
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


def brute_force(g, ll):
    """Minimum over ALL paths of the left-folded fp32 cost, per (frames consumed, state),
    with ties between last arcs broken by the canonical arc order."""
    T = ll.shape[0]
    rank = canonical_rank(g)
    best = {}

    def visit(t, s, c, last):
        cand = (okey(c), last)
        cur = best.get((t, s))
        if cur is None or cand < cur[0]:
            best[(t, s)] = (cand, c)
        for a in range(g.row_offsets[s], g.row_offsets[s + 1]):
            w, d, il = F32(g.weight[a]), int(g.nextstate[a]), int(g.ilabel[a])
            if il == 0:
                visit(t, d, F32(c + w), int(rank[a]))
            elif t < T:
                visit(t + 1, d, F32(F32(c + w) - F32(ll[t, il - 1])), int(rank[a]))

    visit(0, g.start_state, F32(0.0), NO_ARC)
    return best


def decode(g, ll, beam=INF, lattice_beam=INF, alpha=BIG_ALPHA, chunks=None):
    og = oracle.OracleGraph(g)
    d = oracle.OracleDecoder(og, beam, lattice_beam, alpha)
    if chunks is None:
        d.advance(ll)
    else:
        pos = 0
        for n in chunks:
            d.advance(ll[pos:pos + n])
            pos += n
    return d


@pytest.mark.parametrize("seed", range(12))
def test_costs_equal_brute_force_over_all_paths(seed):
    rng = np.random.default_rng(seed)
    g = random_graph(rng, num_states=int(rng.integers(4, 9)), n_emit_per_state=(1, 2), eps_prob=0.25,
                     num_pdfs=5, eps_first=bool(seed % 2))
    T = int(rng.integers(2, 6))
    ll = rng.normal(-3, 2, size=(T, 5)).astype(F32)
    bf = brute_force(g, ll)
    d = decode(g, ll)
    rank = canonical_rank(g)
    assert d.num_frames == T + 1
    for t in range(T + 1):
        st, co, ia = d.tokens(t)
        want = sorted(s for (tt, s) in bf if tt == t)
        assert st.tolist() == want
        for s, c, a in zip(st, co, ia):
            (k, r), cost = bf[(t, int(s))]
            assert okey(c) == k and F32(c) == cost
            assert (NO_ARC if a == NO_ARC else int(rank[a])) == r


@pytest.mark.parametrize("seed", range(6))
def test_integer_ties_equal_brute_force(seed):
    """Integer weights and scores make exact cost ties common: the tie-break is exercised."""
    rng = np.random.default_rng(100 + seed)
    g = random_graph(rng, num_states=6, n_emit_per_state=(2, 3), eps_prob=0.3, num_pdfs=3, wmax=2,
                     integer=True, eps_first=bool(seed % 2))
    ll = -rng.integers(0, 3, size=(4, 3)).astype(F32)
    bf = brute_force(g, ll)
    d = decode(g, ll)
    rank = canonical_rank(g)
    for t in range(5):
        st, co, ia = d.tokens(t)
        assert st.tolist() == sorted(s for (tt, s) in bf if tt == t)
        for s, c, a in zip(st, co, ia):
            (k, r), _ = bf[(t, int(s))]
            assert okey(c) == k
            assert (NO_ARC if a == NO_ARC else int(rank[a])) == r


@pytest.mark.parametrize("seed", range(6))
def test_no_epsilon_equals_dense_min_plus(seed):
    """Without epsilon arcs the token costs are a chain of dense min-plus products."""
    rng = np.random.default_rng(200 + seed)
    n, P, T = 7, 4, 6
    W = rng.uniform(0, 5, size=(n, n)).astype(F32)
    PDF = rng.integers(0, P, size=(n, n))
    arcs = [(s, d, int(PDF[s, d]) + 1, 0, float(W[s, d])) for s in range(n) for d in range(n)]
    g = graph_from_arcs(n, arcs, P)
    ll = rng.normal(-4, 2, size=(T, P)).astype(F32)
    d = decode(g, ll)
    D = np.full(n, np.inf, F32)
    D[0] = 0
    for t in range(T):
        X = (D[:, None] + W) - ll[t][PDF]          # fp32, same association as the decoder
        D = X.min(axis=0)
        st, co, _ = d.tokens(t + 1)
        assert st.tolist() == list(range(n))
        assert np.array_equal(co, D)


@pytest.mark.parametrize("seed", range(5))
def test_closure_idempotent_and_equals_library_shortest_paths(seed):
    from scipy.sparse import csr_matrix
    from scipy.sparse.csgraph import dijkstra
    rng = np.random.default_rng(300 + seed)
    g = random_graph(rng, num_states=30, n_emit_per_state=(0, 1), eps_prob=0.12, num_pdfs=3, wmax=6,
                     integer=True)
    og = oracle.OracleGraph(g)
    seeds = rng.choice(30, 4, replace=False).astype(np.int32)
    scost = rng.integers(0, 5, size=4).astype(F32)
    cutoff = 9.0
    st, co, ia = og.closure(seeds, scost, np.full(4, NO_ARC, np.uint32), cutoff)
    st2, co2, ia2 = og.closure(st, co, ia, cutoff)
    assert np.array_equal(st, st2) and np.array_equal(co, co2) and np.array_equal(ia, ia2)
    # integer weights: fp32 sums are exact, so a float64 library routine must agree exactly
    eps = g.ilabel == 0
    src = arc_sources(g)
    n = g.num_states
    M = np.full((n + 1, n + 1), 0.0)
    big = np.full((n + 1, n + 1), np.inf)
    for s, d, w in zip(src[eps], g.nextstate[eps], g.weight[eps]):
        big[s, d] = min(big[s, d], w + 1e-9)       # keep zero-weight arcs in the sparse matrix
    for s, c in zip(seeds, scost):
        big[n, s] = c + 1e-9                       # super-source
    M = csr_matrix(np.where(np.isfinite(big), big, 0.0))
    dist = dijkstra(M, directed=True, indices=n)[:n]
    dist = np.round(dist)                          # remove the 1e-9 markers
    want = {s: dist[s] for s in range(n) if np.isfinite(dist[s]) and dist[s] <= cutoff}
    assert st.tolist() == sorted(want)
    assert [float(c) for c in co] == [want[s] for s in st.tolist()]


def test_linear_chain_closed_form():
    n, T = 9, 8
    rng = np.random.default_rng(1)
    w = rng.uniform(0, 3, n).astype(F32)
    arcs = [(s, s + 1, s % 3 + 1, s + 1, float(w[s])) for s in range(n - 1)]
    g = graph_from_arcs(n, arcs, 3, finals={n - 1: 0.5})
    ll = rng.normal(-2, 1, size=(T, 3)).astype(F32)
    d = decode(g, ll, beam=5.0, alpha=10)
    c = F32(0)
    for t in range(T):
        c = F32(F32(c + w[t]) - ll[t, t % 3])
        st, co, ia = d.tokens(t + 1)
        assert st.tolist() == [t + 1] and co[0] == c and ia[0] == t
    bp = d.best_path()
    assert bp["reached_final"] and bp["words"].tolist() == list(range(1, n))
    assert bp["total_cost"] == F32(c + F32(0.5))


def test_zero_weights_constant_scores_closed_form():
    rng = np.random.default_rng(2)
    g = random_graph(rng, num_states=12, n_emit_per_state=(1, 3), eps_prob=0.1, num_pdfs=4)
    g.weight[:] = 0
    ell = F32(-1.25)
    T = 7
    d = decode(g, np.full((T, 4), ell, F32), beam=1.0, alpha=100)
    for t in range(T + 1):
        _, co, _ = d.tokens(t)
        assert len(co) > 0 and np.all(co == F32(-ell * t))


def test_max_active_one_is_greedy():
    rng = np.random.default_rng(3)
    g = random_graph(rng, num_states=15, n_emit_per_state=(2, 4), eps_prob=0.0, num_pdfs=6)
    T = 10
    ll = rng.normal(-3, 2, size=(T, 6)).astype(F32)
    d = decode(g, ll, beam=1e9, alpha=1)
    s, c = 0, F32(0)
    for t in range(T):
        cands = []
        for a in range(g.row_offsets[s], g.row_offsets[s + 1]):
            x = F32(F32(c + g.weight[a]) - ll[t, g.ilabel[a] - 1])
            cands.append((okey(x), int(g.nextstate[a]), a, x))
        # greedy: the best token per destination, then the single best (cost, state)
        per_dst = {}
        for k, dst, a, x in cands:
            if dst not in per_dst or (k, a) < per_dst[dst][:2]:
                per_dst[dst] = (k, a, x)
        dst = min(per_dst, key=lambda q: (per_dst[q][0], q))
        s, c = dst, per_dst[dst][2]
        st, co, ia = d.tokens(t + 1)
        assert st.tolist() == [s] and co[0] == c and ia[0] == per_dst[dst][1]


@pytest.mark.parametrize("integer", [False, True])
@pytest.mark.parametrize("seed", range(8))
def test_max_active_is_sort_and_truncate(seed, integer):
    """Decoders with and without the limit agree up to the first frame that exceeds it;
    there the limited one must hold exactly the alpha smallest (cost, state) pairs."""
    rng = np.random.default_rng(400 + seed)
    g = random_graph(rng, num_states=60, n_emit_per_state=(2, 4), eps_prob=0.03, num_pdfs=8,
                     wmax=3, integer=integer)
    T = 12
    ll = (-rng.integers(0, 4, size=(T, 8)).astype(F32)) if integer else rng.normal(-3, 1, size=(T, 8)).astype(F32)
    alpha = 9
    og = oracle.OracleGraph(g)
    lim = oracle.OracleDecoder(og, 50.0, 50.0, alpha)
    unl = oracle.OracleDecoder(og, 50.0, 50.0, BIG_ALPHA)
    checked = False
    for t in range(-1, T):                       # t = -1: frame 0, written by init
        if t >= 0:
            lim.advance(ll[t:t + 1])
            unl.advance(ll[t:t + 1])
        st, co, ia = unl.tokens()
        ls, lc, la = lim.tokens()
        if len(st) <= alpha:
            assert np.array_equal(st, ls) and np.array_equal(co, lc) and np.array_equal(ia, la)
            continue
        keys = np.array([okey(c) for c in co], np.uint64)
        order = np.lexsort((st, keys))[:alpha]
        keep = np.sort(order)
        assert np.array_equal(ls, st[keep]) and np.array_equal(lc, co[keep]) and np.array_equal(la, ia[keep])
        assert lim.last_cutoff == co[order[-1]]
        assert lc.min() == co.min()
        checked = True
        break
    assert checked
    assert lim.max_tokens <= alpha


@pytest.mark.parametrize("seed", range(6))
def test_best_path_cost_is_the_fold_along_its_arcs(seed):
    rng = np.random.default_rng(500 + seed)
    g = random_graph(rng, num_states=40, n_emit_per_state=(2, 4), eps_prob=0.04, num_pdfs=10, n_final=8)
    T = 25
    ll = rng.normal(-5, 2, size=(T, 10)).astype(F32)
    d = decode(g, ll, beam=8.0, lattice_beam=4.0, alpha=25)
    src = arc_sources(g)
    for use_final in (True, False):
        bp = d.best_path(use_final)
        arcs = bp["arcs"]
        c, t, s = F32(0), 0, g.start_state
        for a in arcs:
            assert src[a] == s
            c = F32(c + g.weight[a])
            if g.ilabel[a] != 0:
                c = F32(c - ll[t, g.ilabel[a] - 1])
                t += 1
            s = int(g.nextstate[a])
        assert t == T
        st, co, _ = d.tokens()
        assert c == co[st.tolist().index(s)]
        if use_final and bp["reached_final"]:
            assert np.isfinite(g.final_cost[s])
            assert bp["total_cost"] == F32(c + g.final_cost[s])
            tot = [F32(cc + g.final_cost[ss]) for ss, cc in zip(st, co) if np.isfinite(g.final_cost[ss])]
            assert bp["total_cost"] == min(tot)
        else:
            assert bp["total_cost"] == c == co.min()
        assert bp["words"].tolist() == [int(g.olabel[a]) for a in arcs if g.olabel[a] != 0]


def test_best_path_falls_back_when_no_final_token():
    rng = np.random.default_rng(7)
    g = random_graph(rng, num_states=20, n_emit_per_state=(2, 3), eps_prob=0.0, num_pdfs=5)
    g.final_cost[:] = np.inf
    ll = rng.normal(-3, 1, size=(6, 5)).astype(F32)
    bp = decode(g, ll, beam=6.0, alpha=10).best_path(True)
    assert not bp["reached_final"]


@pytest.mark.parametrize("seed", range(6))
def test_lattice_records_invariants(seed):
    rng = np.random.default_rng(600 + seed)
    integer = bool(seed % 2)
    g = random_graph(rng, num_states=35, n_emit_per_state=(2, 5), eps_prob=0.05, num_pdfs=6, wmax=4,
                     integer=integer)
    T = 15
    ll = (-rng.integers(0, 4, size=(T, 6)).astype(F32)) if integer else rng.normal(-4, 2, size=(T, 6)).astype(F32)
    lbeam = 3.0
    d = decode(g, ll, beam=7.0, lattice_beam=lbeam, alpha=14)
    src = arc_sources(g)
    rank = canonical_rank(g)
    fr, ar, ex = d.lattice()
    assert len(set(zip(fr.tolist(), ar.tolist()))) == len(fr)
    toks = [dict(zip(st.tolist(), zip(co, ia))) for st, co, ia in (d.tokens(t) for t in range(T + 1))]
    zero_extra = {}
    for f, a, e in zip(fr, ar, ex):
        dst = int(g.nextstate[a])
        assert dst in toks[f]
        if g.ilabel[a] != 0:
            assert f >= 1 and int(src[a]) in toks[f - 1]
            x = F32(F32(toks[f - 1][int(src[a])][0] + g.weight[a]) - ll[f - 1, g.ilabel[a] - 1])
        else:
            assert int(src[a]) in toks[f]
            x = F32(toks[f][int(src[a])][0] + g.weight[a])
        assert F32(x - toks[f][dst][0]) == e and 0 <= e <= lbeam
        if e == 0:
            zero_extra.setdefault((int(f), dst), []).append(int(rank[a]))
    for f in range(T + 1):
        for s, (c, ia) in toks[f].items():
            if ia == NO_ARC:
                assert f == 0 and s == g.start_state
                continue
            assert min(zero_extra[(f, s)]) == rank[ia]


def test_lattice_beam_zero_is_the_backpointer_forest():
    rng = np.random.default_rng(8)
    g = random_graph(rng, num_states=50, n_emit_per_state=(2, 4), eps_prob=0.04, num_pdfs=7)
    T = 12
    ll = rng.normal(-4, 2, size=(T, 7)).astype(F32)
    d = decode(g, ll, beam=6.0, lattice_beam=0.0, alpha=20)
    fr, ar, ex = d.lattice()
    got = sorted(zip(fr.tolist(), ar.tolist()))
    want = []
    for t in range(T + 1):
        st, co, ia = d.tokens(t)
        want += [(t, int(a)) for a in ia if a != NO_ARC]
    assert got == sorted(want) and np.all(ex == 0)


@pytest.mark.parametrize("chunks", [[1] * 20, [7, 13], [5, 0, 5, 10], [19, 1]])
def test_chunked_advance_is_identical(chunks):
    rng = np.random.default_rng(9)
    g = random_graph(rng, num_states=40, n_emit_per_state=(2, 4), eps_prob=0.05, num_pdfs=6)
    ll = rng.normal(-4, 2, size=(20, 6)).astype(F32)
    a = decode(g, ll, beam=6.0, lattice_beam=3.0, alpha=15)
    b = decode(g, ll, beam=6.0, lattice_beam=3.0, alpha=15, chunks=chunks)
    assert a.num_frames == b.num_frames == 21
    for t in range(21):
        for x, y in zip(a.tokens(t), b.tokens(t)):
            assert np.array_equal(x, y)
    for x, y in zip(a.lattice(), b.lattice()):
        assert np.array_equal(x, y)
    assert a.arcs_expanded == b.arcs_expanded


def test_arc_order_within_a_state_does_not_change_tokens():
    """Epsilon-first and emitting-first layouts of the same graph decode to the same tokens
    and to the same arcs (by content)."""
    rng1, rng2 = np.random.default_rng(10), np.random.default_rng(10)
    g1 = random_graph(rng1, num_states=30, n_emit_per_state=(2, 3), eps_prob=0.08, num_pdfs=5, wmax=2, integer=True)
    g2 = random_graph(rng2, num_states=30, n_emit_per_state=(2, 3), eps_prob=0.08, num_pdfs=5, wmax=2, integer=True,
                      eps_first=True)
    ll = -np.random.default_rng(11).integers(0, 3, size=(10, 5)).astype(F32)
    d1 = decode(g1, ll, beam=6.0, lattice_beam=2.0, alpha=12)
    d2 = decode(g2, ll, beam=6.0, lattice_beam=2.0, alpha=12)
    r1, r2 = canonical_rank(g1), canonical_rank(g2)
    for t in range(11):
        s1, c1, a1 = d1.tokens(t)
        s2, c2, a2 = d2.tokens(t)
        assert np.array_equal(s1, s2) and np.array_equal(c1, c2)
        m = a1 != NO_ARC
        assert np.array_equal(m, a2 != NO_ARC) and np.array_equal(r1[a1[m]], r2[a2[m]])


def test_dead_channel_and_bad_scores():
    rng = np.random.default_rng(12)
    g = random_graph(rng, num_states=10, n_emit_per_state=(1, 2), eps_prob=0.1, num_pdfs=3)
    ll = rng.normal(-3, 1, size=(4, 3)).astype(F32)
    dead = ll.copy(); dead[2, :] = -np.inf
    d = decode(g, dead, beam=5.0, alpha=10)
    assert d.status == oracle.ST_DEAD and d.num_frames == 4 and len(d.tokens()[0]) == 0
    assert d.best_path() is None
    for bad_value in (np.nan, np.inf):
        bad = ll.copy(); bad[1, :] = bad_value
        d = decode(g, bad, beam=5.0, alpha=10)
        assert d.status == oracle.ST_BAD_INPUT and d.num_frames == 3 and len(d.tokens()[0]) == 0


def test_arcs_expanded_is_the_sum_of_out_degrees():
    rng = np.random.default_rng(13)
    g = random_graph(rng, num_states=30, n_emit_per_state=(1, 4), eps_prob=0.06, num_pdfs=5)
    T = 10
    ll = rng.normal(-3, 1, size=(T, 5)).astype(F32)
    d = decode(g, ll, beam=5.0, alpha=BIG_ALPHA)       # no max-active: kept tokens == closure tokens
    src = arc_sources(g)
    n_emit = np.bincount(src[g.ilabel != 0], minlength=30)
    n_eps = np.bincount(src[g.ilabel == 0], minlength=30)
    total = 0
    for t in range(T + 1):
        st, _, _ = d.tokens(t)
        total += n_eps[st].sum() + (n_emit[st].sum() if t < T else 0)
    assert d.arcs_expanded == total


# ---- final lattice (Section 3.4: the lattice generated at the end of the utterance) ----------

def _final_lattice_by_enumeration(g, d, T, lbeam, use_final):
    """Every recorded arc is kept iff some path of recorded arcs from its destination to the last
    frame, folded from the end in fp32 (v = F32(v + extra) per arc), stays within the lattice
    beam.  All suffix paths are enumerated explicitly."""
    src = arc_sources(g)
    fr, ar, ex = d.lattice()
    out = {}
    for f, a, e in zip(fr.tolist(), ar.tolist(), ex):
        node = (f - (1 if g.ilabel[a] != 0 else 0), int(src[a]))
        out.setdefault(node, []).append(((f, int(g.nextstate[a])), F32(e)))
    st, co, _ = d.tokens(T)
    fin = {int(s): F32(c) + F32(g.final_cost[s]) for s, c in zip(st, co) if np.isfinite(g.final_cost[s])} if use_final else {}
    if fin:
        best = min(fin.values())
        end = {(T, s): F32(v - best) for s, v in fin.items()}
    else:
        best = min(F32(c) for c in co)
        end = {(T, int(s)): F32(F32(c) - best) for s, c in zip(st, co)}

    def suffix_values(node):
        """fp32 right-fold values of all paths from node to an end node."""
        vals = [end[node]] if node in end else []
        for nxt, e in out.get(node, []):
            if nxt[0] == T and nxt not in end and nxt not in out:
                continue
            vals += [F32(v + e) for v in suffix_values(nxt)]
        return vals

    kept = []
    for f, a, e in zip(fr.tolist(), ar.tolist(), ex):
        vals = suffix_values((f, int(g.nextstate[a])))
        if vals and F32(min(vals) + F32(e)) <= lbeam:
            kept.append((f, a))
    return sorted(kept), best


@pytest.mark.parametrize("seed", range(8))
def test_final_lattice_equals_enumeration_of_suffix_paths(seed):
    rng = np.random.default_rng(700 + seed)
    integer = bool(seed % 2)
    g = random_graph(rng, num_states=14, n_emit_per_state=(1, 3), eps_prob=0.06, num_pdfs=4, wmax=3,
                     integer=integer, n_final=4)
    T = 6
    ll = (-rng.integers(0, 3, size=(T, 4)).astype(F32)) if integer else rng.normal(-3, 1.5, size=(T, 4)).astype(F32)
    lbeam = 2.5
    d = decode(g, ll, beam=5.0, lattice_beam=lbeam, alpha=6)
    for use_final in (True, False):
        want, best = _final_lattice_by_enumeration(g, d, T, lbeam, use_final)
        got = d.final_lattice(use_final)
        assert sorted(zip(got["frame"].tolist(), got["arc"].tolist())) == want
        assert got["best_cost"] == best


def test_final_lattice_invariants():
    rng = np.random.default_rng(8)
    g = random_graph(rng, num_states=60, n_emit_per_state=(2, 4), eps_prob=0.03, num_pdfs=8, n_final=12)
    T = 30
    ll = rng.normal(-4, 2, size=(T, 8)).astype(F32)
    sizes = []
    for lbeam in (0.0, 1.0, 4.0):
        d = decode(g, ll, beam=8.0, lattice_beam=lbeam, alpha=25)
        fl = d.final_lattice(True)
        kept = set(zip(fl["frame"].tolist(), fl["arc"].tolist()))
        raw = set(zip(*[x.tolist() for x in d.lattice()[:2]]))
        assert kept <= raw
        bp = d.best_path(True)
        assert fl["best_cost"] == bp["total_cost"] and fl["reached_final"] == bp["reached_final"]
        # every arc of the best path survives, in its frame
        f = 0
        for a in bp["arcs"]:
            if g.ilabel[a] != 0:
                f += 1
            assert (f, int(a)) in kept
        sizes.append(len(kept))
    assert sizes[0] <= sizes[1] <= sizes[2]
