"""Small graph builders and comparison helpers shared by the tests (no decoder arithmetic)."""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np


@dataclass
class G:
    num_states: int
    num_arcs: int
    start_state: int
    num_pdfs: int
    row_offsets: np.ndarray
    ilabel: np.ndarray
    olabel: np.ndarray
    weight: np.ndarray
    nextstate: np.ndarray
    final_cost: np.ndarray


def graph_from_arcs(num_states, arcs, num_pdfs, finals=None, start=0):
    """arcs: list of (src, dst, ilabel, olabel, weight); kept in the given order per state."""
    by_state = [[] for _ in range(num_states)]
    for a in arcs:
        by_state[a[0]].append(a)
    off = [0]
    il, ol, w, ns = [], [], [], []
    for s in range(num_states):
        for (_, d, i, o, wt) in by_state[s]:
            il.append(i); ol.append(o); w.append(wt); ns.append(d)
        off.append(len(il))
    fin = np.full(num_states, np.inf, np.float32)
    for s, c in (finals or {}).items():
        fin[s] = c
    return G(num_states, len(il), start, num_pdfs, np.array(off, np.int64), np.array(il, np.int32),
             np.array(ol, np.int32), np.array(w, np.float32), np.array(ns, np.int32), fin)


def random_graph(rng, num_states, n_emit_per_state, eps_prob, num_pdfs, wmax=5.0, integer=False,
                 eps_first=False, n_final=2):
    """Random graph: emitting arcs anywhere, epsilon arcs only to higher state ids."""
    arcs = []
    for s in range(num_states):
        em = []
        for _ in range(rng.integers(n_emit_per_state[0], n_emit_per_state[1] + 1)):
            wt = float(rng.integers(0, int(wmax) + 1)) if integer else float(np.float32(rng.uniform(0, wmax)))
            em.append((s, int(rng.integers(0, num_states)), int(rng.integers(1, num_pdfs + 1)),
                       int(rng.integers(0, 4)), wt))
        ep = []
        for d in range(s + 1, num_states):
            if rng.uniform() < eps_prob:
                wt = float(rng.integers(0, int(wmax) + 1)) if integer else float(np.float32(rng.uniform(0, wmax)))
                ep.append((s, d, 0, int(rng.integers(0, 4)), wt))
        arcs += (ep + em) if eps_first else (em + ep)
    finals = {int(s): float(np.float32(rng.uniform(0, 3))) for s in rng.choice(num_states, n_final, replace=False)}
    return graph_from_arcs(num_states, arcs, num_pdfs, finals)


def arc_sources(g):
    return np.repeat(np.arange(g.num_states, dtype=np.int32), np.diff(g.row_offsets))


def canonical_rank(g):
    """Position of every arc in the order (source state, emitting before epsilon, caller position)."""
    src = arc_sources(g)
    order = np.lexsort((np.arange(g.num_arcs), g.ilabel == 0, src))
    rank = np.empty(g.num_arcs, np.int64)
    rank[order] = np.arange(g.num_arcs)
    return rank
