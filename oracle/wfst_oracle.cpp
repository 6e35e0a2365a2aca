// CPU checker for beam-pruned Viterbi token passing over a WFST decoding graph.
//
// TEST INFRASTRUCTURE ONLY.  This is the slow, single-threaded, obviously-correct
// implementation the GPU library is compared against.  Only the tests, the smoke check
// and the benchmark's cpu_baseline leg may load it; the GPU library never does, and the
// two share no code.
//
// What it computes follows the paper's order of operations for one frame of acoustic
// scores (Section 3, first paragraph): emitting arcs conditioned on the frame's values,
// then chains of non-emitting arcs, then pruning; and its lattice preprocessing
// (Section 3.4): one representative token per FST state plus an "extra cost" for every
// other arc that reaches that state.  The paper's own implementation prunes in a
// thread-order-dependent way (Section 4.1); where it leaves a rule open, the rule used
// here is order-independent so that a parallel implementation can match it bit for bit:
//
//   costs      fp32, tropical semiring; every add/sub rounded on its own (no FMA).
//   order      costs are compared through the monotone float->uint32 map `okey`;
//              a candidate through arc a is the pair (okey(cost), rank(a)), ordered
//              lexicographically, where rank(a) orders arcs by (source state,
//              emitting before non-emitting, position in the caller's arrays).
//   emitting   for every token (s,c) of frame t and emitting arc a = (s -> d, pdf, w):
//              x = (c + w) - loglike[t][pdf];  best = min x;  cutoff = best + beam;
//              candidates with x > cutoff are dropped; each state d keeps its minimum
//              candidate.                                   (Section 3.3, first paragraph)
//   closure    least fixed point of relaxing non-emitting arcs, x = c + w, kept iff
//              x <= cutoff (the cutoff of the emitting step).          (Section 3.3, 2nd)
//   max-active if more than max_active tokens remain, keep the max_active smallest by
//              (cost, state id); the cost of the last one kept becomes the effective
//              cutoff of the frame (this is the "adaptive beam").   (Fig. 1, Section 4.1)
//   lattice    every arc into a surviving state whose candidate cost, recomputed from
//              final token costs, is within the effective cutoff and within
//              lattice_beam of the state's best cost is recorded as
//              {frame, arc, extra = x - best cost of that state}.        (Section 3.4)
//   best path  arg-min over the last frame of cost (+ final cost), ties to the smaller
//              state id, followed back through each token's best incoming arc.
//
// parity unpinned: that these pruning rules select the same tokens as the paper's own
// decoder cannot be checked (the paper prints no token sets, costs or lattices).
// Everything else is pinned by tests/test_oracle_*.py (brute force over all paths,
// shortest-path library routine, closed forms, sort-and-truncate, invariants; the final
// lattice by brute force over all suffix paths).
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <deque>
#include <limits>
#include <map>
#include <vector>

namespace {

constexpr uint32_t NO_ARC = 0xFFFFFFFFu;
enum { ST_OK = 0, ST_DEAD = 1, ST_BAD_INPUT = 2 };

inline uint32_t okey(float x) {
  uint32_t b; std::memcpy(&b, &x, 4);
  return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}
inline uint64_t pack(float x, uint32_t rank) { return ((uint64_t)okey(x) << 32) | rank; }

struct Graph {
  int32_t ns = 0; int64_t na = 0; int32_t start = 0, npdf = 0;
  std::vector<int64_t> off; std::vector<int32_t> il, ol, dst; std::vector<float> w, fin;
  std::vector<uint32_t> rank;      // caller arc id -> position in the canonical arc order
  std::vector<int64_t> by_rank;    // inverse
  std::vector<int32_t> src;        // caller arc id -> source state
};

struct Tok { float cost; uint32_t in_rank; };     // in_rank = rank of the best incoming arc
typedef std::map<int32_t, Tok> TokMap;            // state -> token, iterated in state order

struct LatRec { int32_t frame; uint32_t arc; float extra; };   // arc = caller's arc id

struct Decoder {
  const Graph *g; float beam, lbeam; int32_t alpha; int lattice_on;
  std::vector<TokMap> frames;      // frames[t] = surviving tokens after t rows of scores
  std::vector<LatRec> lat;
  int status = ST_OK;
  int64_t arcs_expanded = 0;
  int32_t max_pre = 0, max_post = 0;
  float last_cutoff_eff = 0.f;
};

inline uint64_t key_of(const Tok &t) { return pack(t.cost, t.in_rank); }

// Relax non-emitting arcs until nothing changes.  Any processing order reaches the same
// fixed point because rounding is monotone and each state keeps a minimum.
void closure(const Graph &g, TokMap &V, float cutoff) {
  std::deque<int32_t> work;
  for (auto &kv : V) work.push_back(kv.first);
  while (!work.empty()) {
    int32_t s = work.front(); work.pop_front();
    float c = V[s].cost;
    for (int64_t a = g.off[s]; a < g.off[s + 1]; ++a) {
      if (g.il[a] != 0) continue;
      float x = c + g.w[a];
      if (!(x <= cutoff)) continue;
      int32_t d = g.dst[a];
      Tok cand{x, g.rank[a]};
      auto it = V.find(d);
      if (it == V.end()) { V[d] = cand; work.push_back(d); }
      else if (key_of(cand) < key_of(it->second)) { it->second = cand; work.push_back(d); }
    }
  }
}

int64_t eps_degree_sum(const Graph &g, const TokMap &V) {
  int64_t n = 0;
  for (auto &kv : V)
    for (int64_t a = g.off[kv.first]; a < g.off[kv.first + 1]; ++a) n += (g.il[a] == 0);
  return n;
}

// Keep the alpha smallest tokens by (cost, state); returns the effective cutoff.
float max_active(TokMap &V, int32_t alpha, float cutoff) {
  if ((int64_t)V.size() <= (int64_t)alpha) return cutoff;
  std::vector<std::pair<uint32_t, int32_t>> order;
  for (auto &kv : V) order.push_back({okey(kv.second.cost), kv.first});
  std::sort(order.begin(), order.end());
  TokMap kept;
  for (int32_t i = 0; i < alpha; ++i) kept[order[i].second] = V[order[i].second];
  float theta = kept[order[alpha - 1].second].cost;
  V.swap(kept);
  return theta;
}

// Lattice records of the frame whose tokens are `next`.  `prev` (may be null) holds the
// tokens the emitting arcs start from and `ll` that frame's scores.
void lattice_records(Decoder &D, const TokMap *prev, const float *ll, const TokMap &next,
                     int32_t frame, float cutoff_eff) {
  const Graph &g = *D.g;
  auto consider = [&](int64_t a, float x) {
    auto it = next.find(g.dst[a]);
    if (it == next.end()) return;
    if (!(x <= cutoff_eff)) return;
    float extra = x - it->second.cost;
    if (!(extra <= D.lbeam)) return;
    D.lat.push_back({frame, (uint32_t)a, extra});
  };
  if (prev)
    for (auto &kv : *prev)
      for (int64_t a = g.off[kv.first]; a < g.off[kv.first + 1]; ++a)
        if (g.il[a] != 0) { float cw = kv.second.cost + g.w[a]; consider(a, cw - ll[g.il[a] - 1]); }
  for (auto &kv : next)
    for (int64_t a = g.off[kv.first]; a < g.off[kv.first + 1]; ++a)
      if (g.il[a] == 0) consider(a, kv.second.cost + g.w[a]);
}

void finish_frame(Decoder &D, TokMap &V, const TokMap *prev, const float *ll, float cutoff) {
  const Graph &g = *D.g;
  closure(g, V, cutoff);
  D.arcs_expanded += eps_degree_sum(g, V);
  D.max_pre = std::max<int32_t>(D.max_pre, (int32_t)V.size());
  float cutoff_eff = max_active(V, D.alpha, cutoff);
  D.max_post = std::max<int32_t>(D.max_post, (int32_t)V.size());
  D.last_cutoff_eff = cutoff_eff;
  int32_t frame = (int32_t)D.frames.size();
  if (D.lattice_on) lattice_records(D, prev, ll, V, frame, cutoff_eff);
  D.frames.push_back(std::move(V));
}

void init_stream(Decoder &D) {
  D.frames.clear(); D.lat.clear(); D.status = ST_OK; D.arcs_expanded = 0; D.max_pre = D.max_post = 0;
  TokMap V;
  V[D.g->start] = Tok{0.0f, NO_ARC};
  float cutoff = 0.0f + D.beam;
  finish_frame(D, V, nullptr, nullptr, cutoff);
}

void advance_one(Decoder &D, const float *ll) {
  if (D.status != ST_OK) return;
  const Graph &g = *D.g;
  const TokMap &prev = D.frames.back();    // stays valid until finish_frame appends the new frame
  struct Cand { float x; int64_t a; };
  std::vector<Cand> cands;
  bool bad = false;
  for (auto &kv : prev)
    for (int64_t a = g.off[kv.first]; a < g.off[kv.first + 1]; ++a) {
      if (g.il[a] == 0) continue;
      D.arcs_expanded++;
      float cw = kv.second.cost + g.w[a];
      float x = cw - ll[g.il[a] - 1];
      if (x != x || x == -std::numeric_limits<float>::infinity()) bad = true;
      cands.push_back({x, a});
    }
  if (bad) { D.status = ST_BAD_INPUT; D.frames.push_back(TokMap()); return; }
  bool any = false; uint32_t best_key = 0; float best = 0.f;
  for (auto &c : cands) if (!any || okey(c.x) < best_key) { any = true; best_key = okey(c.x); best = c.x; }
  if (!any || best == std::numeric_limits<float>::infinity()) {
    D.status = ST_DEAD; D.frames.push_back(TokMap()); return;
  }
  float cutoff = best + D.beam;
  TokMap V;
  for (auto &c : cands) {
    if (!(c.x <= cutoff)) continue;
    Tok cand{c.x, g.rank[c.a]};
    auto it = V.find(g.dst[c.a]);
    if (it == V.end()) V[g.dst[c.a]] = cand;
    else if (key_of(cand) < key_of(it->second)) it->second = cand;
  }
  finish_frame(D, V, &prev, ll, cutoff);
}

}  // namespace

extern "C" {

void *oracle_graph_new(int32_t num_states, int64_t num_arcs, int32_t start_state, int32_t num_pdfs,
                       const int64_t *row_offsets, const int32_t *ilabel, const int32_t *olabel,
                       const float *weight, const int32_t *nextstate, const float *final_cost) {
  Graph *g = new Graph;
  g->ns = num_states; g->na = num_arcs; g->start = start_state; g->npdf = num_pdfs;
  g->off.assign(row_offsets, row_offsets + num_states + 1);
  g->il.assign(ilabel, ilabel + num_arcs); g->ol.assign(olabel, olabel + num_arcs);
  g->w.assign(weight, weight + num_arcs); g->dst.assign(nextstate, nextstate + num_arcs);
  g->fin.assign(final_cost, final_cost + num_states);
  g->rank.resize(num_arcs); g->by_rank.resize(num_arcs); g->src.resize(num_arcs);
  uint32_t r = 0;
  for (int32_t s = 0; s < num_states; ++s) {
    for (int64_t a = g->off[s]; a < g->off[s + 1]; ++a) { g->src[a] = s; if (g->il[a] != 0) { g->rank[a] = r; g->by_rank[r++] = a; } }
    for (int64_t a = g->off[s]; a < g->off[s + 1]; ++a) if (g->il[a] == 0) { g->rank[a] = r; g->by_rank[r++] = a; }
  }
  return g;
}
void oracle_graph_free(void *g) { delete (Graph *)g; }

void *oracle_decoder_new(const void *graph, float beam, float lattice_beam, int32_t max_active, int32_t lattice_on) {
  Decoder *D = new Decoder;
  D->g = (const Graph *)graph; D->beam = beam; D->lbeam = lattice_beam; D->alpha = max_active; D->lattice_on = lattice_on;
  return D;
}
void oracle_decoder_free(void *d) { delete (Decoder *)d; }

void oracle_init(void *d) { init_stream(*(Decoder *)d); }

// rows: host fp32 [n_frames][stride]
void oracle_advance(void *d, const float *rows, int64_t stride, int32_t n_frames) {
  Decoder &D = *(Decoder *)d;
  for (int32_t f = 0; f < n_frames; ++f) advance_one(D, rows + (int64_t)f * stride);
}

int32_t oracle_status(const void *d) { return ((const Decoder *)d)->status; }
int32_t oracle_num_frames(const void *d) { return (int32_t)((const Decoder *)d)->frames.size(); }
int64_t oracle_arcs_expanded(const void *d) { return ((const Decoder *)d)->arcs_expanded; }
int32_t oracle_max_tokens_pre_prune(const void *d) { return ((const Decoder *)d)->max_pre; }
int32_t oracle_max_tokens(const void *d) { return ((const Decoder *)d)->max_post; }
float oracle_last_cutoff(const void *d) { return ((const Decoder *)d)->last_cutoff_eff; }

int32_t oracle_num_tokens(const void *d, int32_t frame) {
  const Decoder &D = *(const Decoder *)d;
  if (frame < 0) frame += (int32_t)D.frames.size();
  if (frame < 0 || frame >= (int32_t)D.frames.size()) return -1;
  return (int32_t)D.frames[frame].size();
}
// Tokens of one frame in ascending state order; in_arc is the caller's arc id or 0xFFFFFFFF.
int32_t oracle_tokens(const void *d, int32_t frame, int32_t *state, float *cost, uint32_t *in_arc, int32_t cap) {
  const Decoder &D = *(const Decoder *)d;
  if (frame < 0) frame += (int32_t)D.frames.size();
  if (frame < 0 || frame >= (int32_t)D.frames.size()) return -1;
  int32_t n = 0;
  for (auto &kv : D.frames[frame]) {
    if (n >= cap) return -2;
    state[n] = kv.first; cost[n] = kv.second.cost;
    in_arc[n] = kv.second.in_rank == NO_ARC ? NO_ARC : (uint32_t)D.g->by_rank[kv.second.in_rank];
    ++n;
  }
  return n;
}

int64_t oracle_num_lattice(const void *d) { return (int64_t)((const Decoder *)d)->lat.size(); }
// Lattice records with frame >= from_frame, sorted by (frame, arc).
int64_t oracle_lattice(const void *d, int32_t from_frame, int32_t *frame, uint32_t *arc, float *extra, int64_t cap) {
  const Decoder &D = *(const Decoder *)d;
  std::vector<LatRec> v;
  for (auto &r : D.lat) if (r.frame >= from_frame) v.push_back(r);
  std::sort(v.begin(), v.end(), [](const LatRec &a, const LatRec &b) { return a.frame != b.frame ? a.frame < b.frame : a.arc < b.arc; });
  if ((int64_t)v.size() > cap) return -2;
  for (size_t i = 0; i < v.size(); ++i) { frame[i] = v[i].frame; arc[i] = v[i].arc; extra[i] = v[i].extra; }
  return (int64_t)v.size();
}

// Best path.  arcs (caller ids, forward order) and words (non-zero olabels, forward order).
// Returns 0, or -1 if there is no token, -2 if a buffer is too small, -3 if a token's
// best incoming arc starts from a state that holds no token or the back-pointers loop (both
// can only happen on graphs the decoding library refuses or warns about: zero-weight epsilon
// cycles, epsilon arcs into lower state ids with cost ties).
int32_t oracle_best_path(const void *d, int32_t use_final, int32_t *words, int32_t words_cap, int32_t *n_words,
                         int64_t *arcs, int32_t arcs_cap, int32_t *n_arcs, float *total_cost, int32_t *reached_final) {
  const Decoder &D = *(const Decoder *)d; const Graph &g = *D.g;
  if (D.frames.empty() || D.frames.back().empty()) return -1;
  const TokMap &last = D.frames.back();
  bool found = false; int32_t bs = -1; float bc = 0.f; int32_t rf = 0;
  if (use_final) {
    for (auto &kv : last) {
      float f = g.fin[kv.first];
      if (f == std::numeric_limits<float>::infinity()) continue;
      float t = kv.second.cost + f;
      if (!found || okey(t) < okey(bc)) { found = true; bs = kv.first; bc = t; }
    }
    rf = found ? 1 : 0;
  }
  if (!found)
    for (auto &kv : last) if (!found || okey(kv.second.cost) < okey(bc)) { found = true; bs = kv.first; bc = kv.second.cost; }
  std::vector<int64_t> path;
  int32_t f = (int32_t)D.frames.size() - 1, s = bs;
  size_t tokens_in_all = 0;                        // a trace longer than this revisits a token: back-pointers that loop
  for (auto &fr : D.frames) tokens_in_all += fr.size();
  for (;;) {
    if (path.size() > tokens_in_all) return -3;
    auto it = D.frames[f].find(s);
    if (it == D.frames[f].end()) return -3;
    if (it->second.in_rank == NO_ARC) break;
    int64_t a = g.by_rank[it->second.in_rank];
    path.push_back(a);
    if (g.il[a] != 0) --f;
    if (f < 0) return -3;
    s = g.src[a];
  }
  std::reverse(path.begin(), path.end());
  int32_t nw = 0;
  if ((int32_t)path.size() > arcs_cap) return -2;
  for (size_t i = 0; i < path.size(); ++i) {
    arcs[i] = path[i];
    if (g.ol[path[i]] != 0) { if (nw >= words_cap) return -2; words[nw++] = g.ol[path[i]]; }
  }
  *n_words = nw; *n_arcs = (int32_t)path.size(); *total_cost = bc; *reached_final = rf;
  return 0;
}

// Final lattice: backward pruning of the recorded arcs with the lattice beam (the step the
// paper leaves to the end of the utterance, Section 3.4).  Every token gets an extra cost
//   te(n) = min over recorded arcs a: n -> m of (te(m) + extra(a)),
// in the last frame te(n) = (cost(n) + final(n)) - best total (or cost(n) - best cost when no
// final state holds a token, or use_final is 0; non-final tokens get +inf when finals are
// used).  An arc a into m is kept iff te(m) + extra(a) <= lattice_beam.  All fp32, one
// rounded add per step; the minimum makes the result independent of evaluation order.
// Outputs the kept records sorted by (frame, arc); returns their number or -2 (cap).
int64_t oracle_final_lattice(const void *d, int32_t use_final, int32_t *frame, uint32_t *arc, float *extra, int64_t cap,
                             float *best_cost, int32_t *reached_final) {
  const Decoder &D = *(const Decoder *)d; const Graph &g = *D.g;
  const float INF = std::numeric_limits<float>::infinity();
  if (D.frames.empty() || D.frames.back().empty()) return -1;
  const int32_t T = (int32_t)D.frames.size() - 1;
  std::vector<std::map<int32_t, float>> te(T + 1);
  // last frame
  bool any_final = false; float best = INF;
  if (use_final)
    for (auto &kv : D.frames[T]) if (g.fin[kv.first] != INF) { any_final = true; best = std::min(best, kv.second.cost + g.fin[kv.first]); }
  if (!any_final) for (auto &kv : D.frames[T]) best = std::min(best, kv.second.cost);
  for (auto &kv : D.frames[T]) {
    float v;
    if (any_final) v = g.fin[kv.first] != INF ? (kv.second.cost + g.fin[kv.first]) - best : INF;
    else v = kv.second.cost - best;
    te[T][kv.first] = v;
  }
  // records per frame
  std::vector<std::vector<const LatRec *>> by_frame(T + 1);
  for (auto &r : D.lat) if (r.frame >= 0 && r.frame <= T) by_frame[r.frame].push_back(&r);
  for (int32_t f = T; f >= 0; --f) {
    if (f < T) for (auto &kv : D.frames[f]) te[f][kv.first] = INF;
    // arcs that leave frame f by an emitting arc land in frame f + 1
    if (f < T)
      for (const LatRec *r : by_frame[f + 1]) {
        if (g.il[r->arc] == 0) continue;
        float v = te[f + 1][g.dst[r->arc]] + r->extra;
        float &t = te[f][g.src[r->arc]];
        if (v < t) t = v;
      }
    // non-emitting arcs stay inside frame f: relax until nothing changes
    for (bool changed = true; changed;) {
      changed = false;
      for (const LatRec *r : by_frame[f]) {
        if (g.il[r->arc] != 0) continue;
        float v = te[f][g.dst[r->arc]] + r->extra;
        float &t = te[f][g.src[r->arc]];
        if (v < t) { t = v; changed = true; }
      }
    }
  }
  std::vector<LatRec> kept;
  for (auto &r : D.lat) {
    if (r.frame < 0 || r.frame > T) continue;
    float v = te[r.frame][g.dst[r.arc]] + r.extra;
    if (v <= D.lbeam) kept.push_back(r);
  }
  std::sort(kept.begin(), kept.end(), [](const LatRec &a, const LatRec &b) { return a.frame != b.frame ? a.frame < b.frame : a.arc < b.arc; });
  if ((int64_t)kept.size() > cap) return -2;
  for (size_t i = 0; i < kept.size(); ++i) { frame[i] = kept[i].frame; arc[i] = kept[i].arc; extra[i] = kept[i].extra; }
  *best_cost = best; *reached_final = any_final ? 1 : 0;
  return (int64_t)kept.size();
}

// Stand-alone closure of a token set (for tests): in/out arrays of (state, cost, in_arc as
// caller arc id or 0xFFFFFFFF); returns the new count, or -2 if cap is too small.
int32_t oracle_closure(const void *graph, int32_t n, int32_t *state, float *cost, uint32_t *in_arc, int32_t cap, float cutoff) {
  const Graph &g = *(const Graph *)graph;
  TokMap V;
  for (int32_t i = 0; i < n; ++i) V[state[i]] = Tok{cost[i], in_arc[i] == NO_ARC ? NO_ARC : g.rank[in_arc[i]]};
  closure(g, V, cutoff);
  if ((int32_t)V.size() > cap) return -2;
  int32_t m = 0;
  for (auto &kv : V) {
    state[m] = kv.first; cost[m] = kv.second.cost;
    in_arc[m] = kv.second.in_rank == NO_ARC ? NO_ARC : (uint32_t)g.by_rank[kv.second.in_rank];
    ++m;
  }
  return m;
}

}  // extern "C"
