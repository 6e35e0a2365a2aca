// Kernels of the decoder.
//
// One workgroup owns one lane (one audio stream of the batch) for a whole advance call and
// loops over that lane's frames by itself: streams are independent and frames are strictly
// serial (the paper's Section 3.1), so nothing ever has to be agreed between workgroups and
// every synchronisation is a workgroup barrier.  This takes the paper's "one CTA per
// utterance" persistent kernel for the tail of the non-emitting iterations (Section 3.3)
// and applies it to the entire frame: with hundreds of lanes resident the chip is filled by
// lanes rather than by the arcs of one lane, and no kernel launch sits between the stages
// of Fig. 1.
//
// Per frame (Section 3, first paragraph; Fig. 1):
//   1. emitting expansion, load-balanced over arcs (one thread per outgoing arc, Section
//      3.3): x = (cost + weight) - loglike[pdf]; the lane's best cost is tracked in LDS and
//      candidates within (running best + beam) enter the lane's state table through a
//      64-bit atomic minimum over (ordered cost bits, arc index);
//   2. non-emitting closure: rounds over the newly added / improved tokens until a round
//      adds nothing;
//   3. max-active: if more than max_active tokens are within the beam, an exact histogram
//      selection over the ordered cost bits (then over state handles among ties) finds the
//      cut; its cost is the frame's effective cutoff (the adaptive beam);
//   4. contraction: the kept tokens are appended to the channel's token history, which is
//      also the queue the next frame expands from;
//   5. lattice preprocessing (Section 3.4): every candidate arc that reaches a kept token
//      within the effective cutoff and the lattice beam is recorded with its extra cost;
//      the arc equal to the table's minimum fixes the token's back-pointer;
//   6. the touched table slots are cleared.
// A call may cover many chunks of frames: at the boundaries the caller names, the lane seals
// a snapshot of its channel (and hands its lattice records over in the caller's form) and
// goes on, so that partial results can be read beside the decoding and no lane waits for a
// slower one (the role of the paper's second stream, Section 3, Fig. 1).
#pragma once
#include "wfst_device.h"

namespace wfst {

constexpr int NBINS = 1024;
constexpr uint32_t F_NAN = 1, F_TOKOVF = 2, F_LATOVF = 4, F_RESTART = 8;
constexpr uint32_t KEY_NONE = 0xFFFFFFFFu;
constexpr uint32_t KEY_PINF = 0xFF800000u;    // okey(+inf)

__device__ __forceinline__ uint32_t okey(float x) {
  uint32_t b = __float_as_uint(x);
  return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}
__device__ __forceinline__ float key2f(uint32_t k) {
  return __uint_as_float((k & 0x80000000u) ? (k & 0x7FFFFFFFu) : ~k);
}
__device__ __forceinline__ unsigned long long pack(uint32_t key, uint32_t arc) {
  return ((unsigned long long)key << 32) | arc;
}
// Loads that bypass the per-CU vector cache: table words are updated by atomics, which
// execute in L2, so cached copies could be stale.
__device__ __forceinline__ uint32_t ld32(const uint32_t *p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ unsigned long long ld64(const unsigned long long *p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint32_t slot_hash(uint32_t handle, int hbits) {
  return (handle * 2654435761u) >> (32 - hbits);
}

// Table words are read through these: in global memory with loads that bypass the per-CU
// vector cache (see ld32), in LDS with plain loads.
template <bool LDS> __device__ __forceinline__ uint32_t tl32(const uint32_t *p) { return LDS ? *p : ld32(p); }
template <bool LDS> __device__ __forceinline__ unsigned long long tl64(const unsigned long long *p) { return LDS ? *p : ld64(p); }

// Offer candidate K for state `handle`.  Returns the slot, or -1 if the table is full.
template <bool LDS>
__device__ __forceinline__ int ht_insert(Slot *slots, uint32_t mask, int hbits, uint32_t handle,
                                         unsigned long long K, bool &claimed, bool &improved) {
  uint32_t h = slot_hash(handle, hbits);
  claimed = false; improved = false;
  for (uint32_t probe = 0; probe <= mask; ++probe) {
    // one compare-and-swap tells all three cases apart: free (now ours), ours already, another state's
    uint32_t k = atomicCAS(&slots[h].handle, EMPTY, handle);
    if (k == EMPTY) { claimed = true; k = handle; }
    if (k == handle) {
      unsigned long long old = atomicMin(&slots[h].val, K);
      improved = K < old;
      return (int)h;
    }
    h = (h + 1) & mask;
  }
  return -1;
}
// A whole slot at once: in LDS one 16-byte read instead of dependent 8- and 4-byte ones (a
// reader beside concurrent atomic minima gets some value the slot held, which is all the
// callers need); in global memory three independent coherent loads.
template <bool LDS>
__device__ __forceinline__ Slot ld_slot(const Slot *p) {
  Slot r;
  if (LDS) {
    *reinterpret_cast<uint4 *>(&r) = *reinterpret_cast<const uint4 *>(p);
  } else {
    r.val = ld64(&p->val); r.handle = ld32(&p->handle); r.aux = ld32(&p->aux);
  }
  return r;
}
template <bool LDS>
__device__ __forceinline__ int ht_find(const Slot *slots, uint32_t mask, int hbits, uint32_t handle) {
  uint32_t h = slot_hash(handle, hbits);
  for (uint32_t probe = 0; probe <= mask; ++probe) {
    uint32_t k = tl32<LDS>(&slots[h].handle);
    if (k == handle) return (int)h;
    if (k == EMPTY) return -1;
    h = (h + 1) & mask;
  }
  return -1;
}

// Small frames keep the state table in LDS; a frame that outgrows it is redone with the
// lane's table in global memory (nothing is committed before the contraction stage).
// A 512-thread lane shares its compute unit's 160 KB of LDS with another lane, a 1024-thread
// lane has it to itself and takes a table, queue and limits twice as large.
template <int NT> struct LdsCfg {
  static constexpr int SLOTS = NT >= 1024 ? 8192 : 4096;
  static constexpr int HBITS = NT >= 1024 ? 13 : 12;
  static constexpr int CLAIM_LIMIT = SLOTS * 3 / 4;   // states touched in a frame
  static constexpr int NIN_MAX = SLOTS / 4;           // tokens the frame starts from
  static constexpr int QCAP = SLOTS;                  // entries of the LDS token queue (16-bit each)
};
constexpr int EXP_U = 4;                   // arcs per thread and round of the emitting expansion
constexpr int EPS_U = 2;                   // epsilon arcs of a token fetched together
constexpr int LAT_U = 4;                   // candidate records per thread and round of the lattice stage
constexpr uint32_t AUX_EPS = 0x80000000u;  // Aux::slot flag: the record is an epsilon arc
// Slot::aux while a frame is being built (afterwards: index of the kept token, or ~0):
constexpr uint32_t A_FRESH = 0x80000000u;  // epsilon out-degree not counted yet
constexpr uint32_t A_KEPT_MAX = 0x20000000u;  // aux < A_KEPT_MAX: index of the kept token
// LDS queue entry: slot (up to 14 bits) | LQ_EPS | LQ_DUP
constexpr uint32_t LQ_EPS = 0x4000u, LQ_DUP = 0x8000u, LQ_SLOT = 0x3FFFu;

template <int NT>
struct LaneShared {
  int wave_tmp[NT / 64];
  union {                      // the expansion's tile arrays and the selection's histogram never coexist
    struct { int scan[NT]; float cost[NT]; uint32_t base[NT]; };
    uint32_t hist[NBINS];
  };
  // queue entries (low word) and states claimed (high word) of the frame: one 64-bit counter,
  // so that a claim takes one atomic for both
  union { unsigned long long claim_ctr; struct { uint32_t qtail, nclaim; }; };
  uint32_t auxn, best, flags, nvalid, nout, latn, kmin, kmax;
  uint32_t sel_bin, sel_below, sel_cnt;
  unsigned long long emit_arcs, eps_arcs;
  // channel state, cached for the duration of the call
  int status, nf, max_pre, max_post, iters_max, n_in;
  long long in_off, hist_used, lat_room, lat_total, arcs_expanded;
  long long lat_pos;           // ring position of record number lat_total
  long long lat_head, lat_head_pos, blk_pos;   // first record not handed out, its ring position; seal scratch
#ifdef WFST_PHASE_TIMING
  unsigned long long ph[16], tlast, dbg_tok, dbg_iters, dbg_arcs;
#endif
  uint16_t lq[LdsCfg<NT>::QCAP];     // token queue of small frames
  Slot table[LdsCfg<NT>::SLOTS];     // state table of small frames
};

#ifdef WFST_PHASE_TIMING
#define PHASE_MARK(k) do { if (threadIdx.x == 0) { unsigned long long t_ = wall_clock64(); S.ph[k] += t_ - S.tlast; S.tlast = t_; } } while (0)
#else
#define PHASE_MARK(k) do { } while (0)
#endif

// Workgroup barrier for stages that communicate through LDS only: it orders LDS accesses but
// does not wait for global loads or stores in flight, so the score-row touch and the stores of
// notes / tokens / lattice records keep travelling across it.  With LOCAL false it is an
// ordinary __syncthreads() (the global-table path communicates through global memory).
template <bool LOCAL>
__device__ __forceinline__ void wg_sync() {
  if (LOCAL) {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
  } else {
    __syncthreads();
  }
}

// One counter update per wavefront: the lanes that call this together (same call site,
// any subset of the wave) get consecutive indices from a single atomic add.
__device__ __forceinline__ uint32_t wave_alloc(uint32_t *counter) {
  const unsigned long long m = __ballot(1);
  const int lane = threadIdx.x & 63;
  const int leader = __ffsll((long long)m) - 1;
  uint32_t base = 0;
  if (lane == leader) base = atomicAdd(counter, (uint32_t)__popcll(m));
  base = (uint32_t)__shfl((int)base, leader, 64);
  return base + (uint32_t)__popcll(m & ((1ull << lane) - 1ull));
}

template <int NT, bool LOCAL = false>
__device__ __forceinline__ int block_excl_scan(int v, int *s_wave, int &total) {
  const int lane = threadIdx.x & 63, wid = threadIdx.x >> 6;
  int inc = v;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    int t = __shfl_up(inc, d, 64);
    if (lane >= d) inc += t;
  }
  if (lane == 63) s_wave[wid] = inc;
  wg_sync<LOCAL>();
  int base = 0, tot = 0;
#pragma unroll
  for (int i = 0; i < NT / 64; ++i) {
    int t = s_wave[i];
    if (i < wid) base += t;
    tot += t;
  }
  wg_sync<LOCAL>();
  total = tot;
  return base + inc - v;
}

// The need-th smallest (1-based) of the values val(i, v) accepts, all known to lie in
// [lo, hi]: theta, with the number of accepted values below it and equal to it.  Exact:
// only integer histograms, refined until a bin is one value wide.
template <int NT, class F>
__device__ void block_select(LaneShared<NT> &S, int n, uint32_t need, uint32_t lo, uint32_t hi, F val,
                             uint32_t &theta, uint32_t &n_less, uint32_t &n_eq) {
  const int tid = threadIdx.x;
  constexpr int PER = NBINS / NT;
  uint32_t less = 0;
  for (;;) {
    int shift = 0;                           // bins of 2^shift values: the last value, hi, must fall into bin NBINS - 1 at most
    while ((((unsigned long long)hi - lo) >> shift) >= (unsigned long long)NBINS) ++shift;
    for (int b = tid; b < NBINS; b += NT) S.hist[b] = 0;
    __syncthreads();
    for (int i = tid; i < n; i += NT) {
      uint32_t v;
      if (val(i, v) && v >= lo && v <= hi) atomicAdd(&S.hist[(v - lo) >> shift], 1u);
    }
    __syncthreads();
    uint32_t loc[PER], sum = 0;
#pragma unroll
    for (int q = 0; q < PER; ++q) { loc[q] = S.hist[tid * PER + q]; sum += loc[q]; }
    int total;
    uint32_t run = (uint32_t)block_excl_scan<NT>((int)sum, S.wave_tmp, total);
#pragma unroll
    for (int q = 0; q < PER; ++q) {
      if (run < need && run + loc[q] >= need) { S.sel_bin = tid * PER + q; S.sel_below = run; S.sel_cnt = loc[q]; }
      run += loc[q];
    }
    __syncthreads();
    const uint32_t b = S.sel_bin, below = S.sel_below, cnt = S.sel_cnt;
    __syncthreads();
    less += below;
    need -= below;
    lo = lo + (b << shift);
    unsigned long long nhi = (unsigned long long)lo + ((1ull << shift) - 1);
    if (nhi < hi) hi = (uint32_t)nhi;
    if (shift == 0) { theta = lo; n_less = less; n_eq = cnt; return; }
  }
}

// One frame of one lane.  LDS: the state table lives in S.table (small frames), otherwise in
// the lane's global table.  Returns false (LDS mode only) if the frame outgrew the LDS table
// and must be redone with the global one; nothing has been committed in that case.
template <int NT, bool LDS>
__device__ bool lane_frame(const DecDev &D, LaneShared<NT> &S, const float *ll, bool is_init,
                           Slot *gslots, uint32_t *queue, Aux *aux, uint32_t *dkey, uint32_t *dslot,
                           long long *foff, HTok *hist, LatInt *lat) {
  const int tid = threadIdx.x;
  const uint32_t *rec = D.g.rec;
  Slot *slots = LDS ? S.table : gslots;
  const uint32_t mask = LDS ? (uint32_t)(LdsCfg<NT>::SLOTS - 1) : D.H - 1;
  const int hbits = LDS ? LdsCfg<NT>::HBITS : D.hbits;
  const Slot fresh{~0ull, EMPTY, A_FRESH};

  if (tid == 0) {
    S.qtail = 0; S.nclaim = 0; S.auxn = 0; S.best = KEY_NONE; S.flags = 0; S.nvalid = 0; S.nout = 0; S.latn = 0;
    S.kmin = 0xFFFFFFFFu; S.kmax = 0; S.emit_arcs = 0; S.eps_arcs = 0;
  }
  wg_sync<LDS>();
  const int nf = S.nf;                       // index of the frame being written
  const long long out_base = S.hist_used;
  int abort_code = 0;
  if (nf > D.max_frames) abort_code = E_HISTORY_OVERFLOW;

  // the frame's token queue: claimed slots, plus re-expansion requests for improved ones
  const uint32_t qcap = LDS ? (uint32_t)LdsCfg<NT>::QCAP : (uint32_t)D.qcap;
  auto qget = [&](uint32_t i, uint32_t &sl, bool &eps, bool &dup) {
    if (LDS) { const uint32_t e = S.lq[i]; sl = e & LQ_SLOT; eps = e & LQ_EPS; dup = e & LQ_DUP; }
    else { const uint32_t e = queue[i]; sl = e & Q_SLOT; eps = e & Q_EPS; dup = e & Q_DUP; }
  };
  auto on_claim = [&](int sl, uint32_t dw, bool dup) {
    // the lanes of the wave that call this together get consecutive queue entries and, those
    // that claimed a new state, consecutive claim numbers, from a single 64-bit atomic add
    const unsigned long long m_all = __ballot(1), m_new = __ballot(!dup);
    const int wl = threadIdx.x & 63, leader = __ffsll((long long)m_all) - 1;
    unsigned long long base = 0;
    if (wl == leader) base = atomicAdd(&S.claim_ctr, ((unsigned long long)__popcll(m_new) << 32) | (unsigned long long)__popcll(m_all));
    base = __shfl(base, leader, 64);
    const unsigned long long below = (1ull << wl) - 1ull;
    if (!dup) {
      const uint32_t ci = (uint32_t)(base >> 32) + (uint32_t)__popcll(m_new & below);
      if (ci >= (uint32_t)D.tokcap) atomicOr(&S.flags, F_TOKOVF);
      else if (LDS && ci >= (uint32_t)LdsCfg<NT>::CLAIM_LIMIT) atomicOr(&S.flags, F_RESTART);
    }
    const uint32_t q = (uint32_t)base + (uint32_t)__popcll(m_all & below);
    if (q >= qcap) atomicOr(&S.flags, LDS ? F_RESTART : F_TOKOVF);
    else if (LDS) S.lq[q] = (uint16_t)((uint32_t)sl | ((dw & HAS_EPS) ? LQ_EPS : 0u) | (dup ? LQ_DUP : 0u));
    else queue[q] = (uint32_t)sl | ((dw & HAS_EPS) ? Q_EPS : 0u) | (dup ? Q_DUP : 0u);
  };

  // ---- 1. emitting expansion ------------------------------------------------------------
  if (abort_code == 0) {
    if (is_init) {
      if (tid == 0) {
        const uint32_t h = D.g.start_handle;
        bool cl, im;
        const int sl = ht_insert<LDS>(slots, mask, hbits, h, pack(okey(0.0f), NO_ARC), cl, im);
        on_claim(sl, rec[3 * (size_t)h + 1] ? HAS_EPS : 0u, false);
        S.best = okey(0.0f);
      }
    } else {
      const long long in_off = S.in_off;
      const int n_in = S.n_in;
      // touch this frame's row of scores (one 64-byte line per thread) while the tokens'
      // graph records are being fetched, so that the gathers by pdf id below hit L2
      const float touch = tid * 16 < D.g.num_pdfs ? ll[tid * 16] : 0.f;
      float touch_more = 0.f;
      for (int p = (NT + tid) * 16; p < D.g.num_pdfs; p += NT * 16) touch_more += ll[p];
      // this thread's token of a tile: state handle, cost, emitting out-degree
      auto load_token = [&](int i, uint32_t &h, float &c, int &ne) {
        ne = 0; h = 0; c = 0.f;
        if (i < n_in) {
          const HTok t = hist[in_off + i];
          h = t.handle & HMASK; c = t.cost;
          ne = (int)rec[3 * (size_t)h];
        }
      };
      uint32_t h, hn = 0; float c, cn = 0.f; int ne, nen = 0;
      load_token(tid, h, c, ne);
      for (int tb = 0; tb < n_in; tb += NT) {
        int total;
        const int ex = block_excl_scan<NT, LDS>(ne, S.wave_tmp, total);
        S.scan[tid] = ex; S.cost[tid] = c; S.base[tid] = h + 1;
        wg_sync<LDS>();
        PHASE_MARK(8);
        if (tid == 0) S.emit_arcs += (unsigned long long)total;
        if (tb + NT < n_in) load_token(tb + NT + tid, hn, cn, nen);   // next tile, in flight during this one's rounds
        // one thread per arc (Section 3.3), EXP_U arcs of the tile per thread and round so
        // that their loads are in flight together
        for (int j0 = 0; j0 < total; j0 += NT * EXP_U) {
          float x[EXP_U], cw[EXP_U]; uint32_t r[EXP_U], dw[EXP_U], kx[EXP_U], pdf[EXP_U]; int kk[EXP_U];
#pragma unroll
          for (int u = 0; u < EXP_U; ++u) {
            const int j = j0 + u * NT + tid;
            kx[u] = KEY_NONE; kk[u] = -1; r[u] = 0; dw[u] = 0; pdf[u] = 0; cw[u] = 0.f; x[u] = 0.f;
            if (j < total) {
              int lo = 0, hi = NT - 1;             // largest k with scan[k] <= j
              while (lo < hi) { int mid = (lo + hi + 1) >> 1; if (S.scan[mid] <= j) lo = mid; else hi = mid - 1; }
              kk[u] = lo;
              r[u] = S.base[lo] + (uint32_t)(j - S.scan[lo]);
              const uint32_t *a = rec + 3 * (size_t)r[u];
              dw[u] = a[0];
              cw[u] = S.cost[lo] + __uint_as_float(a[1]);
              pdf[u] = a[2];
            }
          }
          uint32_t m = KEY_NONE;
#pragma unroll
          for (int u = 0; u < EXP_U; ++u) {
            if (kk[u] >= 0) {
              x[u] = cw[u] - ll[pdf[u]];
              if (x[u] != x[u] || x[u] == -INFINITY) atomicOr(&S.flags, F_NAN); else kx[u] = okey(x[u]);
              m = min(m, kx[u]);
            }
          }
#pragma unroll
          for (int d = 32; d; d >>= 1) m = min(m, (uint32_t)__shfl_xor((int)m, d, 64));
          if ((tid & 63) == 0 && m != KEY_NONE) atomicMin(&S.best, m);
          wg_sync<LDS>();
          PHASE_MARK(9);
          const float cut = key2f(S.best) + D.beam;     // running bound, never below the final cutoff
#pragma unroll
          for (int u = 0; u < EXP_U; ++u) {
            if (kx[u] == KEY_NONE || !(x[u] <= cut)) continue;
            bool cl, im;
            const int sl = ht_insert<LDS>(slots, mask, hbits, dw[u] & HMASK, pack(kx[u], r[u]), cl, im);
            if (sl < 0) { atomicOr(&S.flags, LDS ? F_RESTART : F_TOKOVF); continue; }
            if (cl) on_claim(sl, dw[u], false);
            if (D.lattice_on || im) {
              const uint32_t ai = wave_alloc(&S.auxn);
              if (ai >= (uint32_t)D.auxcap) atomicOr(&S.flags, F_LATOVF);
              else aux[ai] = Aux{(uint32_t)sl, x[u], r[u], (uint32_t)(tb + kk[u])};
            }
          }
        }
        wg_sync<LDS>();
        PHASE_MARK(10);
        h = hn; c = cn; ne = nen;
      }
      asm volatile("" ::"v"(touch), "v"(touch_more));
    }
  }
  wg_sync<LDS>();
  PHASE_MARK(0);
  const uint32_t bestk = S.best;
  if (abort_code == 0) {
    const uint32_t fl = S.flags;
    if (fl & F_NAN) abort_code = E_NAN_INPUT;
    else if (fl & F_TOKOVF) abort_code = E_TOKEN_OVERFLOW;
    else if (fl & F_LATOVF) abort_code = E_LATTICE_OVERFLOW;
    else if (bestk == KEY_NONE || bestk == KEY_PINF) abort_code = E_DEAD_CHANNEL;
  }
  const float cutoff = key2f(bestk) + D.beam;

  // ---- 2. non-emitting closure ----------------------------------------------------------
  // One epsilon arc of an expanded token: note it for the lattice stage on the token's first
  // expansion (source slot, weight, arc, destination), then offer the candidate.
  auto relax_eps = [&](uint32_t src_slot, float c, uint32_t r, uint32_t dw, float w, uint32_t note_at) {
    if (note_at < (uint32_t)D.auxcap) aux[note_at] = Aux{src_slot | AUX_EPS, w, r, dw & HMASK};
    const float x = c + w;
    if (!(x <= cutoff)) return;
    bool cl, im;
    const int sl = ht_insert<LDS>(slots, mask, hbits, dw & HMASK, pack(okey(x), r), cl, im);
    if (sl < 0) { atomicOr(&S.flags, LDS ? F_RESTART : F_TOKOVF); return; }
    if (cl || im) on_claim(sl, dw, !cl);
  };
  int iters = 0;
  if (abort_code == 0 && !(LDS && (S.flags & F_RESTART))) {
    uint32_t w0 = 0, w1 = min(S.qtail, qcap);
    wg_sync<LDS>();
    while (w0 < w1) {
      // every thread takes one queue entry of the window per pass; the pass is kept convergent
      // (predicated, no early exit) so that the wave can allot note space with one atomic
      for (uint32_t i0 = w0; i0 < w1; i0 += NT) {
        const uint32_t i = i0 + tid;
        bool act = false; uint32_t src = 0; float c = 0.f;
        uint32_t h = 0, ne = 0, np = 0; bool first = false;
        if (i < w1) {
          bool eps, dup;
          qget(i, src, eps, dup);
          if (eps) {
            const Slot sv = ld_slot<LDS>(&slots[src]);
            c = key2f((uint32_t)(sv.val >> 32)); act = c <= cutoff; h = sv.handle;
          }
        }
        if (act) {
          ne = rec[3 * (size_t)h]; np = rec[3 * (size_t)h + 1];
          first = atomicAnd(&slots[src].aux, ~A_FRESH) & A_FRESH;   // first expansion while within the cutoff
        }
        uint32_t dwv[EPS_U]; float wv[EPS_U];                        // the first arcs, loads in flight together
#pragma unroll
        for (int k = 0; k < EPS_U; ++k) {
          dwv[k] = 0; wv[k] = 0.f;
          if (act && (uint32_t)k < np) {
            const uint32_t *a = rec + 3 * (size_t)(h + 1 + ne + k);
            dwv[k] = a[0]; wv[k] = __uint_as_float(a[1]);
          }
        }
        // note space and the arc count, one atomic per wave
        const uint32_t nn = first ? np : 0u;
        uint32_t inc = nn;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) { const uint32_t t = (uint32_t)__shfl_up((int)inc, d, 64); if ((tid & 63) >= d) inc += t; }
        const uint32_t wave_total = (uint32_t)__shfl((int)inc, 63, 64);
        uint32_t note = 0;
        if ((tid & 63) == 0 && wave_total) {
          note = atomicAdd(&S.auxn, wave_total);
          atomicAdd(&S.eps_arcs, (unsigned long long)wave_total);
          if (note + wave_total > (uint32_t)D.auxcap) atomicOr(&S.flags, F_LATOVF);
        }
        note = (uint32_t)__shfl((int)note, 0, 64) + inc - nn;
#pragma unroll
        for (int k = 0; k < EPS_U; ++k)
          if (act && (uint32_t)k < np) relax_eps(src, c, h + 1 + ne + k, dwv[k], wv[k], first ? note + k : 0xFFFFFFFFu);
        for (uint32_t k = EPS_U; act && k < np; ++k) {
          const uint32_t *a = rec + 3 * (size_t)(h + 1 + ne + k);
          relax_eps(src, c, h + 1 + ne + k, a[0], __uint_as_float(a[1]), first ? note + k : 0xFFFFFFFFu);
        }
      }
      wg_sync<LDS>();
      PHASE_MARK(11);
      w0 = w1; w1 = min(S.qtail, qcap);
      ++iters;
      wg_sync<LDS>();
    }
    if (S.flags & F_TOKOVF) abort_code = E_TOKEN_OVERFLOW;
    else if (S.flags & F_LATOVF) abort_code = E_LATTICE_OVERFLOW;
  }
  PHASE_MARK(1);
  if (LDS) {
    wg_sync<true>();
    if (abort_code == 0 && (S.flags & F_RESTART)) {     // outgrew the LDS table: wipe it, redo with the global one
      for (int i = tid; i < LdsCfg<NT>::SLOTS; i += NT) slots[i] = fresh;
      __syncthreads();
      return false;
    }
  }
  const uint32_t n_q = min(S.qtail, qcap);
  auto token_slot = [&](uint32_t i, uint32_t &sl, uint32_t &eps) -> bool {
    bool e, dup;
    qget(i, sl, e, dup);
    eps = e;
    return !dup;
  };

  // ---- 3 + 4. max-active selection and contraction into the token history ---------------
  float cutoff_eff = cutoff;
  if (abort_code == 0) {
    const uint32_t nclaim = S.nclaim;
    const uint32_t room = (uint32_t)min((long long)0x7FFFFFFF, D.hist_cap - out_base);
    if (min(nclaim, (uint32_t)D.max_active) > room) abort_code = E_HISTORY_OVERFLOW;
    else if (nclaim <= (uint32_t)D.max_active) {
      // nothing can be pruned: every token within the beam is kept
      for (uint32_t i = tid; i < n_q; i += NT) {
        uint32_t sl, eps;
        if (!token_slot(i, sl, eps)) continue;
        Slot *sp = slots + sl;
        const Slot sv = ld_slot<LDS>(sp);
        const unsigned long long v = sv.val;
        const float c = key2f((uint32_t)(v >> 32));
        if (!(c <= cutoff)) continue;
        const uint32_t pos = wave_alloc(&S.nout);
        if (pos >= room) continue;
        hist[out_base + pos] = HTok{sv.handle | (eps ? HAS_EPS : 0u), c, (uint32_t)v, NO_ARC};
        sp->aux = pos;
      }
      wg_sync<LDS>();
      if (tid == 0) S.nvalid = S.nout;
    } else {
      for (uint32_t i = tid; i < n_q; i += NT) {
        uint32_t sl, eps;
        if (!token_slot(i, sl, eps)) continue;
        const uint32_t key = (uint32_t)(tl64<LDS>(&slots[sl].val) >> 32);
        if (!(key2f(key) <= cutoff)) continue;
        const uint32_t p = wave_alloc(&S.nvalid);
        dkey[p] = key; dslot[p] = sl | (eps ? Q_EPS : 0u);
        atomicMin(&S.kmin, key); atomicMax(&S.kmax, key);
      }
      __syncthreads();
      const int n = (int)S.nvalid;
      uint32_t theta = KEY_NONE, h_theta = 0xFFFFFFFFu;       // keep key < theta, or == theta with handle <= h_theta
      if (n > D.max_active) {
        uint32_t n_less, n_eq;
        block_select<NT>(S, n, (uint32_t)D.max_active, S.kmin, S.kmax,
                         [&](int i, uint32_t &v) { v = dkey[i]; return true; }, theta, n_less, n_eq);
        const uint32_t need_eq = (uint32_t)D.max_active - n_less;
        if (need_eq < n_eq) {
          uint32_t hl, he;
          block_select<NT>(S, n, need_eq, 0u, HMASK,
                           [&](int i, uint32_t &v) {
                             if (dkey[i] != theta) return false;
                             v = tl32<LDS>(&slots[dslot[i] & Q_SLOT].handle);
                             return true;
                           }, h_theta, hl, he);
        }
        cutoff_eff = key2f(theta);
      }
      for (int i = tid; i < n; i += NT) {
        const uint32_t key = dkey[i], ds = dslot[i];
        Slot *sp = slots + (ds & Q_SLOT);
        const uint32_t h = tl32<LDS>(&sp->handle);
        const bool keep = key < theta || (key == theta && h <= h_theta);
        uint32_t pos = 0xFFFFFFFFu;
        if (keep) pos = wave_alloc(&S.nout);
        if (pos < room) {
          hist[out_base + pos] = HTok{h | ((ds & Q_EPS) ? HAS_EPS : 0u), key2f(key), (uint32_t)tl64<LDS>(&sp->val), NO_ARC};
          sp->aux = pos;
        } else {
          sp->aux = 0xFFFFFFFFu;
        }
      }
    }
  }
  __syncthreads();
  PHASE_MARK(2);
  const uint32_t n_out = (abort_code == 0) ? min(S.nout, (uint32_t)D.max_active) : 0u;

  // ---- 5. lattice records and back-pointers ---------------------------------------------
  if (abort_code == 0) {
    const long long lat_base = S.lat_pos;
    const uint32_t n_aux = min(S.auxn, (uint32_t)D.auxcap);
    auto emit_lat = [&](uint32_t arc, float extra, uint32_t dst, uint32_t src) {
      const uint32_t p = wave_alloc(&S.latn);
      if ((long long)p >= S.lat_room) atomicOr(&S.flags, F_LATOVF);
      else {
        long long at = lat_base + (long long)p;
        if (at >= D.lat_cap) at -= D.lat_cap;
        lat[at] = LatInt{nf, arc, extra, dst, src};
      }
    };
    for (uint32_t i0 = 0; i0 < n_aux; i0 += NT * LAT_U) {
      Aux a[LAT_U];
#pragma unroll
      for (int u = 0; u < LAT_U; ++u) {
        const uint32_t i = i0 + u * NT + tid;
        a[u] = i < n_aux ? aux[i] : Aux{0xFFFFFFFFu, 0.f, 0u, 0u};
      }
#pragma unroll
      for (int u = 0; u < LAT_U; ++u) {
        if (a[u].slot == 0xFFFFFFFFu) continue;
        if (!(a[u].slot & AUX_EPS)) {
          // emitting candidate {slot of the destination, x, arc, index of the source token}
          const Slot sv = ld_slot<LDS>(slots + a[u].slot);
          const uint32_t pos = sv.aux;
          if (pos >= A_KEPT_MAX) continue;
          const unsigned long long v = sv.val;
          if (pack(okey(a[u].x), a[u].arc) == v) hist[out_base + pos].prev = a[u].src;
          if (D.lattice_on && a[u].x <= cutoff_eff) {
            const float extra = a[u].x - key2f((uint32_t)(v >> 32));
            if (extra <= D.lattice_beam) emit_lat(a[u].arc, extra, pos, a[u].src);
          }
        } else {
          // epsilon arc {slot of the source | AUX_EPS, weight, arc, handle of the destination}
          const Slot ssv = ld_slot<LDS>(slots + (a[u].slot & ~AUX_EPS));
          const uint32_t spos = ssv.aux;
          if (spos >= A_KEPT_MAX) continue;                        // the source token was not kept
          const float x = key2f((uint32_t)(ssv.val >> 32)) + a[u].x;
          if (!(x <= cutoff_eff)) continue;
          const int sl = ht_find<LDS>(slots, mask, hbits, a[u].src);
          if (sl < 0) continue;
          const Slot sv = ld_slot<LDS>(slots + sl);
          const uint32_t pos = sv.aux;
          if (pos >= A_KEPT_MAX) continue;
          const unsigned long long v = sv.val;
          if (pack(okey(x), a[u].arc) == v) hist[out_base + pos].prev = spos | PREV_SAME;
          if (D.lattice_on) {
            const float extra = x - key2f((uint32_t)(v >> 32));
            if (extra <= D.lattice_beam) emit_lat(a[u].arc, extra, pos, spos | PREV_SAME);
          }
        }
      }
    }
  }
  wg_sync<LDS>();
  PHASE_MARK(3);

  // ---- 6. clear the table ---------------------------------------------------------------
  if (S.flags & F_TOKOVF) {                                        // untracked claims: wipe everything
    const uint32_t n_all = LDS ? (uint32_t)LdsCfg<NT>::SLOTS : D.H;
    for (uint32_t i = tid; i < n_all; i += NT) slots[i] = fresh;
  } else {
    for (uint32_t i = tid; i < n_q; i += NT) {
      uint32_t sl, eps;
      if (token_slot(i, sl, eps)) slots[sl] = fresh;
    }
  }
  if (tid == 0) {
    if (abort_code == 0 && (S.flags & F_LATOVF)) abort_code = E_LATTICE_OVERFLOW;
    const long long lat_new = min((long long)S.latn, S.lat_room);
    if (nf <= D.max_frames) {
      foff[nf + 1] = out_base + n_out;
      S.nf = nf + 1;
      S.in_off = out_base; S.n_in = (int)n_out;      // the frame just written is what the next one expands
    }
    S.hist_used = out_base + n_out;
    S.lat_total += lat_new; S.lat_room -= lat_new;
    S.lat_pos += lat_new;
    if (S.lat_pos >= D.lat_cap) S.lat_pos -= D.lat_cap;
    S.arcs_expanded += (long long)(S.emit_arcs + S.eps_arcs);
    S.max_pre = max(S.max_pre, (int)S.nvalid);
    S.max_post = max(S.max_post, (int)n_out);
    S.iters_max = max(S.iters_max, iters);
#ifdef WFST_PHASE_TIMING
    S.ph[7] += iters; S.dbg_tok += n_out; S.dbg_iters += iters; S.dbg_arcs += S.emit_arcs + S.eps_arcs;
#endif
    if (abort_code != 0) S.status = abort_code;
  }
  wg_sync<LDS>();
  PHASE_MARK(4);
  return true;
}

// One workgroup per lane.  is_init: (re)start the lane's channel and write frame 0.
template <int NT>
__global__ void __launch_bounds__(NT, 4) k_advance(DecDev D, const LaneParam *__restrict__ lanes, int is_init) {
  __shared__ LaneShared<NT> S;
  const int tid = threadIdx.x;
  const LaneParam lp = lanes[blockIdx.x];
  ChanState *cs = D.chan + lp.chan;
  Slot *slots = D.slots + (size_t)blockIdx.x * D.H;
  uint32_t *queue = D.queue + (size_t)blockIdx.x * (size_t)D.qcap;
  Aux *aux = D.aux + (size_t)blockIdx.x * (size_t)D.auxcap;
  uint32_t *dkey = D.dkey + (size_t)blockIdx.x * (size_t)D.tokcap;
  uint32_t *dslot = D.dslot + (size_t)blockIdx.x * (size_t)D.tokcap;
  long long *foff = D.frame_off + (size_t)lp.chan * (size_t)(D.max_frames + 2);
  HTok *hist = D.hist + (size_t)lp.chan * (size_t)D.hist_cap;
  LatInt *lat = D.lat + (size_t)lp.chan * (size_t)D.lat_cap;

  const Slot fresh{~0ull, EMPTY, A_FRESH};
  for (int i = tid; i < LdsCfg<NT>::SLOTS; i += NT) S.table[i] = fresh;
  if (tid == 0) {
    if (is_init) {
      S.status = 0; S.nf = 0; S.hist_used = 0; S.lat_room = D.lat_cap; S.lat_pos = 0; S.lat_total = 0; S.arcs_expanded = 0;
      S.lat_head = 0; S.lat_head_pos = 0;
      S.max_pre = 0; S.max_post = 0; S.iters_max = 0;
      foff[0] = 0;
    } else {
      S.status = cs->status; S.nf = cs->num_frames; S.hist_used = cs->hist_used;
      S.lat_head = cs->lat_head;
      S.lat_room = D.lat_cap - (cs->lat_total - S.lat_head);
      S.lat_pos = cs->lat_total % D.lat_cap;
      S.lat_head_pos = S.lat_head % D.lat_cap;
      S.lat_total = cs->lat_total; S.arcs_expanded = cs->arcs_expanded; S.max_pre = cs->max_pre;
      S.max_post = cs->max_post; S.iters_max = cs->closure_iters_max;
    }
    S.in_off = 0; S.n_in = 0;
    if (!is_init && S.nf >= 1 && S.nf <= D.max_frames + 1) { S.in_off = foff[S.nf - 1]; S.n_in = (int)(foff[S.nf] - foff[S.nf - 1]); }
#ifdef WFST_PHASE_TIMING
    for (int k = 0; k < 16; ++k) S.ph[k] = 0;
    S.dbg_tok = 0; S.dbg_iters = 0; S.dbg_arcs = 0;
    S.tlast = wall_clock64();
#endif
  }
  __syncthreads();
  // Seal the lane's state as the next snapshot of this call.  With snapshot blocks the lattice
  // records not handed out yet move into the snapshot's block, in the caller's form (the lane
  // reserves its range with one compare-and-swap; the ring is empty afterwards).  Then
  // everything the workgroup has written is made visible to the whole system, then the
  // snapshot entry and the lane's progress word.  Readouts of the snapshot start only after
  // the host has seen the progress words of all lanes, so nothing ever waits inside a kernel.
  int n_sealed = 0;
  auto seal = [&]() {
    __syncthreads();                                  // all waves' stores have been issued and acknowledged
    const long long id = lp.snap_id0 + n_sealed;
    long long blk_start = 0, blk_count = 0;
    if (D.n_blk > 0 && D.lattice_on) {
      const int slot = (int)(id % D.n_blk);
      const long long n = S.lat_total - S.lat_head;
      if (tid == 0) {
        unsigned long long *used = &D.blk[slot].used;
        unsigned long long old = ld64(used);
        long long pos = -1;
        while ((long long)old + n <= D.blk_cap) {     // every failed swap means another lane got its range
          const unsigned long long seen = atomicCAS(used, old, old + (unsigned long long)n);
          if (seen == old) { pos = (long long)old; break; }
          old = seen;
        }
        if (pos < 0 && S.status == 0) S.status = E_LATTICE_OVERFLOW;
        S.blk_pos = pos;
      }
      __syncthreads();
      const long long pos = S.blk_pos;
      if (pos >= 0) {
        LatRec *out = D.blk_recs + (size_t)slot * (size_t)D.blk_cap + (size_t)pos;
        const long long first = S.lat_head_pos;
        constexpr int U = 8;                            // records per thread in flight: the arc-id gathers are HBM round trips
        for (long long i0 = tid; i0 < n; i0 += (long long)NT * U) {
          LatInt r[U];
          uint32_t arc_id[U];
          // loads are unconditional (a lane past the end re-reads the last record) so that all of a
          // round's loads, and then all its gathers, are in flight together
#pragma unroll
          for (int u = 0; u < U; ++u) {
            const long long i = min(i0 + (long long)u * NT, n - 1);
            r[u] = lat[first + i < D.lat_cap ? first + i : first + i - D.lat_cap];
          }
#pragma unroll
          for (int u = 0; u < U; ++u) arc_id[u] = D.g.orig[r[u].arc];
#pragma unroll
          for (int u = 0; u < U; ++u) {
            const long long i = i0 + (long long)u * NT;
            if (i < n) out[i] = LatRec{r[u].frame, arc_id[u], r[u].extra};
          }
        }
        blk_start = pos; blk_count = n;
      }
      __syncthreads();
      if (tid == 0) { S.lat_head = S.lat_total; S.lat_head_pos = S.lat_pos; S.lat_room = D.lat_cap; }
    }
    if (tid == 0) {
      ChanSnap *sp = D.snap + (size_t)lp.chan * SNAP_RING + (size_t)(id % SNAP_RING);
      sp->lat_total = S.lat_total; sp->hist_used = S.hist_used; sp->status = S.status; sp->num_frames = S.nf;
      sp->blk_start = blk_start; sp->blk_count = blk_count;
      sp->id = id;
      __hip_atomic_store(D.lane_sealed + blockIdx.x, id, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
    }
    ++n_sealed;
  };
  const int nframes = is_init ? 1 : lp.n_frames;
  const int n_snaps = is_init ? 0 : lp.n_snaps;
  int until_seal = (!is_init && lp.snap_every > 0) ? lp.snap_every : 0x7FFFFFFF;
  for (int f = 0;;) {
    const bool more = f < nframes && S.status == 0;
    if (more) {
      const float *ll = is_init ? nullptr : lp.ll + (size_t)f * (size_t)lp.stride;
      bool small = is_init != 0;
      if (!small) small = S.n_in <= LdsCfg<NT>::NIN_MAX;
      bool done = false;
      if (small) done = lane_frame<NT, true>(D, S, ll, is_init != 0, slots, queue, aux, dkey, dslot, foff, hist, lat);
      if (!done) {
#ifdef WFST_PHASE_TIMING
        if (tid == 0 && small) S.ph[6] += 1;
#endif
        lane_frame<NT, false>(D, S, ll, is_init != 0, slots, queue, aux, dkey, dslot, foff, hist, lat);
      }
#ifdef WFST_PHASE_TIMING
      if (tid == 0) S.ph[5] += 1;
#endif
      ++f;
      if (--until_seal != 0) continue;
      until_seal = lp.snap_every;
    }
    // a snapshot boundary - or the lane has run out of frames or stopped: it seals the
    // snapshots still due in the state it is in
    if (n_sealed >= n_snaps) { if (more) continue; break; }
    seal();
    PHASE_MARK(12);
  }
  __syncthreads();
  if (tid == 0) {
    cs->status = S.status; cs->num_frames = S.nf; cs->hist_used = S.hist_used;
    cs->lat_total = S.lat_total; cs->arcs_expanded = S.arcs_expanded; cs->max_pre = S.max_pre;
    cs->max_post = S.max_post; cs->closure_iters_max = S.iters_max;
    if (is_init) cs->path_nf = 0;
    cs->lat_head = S.lat_head;
#ifdef WFST_PHASE_TIMING
    if (D.dbg) {
      for (int k = 0; k < 8; ++k) atomicAdd(D.dbg + k, S.ph[k]);
      for (int k = 8; k < 16; ++k) atomicAdd(D.dbg + 8 + 8000 + k, S.ph[k]);
      unsigned long long tot = 0;
      for (int k = 0; k < 5; ++k) tot += S.ph[k];
      for (int k = 8; k < 16; ++k) tot += S.ph[k];
      D.dbg[8 + blockIdx.x] = tot;                      // this lane's time for the call
      if (blockIdx.x < 512) for (int k = 0; k < 16; ++k) D.dbg[8 + 8192 + blockIdx.x * 16 + k] = S.ph[k];
      D.dbg[8 + 2048 + blockIdx.x] = S.dbg_tok;
      D.dbg[8 + 4096 + blockIdx.x] = S.dbg_iters;
      D.dbg[8 + 6144 + blockIdx.x] = S.dbg_arcs;
    }
#endif
  }
}

__global__ void k_fill_slots(Slot *slots, size_t n) {
  const Slot fresh{~0ull, EMPTY, A_FRESH};
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) slots[i] = fresh;
}

// ---- readouts ----------------------------------------------------------------------------
struct PathOut { int32_t status, n_words, n_arcs, reached_final; float total_cost; int32_t pad; long long word_off; };

// Arg-min over the last frame of a channel by the whole wave: packed (ordered cost, handle)
// minimum over all tokens and, if asked for, over tokens in final states (cost + final cost).
// Returns false if the channel has an error or no token; lane 0 gets the start of the walk.
// The channel's state as the readouts see it: live, or as sealed in snapshot `snap_id` (> 0).
struct ChanView { int status, num_frames; long long hist_used, lat_total; };
__device__ __forceinline__ ChanView chan_view(const DecDev &D, int ch, long long snap_id) {
  if (snap_id <= 0) {
    const ChanState *cs = D.chan + ch;
    return ChanView{cs->status, cs->num_frames, cs->hist_used, cs->lat_total};
  }
  const ChanSnap *sp = D.snap + (size_t)ch * SNAP_RING + (size_t)(snap_id % SNAP_RING);
  if (sp->id != snap_id) return ChanView{E_NOT_INIT, 0, 0, 0};     // the channel has no such snapshot (any more)
  return ChanView{sp->status, sp->num_frames, sp->hist_used, sp->lat_total};
}

// W threads work on one channel (a whole wave, or a single thread).
template <int W>
__device__ __forceinline__ bool path_start(const DecDev &D, int ch, int use_final, const ChanView &cv, PathOut &po, int &F, int &cur) {
  const int lane = threadIdx.x % W;
  const long long *foff = D.frame_off + (size_t)ch * (size_t)(D.max_frames + 2);
  const HTok *hist = D.hist + (size_t)ch * (size_t)D.hist_cap;
  const uint32_t *rec = D.g.rec;
  if (cv.status != 0) { po.status = cv.status; return false; }
  F = cv.num_frames - 1;
  if (F < 0) { po.status = E_NOT_INIT; return false; }
  const long long o = foff[F];
  const int n = (int)(foff[F + 1] - o);
  unsigned long long bf = ~0ull, bn = ~0ull; int bfi = -1, bni = -1;
  for (int i = lane; i < n; i += W) {
    const HTok t = hist[o + i];
    const uint32_t h = t.handle & HMASK;
    const unsigned long long kn = pack(okey(t.cost), h);
    if (kn < bn) { bn = kn; bni = i; }
    if (use_final) {
      const float fc = __uint_as_float(rec[3 * (size_t)h + 2]);
      if (fc != INFINITY) {
        const unsigned long long kf = pack(okey(t.cost + fc), h);
        if (kf < bf) { bf = kf; bfi = i; }
      }
    }
  }
  for (int d = W / 2; d; d >>= 1) {
    unsigned long long o2 = __shfl_xor(bn, d, 64); int i2 = __shfl_xor(bni, d, 64);
    if (o2 < bn) { bn = o2; bni = i2; }
    o2 = __shfl_xor(bf, d, 64); i2 = __shfl_xor(bfi, d, 64);
    if (o2 < bf) { bf = o2; bfi = i2; }
  }
  if (n == 0) { po.status = E_DEAD_CHANNEL; return false; }
  if (use_final && bfi >= 0) { cur = bfi; po.total_cost = key2f((uint32_t)(bf >> 32)); po.reached_final = 1; }
  else { cur = bni; po.total_cost = key2f((uint32_t)(bn >> 32)); }
  return true;
}

// Best path of one channel with its arcs (one wave; lane 0 follows the back-pointers over the
// whole utterance).  Words / arcs are written right-aligned into cap-sized regions, so a
// single backward walk leaves them in path order.
__global__ void __launch_bounds__(64) k_best_path(DecDev D, const int32_t *chans, int use_final, long long snap_id,
                                                  int32_t *words, int words_cap, uint32_t *arcs, int arcs_cap,
                                                  PathOut *out) {
  const int ch = chans[blockIdx.x];
  const long long *foff = D.frame_off + (size_t)ch * (size_t)(D.max_frames + 2);
  const HTok *hist = D.hist + (size_t)ch * (size_t)D.hist_cap;
  PathOut po{0, 0, 0, 0, 0.f, 0, 0};
  int F = 0, cur = 0;
  const ChanView cv = chan_view(D, ch, snap_id);
  const bool ok = path_start<64>(D, ch, use_final, cv, po, F, cur);
  if (threadIdx.x != 0) return;
  if (!ok) { out[blockIdx.x] = po; return; }
  int32_t *wout = words ? words + (size_t)blockIdx.x * words_cap : nullptr;
  uint32_t *aout = arcs ? arcs + (size_t)blockIdx.x * arcs_cap : nullptr;
  int f = F, nw = 0, na = 0;
  const long long max_steps = cv.hist_used + 1;
  for (long long step = 0;; ++step) {
    if (cur < 0 || (long long)cur >= foff[f + 1] - foff[f]) { po.status = E_BROKEN_TRACE; break; }
    const HTok t = hist[foff[f] + cur];
    if (t.in_arc == NO_ARC) break;
    if (t.prev == NO_ARC || step > max_steps) { po.status = E_BROKEN_TRACE; break; }
    if (aout && na < arcs_cap) aout[arcs_cap - 1 - na] = D.g.orig[t.in_arc];
    ++na;
    const int32_t w = D.g.label[t.in_arc];
    if (w != 0) { if (wout && nw < words_cap) wout[words_cap - 1 - nw] = w; ++nw; }
    if (t.prev & PREV_SAME) cur = (int)(t.prev & ~PREV_SAME);
    else { cur = (int)t.prev; --f; if (f < 0) { po.status = E_BROKEN_TRACE; break; } }
  }
  po.n_words = nw; po.n_arcs = na;
  if (po.status == 0 && ((wout && nw > words_cap) || (aout && na > arcs_cap))) po.status = E_CAPACITY;
  out[blockIdx.x] = po;
}

// Best-path words of many channels (one wave each).  Back-pointers are unique, so two best
// paths that share a token share everything before it: each channel remembers, per frame,
// the token through which its last traced path entered the frame and the words up to there;
// a new trace walks back only until it meets the remembered path (a chunk of frames plus the
// distance to the merge point, not the whole utterance) and splices the remembered prefix.
// Words of all channels are packed into `words` at po.word_off (allotted with one atomic add).
// W = 64: one wave per channel (fastest when the GPU is otherwise idle).  W = 1: one thread
// per channel, eight waves for 500 channels, which still find room beside a running decode
// kernel whose workgroups hold nearly all wave slots.
template <int W>
__global__ void __launch_bounds__(64) k_best_path_words(DecDev D, const int32_t *chans, int n_ch, int use_final, long long snap_id,
                                                        int32_t *words, int words_cap, unsigned long long *words_used, PathOut *out) {
  const int gi = (int)((blockIdx.x * blockDim.x + threadIdx.x) / W);      // channel of this thread group
  if (gi >= n_ch) return;                                                // (W = 64: one group per block)
  const int ch = chans[gi];
  const int lane = threadIdx.x % W;
  ChanState *cs = D.chan + ch;
  const long long *foff = D.frame_off + (size_t)ch * (size_t)(D.max_frames + 2);
  const HTok *hist = D.hist + (size_t)ch * (size_t)D.hist_cap;
  int32_t *entry = D.pc_entry + (size_t)ch * (size_t)(D.max_frames + 2);
  int32_t *wcount = D.pc_wcount + (size_t)ch * (size_t)(D.max_frames + 2);
  int32_t *cw = D.pc_words + (size_t)ch * (size_t)D.pc_wcap;
  __shared__ int sh[4];                      // status, total words, merge frame, new words (W > 1)
  __shared__ long long sh_off;
  PathOut po{0, 0, 0, 0, 0.f, 0, 0};
  int F = 0, cur = 0;
  const ChanView cv = chan_view(D, ch, snap_id);
  const bool ok = path_start<W>(D, ch, use_final, cv, po, F, cur);
  if (!ok) { if (lane == 0) out[gi] = po; return; }
  int status = 0, total = 0, merge_f = 0, k = 0;
  if (lane == 0) {
    const int cached_nf = cs->path_nf;
    int f = F, base = 0;
    const long long max_steps = cv.hist_used + 1;
    // the token of the next step is fetched while this step's word label is still on its way
    auto in_frame = [&](int ff, int c) { return ff >= 0 && c >= 0 && (long long)c < foff[ff + 1] - foff[ff]; };
    HTok t{};
    if (!in_frame(f, cur)) status = E_BROKEN_TRACE; else t = hist[foff[f] + cur];
    for (long long step = 0; status == 0; ++step) {
      if (t.in_arc == NO_ARC) break;
      if (t.prev == NO_ARC || step > max_steps) { status = E_BROKEN_TRACE; break; }
      const bool is_entry = !(t.prev & PREV_SAME);
      if (is_entry) {
        if (f < cached_nf && entry[f] == cur) { base = wcount[f]; merge_f = f; break; }
        entry[f] = cur; wcount[f] = k;        // k: words found so far, all later on the path; fixed up below
      }
      const int32_t w = D.g.label[t.in_arc];
      const int ncur = is_entry ? (int)t.prev : (int)(t.prev & ~PREV_SAME);
      const int nf = is_entry ? f - 1 : f;
      HTok tn{};
      const bool ok2 = in_frame(nf, ncur);
      if (ok2) tn = hist[foff[nf] + ncur];
      if (w != 0) {
        if (k < D.pc_wcap) cw[D.pc_wcap - 1 - k] = w;
        ++k;
      }
      if (!ok2) { status = E_BROKEN_TRACE; break; }
      cur = ncur; f = nf; t = tn;
    }
    if (status == 0 && (long long)base + 2ll * k > (long long)D.pc_wcap) status = E_CAPACITY;
    total = base + k;
  }
  if constexpr (W > 1) {
    if (lane == 0) { sh[0] = status; sh[1] = total; sh[2] = merge_f; sh[3] = k; }
    __syncthreads();
    status = sh[0]; total = sh[1]; merge_f = sh[2]; k = sh[3];
  }
  if (status != 0) {
    if (lane == 0) { cs->path_nf = 0; po.status = status; po.n_words = total; out[gi] = po; }
    return;
  }
  for (int f = merge_f + 1 + lane; f <= F; f += W) wcount[f] = total - wcount[f];
  const int base = total - k;
  for (int j = lane; j < k; j += W) cw[base + j] = cw[D.pc_wcap - k + j];
  if constexpr (W > 1) __syncthreads();
  long long off = 0;
  if (lane == 0) {
    cs->path_nf = F + 1;
    po.n_words = total;
    if (total > words_cap) po.status = E_CAPACITY;
    else po.word_off = (long long)atomicAdd(words_used, (unsigned long long)total);
    off = po.word_off;
    out[gi] = po;
  }
  if constexpr (W > 1) {
    if (lane == 0) { sh[0] = po.status; sh_off = off; }
    __syncthreads();
    po.status = sh[0]; off = sh_off;
  }
  if (po.status != 0) return;
  for (int j = lane; j < total; j += W) words[off + j] = cw[j];
}

// Tokens of one frame in the public form: state id and caller's arc id.
struct TokOut { int32_t state; float cost; uint32_t in_arc; };
__global__ void k_export_tokens(DecDev D, int ch, long long off, int n, TokOut *out) {
  const HTok *hist = D.hist + (size_t)ch * (size_t)D.hist_cap;
  for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) {
    const HTok t = hist[off + i];
    out[i] = TokOut{D.g.label[t.handle & HMASK], t.cost, t.in_arc == NO_ARC ? NO_ARC : D.g.orig[t.in_arc]};
  }
}

// Lattice records with frame >= from_frame, arc ids translated to the caller's; cnt is
// the running output count (zeroed by the host).
// (the n records start at ring position `start`)
__global__ void k_export_lattice(DecDev D, int ch, long long start, long long n, int from_frame, LatRec *out, long long cap,
                                 unsigned long long *cnt) {
  const LatInt *lat = D.lat + (size_t)ch * (size_t)D.lat_cap;
  for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (long long)gridDim.x * blockDim.x) {
    const LatInt r = lat[start + i < D.lat_cap ? start + i : start + i - D.lat_cap];
    if (r.frame < from_frame) continue;
    const unsigned long long p = atomicAdd(cnt, 1ull);
    if ((long long)p < cap) out[p] = LatRec{r.frame, D.g.orig[r.arc], r.extra};
  }
}
// Records a live drain hands out.  A channel stopped by an overflow hands out nothing.
__device__ __forceinline__ long long lattice_pending(const DecDev &D, int ch) {
  const ChanState *cs = D.chan + ch;
  const bool readable = cs->status == 0 || cs->status == E_DEAD_CHANNEL || cs->status == E_NAN_INPUT;
  return readable ? cs->lat_total - cs->lat_head : 0;
}
__global__ void k_reset_lattice(DecDev D, int ch) { D.chan[ch].lat_head = D.chan[ch].lat_total; }

// Batched drain: counts of the listed channels, then one copy kernel (grid.x = channel,
// grid.y = slices of that channel's buffer), then the reset.
// offs[0..n]: exclusive prefix sums of the buffered record counts of the listed channels
// (channels stopped by an overflow count as empty).  One block.
__global__ void __launch_bounds__(1024) k_lattice_offsets(DecDev D, const int32_t *chans, int n, long long *offs) {
  __shared__ long long part[1024];
  const int tid = threadIdx.x;
  const int per = (n + 1023) / 1024;
  const int b = tid * per, e = min(n, b + per);
  long long sum = 0;
  for (int i = b; i < e; ++i) {
    sum += lattice_pending(D, chans[i]);
  }
  part[tid] = sum;
  __syncthreads();
  for (int d = 1; d < 1024; d <<= 1) {
    const long long v = tid >= d ? part[tid - d] : 0;
    __syncthreads();
    part[tid] += v;
    __syncthreads();
  }
  long long run = part[tid] - sum;
  for (int i = b; i < e; ++i) {
    offs[i] = run;
    run += lattice_pending(D, chans[i]);
  }
  if (tid == 1023) offs[n] = part[1023];
}
__global__ void k_export_lattice_batch(DecDev D, const int32_t *chans, int n_ch, const long long *offs, LatRec *out, long long cap) {
  if (offs[n_ch] > cap) return;                       // caller's buffer too small: nothing is copied or drained
  const int ch = chans[blockIdx.x];
  const LatInt *lat = D.lat + (size_t)ch * (size_t)D.lat_cap;
  const long long o = offs[blockIdx.x], n = offs[blockIdx.x + 1] - o;
  if (n <= 0) return;
  const long long start = D.chan[ch].lat_head % D.lat_cap;
  for (long long i = (long long)blockIdx.y * blockDim.x + threadIdx.x; i < n; i += (long long)gridDim.y * blockDim.x) {
    const LatInt r = lat[start + i < D.lat_cap ? start + i : start + i - D.lat_cap];
    out[o + i] = LatRec{r.frame, D.g.orig[r.arc], r.extra};
  }
}
__global__ void k_reset_lattice_batch(DecDev D, const int32_t *chans, int n, const long long *offs, long long cap) {
  if (offs[n] > cap) return;
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) D.chan[chans[i]].lat_head += offs[i + 1] - offs[i];
}

// Snapshot blocks: the slots of a call's snapshots are emptied before its lanes start.
__global__ void k_reset_blocks(DecDev D, long long id0, int n) {
  const int j = blockIdx.x * blockDim.x + threadIdx.x;
  if (j < n) D.blk[(id0 + j) % D.n_blk] = SnapBlock{0ull, id0 + j};
}
// Where each listed channel's lattice records sit in the block of snapshot `id`:
// out[2i] = start, out[2i+1] = count (0, 0 for a channel without that snapshot);
// out[2n] = records in the block, all lanes together.
__global__ void k_snapshot_ranges(DecDev D, const int32_t *chans, int n, long long id, long long *out) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) {
    const ChanSnap *sp = D.snap + (size_t)chans[i] * SNAP_RING + (size_t)(id % SNAP_RING);
    const bool have = sp->id == id;
    out[2 * i] = have ? sp->blk_start : 0;
    out[2 * i + 1] = have ? sp->blk_count : 0;
  }
  if (i == 0) {
    const SnapBlock b = D.blk[id % D.n_blk];
    out[2 * n] = b.id == id ? (long long)b.used : -1;
  }
}

// ---- final lattice -------------------------------------------------------------------------
// Backward pruning of a channel's buffered lattice arcs with the lattice beam (the paper's
// Section 3.4 leaves this to the end of the utterance).  te(n), the extra cost of token n, is
// the minimum over recorded arcs a: n -> m of te(m) + extra(a); in the last frame it is the
// token's distance to the best (final) cost.  An arc into m is kept iff te(m) + extra(a) <=
// lattice_beam.  fp32, one rounded add per step; minima via integer atomics on the (non-
// negative) float bits, so the result does not depend on thread order.  One workgroup.
struct LatticeInfoDev { long long arcs_in, arcs_kept; int32_t frames, reached_final, status, pad; float best_cost, pad2; };

__global__ void __launch_bounds__(1024) k_final_lattice(DecDev D, int ch, int use_final, uint32_t *te, long long *rec_start,
                                                        LatRec *out, long long cap, LatticeInfoDev *info) {
  const int tid = threadIdx.x, NTH = 1024;
  const ChanState *cs = D.chan + ch;
  const long long *foff = D.frame_off + (size_t)ch * (size_t)(D.max_frames + 2);
  const HTok *hist = D.hist + (size_t)ch * (size_t)D.hist_cap;
  const LatInt *lat_ring = D.lat + (size_t)ch * (size_t)D.lat_cap;
  const long long lat_first = cs->lat_head % D.lat_cap, lat_cap = D.lat_cap;
  // record i of the buffered ones (they start at ring position lat_first)
  auto lat = [&](long long i) -> const LatInt & { return lat_ring[lat_first + i < lat_cap ? lat_first + i : lat_first + i - lat_cap]; };
  const uint32_t *rec = D.g.rec;
  __shared__ uint32_t s_best_f, s_best_n, s_changed;
  __shared__ unsigned long long s_kept;
  const int st = cs->status;
  const bool readable = st == 0;
  const int T = cs->num_frames - 1;
  const long long n_rec = cs->lat_total - cs->lat_head;
  const long long n_tok = cs->hist_used;
  const long long oT = T >= 0 ? foff[T] : 0;
  const int nT = T >= 0 ? (int)(foff[T + 1] - oT) : 0;
  if (!readable || nT == 0) {
    if (tid == 0) { LatticeInfoDev li{n_rec, 0, T + 1, 0, readable ? E_DEAD_CHANNEL : st, 0, 0.f, 0.f}; *info = li; }
    return;
  }
  if (tid == 0) { s_best_f = KEY_NONE; s_best_n = KEY_NONE; s_kept = 0; }
  for (long long i = tid; i < n_tok; i += NTH) te[i] = 0x7F800000u;            // +inf
  for (int f = tid; f <= T + 2; f += NTH) rec_start[f] = f > T ? n_rec : -1;
  __syncthreads();
  // start of each frame's run of records (records are appended frame by frame)
  for (long long i = tid; i < n_rec; i += NTH) {
    const int f = lat(i).frame;
    if (i == 0 || lat(i - 1).frame != f) rec_start[f] = i;
  }
  // best cost over the last frame
  for (int i = tid; i < nT; i += NTH) {
    const HTok t = hist[oT + i];
    atomicMin(&s_best_n, okey(t.cost));
    if (use_final) {
      const float fc = __uint_as_float(rec[3 * (size_t)(t.handle & HMASK) + 2]);
      if (fc != INFINITY) atomicMin(&s_best_f, okey(t.cost + fc));
    }
  }
  __syncthreads();
  if (tid == 0) {                                   // frames without records inherit the next start
    long long nxt = n_rec;
    for (int f = T; f >= 0; --f) { if (rec_start[f] < 0) rec_start[f] = nxt; else nxt = rec_start[f]; }
  }
  const bool any_final = use_final && s_best_f != KEY_NONE;
  const float best = key2f(any_final ? s_best_f : s_best_n);
  for (int i = tid; i < nT; i += NTH) {
    const HTok t = hist[oT + i];
    float v;
    if (any_final) {
      const float fc = __uint_as_float(rec[3 * (size_t)(t.handle & HMASK) + 2]);
      v = fc != INFINITY ? (t.cost + fc) - best : INFINITY;
    } else {
      v = t.cost - best;
    }
    te[oT + i] = __float_as_uint(v);
  }
  __syncthreads();
  for (int f = T; f >= 0; --f) {
    const long long of = foff[f];
    if (f < T) {                                    // emitting arcs recorded with frame f + 1 start in frame f
      const long long of1 = foff[f + 1];
      for (long long i = rec_start[f + 1] + tid; i < rec_start[f + 2]; i += NTH) {
        const LatInt r = lat(i);
        if (r.src & PREV_SAME) continue;
        const float v = __uint_as_float(ld32(&te[of1 + r.dst])) + r.extra;
        atomicMin(&te[of + r.src], __float_as_uint(v));
      }
      __syncthreads();
    }
    const long long e0 = rec_start[f], e1 = rec_start[f + 1];
    for (;;) {                                      // epsilon arcs inside frame f, to the fixed point
      if (tid == 0) s_changed = 0;
      __syncthreads();
      for (long long i = e0 + tid; i < e1; i += NTH) {
        const LatInt r = lat(i);
        if (!(r.src & PREV_SAME)) continue;
        const uint32_t v = __float_as_uint(__uint_as_float(ld32(&te[of + r.dst])) + r.extra);
        if (v < atomicMin(&te[of + (r.src & ~PREV_SAME)], v)) s_changed = 1;
      }
      __syncthreads();
      if (!s_changed) break;
      __syncthreads();
    }
  }
  for (long long i = tid; i < n_rec; i += NTH) {
    const LatInt r = lat(i);
    const float v = __uint_as_float(ld32(&te[foff[r.frame] + r.dst])) + r.extra;
    if (v <= D.lattice_beam) {
      const unsigned long long p = atomicAdd(&s_kept, 1ull);
      if ((long long)p < cap) out[p] = LatRec{r.frame, D.g.orig[r.arc], r.extra};
    }
  }
  __syncthreads();
  if (tid == 0) {
    LatticeInfoDev li{n_rec, (long long)s_kept, T + 1, any_final ? 1 : 0, 0, 0, best, 0.f};
    if ((long long)s_kept > cap) li.status = E_CAPACITY;
    *info = li;
  }
}

}  // namespace wfst
