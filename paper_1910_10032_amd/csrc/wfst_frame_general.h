// The general form of a lane's frame (any size, any graph).
#pragma once
#include "wfst_lane.h"

namespace wfst {

// Several workgroups on one lane (Section 3.1: a batch too small to fill the device is bound by
// latency; Section 3.3: the persistent kernel): workgroup g of the lane's G takes every G-th
// tile of tokens, window of queue entries and block of notes; the frame's counters and the
// selection's histogram live in global memory (WideLane), and where one workgroup would pass a
// workgroup barrier the lane's workgroups meet at a lane barrier: each makes its stores visible
// device-wide, counts itself in, and waits (a bounded number of polls) until all have.
struct WideCtx {
  int g, G;                    // this workgroup's number among the lane's, and how many there are
  WideLane *wl;
  unsigned long long epoch;    // arrivals expected at the next barrier (thread 0 keeps count)
  unsigned spin_limit;
};
constexpr unsigned WIDE_SPIN_LIMIT = 1u << 22;      // default number of polls before a barrier is given up (seconds)

// Returns false (to every thread of the workgroup) if a barrier of the lane was given up: the
// workgroup must then stop working on the lane (what it would read may be incomplete).
template <int NT>
__device__ __forceinline__ bool lane_sync(WideCtx &W, LaneShared<NT> &S) {
  __syncthreads();                                  // every wave's stores have been acknowledged
  if (threadIdx.x == 0) {
    W.epoch += (unsigned long long)W.G;
    bool ok = !ld32(&W.wl->broken);
    if (ok) {
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
      atomicAdd(&W.wl->arrived, 1ull);
      unsigned spins = 0;
      while (ld64(&W.wl->arrived) < W.epoch) {
        if (++spins > W.spin_limit || ld32(&W.wl->broken)) { atomicExch(&W.wl->broken, 1u); ok = false; break; }
        __builtin_amdgcn_s_sleep(4);
      }
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    }
    S.wide_ok = ok ? 1u : 0u;
  }
  __syncthreads();
  return S.wide_ok != 0;
}

// The exact selection by all workgroups of a lane together (see block_select); every workgroup
// arrives at the same result.  Each workgroup counts its share in LDS and adds the bins it
// filled to the pass's histogram in global memory.  Passes rotate through three histograms, so
// that one lane barrier per pass is enough: pass p counts into histogram p % 3 (zero since pass
// p - 1 at the latest), the barrier, then every workgroup reads it and zeroes histogram
// (p + 2) % 3, which nobody reads any more (its readers passed the barrier of pass p) and nobody
// counts into before the barrier of pass p + 1.  `pass` is the lane's running pass number (the
// same in all workgroups); histograms 0 and 1 are zero at the start of a frame.
template <int NT, class F>
__device__ bool wide_select(LaneShared<NT> &S, WideCtx &W, uint32_t &pass, int n, uint32_t need, uint32_t lo, uint32_t hi, F val,
                            uint32_t &theta, uint32_t &n_less, uint32_t &n_eq, bool one_pass) {
  const int tid = threadIdx.x;
  constexpr int PER = NBINS / NT;
  const uint32_t gtid = (uint32_t)W.g * NT + tid, gstr = (uint32_t)W.G * NT;
  uint32_t less = 0;
  for (;;) {
    int shift = 0;
    while ((((unsigned long long)hi - lo) >> shift) >= (unsigned long long)NBINS) ++shift;
    uint32_t *hist = W.wl->hist[pass % 3], *hist_next = W.wl->hist[(pass + 2) % 3];
    ++pass;
    for (int b = tid; b < NBINS; b += NT) S.hist[b] = 0;
    __syncthreads();
    for (uint32_t i = gtid; i < (uint32_t)n; i += gstr) {
      uint32_t v;
      if (val((int)i, v) && v >= lo && v <= hi) atomicAdd(&S.hist[(v - lo) >> shift], 1u);
    }
    __syncthreads();
    for (int b = tid; b < NBINS; b += NT) { const uint32_t cnt = S.hist[b]; if (cnt) atomicAdd(&hist[b], cnt); }
    if (!lane_sync<NT>(W, S)) return false;
    uint32_t loc[PER], sum = 0;
#pragma unroll
    for (int q = 0; q < PER; ++q) { loc[q] = ld32(&hist[tid * PER + q]); sum += loc[q]; }
    for (uint32_t b = gtid; b < (uint32_t)NBINS; b += gstr) hist_next[b] = 0;
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
    if (one_pass) {                                 // the approximate cut: the bin's upper edge
      const unsigned long long edge = (unsigned long long)lo + ((unsigned long long)(b + 1) << shift) - 1ull;
      theta = edge < hi ? (uint32_t)edge : hi; n_less = 0; n_eq = 0;
      return true;
    }
    less += below;
    need -= below;
    lo = lo + (b << shift);
    unsigned long long nhi = (unsigned long long)lo + ((1ull << shift) - 1);
    if (nhi < hi) hi = (uint32_t)nhi;
    if (shift == 0) { theta = lo; n_less = less; n_eq = cnt; return true; }
  }
}

// One frame of one lane in its general form: state table, token queue and candidate notes in
// the lane's global scratch, tokens and state headers read from memory.  It handles frames of
// any size (up to the decoder's capacities) and every graph; light frames take the LDS form
// in wfst_frame_light.h instead.  Stages as listed at the top of wfst_kernels.h.  WIDE: the
// lane is shared by W.G workgroups (each with its own replica of the lane's state in S).
template <int NT, bool WIDE>
__device__ void general_frame(const DecDev &D, LaneShared<NT> &S, WideCtx &W, const float *ll, bool is_init,
                           Slot *gslots, uint32_t *queue, Aux *aux, uint32_t *dkey, uint32_t *dslot,
                           long long *foff, HTok *hist, LatInt *lat) {
  const int tid = threadIdx.x;
  GenCtr *Cp;
  if constexpr (WIDE) Cp = &W.wl->c; else Cp = &S.gen;
  GenCtr &C = *Cp;
  // counters are read through these: plain in LDS, past the vector cache in global memory
  auto R32 = [&](const uint32_t *p) -> uint32_t { if constexpr (WIDE) return ld32(p); else return *p; };
  auto R64 = [&](const unsigned long long *p) -> unsigned long long { if constexpr (WIDE) return ld64(p); else return *p; };
  // the lane's barrier; a workgroup leaves the frame (and the lane) if the barrier was given up
#define LSYNC() do { if constexpr (WIDE) { if (!lane_sync<NT>(W, S)) { if (threadIdx.x == 0) S.status = E_DEVICE; __syncthreads(); return; } } \
                     else __syncthreads(); } while (0)
  const uint32_t wg = WIDE ? (uint32_t)W.g : 0u, nwg = WIDE ? (uint32_t)W.G : 1u;
  const uint32_t gtid = wg * NT + (uint32_t)tid, gstr = nwg * NT;
  const bool lead = wg == 0 && tid == 0;            // the one thread of the lane that writes what exists once
  const uint32_t *rec = D.g.rec;
  constexpr bool LDS = false;                // table words are read with coherent global loads
#ifdef WFST_PHASE_TIMING
  if (threadIdx.x == 0) S.gtlast = wall_clock64();
#endif
  Slot *slots = gslots;
  const uint32_t mask = D.H - 1;
  const int hbits = D.hbits;
  const Slot fresh{~0ull, EMPTY, A_FRESH};

  if constexpr (WIDE) {                             // the first two histograms of the selection start at zero
    for (uint32_t b = gtid; b < 2u * NBINS; b += gstr) W.wl->hist[b / NBINS][b % NBINS] = 0;
  }
  uint32_t sel_pass = 0;
  if (lead) {
    C.claim_ctr = 0; C.auxn = 0; C.best = KEY_NONE; C.flags = 0; C.nvalid = 0; C.nout = 0; C.latn = 0;
    C.kmin = 0xFFFFFFFFu; C.kmax = 0; C.emit_arcs = 0; C.eps_arcs = 0;
  }
  LSYNC();
  const int nf = S.nf;                       // index of the frame being written
  const long long out_base = S.hist_used;
  int abort_code = 0;
  if (nf > D.max_frames) abort_code = E_HISTORY_OVERFLOW;

  // the frame's token queue: claimed slots, plus re-expansion requests for improved ones
  const uint32_t qcap = (uint32_t)D.qcap;
  auto qget = [&](uint32_t i, uint32_t &sl, bool &eps, bool &dup) {
    const uint32_t e = queue[i]; sl = e & Q_SLOT; eps = e & Q_EPS; dup = e & Q_DUP;
  };
  auto on_claim = [&](int sl, uint32_t dw, bool dup) {
    // the lanes of the wave that call this together get consecutive queue entries and, those
    // that claimed a new state, consecutive claim numbers, from a single 64-bit atomic add
    const unsigned long long m_all = __ballot(1), m_new = __ballot(!dup);
    const int wl = threadIdx.x & 63, leader = __ffsll((long long)m_all) - 1;
    unsigned long long base = 0;
    if (wl == leader) base = atomicAdd(&C.claim_ctr, ((unsigned long long)__popcll(m_new) << 32) | (unsigned long long)__popcll(m_all));
    base = __shfl(base, leader, 64);
    const unsigned long long below = (1ull << wl) - 1ull;
    if (!dup) {
      const uint32_t ci = (uint32_t)(base >> 32) + (uint32_t)__popcll(m_new & below);
      if (ci >= (uint32_t)D.tokcap) atomicOr(&C.flags, F_TOKOVF);
    }
    const uint32_t q = (uint32_t)base + (uint32_t)__popcll(m_all & below);
    if (q >= qcap) atomicOr(&C.flags, F_TOKOVF);
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
        C.best = okey(0.0f);
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
      const int tb0 = (int)(wg * NT), tstep = (int)gstr;     // this workgroup's tiles
      load_token(tb0 + tid, h, c, ne);
      for (int tb = tb0; tb < n_in; tb += tstep) {
        int total;
        const int ex = block_excl_scan<NT, LDS>(ne, S.wave_tmp, total);
        S.scan[tid] = ex; S.cost[tid] = c; S.base[tid] = h + 1;
        wg_sync<LDS>();
        GEN_MARK(8);
        if (tid == 0 && total) { if constexpr (WIDE) atomicAdd(&C.emit_arcs, (unsigned long long)total); else C.emit_arcs += (unsigned long long)total; }
        if (tb + tstep < n_in) load_token(tb + tstep + tid, hn, cn, nen);   // next tile, in flight during this one's rounds
        // one thread per arc (Section 3.3), EXP_U arcs of the tile per thread and round so
        // that their loads are in flight together
        for (int j0 = 0; j0 < total; j0 += NT * EXP_U) {
          float x[EXP_U], ct[EXP_U], sll[EXP_U]; uint32_t r[EXP_U], dw[EXP_U], kx[EXP_U], wt[EXP_U], w2[EXP_U]; int kk[EXP_U];
          int lo[EXP_U], hi[EXP_U], jc[EXP_U];
          // (a lane past the end re-reads the tile's last arc, so that no load is conditional and all
          // record loads, then all score loads, of a round are in flight together)
#pragma unroll
          for (int u = 0; u < EXP_U; ++u) { jc[u] = min(j0 + u * NT + tid, total - 1); lo[u] = 0; hi[u] = NT - 1; }
          constexpr int STEPS = NT >= 1024 ? 10 : NT >= 512 ? 9 : 8;
#pragma unroll
          for (int it = 0; it < STEPS; ++it) {     // largest k with scan[k] <= j, the searches step by step side by side
            int v[EXP_U];
#pragma unroll
            for (int u = 0; u < EXP_U; ++u) v[u] = S.scan[(lo[u] + hi[u] + 1) >> 1];
#pragma unroll
            for (int u = 0; u < EXP_U; ++u) { const int mid = (lo[u] + hi[u] + 1) >> 1; if (v[u] <= jc[u]) lo[u] = mid; else hi[u] = mid - 1; }
          }
#pragma unroll
          for (int u = 0; u < EXP_U; ++u) {
            kk[u] = lo[u];
            r[u] = S.base[lo[u]] + (uint32_t)(jc[u] - S.scan[lo[u]]);
            ct[u] = S.cost[lo[u]];
          }
#pragma unroll
          for (int u = 0; u < EXP_U; ++u) {
            const uint32_t *a = rec + 3 * (size_t)r[u];
            dw[u] = a[0]; wt[u] = a[1]; w2[u] = a[2];
          }
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int u = 0; u < EXP_U; ++u) sll[u] = ll[w2[u] & D.g.pdf_mask];
          __builtin_amdgcn_sched_barrier(0);
          uint32_t m = KEY_NONE;
          bool bad = false;
#pragma unroll
          for (int u = 0; u < EXP_U; ++u) {
            x[u] = (ct[u] + __uint_as_float(wt[u])) - sll[u];
            const bool have = j0 + u * NT + tid < total;
            const bool nan = x[u] != x[u] || x[u] == -INFINITY;
            bad |= have && nan;
            kx[u] = (have && !nan) ? okey(x[u]) : KEY_NONE;
            m = min(m, kx[u]);
          }
          if (bad) atomicOr(&C.flags, F_NAN);
          m = wave_min_u32(m);
          if ((tid & 63) == 0 && m != KEY_NONE) atomicMin(&C.best, m);
          wg_sync<LDS>();
          GEN_MARK(9);
          const float cut = key2f(R32(&C.best)) + D.beam;     // running bound, never below the final cutoff
#pragma unroll
          for (int u = 0; u < EXP_U; ++u) {
            if (kx[u] == KEY_NONE || !(x[u] <= cut)) continue;
            bool cl, im;
            const int sl = ht_insert<LDS>(slots, mask, hbits, dw[u] & HMASK, pack(kx[u], r[u]), cl, im);
            if (sl < 0) { atomicOr(&C.flags, F_TOKOVF); continue; }
            if (cl) on_claim(sl, dw[u], false);
            if (D.lattice_on || im) {
              const uint32_t ai = wave_alloc(&C.auxn);
              if (ai >= (uint32_t)D.auxcap) atomicOr(&C.flags, F_LATOVF);
              else aux[ai] = Aux{(uint32_t)sl, x[u], r[u], (uint32_t)(tb + kk[u])};
            }
          }
        }
        wg_sync<LDS>();
        GEN_MARK(10);
        h = hn; c = cn; ne = nen;
      }
      asm volatile("" ::"v"(touch), "v"(touch_more));
    }
  }
  LSYNC();
  GEN_MARK(0);
  const uint32_t bestk = R32(&C.best);
  if (abort_code == 0) {
    const uint32_t fl = R32(&C.flags);
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
    if (sl < 0) { atomicOr(&C.flags, F_TOKOVF); return; }
    if (cl || im) on_claim(sl, dw, !cl);
  };
  int iters = 0;
  if (abort_code == 0) {
    uint32_t w0 = 0, w1 = min((uint32_t)R64(&C.claim_ctr), qcap);
    LSYNC();
    while (w0 < w1) {
      // every thread takes CU queue entries of the window per pass, their loads side by side; the
      // pass is kept convergent (predicated, no early exit) so that the wave can allot note space
      // with one atomic
      constexpr int CU = 4;
      for (uint32_t i0 = w0; i0 < w1; i0 += gstr * CU) {
        bool act[CU], first[CU]; uint32_t src[CU], h[CU], ne[CU], np[CU]; float c[CU]; Slot sv[CU];
#pragma unroll
        for (int u = 0; u < CU; ++u) {
          const uint32_t i = i0 + (uint32_t)u * gstr + gtid;
          act[u] = false; first[u] = false; src[u] = 0; h[u] = 0; ne[u] = 0; np[u] = 0; c[u] = 0.f;
          if (i < w1) {
            bool eps, dup;
            qget(i, src[u], eps, dup);
            act[u] = eps;
          }
        }
#pragma unroll
        for (int u = 0; u < CU; ++u) if (act[u]) sv[u] = ld_slot<LDS>(&slots[src[u]]);
#pragma unroll
        for (int u = 0; u < CU; ++u)
          if (act[u]) { c[u] = key2f((uint32_t)(sv[u].val >> 32)); act[u] = c[u] <= cutoff; h[u] = sv[u].handle; }
#pragma unroll
        for (int u = 0; u < CU; ++u) if (act[u]) { ne[u] = rec[3 * (size_t)h[u]]; np[u] = rec[3 * (size_t)h[u] + 1]; }
        uint32_t fr[CU];
#pragma unroll
        for (int u = 0; u < CU; ++u) fr[u] = act[u] ? atomicAnd(&slots[src[u]].aux, ~A_FRESH) : 0u;   // first expansion while within the cutoff
#pragma unroll
        for (int u = 0; u < CU; ++u) first[u] = (fr[u] & A_FRESH) != 0;
        uint32_t dwv[CU][EPS_U]; float wv[CU][EPS_U];                // the first arcs, loads in flight together
#pragma unroll
        for (int u = 0; u < CU; ++u)
#pragma unroll
          for (int k = 0; k < EPS_U; ++k) {
            dwv[u][k] = 0; wv[u][k] = 0.f;
            if (act[u] && (uint32_t)k < np[u]) {
              const uint32_t *a = rec + 3 * (size_t)(h[u] + 1 + ne[u] + k);
              dwv[u][k] = a[0]; wv[u][k] = __uint_as_float(a[1]);
            }
          }
        // note space and the arc count, one atomic per wave
        uint32_t nn = 0;
#pragma unroll
        for (int u = 0; u < CU; ++u) nn += first[u] ? np[u] : 0u;
        const uint32_t inc = (uint32_t)wave_incl_scan((int)nn);
        const uint32_t wave_total = (uint32_t)__builtin_amdgcn_readlane((int)inc, 63);
        uint32_t note = 0;
        if ((tid & 63) == 0 && wave_total) {
          note = atomicAdd(&C.auxn, wave_total);
          atomicAdd(&C.eps_arcs, (unsigned long long)wave_total);
          if (note + wave_total > (uint32_t)D.auxcap) atomicOr(&C.flags, F_LATOVF);
        }
        note = (uint32_t)__builtin_amdgcn_readlane((int)note, 0) + inc - nn;
#pragma unroll
        for (int u = 0; u < CU; ++u) {
#pragma unroll
          for (int k = 0; k < EPS_U; ++k)
            if (act[u] && (uint32_t)k < np[u]) relax_eps(src[u], c[u], h[u] + 1 + ne[u] + k, dwv[u][k], wv[u][k], first[u] ? note + k : 0xFFFFFFFFu);
          for (uint32_t k = EPS_U; act[u] && k < np[u]; ++k) {
            const uint32_t *a = rec + 3 * (size_t)(h[u] + 1 + ne[u] + k);
            relax_eps(src[u], c[u], h[u] + 1 + ne[u] + k, a[0], __uint_as_float(a[1]), first[u] ? note + k : 0xFFFFFFFFu);
          }
          if (first[u]) note += np[u];
        }
      }
      LSYNC();
      GEN_MARK(11);
      w0 = w1; w1 = min((uint32_t)R64(&C.claim_ctr), qcap);
      ++iters;
      LSYNC();
    }
    const uint32_t fl2 = R32(&C.flags);
    if (fl2 & F_TOKOVF) abort_code = E_TOKEN_OVERFLOW;
    else if (fl2 & F_LATOVF) abort_code = E_LATTICE_OVERFLOW;
  }
  GEN_MARK(1);
  const uint32_t n_q = min((uint32_t)R64(&C.claim_ctr), qcap);
  auto token_slot = [&](uint32_t i, uint32_t &sl, uint32_t &eps) -> bool {
    bool e, dup;
    qget(i, sl, e, dup);
    eps = e;
    return !dup;
  };

  // ---- 3 + 4. max-active selection and contraction into the token history ---------------
  float cutoff_eff = cutoff;
  if (abort_code == 0) {
    const uint32_t nclaim = (uint32_t)(R64(&C.claim_ctr) >> 32);
    const uint32_t room = (uint32_t)min((long long)0x7FFFFFFF, D.hist_cap - out_base);
    if ((D.approximate ? nclaim : min(nclaim, (uint32_t)D.max_active)) > room) abort_code = E_HISTORY_OVERFLOW;
    else if (nclaim <= (uint32_t)D.max_active) {
      // nothing can be pruned: every token within the beam is kept
      for (uint32_t i = gtid; i < n_q; i += gstr) {
        uint32_t sl, eps;
        if (!token_slot(i, sl, eps)) continue;
        Slot *sp = slots + sl;
        const Slot sv = ld_slot<LDS>(sp);
        const unsigned long long v = sv.val;
        const float c = key2f((uint32_t)(v >> 32));
        if (!(c <= cutoff)) continue;
        const uint32_t pos = wave_alloc(&C.nout);
        if (pos >= room) continue;
        hist[out_base + pos] = HTok{sv.handle | (eps ? HAS_EPS : 0u), c, (uint32_t)v, NO_ARC};
        sp->aux = pos;
      }
      LSYNC();
      if (lead) C.nvalid = R32(&C.nout);
    } else {
      for (uint32_t i = gtid; i < n_q; i += gstr) {
        uint32_t sl, eps;
        if (!token_slot(i, sl, eps)) continue;
        const uint32_t key = (uint32_t)(tl64<LDS>(&slots[sl].val) >> 32);
        if (!(key2f(key) <= cutoff)) continue;
        const uint32_t p = wave_alloc(&C.nvalid);
        dkey[p] = key; dslot[p] = sl | (eps ? Q_EPS : 0u);
        atomicMin(&C.kmin, key); atomicMax(&C.kmax, key);
      }
      LSYNC();
      const int n = (int)R32(&C.nvalid);
      const uint32_t kmin = R32(&C.kmin), kmax = R32(&C.kmax);
      uint32_t theta = KEY_NONE, h_theta = 0xFFFFFFFFu;       // keep key < theta, or == theta with handle <= h_theta
      auto by_key = [&](int i, uint32_t &v) { v = dkey[i]; return true; };
      auto by_handle_at_theta = [&](int i, uint32_t &v) {
        if (dkey[i] != theta) return false;
        v = tl32<LDS>(&slots[dslot[i] & Q_SLOT].handle);
        return true;
      };
      if (n > D.max_active && D.approximate) {
        uint32_t nl, nq;
        if constexpr (WIDE) { if (!wide_select<NT>(S, W, sel_pass, n, (uint32_t)D.max_active, kmin, kmax, by_key, theta, nl, nq, true)) { if (tid == 0) S.status = E_DEVICE; __syncthreads(); return; } }
        else theta = block_histogram_cut<NT>(S, n, (uint32_t)D.max_active, kmin, kmax, by_key);
        cutoff_eff = key2f(theta);                            // (every key <= theta is kept)
      } else if (n > D.max_active) {
        uint32_t n_less, n_eq;
        if constexpr (WIDE) { if (!wide_select<NT>(S, W, sel_pass, n, (uint32_t)D.max_active, kmin, kmax, by_key, theta, n_less, n_eq, false)) { if (tid == 0) S.status = E_DEVICE; __syncthreads(); return; } }
        else block_select<NT>(S, n, (uint32_t)D.max_active, kmin, kmax, by_key, theta, n_less, n_eq);
        const uint32_t need_eq = (uint32_t)D.max_active - n_less;
        if (need_eq < n_eq) {
          uint32_t hl, he;
          if constexpr (WIDE) { if (!wide_select<NT>(S, W, sel_pass, n, need_eq, 0u, HMASK, by_handle_at_theta, h_theta, hl, he, false)) { if (tid == 0) S.status = E_DEVICE; __syncthreads(); return; } }
          else block_select<NT>(S, n, need_eq, 0u, HMASK, by_handle_at_theta, h_theta, hl, he);
        }
        cutoff_eff = key2f(theta);
      }
      for (uint32_t i = gtid; i < (uint32_t)n; i += gstr) {
        const uint32_t key = dkey[i], ds = dslot[i];
        Slot *sp = slots + (ds & Q_SLOT);
        const uint32_t h = tl32<LDS>(&sp->handle);
        const bool keep = key < theta || (key == theta && h <= h_theta);
        uint32_t pos = 0xFFFFFFFFu;
        if (keep) pos = wave_alloc(&C.nout);
        if (pos < room) {
          hist[out_base + pos] = HTok{h | ((ds & Q_EPS) ? HAS_EPS : 0u), key2f(key), (uint32_t)tl64<LDS>(&sp->val), NO_ARC};
          sp->aux = pos;
        } else {
          sp->aux = 0xFFFFFFFFu;
        }
      }
    }
  }
  LSYNC();
  GEN_MARK(2);
  const uint32_t nout_all = R32(&C.nout);
  const uint32_t n_out = (abort_code == 0) ? (D.approximate ? nout_all : min(nout_all, (uint32_t)D.max_active)) : 0u;

  // ---- 5. lattice records and back-pointers ---------------------------------------------
  if (abort_code == 0) {
    const long long lat_base = S.lat_pos;
    const uint32_t n_aux = min(R32(&C.auxn), (uint32_t)D.auxcap);
    auto emit_lat = [&](uint32_t arc, float extra, uint32_t dst, uint32_t src) {
      const uint32_t p = wave_alloc(&C.latn);
      if ((long long)p >= S.lat_room) atomicOr(&C.flags, F_LATOVF);
      else {
        long long at = lat_base + (long long)p;
        if (at >= D.lat_cap) at -= D.lat_cap;
        lat[at] = LatInt{nf, arc, extra, dst, src};
      }
    };
    for (uint32_t i0 = 0; i0 < n_aux; i0 += gstr * LAT_U) {
      Aux a[LAT_U];
#pragma unroll
      for (int u = 0; u < LAT_U; ++u) {
        const uint32_t i = i0 + (uint32_t)u * gstr + gtid;
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
  LSYNC();
  GEN_MARK(3);

  // ---- 6. clear the table ---------------------------------------------------------------
  const uint32_t fl3 = R32(&C.flags);
  if (fl3 & F_TOKOVF) {                                            // untracked claims: wipe everything
    const uint32_t n_all = D.H;
    for (uint32_t i = gtid; i < n_all; i += gstr) slots[i] = fresh;
  } else {
    for (uint32_t i = gtid; i < n_q; i += gstr) {
      uint32_t sl, eps;
      if (token_slot(i, sl, eps)) slots[sl] = fresh;
    }
  }
  if (tid == 0) {                                   // (every workgroup of the lane keeps its own replica of the lane's state)
    if (abort_code == 0 && (fl3 & F_LATOVF)) abort_code = E_LATTICE_OVERFLOW;
    const long long lat_new = min((long long)R32(&C.latn), S.lat_room);
    if (nf <= D.max_frames) {
      if (wg == 0) foff[nf + 1] = out_base + n_out;
      S.nf = nf + 1;
      S.in_off = out_base; S.n_in = (int)n_out;      // the frame just written is what the next one expands
    }
    S.hist_used = out_base + n_out;
    S.lat_total += lat_new; S.lat_room -= lat_new;
    S.lat_pos += lat_new;
    if (S.lat_pos >= D.lat_cap) S.lat_pos -= D.lat_cap;
    S.arcs_expanded += (long long)(R64(&C.emit_arcs) + R64(&C.eps_arcs));
    S.max_pre = max(S.max_pre, (int)R32(&C.nvalid));
    S.max_post = max(S.max_post, (int)n_out);
    S.iters_max = max(S.iters_max, iters);
#ifdef WFST_PHASE_TIMING
    S.ph[7] += iters; S.dbg_tok += n_out; S.dbg_iters += iters; S.dbg_arcs += C.emit_arcs + C.eps_arcs;
#endif
    if (abort_code != 0) S.status = abort_code;
  }
  LSYNC();
  GEN_MARK(4);
#undef LSYNC
}

}  // namespace wfst
