// The frame of a lane whose working set fits in LDS ("light" frames: at the benchmark's
// operating point nearly all of them).
//
// What a frame computes is the paper's Section 3 / Fig. 1 sequence (emitting expansion with one
// thread per arc, adaptive beam, non-emitting iterations to convergence, contraction, lattice
// preprocessing of Section 3.4) - the same as the general frame.  How it is laid out differs,
// because at a few hundred tokens per lane a frame is not limited by bandwidth but by its
// chain of dependent steps, and this form is built to shorten that chain:
//   * the kept tokens of a frame stay in LDS (state handle, cost, degree info) and are the
//     next frame's queue, so a frame starts without any global read;
//   * every arc record carries the out-degrees of its destination, so a token is expanded
//     without fetching its state's header, and the epsilon arcs of a newly claimed state are
//     fetched by the claiming thread at once and parked in LDS: a closure round then works on
//     LDS alone, and only the arcs of the states it claims itself cost a memory round trip;
//   * a frame whose arcs fit one round (<= threads x EXP_U) knows the final cutoff before its
//     first insertion and keeps its candidate notes in registers for the lattice stage;
//   * the per-frame counters come in two sets used alternately and the clearing of the state
//     table is deferred into the next frame's first stage, so a frame has five workgroup
//     barriers plus one per closure round, all of them LDS-only (global stores keep
//     travelling across them); wavefront scans and reductions use DPP row shifts;
//   * a kept token is written to the channel's history exactly once, by the thread that holds
//     the candidate equal to the table's minimum (its best incoming arc), with the
//     back-pointer already in it.
// A frame that outgrows the LDS structures, or meets a state whose out-degrees do not fit the
// degree info, is redone by the general frame; nothing has been committed at that point.
#pragma once
#include <type_traits>
#include "wfst_lane.h"

namespace wfst {

// Returns false if the frame must be redone by the general frame.
template <int NT>
__device__ bool light_frame(const DecDev &D, LaneShared<NT> &S, LaneCtx &ctx, const float *ll, const float *ll_next,
                            bool is_init, int chan) {
  using L = LightCfg<NT>;
  constexpr int NW = NT / 64, U = L::EXP_U;
  constexpr uint32_t mask = L::SLOTS - 1;
  constexpr int hbits = L::HBITS;
  constexpr uint32_t NOSLOT = 0xFFFFFFFFu;
  const int tid = threadIdx.x, lane = tid & 63, wid = tid >> 6;
  const uint32_t *rec = D.g.rec;
  Slot *slots = S.table;
  const Slot fresh{~0ull, EMPTY, 0xFFFFFFFFu};
  FrameCtr &C = S.fc[ctx.par];
  const int nf = ctx.nf;                       // index of the frame being written
  const long long out_base = ctx.hist_used;
  const int n_in = is_init ? 0 : ctx.n_in;
  const int info_shift = D.g.info_shift;
  const uint32_t sink = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) float *)S.sink;
  // (the lane's buffers are addressed from the decoder's arrays where they are used: eight
  // pointers less to keep in registers across the whole kernel)
  HTok *const hist = D.hist + (size_t)chan * (size_t)D.hist_cap;
  LatInt *const lat = D.lat + (size_t)chan * (size_t)D.lat_cap;
  const uint32_t claim_limit = min((uint32_t)L::CLAIM_LIMIT, (uint32_t)D.tokcap);

  // ---- 0. what the previous light frame left: its table entries are cleared here, beside the
  //         first memory round trip of this frame ---------------------------------------------
  for (uint32_t i = tid; i < ctx.pending_clear; i += NT) {
    const uint32_t e = S.lq[i];
    if (!(e & LQ_DUP)) slots[e & LQ_SLOT] = fresh;
  }
  ctx.pending_clear = 0;
  if (nf > D.max_frames) { ctx.status = E_HISTORY_OVERFLOW; return true; }
  if (!is_init && !ctx.tok_valid) {            // the token list is not in LDS (first frame of a call, or after a general frame)
    for (int i = tid; i < n_in; i += NT) {
      const HTok t = hist[ctx.in_off + i];
      const uint32_t h = t.handle & HMASK;
      S.tok_h[i] = t.handle; S.tok_c[i] = t.cost;
      S.tok_i[i] = (uint16_t)degree_info(rec[3 * (size_t)h], rec[3 * (size_t)h + 1]);
    }
    ctx.tok_valid = true;
    ctx.scan_ready = false;
    lds_barrier();
  }

  PHASE_MARK(0);
  // A state has been claimed (dup false) or improved and must be expanded again (dup true): it
  // gets a queue entry and, when claimed, a claim number - the lanes of the wave that call this
  // together take consecutive ones from a single 64-bit atomic add.  The claiming thread also
  // fetches the state's epsilon arcs and parks them in LDS.
  auto claim = [&](int sl, uint32_t dw, uint32_t info, bool dup, unsigned long long *ctr, uint32_t qbase, uint32_t cbase) {
    const unsigned long long m_all = __ballot(1), m_new = __ballot(!dup);
    const unsigned long long m_eps = __ballot(dup || ((info >> INFO_NP_SHIFT) & INFO_NP) != 0);   // entries a closure round has work for
    const int leader = __ffsll((long long)m_all) - 1;
    unsigned long long base = 0;
    if (lane == leader)
      base = atomicAdd(ctr, ((unsigned long long)__popcll(m_new) << CNT_CLAIM_SHIFT) | ((unsigned long long)__popcll(m_eps) << CNT_EPS_SHIFT) |
                                (unsigned long long)__popcll(m_all));
    const uint32_t base_q = (uint32_t)__builtin_amdgcn_readlane((int)((uint32_t)base & CNT_ENTRIES), leader);
    const uint32_t base_c = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(base >> CNT_CLAIM_SHIFT), leader);
    const unsigned long long below = (1ull << lane) - 1ull;
    const uint32_t q = qbase + base_q + (uint32_t)__popcll(m_all & below);
    if (q >= (uint32_t)L::QCAP) atomicOr(ctr, CNT_RESTART);
    else S.lq[q] = (uint16_t)((uint32_t)sl | (dup ? LQ_DUP : 0u));
    if (dup) return;
    const uint32_t ci = cbase + base_c + (uint32_t)__popcll(m_new & below);
    if (ci >= claim_limit) atomicOr(ctr, CNT_RESTART);
    const uint32_t ne = info & INFO_NE, np = (info >> INFO_NP_SHIFT) & INFO_NP;
    uint32_t e0 = 0;
    if (ne == INFO_NE || np == INFO_NP) {
      atomicOr(ctr, CNT_RESTART);                // degrees too large for the info: the general frame reads the header
    } else if (np) {
      e0 = atomicAdd(&C.enote_n, np);
      if (e0 + np > (uint32_t)L::ECAP) atomicOr(ctr, CNT_RESTART);
      else {
        const uint32_t r0 = (dw & HMASK) + 1 + ne;
        const uint32_t *a0 = rec + 3 * (size_t)r0;
        uint32_t b0[3], b1[3] = {0, 0, 0};       // the first two arcs' loads in flight together
        b0[0] = a0[0]; b0[1] = a0[1]; b0[2] = a0[2];
        if (np > 1) { b1[0] = a0[3]; b1[1] = a0[4]; b1[2] = a0[5]; }
        auto park = [&](uint32_t e, uint32_t rr, uint32_t c0, uint32_t c1, uint32_t c2) {
          S.enote[e] = ENote{__uint_as_float(c1), rr, c0, ((info_shift ? (c2 >> 16) : INFO_UNKNOWN) << 16) | 0xFFFFu};
        };
        park(e0, r0, b0[0], b0[1], b0[2]);
        if (np > 1) park(e0 + 1, r0 + 1, b1[0], b1[1], b1[2]);
        for (uint32_t k = 2; k < np; ++k) {
          const uint32_t *a = a0 + 3 * (size_t)k;
          const uint32_t c0 = a[0], c1 = a[1], c2 = a[2];
          park(e0 + k, r0 + k, c0, c1, c2);
        }
      }
    }
    slots[sl].aux = (e0 << 16) | (info & 0xFFFFu);
  };

  // ---- 1. emitting expansion ------------------------------------------------------------------
  // candidate notes of a one-round frame, kept in registers until the lattice stage
  float x[U]; uint32_t r[U], nslot[U]; int kk[U];
#pragma unroll
  for (int u = 0; u < U; ++u) { nslot[u] = NOSLOT; x[u] = 0.f; r[u] = 0; kk[u] = 0; }
  bool simple = true;                          // one tile, one round: notes in registers, cutoff final before the first insertion
  unsigned long long emit_arcs = 0;
  if (is_init) {
    if (tid == 0) C.best = okey(0.0f);
    lds_barrier();
    if (tid == 0) {
      const uint32_t h = D.g.start_handle;
      bool cl, im;
      const int sl = ht_insert<true>(slots, mask, hbits, h, pack(okey(0.0f), NO_ARC), cl, im);
      claim(sl, h, D.g.start_info, false, &C.cnt[0], 0u, 0u);
    }
  } else {
    for (int tb = 0; tb < n_in; tb += NT) {
      if (tb > 0 || !ctx.scan_ready) {         // (the first tile's sums are usually left by the previous frame)
        const int i = tb + tid;
        int ne = i < n_in ? (int)(S.tok_i[i] & INFO_NE) : 0;
        if (ne == (int)INFO_NE) { atomicOr(&C.cnt[0], CNT_RESTART); ne = 0; }
        const int inc = wave_incl_scan(ne);
        S.scan[tid] = inc - ne;                // exclusive within the wave
        if (lane == 63) S.wtot[wid] = inc;
        lds_barrier();
      }
      PHASE_MARK(1);
      int wb[NW];                              // arcs before each wave of the tile
      int total = 0;
#pragma unroll
      for (int w = 0; w < NW; ++w) { wb[w] = total; total += uni(S.wtot[w]); }
      emit_arcs += (unsigned long long)total;
      if (tb == 0) simple = n_in <= NT && total <= NT * U;
      for (int j0 = 0; j0 < total; j0 += NT * U) {
        uint32_t dw[U], kx[U], w2[U];
#pragma unroll
        for (int u = 0; u < U; ++u) { kx[u] = KEY_NONE; dw[u] = 0; w2[u] = 0; nslot[u] = NOSLOT; }
        uint32_t m = KEY_NONE;
        bool bad = false;
        // Arc j0 + u * NT + tid is this thread's u-th arc of the round.  A wave runs only as many
        // of the U slots as it has arcs for (the same number for all its lanes), and runs them
        // side by side: the steps of the searches, then all record loads, then all score loads.
        auto expand = [&](auto ua_const) {
          constexpr int UA = decltype(ua_const)::value;
          uint32_t wt[UA]; float ct[UA], sc_ll[UA];
          int jj[UA], lo[UA], hi[UA], wv[UA];
#pragma unroll
          for (int u = 0; u < UA; ++u) {
            // (a lane past the end re-reads the last arc, so that no load is conditional)
            const int j = min(j0 + u * NT + tid, total - 1);
            int w = 0;                         // the wave whose tokens own arc j, then the token inside it
#pragma unroll
            for (int q = 1; q < NW; ++q) w += (j >= wb[q]) ? 1 : 0;
            int base = 0;
#pragma unroll
            for (int q = 1; q < NW; ++q) base = (w == q) ? wb[q] : base;
            jj[u] = j - base; wv[u] = w * 64; lo[u] = 0; hi[u] = 63;
          }
#pragma unroll
          for (int it = 0; it < 6; ++it) {     // largest k with scan[k] <= jj
            int v[UA];
#pragma unroll
            for (int u = 0; u < UA; ++u) v[u] = S.scan[wv[u] + ((lo[u] + hi[u] + 1) >> 1)];
#pragma unroll
            for (int u = 0; u < UA; ++u) { const int mid = (lo[u] + hi[u] + 1) >> 1; if (v[u] <= jj[u]) lo[u] = mid; else hi[u] = mid - 1; }
          }
#pragma unroll
          for (int u = 0; u < UA; ++u) {
            const int k = tb + wv[u] + lo[u];
            kk[u] = k;
            r[u] = (S.tok_h[k] & HMASK) + 1u + (uint32_t)(jj[u] - S.scan[wv[u] + lo[u]]);
            ct[u] = S.tok_c[k];
          }
#pragma unroll
          for (int u = 0; u < UA; ++u) {
            const uint32_t *a = rec + 3 * (size_t)r[u];
            dw[u] = a[0]; wt[u] = a[1]; w2[u] = a[2];
          }
          __builtin_amdgcn_sched_barrier(0);   // (keeps the loads above together and their uses below them)
#pragma unroll
          for (int u = 0; u < UA; ++u) sc_ll[u] = ll[w2[u] & D.g.pdf_mask];
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int u = 0; u < UA; ++u) {
            x[u] = (ct[u] + __uint_as_float(wt[u])) - sc_ll[u];
            const bool have = j0 + u * NT + tid < total;
            const bool nan = x[u] != x[u] || x[u] == -INFINITY;
            bad |= have && nan;
            kx[u] = (have && !nan) ? okey(x[u]) : KEY_NONE;
            m = min(m, kx[u]);
          }
        };
        const int left = total - j0 - uni(wid) * 64;        // arcs of the round from this wave's first lane on
        const int ua = left <= 0 ? 0 : min(U, (left + NT - 1) / NT);
        static_assert(U == 4 || U == 8, "slots per thread");
        switch (ua) {
          case 0: break;
          case 1: expand(std::integral_constant<int, 1>{}); break;
          case 2: expand(std::integral_constant<int, 2>{}); break;
          case 3: expand(std::integral_constant<int, 3>{}); break;
          case 4: expand(std::integral_constant<int, 4>{}); break;
          default:
            if constexpr (U > 4) expand(std::integral_constant<int, U>{});
            break;
        }
        if (bad) atomicOr(&C.flags, F_NAN);
        m = wave_min_u32(m);
        if (lane == 0 && m != KEY_NONE) atomicMin(&C.best, m);
        lds_barrier();
        PHASE_MARK(2);
        // within (best so far + beam): with one round that is the frame's final cutoff, with
        // more rounds a bound that is never below it (entries above the final one are ignored later)
        const float cut = key2f(uni(C.best)) + D.beam;
        const bool stop = (C.flags & F_NAN) != 0 || (C.cnt[0] & CNT_RESTART) != 0;   // (only saves work: the frame is given up later)
#pragma unroll
        for (int u = 0; u < U; ++u) {
          if (stop || kx[u] == KEY_NONE || !(x[u] <= cut)) continue;
          bool cl, im;
          const int sl = ht_insert<true>(slots, mask, hbits, dw[u] & HMASK, pack(kx[u], r[u]), cl, im);
          if (sl < 0) { atomicOr(&C.cnt[0], CNT_RESTART); continue; }
          if (cl) claim(sl, dw[u], info_shift ? (w2[u] >> 16) : INFO_UNKNOWN, false, &C.cnt[0], 0u, 0u);
          if (simple) nslot[u] = (uint32_t)sl;
          else if (D.lattice_on || im) {
            const uint32_t ai = wave_alloc(&C.auxn);
            if (ai >= (uint32_t)D.auxcap) atomicOr(&C.flags, F_LATOVF);
            else (D.aux + (size_t)blockIdx.x * (size_t)D.auxcap)[ai] = Aux{(uint32_t)sl, x[u], r[u], (uint32_t)kk[u]};
          }
        }
      }
      if (tb + NT < n_in) lds_barrier();       // the next tile overwrites the scan
    }
  }
  if (simple) lds_barrier(); else __syncthreads();   // (notes in global memory must have arrived before the lattice stage)
  PHASE_MARK(3);
  if (tid == 0) reset_ctr(S.fc[ctx.par ^ 1]);  // the previous frame's counters: nobody reads them any more

  // (from here on the frame's flags and its first counter are stable: closure rounds report
  // through their own counters)
  const uint32_t bestk = uni(C.best);
  const unsigned long long c0 = uni(C.cnt[0]);
  int abort_code = 0;                          // 1: give the frame to the general form
  {
    const uint32_t fl = uni(C.flags);
    if (c0 & CNT_RESTART) abort_code = 1;
    else if (fl & F_NAN) abort_code = E_NAN_INPUT;
    else if (fl & F_LATOVF) abort_code = E_LATTICE_OVERFLOW;
    else if (bestk == KEY_NONE || bestk == KEY_PINF) abort_code = E_DEAD_CHANNEL;
  }
  const float cutoff = key2f(bestk) + D.beam;

  // ---- 2. non-emitting closure ----------------------------------------------------------------
  // Round k works on the queue entries the round before appended: for each, the state's parked
  // epsilon arcs are relaxed from its current cost.  Entries appended in round k are counted by
  // counter (k + 1) % 3, which nobody touches in round k + 1, so one barrier per round is enough.
  uint32_t w0 = 0, w1 = min((uint32_t)c0 & CNT_ENTRIES, (uint32_t)L::QCAP), nclaim = (uint32_t)(c0 >> CNT_CLAIM_SHIFT);
  uint32_t n_eps = (uint32_t)(c0 >> CNT_EPS_SHIFT) & CNT_EPS;      // entries of the window with epsilon arcs to relax
  int iters = 0;
  if (abort_code == 0) {
    while (n_eps > 0) {                        // (a window without such entries needs no round)
      unsigned long long *ctr = &C.cnt[(iters + 1) % 3];
      if (tid == 0) C.cnt[(iters + 2) % 3] = 0;
      for (uint32_t i = w0 + tid; i < w1; i += NT) {
        const uint32_t sl = S.lq[i] & LQ_SLOT;
        const Slot sv = ld_slot<true>(slots + sl);
        const float c = key2f((uint32_t)(sv.val >> 32));
        const uint32_t np = (sv.aux >> INFO_NP_SHIFT) & INFO_NP, e0 = sv.aux >> 16;
        if (!np || !(c <= cutoff)) continue;
        for (uint32_t k = 0; k < np; ++k) {
          const ENote en = S.enote[e0 + k];
          const float xe = c + en.w;
          if (!(xe <= cutoff)) continue;
          bool cl, im;
          const int sl2 = ht_insert<true>(slots, mask, hbits, en.dest & HMASK, pack(okey(xe), en.arc), cl, im);
          if (sl2 < 0) { atomicOr(ctr, CNT_RESTART); continue; }
          if ((en.dinfo_dslot & 0xFFFFu) == 0xFFFFu) S.enote[e0 + k].dinfo_dslot = (en.dinfo_dslot & 0xFFFF0000u) | (uint32_t)sl2;
          if (cl) claim(sl2, en.dest, en.dinfo_dslot >> 16, false, ctr, w1, nclaim);
          else if (im && (en.dest & HAS_EPS)) claim(sl2, en.dest, 0u, true, ctr, w1, nclaim);
        }
      }
      lds_barrier();
      const unsigned long long cv = uni(*ctr);   // stable: the next round appends to another counter
      w0 = w1; w1 = min(w1 + ((uint32_t)cv & CNT_ENTRIES), (uint32_t)L::QCAP); nclaim += (uint32_t)(cv >> CNT_CLAIM_SHIFT);
      n_eps = (uint32_t)(cv >> CNT_EPS_SHIFT) & CNT_EPS;
      ++iters;
      if (cv & CNT_RESTART) { abort_code = 1; break; }
    }
  }
  if (abort_code == 1) {                       // outgrew the LDS structures: wipe the table, the general frame redoes it
    for (int i = tid; i < L::SLOTS; i += NT) slots[i] = fresh;
    if (tid == 0) reset_ctr(C);
    ctx.tok_valid = false; ctx.scan_ready = false;
    __syncthreads();
#ifdef WFST_PHASE_TIMING
    if (tid == 0) S.ph[13] += 1;
#endif
    PHASE_MARK(14);
    return false;
  }
  const uint32_t n_q = w1;

  PHASE_MARK(4);
  // fetch ahead the next frame's row of scores (one 64-byte line per load): by the next
  // expansion its gathers by pdf id hit L2
  if (ll_next)
    for (int p = tid * 16; p < D.g.num_pdfs; p += NT * 16) fetch_ahead(ll_next + p, sink);

  // ---- 3 + 4. max-active selection and contraction ------------------------------------------
  // A kept token gets its index in the new frame (low bits of its slot's aux) and its entry in
  // the LDS token list; its history record is written in stage 5.
  float cutoff_eff = cutoff;
  uint32_t eps_cnt = 0;
  if (abort_code == 0) {
    const uint32_t room = (uint32_t)min((long long)0x7FFFFFFF, D.hist_cap - out_base);
    if ((D.approximate ? nclaim : min(nclaim, (uint32_t)D.max_active)) > room) abort_code = E_HISTORY_OVERFLOW;
    else if (nclaim <= (uint32_t)D.max_active) {
      // nothing can be pruned: every token within the beam is kept
      for (uint32_t i = tid; i < n_q; i += NT) {
        const uint32_t e = S.lq[i];
        if (e & LQ_DUP) continue;
        const uint32_t sl = e & LQ_SLOT;
        const Slot sv = ld_slot<true>(slots + sl);
        const float c = key2f((uint32_t)(sv.val >> 32));
        if (!(c <= cutoff)) { slots[sl].aux = sv.aux | POS_MASK; continue; }
        const uint32_t np = (sv.aux >> INFO_NP_SHIFT) & INFO_NP;
        eps_cnt += np;
        const uint32_t pos = wave_alloc(&C.nout);
        S.tok_h[pos] = sv.handle | (np ? HAS_EPS : 0u); S.tok_c[pos] = c; S.tok_i[pos] = (uint16_t)sv.aux;
        slots[sl].aux = (sv.aux & ~POS_MASK) | pos;
      }
    } else {
      uint32_t *const dkey = D.dkey + (size_t)blockIdx.x * (size_t)D.tokcap;
      uint32_t *const dslot = D.dslot + (size_t)blockIdx.x * (size_t)D.tokcap;
      for (uint32_t i = tid; i < n_q; i += NT) {
        const uint32_t e = S.lq[i];
        if (e & LQ_DUP) continue;
        const uint32_t sl = e & LQ_SLOT;
        const Slot sv = ld_slot<true>(slots + sl);
        const uint32_t key = (uint32_t)(sv.val >> 32);
        if (!(key2f(key) <= cutoff)) { slots[sl].aux = sv.aux | POS_MASK; continue; }
        eps_cnt += (sv.aux >> INFO_NP_SHIFT) & INFO_NP;
        const uint32_t p = wave_alloc(&C.nvalid);
        dkey[p] = key; dslot[p] = sl;
        atomicMin(&C.kmin, key); atomicMax(&C.kmax, key);
      }
      __syncthreads();
      const int n = (int)uni(C.nvalid);
      uint32_t theta = KEY_NONE, h_theta = 0xFFFFFFFFu;       // keep key < theta, or == theta with handle <= h_theta
      if (n > D.max_active && D.approximate) {
        theta = block_histogram_cut<NT>(S, n, (uint32_t)D.max_active, uni(C.kmin), uni(C.kmax),
                                        [&](int i, uint32_t &v) { v = dkey[i]; return true; });
        cutoff_eff = key2f(theta);                            // (every key <= theta is kept)
      } else if (n > D.max_active) {
        uint32_t n_less, n_eq;
        block_select<NT>(S, n, (uint32_t)D.max_active, uni(C.kmin), uni(C.kmax),
                         [&](int i, uint32_t &v) { v = dkey[i]; return true; }, theta, n_less, n_eq);
        const uint32_t need_eq = (uint32_t)D.max_active - n_less;
        if (need_eq < n_eq) {
          uint32_t hl, he;
          block_select<NT>(S, n, need_eq, 0u, HMASK,
                           [&](int i, uint32_t &v) {
                             if (dkey[i] != theta) return false;
                             v = slots[dslot[i]].handle;
                             return true;
                           }, h_theta, hl, he);
        }
        cutoff_eff = key2f(theta);
      }
      for (int i = tid; i < n; i += NT) {
        const uint32_t key = dkey[i], sl = dslot[i];
        const Slot sv = ld_slot<true>(slots + sl);
        const bool keep = key < theta || (key == theta && sv.handle <= h_theta);
        if (keep) {
          const uint32_t pos = wave_alloc(&C.nout);
          const uint32_t np = (sv.aux >> INFO_NP_SHIFT) & INFO_NP;
          S.tok_h[pos] = sv.handle | (np ? HAS_EPS : 0u); S.tok_c[pos] = key2f(key); S.tok_i[pos] = (uint16_t)sv.aux;
          slots[sl].aux = (sv.aux & ~POS_MASK) | pos;
        } else {
          slots[sl].aux = sv.aux | POS_MASK;
        }
      }
    }
  }
  eps_cnt = wave_sum_u32(eps_cnt);
  if (lane == 0 && eps_cnt) atomicAdd(&C.eps_arcs, eps_cnt);
  lds_barrier();
  PHASE_MARK(8);
  const uint32_t nout_all = uni(C.nout);
  const uint32_t n_out = (abort_code == 0) ? (D.approximate ? nout_all : min(nout_all, (uint32_t)D.max_active)) : 0u;
  const uint32_t n_valid = (abort_code == 0) ? max(uni(C.nvalid), nout_all) : 0u;

  // ---- 5. history records, back-pointers and lattice records ---------------------------------
  // Every candidate arc is looked at once more, with final costs.  The one equal to the table's
  // minimum is the token's best incoming arc: its thread writes the token's history record.
  // Every arc into a kept token within the effective cutoff and the lattice beam is recorded
  // with its extra cost (Section 3.4).
  if (abort_code == 0) {
    const long long lat_base = ctx.lat_pos, lat_room = ctx.lat_room;
    auto emit_lat = [&](uint32_t arc, float extra, uint32_t dst, uint32_t src) {
      const uint32_t p = wave_alloc(&C.latn);
      if ((long long)p >= lat_room) atomicOr(&C.flags, F_LATOVF);
      else {
        long long at = lat_base + (long long)p;
        if (at >= D.lat_cap) at -= D.lat_cap;
        lat[at] = LatInt{nf, arc, extra, dst, src};
      }
    };
    // emitting candidate: slot of the destination, cost, arc, index of the source token
    auto emitting_note = [&](uint32_t slot, float xn, uint32_t arc, uint32_t src) {
      const Slot sv = ld_slot<true>(slots + slot);
      const uint32_t pos = sv.aux & POS_MASK;
      if (pos == POS_NONE) return;
      if (pack(okey(xn), arc) == sv.val) hist[out_base + pos] = HTok{S.tok_h[pos], xn, arc, src};
      if (D.lattice_on && xn <= cutoff_eff) {
        const float extra = xn - key2f((uint32_t)(sv.val >> 32));
        if (extra <= D.lattice_beam) emit_lat(arc, extra, pos, src);
      }
    };
    if (simple) {
#pragma unroll
      for (int u = 0; u < U; ++u)
        if (nslot[u] != NOSLOT) emitting_note(nslot[u], x[u], r[u], (uint32_t)kk[u]);
    } else {
      const Aux *const aux = D.aux + (size_t)blockIdx.x * (size_t)D.auxcap;
      const uint32_t n_aux = min(uni(C.auxn), (uint32_t)D.auxcap);
      for (uint32_t i0 = 0; i0 < n_aux; i0 += NT * LAT_U) {
        Aux a[LAT_U];
#pragma unroll
        for (int u = 0; u < LAT_U; ++u) {
          const uint32_t i = i0 + u * NT + tid;
          a[u] = i < n_aux ? aux[i] : Aux{NOSLOT, 0.f, 0u, 0u};
        }
#pragma unroll
        for (int u = 0; u < LAT_U; ++u)
          if (a[u].slot != NOSLOT) emitting_note(a[u].slot, a[u].x, a[u].arc, a[u].src);
      }
    }
    // epsilon arcs, through the states that own them
    for (uint32_t i = tid; i < n_q; i += NT) {
      const uint32_t e = S.lq[i];
      if (e & LQ_DUP) continue;
      const Slot ssv = ld_slot<true>(slots + (e & LQ_SLOT));
      const uint32_t np = (ssv.aux >> INFO_NP_SHIFT) & INFO_NP, e0 = ssv.aux >> 16;
      const float c = key2f((uint32_t)(ssv.val >> 32));
      if (!np || !(c <= cutoff)) continue;
      const uint32_t spos = ssv.aux & POS_MASK;
      for (uint32_t k = 0; k < np; ++k) {
        const ENote en = S.enote[e0 + k];
        const float xe = c + en.w;
        const uint32_t dsl = en.dinfo_dslot & 0xFFFFu;
        if (!(xe <= cutoff_eff) || dsl == 0xFFFFu) continue;
        const Slot sv = ld_slot<true>(slots + dsl);
        const uint32_t pos = sv.aux & POS_MASK;
        if (pos == POS_NONE) continue;
        // a best incoming arc whose source was cut by max-active leaves the token without a
        // back-pointer (a best path through it reports a broken trace)
        if (pack(okey(xe), en.arc) == sv.val)
          hist[out_base + pos] = HTok{S.tok_h[pos], xe, en.arc, spos == POS_NONE ? NO_ARC : (spos | PREV_SAME)};
        if (spos == POS_NONE) continue;
        if (D.lattice_on) {
          const float extra = xe - key2f((uint32_t)(sv.val >> 32));
          if (extra <= D.lattice_beam) emit_lat(en.arc, extra, pos, spos | PREV_SAME);
        }
      }
    }
    if (is_init && tid == 0) {                 // the start token has no incoming arc
      const int sl = ht_find<true>(slots, mask, hbits, D.g.start_handle);
      const uint32_t pos = sl >= 0 ? (slots[sl].aux & POS_MASK) : POS_NONE;
      if (pos != POS_NONE && (uint32_t)slots[sl].val == NO_ARC) hist[out_base + pos] = HTok{S.tok_h[pos], 0.0f, NO_ARC, NO_ARC};
    }
  }
  // the out-degree prefix sums the next frame's expansion starts from (its first tile), while
  // this frame's stores drain: the barrier below publishes them with everything else
  const bool scan_next = abort_code == 0 && ll_next != nullptr;
  if (scan_next) {
    int ne = (uint32_t)tid < n_out ? (int)(S.tok_i[tid] & INFO_NE) : 0;
    if (ne == (int)INFO_NE) { atomicOr(&S.fc[ctx.par ^ 1].cnt[0], CNT_RESTART); ne = 0; }   // (the next frame's counter: reset long ago)
    const int inc = wave_incl_scan(ne);
    S.scan[tid] = inc - ne;
    if (lane == 63) S.wtot[wid] = inc;
  }
  lds_barrier();
  PHASE_MARK(9);

  // ---- 6. the lane's state after the frame (every thread computes the same values) -----------
  if (abort_code == 0 && (uni(C.flags) & F_LATOVF)) abort_code = E_LATTICE_OVERFLOW;
  const long long lat_new = min((long long)uni(C.latn), ctx.lat_room);
  if (tid == 0) (D.frame_off + (size_t)chan * (size_t)(D.max_frames + 2))[nf + 1] = out_base + n_out;
  ctx.nf = nf + 1;
  ctx.in_off = out_base; ctx.n_in = (int)n_out;
  ctx.hist_used = out_base + n_out;
  ctx.lat_total += lat_new; ctx.lat_room -= lat_new;
  ctx.lat_pos += lat_new;
  if (ctx.lat_pos >= D.lat_cap) ctx.lat_pos -= D.lat_cap;
  ctx.arcs_expanded += (long long)(emit_arcs + (unsigned long long)uni(C.eps_arcs));
  ctx.max_pre = max(ctx.max_pre, (int)n_valid);
  ctx.max_post = max(ctx.max_post, (int)n_out);
  ctx.iters_max = max(ctx.iters_max, iters);
#ifdef WFST_PHASE_TIMING
  if (tid == 0) { S.ph[7] += iters; S.dbg_tok += n_out; S.dbg_arcs += emit_arcs + C.eps_arcs; }
#endif
  if (abort_code != 0) ctx.status = abort_code;
  ctx.tok_valid = abort_code == 0;
  ctx.scan_ready = scan_next;
  ctx.pending_clear = n_q;
  ctx.par ^= 1;
  return true;
}

}  // namespace wfst
