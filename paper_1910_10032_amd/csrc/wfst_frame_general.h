// The general form of a lane's frame (any size, any graph).
#pragma once
#include "wfst_lane.h"

namespace wfst {

// One frame of one lane in its general form: state table, token queue and candidate notes in
// the lane's global scratch, tokens and state headers read from memory.  It handles frames of
// any size (up to the decoder's capacities) and every graph; light frames take the LDS form
// in wfst_frame_light.h instead.  Stages as listed at the top of wfst_kernels.h.
template <int NT>
__device__ void general_frame(const DecDev &D, LaneShared<NT> &S, const float *ll, bool is_init,
                           Slot *gslots, uint32_t *queue, Aux *aux, uint32_t *dkey, uint32_t *dslot,
                           long long *foff, HTok *hist, LatInt *lat) {
  const int tid = threadIdx.x;
  const uint32_t *rec = D.g.rec;
  constexpr bool LDS = false;                // table words are read with coherent global loads
  Slot *slots = gslots;
  const uint32_t mask = D.H - 1;
  const int hbits = D.hbits;
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
    if (wl == leader) base = atomicAdd(&S.claim_ctr, ((unsigned long long)__popcll(m_new) << 32) | (unsigned long long)__popcll(m_all));
    base = __shfl(base, leader, 64);
    const unsigned long long below = (1ull << wl) - 1ull;
    if (!dup) {
      const uint32_t ci = (uint32_t)(base >> 32) + (uint32_t)__popcll(m_new & below);
      if (ci >= (uint32_t)D.tokcap) atomicOr(&S.flags, F_TOKOVF);
    }
    const uint32_t q = (uint32_t)base + (uint32_t)__popcll(m_all & below);
    if (q >= qcap) atomicOr(&S.flags, F_TOKOVF);
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
        GEN_MARK(8);
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
              pdf[u] = a[2] & D.g.pdf_mask;
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
          GEN_MARK(9);
          const float cut = key2f(S.best) + D.beam;     // running bound, never below the final cutoff
#pragma unroll
          for (int u = 0; u < EXP_U; ++u) {
            if (kx[u] == KEY_NONE || !(x[u] <= cut)) continue;
            bool cl, im;
            const int sl = ht_insert<LDS>(slots, mask, hbits, dw[u] & HMASK, pack(kx[u], r[u]), cl, im);
            if (sl < 0) { atomicOr(&S.flags, F_TOKOVF); continue; }
            if (cl) on_claim(sl, dw[u], false);
            if (D.lattice_on || im) {
              const uint32_t ai = wave_alloc(&S.auxn);
              if (ai >= (uint32_t)D.auxcap) atomicOr(&S.flags, F_LATOVF);
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
  wg_sync<LDS>();
  GEN_MARK(0);
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
    if (sl < 0) { atomicOr(&S.flags, F_TOKOVF); return; }
    if (cl || im) on_claim(sl, dw, !cl);
  };
  int iters = 0;
  if (abort_code == 0) {
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
      GEN_MARK(11);
      w0 = w1; w1 = min(S.qtail, qcap);
      ++iters;
      wg_sync<LDS>();
    }
    if (S.flags & F_TOKOVF) abort_code = E_TOKEN_OVERFLOW;
    else if (S.flags & F_LATOVF) abort_code = E_LATTICE_OVERFLOW;
  }
  GEN_MARK(1);
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
    if ((D.approximate ? nclaim : min(nclaim, (uint32_t)D.max_active)) > room) abort_code = E_HISTORY_OVERFLOW;
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
      if (n > D.max_active && D.approximate) {
        theta = block_histogram_cut<NT>(S, n, (uint32_t)D.max_active, S.kmin, S.kmax,
                                        [&](int i, uint32_t &v) { v = dkey[i]; return true; });
        cutoff_eff = key2f(theta);                            // (every key <= theta is kept)
      } else if (n > D.max_active) {
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
  GEN_MARK(2);
  const uint32_t n_out = (abort_code == 0) ? (D.approximate ? S.nout : min(S.nout, (uint32_t)D.max_active)) : 0u;

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
  GEN_MARK(3);

  // ---- 6. clear the table ---------------------------------------------------------------
  if (S.flags & F_TOKOVF) {                                        // untracked claims: wipe everything
    const uint32_t n_all = D.H;
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
  GEN_MARK(4);
}

}  // namespace wfst
