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
#include "wfst_frame_general.h"
#include "wfst_frame_light.h"

namespace wfst {

// One workgroup per lane.  is_init: (re)start the lane's channel and write frame 0.
// Between frames the lane's state is held in registers by every thread (LaneCtx, all values
// uniform); a general frame gets it through LDS.
template <int NT>
__global__ void __launch_bounds__(NT, NT >= 512 ? 4 : 2) k_advance(DecDev D, const LaneParam *__restrict__ lanes, int is_init) {
  __shared__ LaneShared<NT> S;
  const int tid = threadIdx.x;
  LaneParam lp = lanes[blockIdx.x];
  lp.ll = (const float *)uni((unsigned long long)lp.ll); lp.chan = uni(lp.chan); lp.n_frames = uni(lp.n_frames); lp.stride = uni(lp.stride);
  lp.snap_every = uni(lp.snap_every); lp.snap_id0 = uni(lp.snap_id0); lp.n_snaps = uni(lp.n_snaps);
  ChanState *cs = D.chan + lp.chan;
  long long *foff = D.frame_off + (size_t)lp.chan * (size_t)(D.max_frames + 2);
  LatInt *lat = D.lat + (size_t)lp.chan * (size_t)D.lat_cap;

  const Slot fresh{~0ull, EMPTY, 0xFFFFFFFFu};
  for (int i = tid; i < LightCfg<NT>::SLOTS; i += NT) S.table[i] = fresh;
  if (tid == 0) {
    reset_ctr(S.fc[0]); reset_ctr(S.fc[1]);
    if (is_init) foff[0] = 0;
#ifdef WFST_PHASE_TIMING
    for (int k = 0; k < 16; ++k) { S.ph[k] = 0; S.gph[k] = 0; }
    S.dbg_tok = 0; S.dbg_iters = 0; S.dbg_arcs = 0;
#endif
  }
  LaneCtx ctx;
#ifdef WFST_PHASE_TIMING
  ctx.tlast = wall_clock64();
#endif
  if (is_init) {
    ctx.status = 0; ctx.nf = 0; ctx.hist_used = 0; ctx.lat_room = D.lat_cap; ctx.lat_pos = 0; ctx.lat_total = 0;
    ctx.arcs_expanded = 0; ctx.lat_head = 0; ctx.lat_head_pos = 0; ctx.max_pre = 0; ctx.max_post = 0; ctx.iters_max = 0;
  } else {
    ctx.status = uni(cs->status); ctx.nf = uni(cs->num_frames); ctx.hist_used = uni(cs->hist_used);
    ctx.lat_head = uni(cs->lat_head); ctx.lat_total = uni(cs->lat_total);
    ctx.lat_room = D.lat_cap - (ctx.lat_total - ctx.lat_head);
    ctx.lat_pos = ctx.lat_total % D.lat_cap;
    ctx.lat_head_pos = ctx.lat_head % D.lat_cap;
    ctx.arcs_expanded = uni(cs->arcs_expanded); ctx.max_pre = uni(cs->max_pre);
    ctx.max_post = uni(cs->max_post); ctx.iters_max = uni(cs->closure_iters_max);
  }
  ctx.in_off = 0; ctx.n_in = 0;
  if (!is_init && ctx.nf >= 1 && ctx.nf <= D.max_frames + 1) {
    const long long o0 = uni(foff[ctx.nf - 1]), o1 = uni(foff[ctx.nf]);
    ctx.in_off = o0; ctx.n_in = (int)(o1 - o0);
  }
  ctx.pending_clear = 0; ctx.par = 0; ctx.tok_valid = false; ctx.scan_ready = false;
  __syncthreads();
  // Seal the lane's state as the next snapshot of this call.  With snapshot blocks the lattice
  // records not handed out yet move into the snapshot's block, in the caller's form (the lane
  // reserves its range with one compare-and-swap; the ring is empty afterwards).  Then
  // everything the workgroup has written is made visible to the whole system, then the
  // snapshot entry and the lane's progress word.  Readouts of the snapshot start only after
  // the host has seen the progress words of all lanes, so nothing ever waits inside a kernel.
  int n_sealed = 0;
  auto seal = [&]() {
    __syncthreads();                                  // every wave has issued its stores of the frames so far
    const long long id = lp.snap_id0 + n_sealed;
    long long blk_start = 0, blk_count = 0;
    if (D.n_blk > 0 && D.lattice_on) {
      const int slot = (int)(id % D.n_blk);
      const long long n = ctx.lat_total - ctx.lat_head;
      if (tid == 0) {
        unsigned long long *used = &D.blk[slot].used;
        unsigned long long old = ld64(used);
        long long pos = -1;
        while ((long long)old + n <= D.blk_cap) {     // every failed swap means another lane got its range
          const unsigned long long seen = atomicCAS(used, old, old + (unsigned long long)n);
          if (seen == old) { pos = (long long)old; break; }
          old = seen;
        }
        S.blk_pos = pos;
      }
      __syncthreads();
      const long long pos = uni(S.blk_pos);
      if (pos < 0 && ctx.status == 0) ctx.status = E_LATTICE_OVERFLOW;
      if (pos >= 0) {
        LatRec *out = D.blk_recs + (size_t)slot * (size_t)D.blk_cap + (size_t)pos;
        const long long first = ctx.lat_head_pos;
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
      ctx.lat_head = ctx.lat_total; ctx.lat_head_pos = ctx.lat_pos; ctx.lat_room = D.lat_cap;
    }
    // Every thread's stores (tokens, lattice records, the block) must have reached the L2 before
    // thread 0 publishes: each wave waits until its own stores have been acknowledged, then the
    // barrier, then thread 0's system-scope release, which writes the L2's dirty lines back.
    // (One release per lane and snapshot: a device-scope fence in every thread would flush and
    // invalidate the cache eight times over and slows all lanes of the chip down noticeably.)
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (tid == 0) {
      ChanSnap *sp = D.snap + (size_t)lp.chan * SNAP_RING + (size_t)(id % SNAP_RING);
      sp->lat_total = ctx.lat_total; sp->hist_used = ctx.hist_used; sp->status = ctx.status; sp->num_frames = ctx.nf;
      sp->blk_start = blk_start; sp->blk_count = blk_count;
      sp->id = id;
      __hip_atomic_store(D.lane_sealed + blockIdx.x, id, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
    }
    ++n_sealed;
  };
  // a frame in the general form: the lane's state goes through LDS
  auto run_general = [&](const float *ll) {
    if (tid == 0) {
      S.status = ctx.status; S.nf = ctx.nf; S.n_in = ctx.n_in; S.max_pre = ctx.max_pre; S.max_post = ctx.max_post;
      S.iters_max = ctx.iters_max; S.in_off = ctx.in_off; S.hist_used = ctx.hist_used; S.lat_room = ctx.lat_room;
      S.lat_total = ctx.lat_total; S.lat_pos = ctx.lat_pos; S.arcs_expanded = ctx.arcs_expanded;
    }
    __syncthreads();                                  // (also: the light frames' history stores have arrived)
    WideCtx none{0, 1, nullptr, 0ull, 0u};
    general_frame<NT, false>(D, S, none, ll, is_init != 0, D.slots + (size_t)blockIdx.x * D.H, D.queue + (size_t)blockIdx.x * (size_t)D.qcap,
                      D.aux + (size_t)blockIdx.x * (size_t)D.auxcap, D.dkey + (size_t)blockIdx.x * (size_t)D.tokcap,
                      D.dslot + (size_t)blockIdx.x * (size_t)D.tokcap, foff, D.hist + (size_t)lp.chan * (size_t)D.hist_cap, lat);
    ctx.status = uni(S.status); ctx.nf = uni(S.nf); ctx.n_in = uni(S.n_in); ctx.max_pre = uni(S.max_pre); ctx.max_post = uni(S.max_post);
    ctx.iters_max = uni(S.iters_max); ctx.in_off = uni(S.in_off); ctx.hist_used = uni(S.hist_used); ctx.lat_room = uni(S.lat_room);
    ctx.lat_total = uni(S.lat_total); ctx.lat_pos = uni(S.lat_pos); ctx.arcs_expanded = uni(S.arcs_expanded);
    ctx.tok_valid = false; ctx.scan_ready = false;
    __syncthreads();                                  // all have read the state before the next general frame rewrites it
  };
  const int nframes = is_init ? 1 : lp.n_frames;
  const int n_snaps = is_init ? 0 : lp.n_snaps;
  const bool light_ok = D.g.info_shift != 0 && D.force_general == 0;
  int until_seal = (!is_init && lp.snap_every > 0) ? lp.snap_every : 0x7FFFFFFF;
  for (int f = 0;;) {
    const bool more = f < nframes && ctx.status == 0;
    if (more) {
      const float *ll = is_init ? nullptr : lp.ll + (size_t)f * (size_t)lp.stride;
      const float *ll_next = (!is_init && f + 1 < nframes) ? ll + lp.stride : nullptr;
      bool done = false;
      if (light_ok && (is_init || ctx.n_in <= LightCfg<NT>::NIN_MAX))
        done = light_frame<NT>(D, S, ctx, ll, ll_next, is_init != 0, lp.chan);
      if (!done) {
#ifdef WFST_PHASE_TIMING
        if (tid == 0) S.ph[6] += 1;
#endif
        run_general(ll);
        PHASE_MARK(11);
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
    cs->status = ctx.status; cs->num_frames = ctx.nf; cs->hist_used = ctx.hist_used;
    cs->lat_total = ctx.lat_total; cs->arcs_expanded = ctx.arcs_expanded; cs->max_pre = ctx.max_pre;
    cs->max_post = ctx.max_post; cs->closure_iters_max = ctx.iters_max;
    if (is_init) cs->path_nf = 0;
    cs->lat_head = ctx.lat_head;
#ifdef WFST_PHASE_TIMING
    if (D.dbg) {
      for (int k = 0; k < 16; ++k) { atomicAdd(D.dbg + k, S.ph[k]); atomicAdd(D.dbg + 16 + 10240 + k, S.gph[k]); }
      unsigned long long tot = 0;
      for (int k = 0; k < 16; ++k) if (k != 5 && k != 6 && k != 7 && k != 13) tot += S.ph[k];
      D.dbg[16 + blockIdx.x] = tot;                     // this lane's time for the call
      D.dbg[16 + 2048 + blockIdx.x] = S.dbg_tok;
      D.dbg[16 + 4096 + blockIdx.x] = S.dbg_arcs;
      D.dbg[16 + 6144 + blockIdx.x] = S.ph[6];            // frames in the general form
      D.dbg[16 + 8192 + blockIdx.x] = S.ph[11];           // time in them
    }
#endif
  }
}

// Several workgroups per lane (blockIdx.x = lane * G + g): every frame in the general form, the
// lane's G workgroups working through it together (see WideCtx).  Every workgroup keeps its own
// replica of the lane's state; workgroup 0 of the lane writes it back.  For calls with so few
// lanes that the device would otherwise stand idle; no snapshots.
template <int NT>
__global__ void __launch_bounds__(NT, 4) k_advance_wide(DecDev D, const LaneParam *__restrict__ lanes, WideLane *wide, int G) {
  __shared__ LaneShared<NT> S;
  const int tid = threadIdx.x;
  const int lane = blockIdx.x / G, g = blockIdx.x % G;
  const LaneParam lp = lanes[lane];
  ChanState *cs = D.chan + lp.chan;
  long long *foff = D.frame_off + (size_t)lp.chan * (size_t)(D.max_frames + 2);
  if (tid == 0) {
    S.status = cs->status; S.nf = cs->num_frames; S.hist_used = cs->hist_used;
    S.lat_total = cs->lat_total;
    S.lat_room = D.lat_cap - (cs->lat_total - cs->lat_head);
    S.lat_pos = cs->lat_total % D.lat_cap;
    S.arcs_expanded = cs->arcs_expanded; S.max_pre = cs->max_pre; S.max_post = cs->max_post; S.iters_max = cs->closure_iters_max;
    S.in_off = 0; S.n_in = 0;
    if (S.nf >= 1 && S.nf <= D.max_frames + 1) { S.in_off = foff[S.nf - 1]; S.n_in = (int)(foff[S.nf] - foff[S.nf - 1]); }
#ifdef WFST_PHASE_TIMING
    for (int k = 0; k < 16; ++k) { S.ph[k] = 0; S.gph[k] = 0; }
    S.dbg_tok = 0; S.dbg_iters = 0; S.dbg_arcs = 0;
#endif
  }
  __syncthreads();
  WideCtx W{g, G, wide + lane, 0ull, D.wide_spin_limit};
  for (int f = 0; f < lp.n_frames && S.status == 0; ++f) {
    general_frame<NT, true>(D, S, W, lp.ll + (size_t)f * (size_t)lp.stride, false, D.slots + (size_t)lane * D.H,
                            D.queue + (size_t)lane * (size_t)D.qcap, D.aux + (size_t)lane * (size_t)D.auxcap,
                            D.dkey + (size_t)lane * (size_t)D.tokcap, D.dslot + (size_t)lane * (size_t)D.tokcap, foff,
                            D.hist + (size_t)lp.chan * (size_t)D.hist_cap, D.lat + (size_t)lp.chan * (size_t)D.lat_cap);
  }
  __syncthreads();
  if (g == 0 && tid == 0) {
    // (a barrier that was given up leaves the lane's state incomplete: the channel stops with a device error)
    cs->status = ld32(&wide[lane].broken) && S.status == 0 ? E_DEVICE : S.status;
    cs->num_frames = S.nf; cs->hist_used = S.hist_used;
    cs->lat_total = S.lat_total; cs->arcs_expanded = S.arcs_expanded; cs->max_pre = S.max_pre;
    cs->max_post = S.max_post; cs->closure_iters_max = S.iters_max;
#ifdef WFST_PHASE_TIMING
    if (D.dbg) { for (int k = 0; k < 16; ++k) atomicAdd(D.dbg + 16 + 10240 + k, S.gph[k]); atomicAdd(D.dbg + 6, (unsigned long long)lp.n_frames); atomicAdd(D.dbg + 5, (unsigned long long)lp.n_frames); }
#endif
  }
}
__global__ void k_zero_wide(WideLane *wide, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) { wide[i].arrived = 0ull; wide[i].broken = 0u; }
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

// Pass 1, one workgroup per listed channel: the extra cost te of every kept token (into the
// channel's scratch: te one word per token, rec_start one offset per frame) and the number of
// arcs that survive, into info[blockIdx.x].  te_stride / rs_stride: distance between the
// scratch areas of consecutive channel ids (0: a single area, for a call on one channel).
__global__ void __launch_bounds__(1024) k_final_lattice_te(DecDev D, const int32_t *chans, int use_final, uint32_t *te_base,
                                                           long long te_stride, long long *rs_base, long long rs_stride,
                                                           LatticeInfoDev *info) {
  const int tid = threadIdx.x, NTH = 1024;
  const int ch = chans[blockIdx.x];
  uint32_t *te = te_base + (size_t)ch * (size_t)te_stride;
  long long *rec_start = rs_base + (size_t)ch * (size_t)rs_stride;
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
    if (tid == 0) { LatticeInfoDev li{n_rec, 0, T + 1, 0, readable ? E_DEAD_CHANNEL : st, 0, 0.f, 0.f}; info[blockIdx.x] = li; }
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
  unsigned long long kept = 0;
  for (long long i = tid; i < n_rec; i += NTH) {
    const LatInt r = lat(i);
    const float v = __uint_as_float(ld32(&te[foff[r.frame] + r.dst])) + r.extra;
    kept += v <= D.lattice_beam ? 1 : 0;
  }
  if (kept) atomicAdd(&s_kept, kept);
  __syncthreads();
  if (tid == 0) {
    LatticeInfoDev li{n_rec, (long long)s_kept, T + 1, any_final ? 1 : 0, 0, 0, best, 0.f};
    info[blockIdx.x] = li;
  }
}

// offs[0..n]: exclusive prefix sums of the kept-arc counts of pass 1 (one block).
__global__ void __launch_bounds__(1024) k_final_lattice_offsets(const LatticeInfoDev *info, int n, long long *offs) {
  __shared__ long long part[1024];
  const int tid = threadIdx.x;
  const int per = (n + 1023) / 1024;
  const int b = tid * per, e = min(n, b + per);
  long long sum = 0;
  for (int i = b; i < e; ++i) sum += info[i].status == 0 ? info[i].arcs_kept : 0;
  part[tid] = sum;
  __syncthreads();
  for (int d = 1; d < 1024; d <<= 1) {
    const long long v = tid >= d ? part[tid - d] : 0;
    __syncthreads();
    part[tid] += v;
    __syncthreads();
  }
  long long run = part[tid] - sum;
  for (int i = b; i < e; ++i) { offs[i] = run; run += info[i].status == 0 ? info[i].arcs_kept : 0; }
  if (tid == 1023) offs[n] = part[1023];
}

// Pass 2: the surviving arcs of listed channel blockIdx.x, in the caller's form, at out[offs[blockIdx.x] ..).
// Nothing is written if the caller's buffer cannot take all channels' arcs.
__global__ void __launch_bounds__(1024) k_final_lattice_emit(DecDev D, const int32_t *chans, int n_ch, const uint32_t *te_base,
                                                             long long te_stride, const long long *offs, LatRec *out,
                                                             long long cap, const LatticeInfoDev *info) {
  if (offs[n_ch] > cap || info[blockIdx.x].status != 0) return;
  const int tid = threadIdx.x, NTH = 1024;
  const int ch = chans[blockIdx.x];
  const uint32_t *te = te_base + (size_t)ch * (size_t)te_stride;
  const ChanState *cs = D.chan + ch;
  const long long *foff = D.frame_off + (size_t)ch * (size_t)(D.max_frames + 2);
  const LatInt *lat_ring = D.lat + (size_t)ch * (size_t)D.lat_cap;
  const long long lat_first = cs->lat_head % D.lat_cap, lat_cap = D.lat_cap;
  const long long n_rec = cs->lat_total - cs->lat_head;
  LatRec *dst = out + offs[blockIdx.x];
  __shared__ unsigned long long s_pos;
  if (tid == 0) s_pos = 0;
  __syncthreads();
  for (long long i = tid; i < n_rec; i += NTH) {
    const LatInt r = lat_ring[lat_first + i < lat_cap ? lat_first + i : lat_first + i - lat_cap];
    const float v = __uint_as_float(te[foff[r.frame] + r.dst]) + r.extra;
    if (v <= D.lattice_beam) {
      const unsigned long long p = atomicAdd(&s_pos, 1ull);
      dst[p] = LatRec{r.frame, D.g.orig[r.arc], r.extra};
    }
  }
}

}  // namespace wfst
