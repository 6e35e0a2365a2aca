// What both forms of a lane's frame share: cost keys, the state table, wavefront and workgroup
// primitives, and the LDS block of a lane.
#pragma once
#include "wfst_device.h"

namespace wfst {

constexpr int NBINS = 1024;
// ---- wavefront primitives (all 64 lanes must be active) ------------------------------------
template <int CTRL> __device__ __forceinline__ int dpp_mov(int old, int v) {
  return __builtin_amdgcn_update_dpp(old, v, CTRL, 0xF, 0xF, false);
}
// inclusive prefix sum over the wavefront
__device__ __forceinline__ int wave_incl_scan(int v) {
  v += dpp_mov<0x111>(0, v);                 // row_shr:1, lanes without a source add 0
  v += dpp_mov<0x112>(0, v);
  v += dpp_mov<0x114>(0, v);
  v += dpp_mov<0x118>(0, v);                 // inclusive within each row of 16
  const int t0 = __builtin_amdgcn_readlane(v, 15), t1 = __builtin_amdgcn_readlane(v, 31), t2 = __builtin_amdgcn_readlane(v, 47);
  const int row = (threadIdx.x & 63) >> 4;
  return v + (row >= 1 ? t0 : 0) + (row >= 2 ? t1 : 0) + (row >= 3 ? t2 : 0);
}
__device__ __forceinline__ uint32_t wave_min_u32(uint32_t v) {
  v = min(v, (uint32_t)dpp_mov<0x111>((int)v, (int)v));
  v = min(v, (uint32_t)dpp_mov<0x112>((int)v, (int)v));
  v = min(v, (uint32_t)dpp_mov<0x114>((int)v, (int)v));
  v = min(v, (uint32_t)dpp_mov<0x118>((int)v, (int)v));      // lane 15 of each row: the row's minimum
  const uint32_t a = (uint32_t)__builtin_amdgcn_readlane((int)v, 15), b = (uint32_t)__builtin_amdgcn_readlane((int)v, 31);
  const uint32_t c = (uint32_t)__builtin_amdgcn_readlane((int)v, 47), d = (uint32_t)__builtin_amdgcn_readlane((int)v, 63);
  return min(min(a, b), min(c, d));
}
__device__ __forceinline__ uint32_t wave_sum_u32(uint32_t v) {
  return (uint32_t)__builtin_amdgcn_readlane(wave_incl_scan((int)v), 63);
}
// One counter update per wavefront: the lanes that call this together (same call site, any
// subset of the wave) get consecutive indices from a single atomic add.
__device__ __forceinline__ uint32_t wave_alloc(uint32_t *counter) {
  const unsigned long long m = __ballot(1);
  const int lane = threadIdx.x & 63;
  const int leader = __ffsll((long long)m) - 1;
  uint32_t base = 0;
  if (lane == leader) base = atomicAdd(counter, (uint32_t)__popcll(m));
  base = (uint32_t)__builtin_amdgcn_readlane((int)base, leader);
  return base + (uint32_t)__popcll(m & ((1ull << lane) - 1ull));
}
// Fetch ahead: start the load of the line that holds *p without waiting for it and without
// tying up a register - the value is delivered to a scratch word in LDS (`sink`: the LDS
// address of 64 floats nobody reads) by the LDS-direct form of the load.  A later ordinary
// load of the same line finds it in the cache or on its way.  The compiler does not count this
// load in its vmcnt bookkeeping; since vector memory operations complete in order, the waits
// it inserts for its own loads stay correct (an older operation in the queue can only make
// them wait for slightly more than they need).
__device__ __forceinline__ void fetch_ahead(const void *p, uint32_t sink) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dword %0, off" ::"v"(p), "s"(sink) : "m0", "memory");
}
__device__ __forceinline__ void lds_barrier() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// ---- LDS structures of a light frame ----------------------------------------------------------
// A 512-thread lane shares its compute unit's 160 KB of LDS with another lane; a 1024-thread
// lane has the unit to itself and takes structures twice as large.
template <int NT> struct LightCfg {
  static constexpr int SLOTS = NT >= 1024 ? 4096 : 2048;   // state table
  static constexpr int HBITS = NT >= 1024 ? 12 : 11;
  static constexpr int CLAIM_LIMIT = SLOTS * 3 / 4;        // states touched in a frame
  static constexpr int NIN_MAX = SLOTS / 2;                // tokens a light frame starts from
  static constexpr int QCAP = SLOTS;                       // queue entries: claims + re-expansion requests
  static constexpr int ECAP = NT >= 1024 ? 1536 : 768;     // epsilon arcs parked in LDS
  static constexpr int EXP_U = NT >= 512 ? 4 : 8;          // arcs per thread and round of the expansion
};
// queue entry (16 bits): slot | LQ_DUP (a re-expansion request for a state claimed earlier)
constexpr uint32_t LQ_DUP = 0x8000u, LQ_SLOT = 0x7FFFu;
// Slot::aux of the light table:  [31:16] first parked epsilon arc of the state
//                                [15:12] its epsilon out-degree
//                                [11:0]  its emitting out-degree; after contraction: index of
//                                        the kept token in the new frame, POS_NONE if dropped
constexpr uint32_t POS_MASK = 0xFFFu, POS_NONE = 0xFFFu;
// a round's counter: [63:42] states claimed, [41:21] entries appended that have epsilon arcs to
// relax (claims of such states, re-expansion requests), [20] give the frame up, [19:0] entries appended
constexpr unsigned long long CNT_RESTART = 1ull << 20;
constexpr uint32_t CNT_ENTRIES = 0xFFFFFu;
constexpr int CNT_EPS_SHIFT = 21, CNT_CLAIM_SHIFT = 42;
constexpr uint32_t CNT_EPS = 0x1FFFFFu;
constexpr uint32_t F_NAN = 1, F_TOKOVF = 2, F_LATOVF = 4, F_RESTART = 8;
constexpr uint32_t KEY_NONE = 0xFFFFFFFFu;
constexpr uint32_t KEY_PINF = 0xFF800000u;    // okey(+inf)

// An epsilon arc parked in LDS by the thread that claimed its source state.
struct __align__(16) ENote {
  float w; uint32_t arc;
  uint32_t dest;             // dest handle | HAS_EPS
  uint32_t dinfo_dslot;      // degree info of the dest << 16 | slot of the dest once a candidate over
                             // this arc has entered the table (0xFFFF before)
};

// Counters of one frame.  Two sets are used alternately, so that a frame can start while the
// previous frame's values are still being read; the set not in use is reset in between.
struct FrameCtr {
  // per closure round: states claimed | entries with epsilon work | CNT_RESTART | entries appended.  A round's
  // counter is final at the round's barrier (the next round uses another one), so every thread
  // reads the same value there - also the request to give the frame up.
  unsigned long long cnt[3];
  uint32_t best, flags, auxn, nout, latn, enote_n, nvalid, kmin, kmax, eps_arcs;
};
__device__ __forceinline__ void reset_ctr(FrameCtr &c) {
  c.cnt[0] = 0; c.cnt[1] = 0; c.cnt[2] = 0;
  c.best = KEY_NONE; c.flags = 0; c.auxn = 0; c.nout = 0; c.latn = 0; c.enote_n = 0; c.nvalid = 0;
  c.kmin = 0xFFFFFFFFu; c.kmax = 0; c.eps_arcs = 0;
}

// State of a lane that every thread of its workgroup holds in registers (all values uniform).
struct LaneCtx {
  int status, nf, n_in, max_pre, max_post, iters_max;
  long long in_off, hist_used, lat_room, lat_total, lat_pos, lat_head, lat_head_pos, arcs_expanded;
  uint32_t pending_clear;    // queue entries of the last light frame whose table slots are still to be cleared
  int par;                   // counter set the next light frame uses
  bool tok_valid;            // the LDS token list holds the frame the next one starts from
  bool scan_ready;           // ... and the prefix sums of its first tile's out-degrees are in LDS too
#ifdef WFST_PHASE_TIMING
  unsigned long long tlast;
#endif
};
// A value every lane of the wavefront holds alike, moved to a scalar register (values that
// come from LDS or from vector loads sit in vector registers otherwise, and so would
// everything computed from them: the lane's whole state and its arithmetic).
__device__ __forceinline__ uint32_t uni(uint32_t v) { return (uint32_t)__builtin_amdgcn_readfirstlane((int)v); }
__device__ __forceinline__ int uni(int v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ __forceinline__ unsigned long long uni(unsigned long long v) {
  return ((unsigned long long)uni((uint32_t)(v >> 32)) << 32) | uni((uint32_t)v);
}
__device__ __forceinline__ long long uni(long long v) { return (long long)uni((unsigned long long)v); }
__device__ __forceinline__ float uni(float v) { return __uint_as_float(uni(__float_as_uint(v))); }




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

constexpr int EXP_U = 4;                   // general frame: arcs per thread and round of the emitting expansion
constexpr int EPS_U = 2;                   // epsilon arcs of a token fetched together
constexpr int LAT_U = 4;                   // candidate records per thread and round of the lattice stage
constexpr uint32_t AUX_EPS = 0x80000000u;  // Aux::slot flag: the record is an epsilon arc
// Slot::aux of the general frame while a frame is being built (afterwards: index of the kept token, or ~0):
constexpr uint32_t A_FRESH = 0x80000000u;  // epsilon out-degree not counted yet
constexpr uint32_t A_KEPT_MAX = 0x20000000u;  // aux < A_KEPT_MAX: index of the kept token

// Counters of a general frame: in LDS when one workgroup owns the lane, in global memory when
// several do (then read with loads that bypass the vector cache).
struct GenCtr {
  // queue entries (low word) and states claimed (high word) of the frame: one 64-bit counter,
  // so that a claim takes one atomic for both
  unsigned long long claim_ctr;
  unsigned long long emit_arcs, eps_arcs;
  uint32_t auxn, best, flags, nvalid, nout, latn, kmin, kmax;
};
// A lane shared by several workgroups: its counters, the selection's histogram and the count
// of workgroups that have arrived at the lane's barriers so far.
struct WideLane {
  GenCtr c;
  uint32_t hist[3][NBINS];     // the selection's passes rotate through three histograms (see wide_select)
  unsigned long long arrived;
  uint32_t broken, pad;
};

// LDS of a lane's workgroup.
template <int NT>
struct LaneShared {
  int wave_tmp[NT / 64];
  int wtot[NT / 64];
  float sink[64];              // where fetch_ahead delivers; never read
  union {                      // the expansion's tile arrays and the selection's histogram never coexist
    struct { int scan[NT]; float cost[NT]; uint32_t base[NT]; };
    uint32_t hist[NBINS];
  };
  // -- general frame: its counters, and the lane's state while such a frame runs (between light
  //    frames the state lives in registers, see LaneCtx)
  GenCtr gen;                  // the general frame's counters (one workgroup per lane)
  uint32_t sel_bin, sel_below, sel_cnt;
  uint32_t wide_ok;            // outcome of the last lane barrier (lanes shared by several workgroups)
  int status, nf, max_pre, max_post, iters_max, n_in;
  long long in_off, hist_used, lat_room, lat_total, arcs_expanded;
  long long lat_pos;           // ring position of record number lat_total
  long long blk_pos;           // seal scratch
#ifdef WFST_PHASE_TIMING
  unsigned long long ph[16], gph[16], gtlast, dbg_tok, dbg_iters, dbg_arcs;
#endif
  // -- light frame
  FrameCtr fc[2];
  uint32_t tok_h[LightCfg<NT>::CLAIM_LIMIT];   // kept tokens of the last frame = queue of the next:
  float tok_c[LightCfg<NT>::CLAIM_LIMIT];      //   state handle | HAS_EPS, cost,
  uint16_t tok_i[LightCfg<NT>::CLAIM_LIMIT];   //   degree info
  uint16_t lq[LightCfg<NT>::QCAP];             // the frame's queue: claimed slots and re-expansion requests
  ENote enote[LightCfg<NT>::ECAP];             // epsilon arcs of the claimed states
  Slot table[LightCfg<NT>::SLOTS];             // state table
};

#ifdef WFST_PHASE_TIMING
// (instrumented builds) thread 0 adds the time since its previous mark to phase k
#define PHASE_MARK(k) do { if (threadIdx.x == 0) { unsigned long long t_ = wall_clock64(); atomicAdd(&S.ph[k], t_ - ctx.tlast); ctx.tlast = t_; } } while (0)
#else
#define PHASE_MARK(k) do { } while (0)
#endif
#ifdef WFST_PHASE_TIMING
#define GEN_MARK(k) do { if (threadIdx.x == 0) { unsigned long long t_ = wall_clock64(); S.gph[k] += t_ - S.gtlast; S.gtlast = t_; } } while (0)
#else
#define GEN_MARK(k) do { } while (0)
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

// The approximate form of the selection (the paper's histogram-based max-active, Section 4.1):
// ONE histogram of NBINS equal-width bins over [lo, hi]; the cut is the upper edge of the bin in
// which the running count reaches `need`, so up to that bin's population more than `need`
// values lie at or below it.  Integer counting only: the same cut whatever the thread order.
template <int NT, class F>
__device__ uint32_t block_histogram_cut(LaneShared<NT> &S, int n, uint32_t need, uint32_t lo, uint32_t hi, F val) {
  const int tid = threadIdx.x;
  constexpr int PER = NBINS / NT;
  int shift = 0;
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
    if (run < need && run + loc[q] >= need) S.sel_bin = tid * PER + q;
    run += loc[q];
  }
  __syncthreads();
  const uint32_t b = S.sel_bin;
  __syncthreads();
  const unsigned long long edge = (unsigned long long)lo + ((unsigned long long)(b + 1) << shift) - 1ull;
  return edge < hi ? (uint32_t)edge : hi;
}

}  // namespace wfst
