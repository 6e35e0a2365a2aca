// Host side of the wfst_decode C ABI (declared in include/wfst_decode.h): graph validation
// and device layout, decoder memory, launches and readouts.  Every step of the decoding
// path itself runs in the kernels of wfst_kernels.h.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstdlib>
#include <cstring>
#include <new>
#include <deque>
#include <thread>
#include <vector>

#include "../../include/wfst_decode.h"
#include "wfst_kernels.h"

using namespace wfst;

#define HIP_TRY(expr) do { if ((expr) != hipSuccess) { (void)hipGetLastError(); return WFST_E_DEVICE; } } while (0)

static_assert(sizeof(LatRec) == sizeof(wfst_lat_arc_t), "lattice record layout");
static_assert(sizeof(TokOut) == sizeof(wfst_token_t), "token layout");
static_assert(sizeof(Slot) == 16 && sizeof(HTok) == 16 && sizeof(Aux) == 16, "16-byte records");

constexpr int NT = 512;          // threads of the workgroup that owns a lane
constexpr int PARAM_RING = 8;    // pinned staging buffers for lane parameters

struct wfst_graph {
  GraphDev dev{};
  int device = 0;
  int32_t num_states = 0;
  int64_t num_arcs = 0;
  int64_t decode_bytes = 0, readout_bytes = 0;
};

struct wfst_decoder {
  const wfst_graph *graph = nullptr;
  wfst_config_t cfg{};
  DecDev dev{};
  int64_t per_channel_bytes = 0, per_lane_bytes = 0, total_bytes = 0;
  std::vector<void *> allocs;
  std::vector<uint8_t> inited;          // host mirror: channel has been initialised
  std::vector<int64_t> frames_fed;      // host mirror: rows of scores handed to the channel
  std::vector<uint32_t> stamp;          // duplicate detection within a call
  uint32_t stamp_now = 0;
  LaneParam *d_params = nullptr;        // [max_lanes]
  WideLane *d_wide = nullptr;           // [max_lanes] lanes shared by several workgroups (lane_workgroups > 1)
  LaneParam *h_params[PARAM_RING] = {};
  hipEvent_t param_ev[PARAM_RING] = {};
  int ring_pos = 0;
  int32_t *d_chans = nullptr;           // readout scratch [max(num_channels, max_lanes)]
  std::vector<int32_t> staged_chans;    // what d_chans currently holds
  PathOut *d_pathout = nullptr;
  void *d_stage = nullptr; size_t stage_bytes = 0;
  uint32_t *fl_te = nullptr;            // final-lattice scratch [num_channels][hist_cap]: extra cost of every kept token
  long long *fl_rs = nullptr;           // [num_channels][max_frames + 3]: first lattice record of every frame
  LatticeInfoDev *fl_info = nullptr;    // [num_channels]
  unsigned long long *d_cnt = nullptr;
  long long *d_offs = nullptr;          // readout scratch [max(num_channels, max_lanes) + 1]
  hipStream_t last_stream = nullptr;    // stream of the last advance call; readouts use it
  hipEvent_t last_advance = nullptr;    // recorded behind the last advance call
  bool have_last_advance = false;
  hipStream_t side_stream = nullptr;    // snapshot readouts run here, beside the decoding
  long long *h_sealed = nullptr;        // pinned [max_lanes]: id of the last snapshot each lane sealed
  int64_t next_snap_id = 1;
  struct SnapCall { int64_t id0; int32_t n_snaps, n_lanes; hipStream_t stream; };
  std::deque<SnapCall> snap_calls;      // the advance calls that seal snapshots, newest last
  std::vector<int64_t> blk_ids;         // host mirror: snapshot id each block slot is assigned to
  long long *d_ranges = nullptr;        // readout scratch [2 * max(num_channels, max_lanes) + 1]
  bool profiling = false;
  int num_cus = 0;                      // compute units of the device
  void *noalloc_scratch = nullptr;      // this device's copy of `scratch`
  std::vector<std::pair<hipEvent_t, hipEvent_t>> prof_events;
};

// Scratch of the allocation-free entry point (wfst_decode_final_lattice_noalloc): a fixed
// array in the library's device image.  Every GPU the library runs on holds its own copy at
// its own address until the process ends; in host code the array's name is only a stand-in for
// the symbol, so the address is looked up once per device and used from then on.
constexpr size_t NOALLOC_SCRATCH_BYTES = (size_t)8 << 20;
constexpr int MAX_DEVICES = 64;
static __device__ __align__(256) unsigned char scratch[NOALLOC_SCRATCH_BYTES];
static void *g_scratch_ptr[MAX_DEVICES] = {};

namespace {

// Address of `scratch` on the current device (looked up on first use, with that device current).
int scratch_address(void **out) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) { (void)hipGetLastError(); return WFST_E_DEVICE; }
  if (dev < 0 || dev >= MAX_DEVICES) return WFST_E_DEVICE;
  if (!g_scratch_ptr[dev]) {
    void *p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) { (void)hipGetLastError(); return WFST_E_DEVICE; }
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return 0;
}

template <class T> int dev_alloc(wfst_decoder *d, T **p, size_t n) {
  void *q = nullptr;
  size_t bytes = std::max<size_t>(n, 1) * sizeof(T);
  if (hipMalloc(&q, bytes) != hipSuccess) { (void)hipGetLastError(); return WFST_E_DEVICE; }
  d->allocs.push_back(q);
  d->total_bytes += (int64_t)bytes;
  *p = (T *)q;
  return 0;
}

int ensure_stage(wfst_decoder *d, size_t bytes) {
  if (bytes <= d->stage_bytes) return 0;
  if (d->d_stage) HIP_TRY(hipFree(d->d_stage));
  d->d_stage = nullptr; d->stage_bytes = 0;
  size_t want = std::max<size_t>(bytes, 1 << 20);
  HIP_TRY(hipMalloc(&d->d_stage, want));
  d->stage_bytes = want;
  return 0;
}

int check_channels(wfst_decoder *d, const int32_t *channels, int32_t n, bool need_init) {
  if (!channels && n > 0) return WFST_E_INVALID_ARG;
  if (++d->stamp_now == 0) { std::fill(d->stamp.begin(), d->stamp.end(), 0u); d->stamp_now = 1; }
  for (int32_t i = 0; i < n; ++i) {
    const int32_t c = channels[i];
    if (c < 0 || c >= d->cfg.num_channels) return WFST_E_BAD_CHANNEL;
    if (d->stamp[c] == d->stamp_now) return WFST_E_BAD_CHANNEL;
    d->stamp[c] = d->stamp_now;
    if (need_init && !d->inited[c]) return WFST_E_NOT_INIT;
  }
  return 0;
}

// Stage lane parameters through a pinned ring and launch the lane kernel.  wide: several
// workgroups per lane (only for calls without snapshots whose lanes x workgroups fit the device
// at one workgroup per compute unit, so that all of them are resident and can wait for each other).
int launch_lanes(wfst_decoder *d, const std::vector<LaneParam> &lp, int is_init, hipStream_t stream, bool wide = false) {
  const int n = (int)lp.size();
  if (n == 0) return 0;
  const int slot = d->ring_pos;
  d->ring_pos = (d->ring_pos + 1) % PARAM_RING;
  HIP_TRY(hipEventSynchronize(d->param_ev[slot]));           // its previous copy has been consumed
  std::memcpy(d->h_params[slot], lp.data(), sizeof(LaneParam) * (size_t)n);
  HIP_TRY(hipMemcpyAsync(d->d_params, d->h_params[slot], sizeof(LaneParam) * (size_t)n, hipMemcpyHostToDevice, stream));
  HIP_TRY(hipEventRecord(d->param_ev[slot], stream));
  hipEvent_t e0 = nullptr, e1 = nullptr;
  if (d->profiling && !is_init) {
    HIP_TRY(hipEventCreate(&e0)); HIP_TRY(hipEventCreate(&e1));
    HIP_TRY(hipEventRecord(e0, stream));
  }
  // A lane is one workgroup.  With at most one lane per compute unit a lane can have the whole
  // unit: 1024 threads; with more lanes two 512-thread workgroups share a unit.  The results
  // do not depend on the choice.
  if (wide) {
    const int G = std::min(d->cfg.lane_workgroups, d->num_cus / n);
    hipLaunchKernelGGL(k_zero_wide, dim3((n + 63) / 64), dim3(64), 0, stream, d->d_wide, n);
    hipLaunchKernelGGL(k_advance_wide<1024>, dim3(n * G), dim3(1024), 0, stream, d->dev, (const LaneParam *)d->d_params, d->d_wide, G);
    HIP_TRY(hipGetLastError());
    if (e0) { HIP_TRY(hipEventRecord(e1, stream)); d->prof_events.push_back({e0, e1}); }
    return 0;
  }
  int threads = d->cfg.lane_threads;
  if (threads == 0) threads = n <= d->num_cus ? 1024 : NT;
  if (threads == 1024)
    hipLaunchKernelGGL(k_advance<1024>, dim3(n), dim3(1024), 0, stream, d->dev, (const LaneParam *)d->d_params, is_init);
  else if (threads == 256)
    hipLaunchKernelGGL(k_advance<256>, dim3(n), dim3(256), 0, stream, d->dev, (const LaneParam *)d->d_params, is_init);
  else
    hipLaunchKernelGGL(k_advance<NT>, dim3(n), dim3(NT), 0, stream, d->dev, (const LaneParam *)d->d_params, is_init);
  HIP_TRY(hipGetLastError());
  if (e0) { HIP_TRY(hipEventRecord(e1, stream)); d->prof_events.push_back({e0, e1}); }
  return 0;
}

}  // namespace

extern "C" {

const char *wfst_decode_strerror(int code) {
  switch (code) {
    case WFST_OK: return "ok";
    case WFST_E_INVALID_ARG: return "invalid argument";
    case WFST_E_BAD_GRAPH: return "malformed graph";
    case WFST_E_BAD_CHANNEL: return "channel id out of range or repeated";
    case WFST_E_NOT_INIT: return "channel not initialised, or no such snapshot";
    case WFST_E_CAPACITY: return "caller buffer too small";
    case WFST_E_TOKEN_OVERFLOW: return "token capacity exceeded";
    case WFST_E_LATTICE_OVERFLOW: return "lattice capacity exceeded";
    case WFST_E_DEAD_CHANNEL: return "no token survived";
    case WFST_E_NAN_INPUT: return "NaN or +inf acoustic score";
    case WFST_E_BROKEN_TRACE: return "back-pointer chain is broken";
    case WFST_E_DEVICE: return "HIP runtime error";
    case WFST_E_HISTORY_OVERFLOW: return "token history or max_frames exceeded";
    case WFST_E_SCRATCH_LIMIT: return "channel too large for the fixed scratch of the allocation-free entry point";
    default: return "unknown error";
  }
}

int wfst_decode_graph_load(const wfst_csr_t *csr, wfst_graph_t **out) {
  if (!csr || !out) return WFST_E_INVALID_ARG;
  const int32_t Q = csr->num_states;
  const int64_t E = csr->num_arcs;
  if (Q < 1 || E < 0 || csr->num_pdfs < 1) return WFST_E_INVALID_ARG;
  if (!csr->row_offsets || !csr->final_cost) return WFST_E_INVALID_ARG;
  if (E > 0 && (!csr->ilabel || !csr->olabel || !csr->weight || !csr->nextstate)) return WFST_E_INVALID_ARG;
  if ((int64_t)Q + E >= 0x7FFFFFFFll - 1) return WFST_E_BAD_GRAPH;
  if (csr->start_state < 0 || csr->start_state >= Q) return WFST_E_BAD_GRAPH;
  if (csr->row_offsets[0] != 0 || csr->row_offsets[Q] != E) return WFST_E_BAD_GRAPH;
  for (int32_t s = 0; s < Q; ++s) {
    if (csr->row_offsets[s + 1] < csr->row_offsets[s] || csr->row_offsets[s + 1] > E) return WFST_E_BAD_GRAPH;
    const float f = csr->final_cost[s];
    if (f != f || f == -INFINITY) return WFST_E_BAD_GRAPH;
  }
  for (int64_t a = 0; a < E; ++a) {
    if (csr->nextstate[a] < 0 || csr->nextstate[a] >= Q) return WFST_E_BAD_GRAPH;
    if (csr->ilabel[a] < 0 || csr->ilabel[a] > csr->num_pdfs) return WFST_E_BAD_GRAPH;
    if (!std::isfinite(csr->weight[a])) return WFST_E_BAD_GRAPH;
    if (csr->ilabel[a] == 0 && csr->weight[a] < 0.f) return WFST_E_BAD_GRAPH;
  }
  // Zero-weight epsilon cycles are refused: around such a cycle all candidates tie in cost, the
  // tie goes to the smaller arc index, and a token's best incoming arc can then be the cycle's own
  // arc - back-pointers that loop.  (Kahn's algorithm on the sub-graph of zero-weight epsilon arcs.)
  {
    std::vector<int64_t> zero_arcs;
    try {
      for (int64_t a = 0; a < E; ++a) if (csr->ilabel[a] == 0 && csr->weight[a] == 0.f) zero_arcs.push_back(a);
      if (!zero_arcs.empty()) {
        std::vector<int32_t> src_of(zero_arcs.size()), indeg(Q, 0), order;
        std::vector<int64_t> first(Q + 1, 0);
        for (size_t k = 0; k < zero_arcs.size(); ++k) {
          const int64_t a = zero_arcs[k];
          const int32_t s = (int32_t)(std::upper_bound(csr->row_offsets, csr->row_offsets + Q + 1, a) - csr->row_offsets) - 1;
          src_of[k] = s; ++first[s + 1]; ++indeg[csr->nextstate[a]];
        }
        for (int32_t s = 0; s < Q; ++s) first[s + 1] += first[s];
        std::vector<int32_t> dst_by_src(zero_arcs.size());
        std::vector<int64_t> fill(first.begin(), first.end() - 1);
        for (size_t k = 0; k < zero_arcs.size(); ++k) dst_by_src[(size_t)fill[src_of[k]]++] = csr->nextstate[zero_arcs[k]];
        for (int32_t s = 0; s < Q; ++s) if (indeg[s] == 0) order.push_back(s);
        size_t done = 0;
        while (done < order.size()) {
          const int32_t s = order[done++];
          for (int64_t k = first[s]; k < first[s + 1]; ++k) if (--indeg[dst_by_src[(size_t)k]] == 0) order.push_back(dst_by_src[(size_t)k]);
        }
        if (order.size() != (size_t)Q) return WFST_E_BAD_GRAPH;
      }
    } catch (const std::bad_alloc &) { return WFST_E_DEVICE; }
  }
  // record layout: header of state s at handle[s] = s + (arcs of earlier states)
  const size_t R = (size_t)Q + (size_t)E;
  std::vector<uint32_t> rec, orig; std::vector<int32_t> label; std::vector<uint8_t> has_eps;
  try {
    rec.resize(3 * R); orig.assign(R, NO_ARC); label.resize(R); has_eps.assign(Q, 0);
  } catch (const std::bad_alloc &) { return WFST_E_DEVICE; }
  auto handle_of = [&](int32_t s) { return (uint32_t)((int64_t)s + csr->row_offsets[s]); };
  std::vector<uint32_t> n_emit, n_eps;
  try { n_emit.assign(Q, 0); n_eps.assign(Q, 0); } catch (const std::bad_alloc &) { return WFST_E_DEVICE; }
  for (int32_t s = 0; s < Q; ++s) {
    for (int64_t a = csr->row_offsets[s]; a < csr->row_offsets[s + 1]; ++a) (csr->ilabel[a] ? n_emit[s] : n_eps[s])++;
    has_eps[s] = n_eps[s] != 0;
  }
  const bool packed = csr->num_pdfs <= 65536;      // pdf ids leave the upper half of the third word free
  auto f2u = [](float x) { uint32_t u; std::memcpy(&u, &x, 4); return u; };
  for (int32_t s = 0; s < Q; ++s) {
    const uint32_t h = handle_of(s);
    const uint32_t ne = n_emit[s], np = n_eps[s];
    rec[3 * (size_t)h] = ne; rec[3 * (size_t)h + 1] = np; rec[3 * (size_t)h + 2] = f2u(csr->final_cost[s]);
    label[h] = s;
    uint32_t re = h + 1, rp = h + 1 + ne;            // next emitting / epsilon record
    for (int64_t a = csr->row_offsets[s]; a < csr->row_offsets[s + 1]; ++a) {
      const int32_t d = csr->nextstate[a];
      const uint32_t r = csr->ilabel[a] ? re++ : rp++;
      rec[3 * (size_t)r] = handle_of(d) | (has_eps[d] ? HAS_EPS : 0u);
      rec[3 * (size_t)r + 1] = f2u(csr->weight[a]);
      // third word: pdf id of an emitting arc, and above it the out-degrees of the destination
      const uint32_t info = packed ? (degree_info(n_emit[d], n_eps[d]) << 16) : 0u;
      rec[3 * (size_t)r + 2] = (csr->ilabel[a] ? (uint32_t)(csr->ilabel[a] - 1) : 0u) | info;
      label[r] = csr->olabel[a];
      orig[r] = (uint32_t)a;
    }
  }
  wfst_graph *g = new (std::nothrow) wfst_graph;
  if (!g) return WFST_E_DEVICE;
  (void)hipGetDevice(&g->device);
  uint32_t *d_rec = nullptr, *d_orig = nullptr; int32_t *d_label = nullptr;
  bool ok = hipMalloc((void **)&d_rec, sizeof(uint32_t) * 3 * R) == hipSuccess &&
            hipMalloc((void **)&d_orig, sizeof(uint32_t) * R) == hipSuccess &&
            hipMalloc((void **)&d_label, sizeof(int32_t) * R) == hipSuccess &&
            hipMemcpy(d_rec, rec.data(), sizeof(uint32_t) * 3 * R, hipMemcpyHostToDevice) == hipSuccess &&
            hipMemcpy(d_orig, orig.data(), sizeof(uint32_t) * R, hipMemcpyHostToDevice) == hipSuccess &&
            hipMemcpy(d_label, label.data(), sizeof(int32_t) * R, hipMemcpyHostToDevice) == hipSuccess;
  if (!ok) {
    (void)hipGetLastError();
    if (d_rec) (void)hipFree(d_rec);
    if (d_orig) (void)hipFree(d_orig);
    if (d_label) (void)hipFree(d_label);
    delete g;
    return WFST_E_DEVICE;
  }
  g->dev.rec = d_rec; g->dev.orig = d_orig; g->dev.label = d_label;
  g->dev.num_records = (uint32_t)R; g->dev.start_handle = handle_of(csr->start_state); g->dev.num_pdfs = csr->num_pdfs;
  g->dev.pdf_mask = packed ? 0xFFFFu : 0xFFFFFFFFu; g->dev.info_shift = packed ? 16 : 0;
  g->dev.start_info = degree_info(n_emit[csr->start_state], n_eps[csr->start_state]);
  g->num_states = Q; g->num_arcs = E;
  g->decode_bytes = (int64_t)(12 * R); g->readout_bytes = (int64_t)(8 * R);
  *out = g;
  return 0;
}

void wfst_decode_graph_free(wfst_graph_t *g) {
  if (!g) return;
  (void)hipFree((void *)g->dev.rec); (void)hipFree((void *)g->dev.orig); (void)hipFree((void *)g->dev.label);
  delete g;
}

int wfst_decode_graph_bytes(const wfst_graph_t *g, int64_t *decode_bytes, int64_t *readout_bytes) {
  if (!g) return WFST_E_INVALID_ARG;
  if (decode_bytes) *decode_bytes = g->decode_bytes;
  if (readout_bytes) *readout_bytes = g->readout_bytes;
  return 0;
}

int wfst_decode_create(const wfst_graph_t *graph, const wfst_config_t *config, wfst_decoder_t **out) {
  if (!graph || !config || !out) return WFST_E_INVALID_ARG;
  wfst_config_t c = *config;
  if (!(c.beam > 0.f) || !(c.lattice_beam >= 0.f) || c.max_active < 1 || c.num_channels < 1 || c.max_lanes < 1 ||
      c.max_frames < 1 || c.token_capacity < 0 || c.aux_capacity < 0 || c.history_capacity < 0 || c.lattice_capacity < 0)
    return WFST_E_INVALID_ARG;
  if (c.max_active > (1 << 26)) return WFST_E_INVALID_ARG;
  if (c.token_capacity == 0) c.token_capacity = (int32_t)std::min<int64_t>(4ll * c.max_active, 1 << 28);
  if (c.token_capacity < 2 || c.token_capacity > (1 << 28)) return WFST_E_INVALID_ARG;
  if (c.aux_capacity == 0) c.aux_capacity = (int32_t)std::min<int64_t>(2ll * c.token_capacity, 1 << 29);
  if (c.history_capacity == 0)          // (the approximate cut keeps somewhat more than max_active per frame)
    c.history_capacity = ((int64_t)c.max_frames + 1) * (c.approximate ? (int64_t)c.max_active + c.max_active / 4 + 64 : (int64_t)c.max_active);
  if (c.lattice_capacity == 0) c.lattice_capacity = 64ll * c.max_active;
  if (c.snapshot_blocks < 0 || c.snapshot_block_capacity < 0) return WFST_E_INVALID_ARG;
  if (c.lane_threads != 0 && c.lane_threads != 256 && c.lane_threads != 512 && c.lane_threads != 1024) return WFST_E_INVALID_ARG;
  if (c.frame_form != 0 && c.frame_form != 1) return WFST_E_INVALID_ARG;
  if (c.approximate != 0 && c.approximate != 1) return WFST_E_INVALID_ARG;
  if (c.lane_workgroups < 0 || c.lane_workgroups > 64) return WFST_E_INVALID_ARG;
  if (!c.lattice_on) c.snapshot_blocks = 0;
  if (c.snapshot_blocks > 0 && c.snapshot_block_capacity == 0)
    c.snapshot_block_capacity = std::min<int64_t>(c.lattice_capacity, 4096ll * c.max_lanes);
  wfst_decoder *d = new (std::nothrow) wfst_decoder;
  if (!d) return WFST_E_DEVICE;
  d->graph = graph; d->cfg = c;
  {
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) {
      (void)hipGetLastError(); delete d; return WFST_E_DEVICE;
    }
    d->num_cus = cus;
    const int src = scratch_address(&d->noalloc_scratch);
    if (src) { delete d; return src; }
  }
  DecDev &D = d->dev;
  D.g = graph->dev;
  int hbits = 4;
  while ((1ll << hbits) < 2ll * c.token_capacity) ++hbits;
  D.H = 1u << hbits; D.hbits = hbits;
  D.qcap = (int32_t)std::min<int64_t>(2ll * c.token_capacity, 0x3FFFFFFF);
  D.auxcap = c.aux_capacity; D.tokcap = c.token_capacity; D.max_frames = c.max_frames; D.max_active = c.max_active;
  D.lattice_on = c.lattice_on ? 1 : 0; D.beam = c.beam; D.lattice_beam = c.lattice_beam;
  D.force_general = c.frame_form == 1 ? 1 : 0;
  D.approximate = c.approximate;
  D.wide_spin_limit = WIDE_SPIN_LIMIT;
  if (const char *e = std::getenv("WFST_DECODE_WIDE_SPIN_LIMIT")) {   // a testing aid: give lane barriers up early
    const long v = std::strtol(e, nullptr, 10);
    if (v >= 1 && v <= (long)WIDE_SPIN_LIMIT) D.wide_spin_limit = (uint32_t)v;
  }
  D.hist_cap = c.history_capacity; D.lat_cap = c.lattice_on ? c.lattice_capacity : 1;
  const size_t nc = (size_t)c.num_channels, nl = (size_t)c.max_lanes;
  int rc = 0;
  if (!rc) rc = dev_alloc(d, &D.chan, nc);
  if (!rc) rc = dev_alloc(d, &D.snap, nc * (size_t)SNAP_RING);
  if (!rc) rc = dev_alloc(d, &D.frame_off, nc * (size_t)(c.max_frames + 2));
  if (!rc) rc = dev_alloc(d, &D.hist, nc * (size_t)D.hist_cap);
  if (!rc) rc = dev_alloc(d, &D.lat, nc * (size_t)D.lat_cap);
  D.pc_wcap = 4 * (c.max_frames + 1) + 64;
  if (!rc) rc = dev_alloc(d, &D.pc_entry, nc * (size_t)(c.max_frames + 2));
  if (!rc) rc = dev_alloc(d, &D.pc_wcount, nc * (size_t)(c.max_frames + 2));
  if (!rc) rc = dev_alloc(d, &D.pc_words, nc * (size_t)D.pc_wcap);
  d->per_channel_bytes = d->total_bytes / (int64_t)nc;
  const int64_t before_lanes = d->total_bytes;
  if (!rc) rc = dev_alloc(d, &D.slots, nl * (size_t)D.H);
  if (!rc) rc = dev_alloc(d, &D.queue, nl * (size_t)D.qcap);
  if (!rc) rc = dev_alloc(d, &D.aux, nl * (size_t)D.auxcap);
  if (!rc) rc = dev_alloc(d, &D.dkey, nl * (size_t)D.tokcap);
  if (!rc) rc = dev_alloc(d, &D.dslot, nl * (size_t)D.tokcap);
  if (!rc) rc = dev_alloc(d, &d->d_params, nl);
  if (!rc && c.lane_workgroups > 1) rc = dev_alloc(d, &d->d_wide, nl);
  d->per_lane_bytes = (d->total_bytes - before_lanes) / (int64_t)nl;
  if (!rc) rc = dev_alloc(d, &d->d_chans, std::max(nc, nl));
  if (!rc) rc = dev_alloc(d, &d->d_pathout, std::max(nc, nl));
  if (!rc) rc = dev_alloc(d, &d->d_cnt, 1);
#ifdef WFST_PHASE_TIMING
  if (!rc) rc = dev_alloc(d, &D.dbg, 8 + 16384);
  if (!rc && hipMemset(D.dbg, 0, 8 * (8 + 16384)) != hipSuccess) rc = WFST_E_DEVICE;
#endif
  if (!rc) rc = dev_alloc(d, &d->d_offs, std::max(nc, nl) + 1);
  if (!rc) rc = dev_alloc(d, &d->d_ranges, 2 * std::max(nc, nl) + 1);
  if (!rc && c.lattice_on) {
    rc = dev_alloc(d, &d->fl_te, nc * (size_t)D.hist_cap);
    if (!rc) rc = dev_alloc(d, &d->fl_rs, nc * (size_t)(c.max_frames + 3));
    if (!rc) rc = dev_alloc(d, &d->fl_info, nc);
  }
  D.n_blk = c.snapshot_blocks; D.blk_cap = c.snapshot_block_capacity;
  if (!rc && D.n_blk > 0) {
    rc = dev_alloc(d, &D.blk, (size_t)D.n_blk);
    if (!rc) rc = dev_alloc(d, &D.blk_recs, (size_t)D.n_blk * (size_t)D.blk_cap);
    if (!rc && hipMemset(D.blk, 0, sizeof(SnapBlock) * (size_t)D.n_blk) != hipSuccess) rc = WFST_E_DEVICE;
    d->blk_ids.assign((size_t)D.n_blk, 0);
  }
  if (!rc) {
    bool ok = hipMemset(D.chan, 0, sizeof(ChanState) * nc) == hipSuccess;
    for (int i = 0; ok && i < PARAM_RING; ++i)
      ok = hipHostMalloc((void **)&d->h_params[i], sizeof(LaneParam) * nl) == hipSuccess &&
           hipEventCreateWithFlags(&d->param_ev[i], hipEventDisableTiming) == hipSuccess;
    ok = ok && hipMemset(D.snap, 0, sizeof(ChanSnap) * nc * SNAP_RING) == hipSuccess &&
         hipStreamCreateWithFlags(&d->side_stream, hipStreamNonBlocking) == hipSuccess &&
         hipEventCreateWithFlags(&d->last_advance, hipEventDisableTiming) == hipSuccess &&
         hipHostMalloc((void **)&d->h_sealed, sizeof(long long) * nl) == hipSuccess;
    if (ok) {
      std::memset(d->h_sealed, 0, sizeof(long long) * nl);
      ok = hipHostGetDevicePointer((void **)&D.lane_sealed, d->h_sealed, 0) == hipSuccess;
    }
    if (ok) {
      hipLaunchKernelGGL(k_fill_slots, dim3(1024), dim3(256), 0, 0, D.slots, nl * (size_t)D.H);
      ok = hipGetLastError() == hipSuccess && hipDeviceSynchronize() == hipSuccess;
    }
    if (!ok) { (void)hipGetLastError(); rc = WFST_E_DEVICE; }
  }
  if (rc) { wfst_decode_destroy(d); return rc; }
  d->inited.assign(nc, 0); d->frames_fed.assign(nc, 0); d->stamp.assign(nc, 0);
  *out = d;
  return 0;
}

void wfst_decode_destroy(wfst_decoder_t *d) {
  if (!d) return;
  (void)hipDeviceSynchronize();
  for (void *p : d->allocs) (void)hipFree(p);
  if (d->d_stage) (void)hipFree(d->d_stage);
  for (int i = 0; i < PARAM_RING; ++i) {
    if (d->h_params[i]) (void)hipHostFree(d->h_params[i]);
    if (d->param_ev[i]) (void)hipEventDestroy(d->param_ev[i]);
  }
  for (auto &p : d->prof_events) { (void)hipEventDestroy(p.first); (void)hipEventDestroy(p.second); }
  if (d->side_stream) (void)hipStreamDestroy(d->side_stream);
  if (d->last_advance) (void)hipEventDestroy(d->last_advance);
  if (d->h_sealed) (void)hipHostFree(d->h_sealed);
  delete d;
}

int wfst_decode_state_bytes(const wfst_decoder_t *d, int64_t *per_channel, int64_t *per_lane, int64_t *total) {
  if (!d) return WFST_E_INVALID_ARG;
  if (per_channel) *per_channel = d->per_channel_bytes;
  if (per_lane) *per_lane = d->per_lane_bytes;
  if (total) *total = d->total_bytes;
  return 0;
}

int wfst_decode_init_channels(wfst_decoder_t *d, const int32_t *channels, int32_t n) {
  if (!d || n < 0) return WFST_E_INVALID_ARG;
  int rc = check_channels(d, channels, n, false);
  if (rc) return rc;
  HIP_TRY(hipStreamSynchronize(d->last_stream));      // earlier work on these channels must be over
  HIP_TRY(hipStreamSynchronize(d->side_stream));
  std::vector<LaneParam> lp;
  for (int32_t i = 0; i < n; i += d->cfg.max_lanes) {
    const int32_t m = std::min(d->cfg.max_lanes, n - i);
    lp.clear();
    for (int32_t k = 0; k < m; ++k) lp.push_back(LaneParam{nullptr, channels[i + k], 1, 0, 0, 0, 0, 0});
    rc = launch_lanes(d, lp, 1, nullptr);
    if (rc) return rc;
  }
  HIP_TRY(hipStreamSynchronize(nullptr));
  for (int32_t i = 0; i < n; ++i) { d->inited[channels[i]] = 1; d->frames_fed[channels[i]] = 0; }
  return 0;
}

int wfst_decode_free_channels(wfst_decoder_t *d, const int32_t *channels, int32_t n) {
  if (!d || n < 0) return WFST_E_INVALID_ARG;
  int rc = check_channels(d, channels, n, false);
  if (rc) return rc;
  for (int32_t i = 0; i < n; ++i) d->inited[channels[i]] = 0;
  return 0;
}

static int advance_impl(wfst_decoder_t *d, const int32_t *channels, int32_t n_lanes, const float *const *loglikes,
                        const int32_t *strides, const int32_t *n_frames, int32_t snapshot_every, void *stream,
                        int64_t *first_id, int32_t *n_snapshots) {
  if (!d || n_lanes < 0 || n_lanes > d->cfg.max_lanes || snapshot_every < 0) return WFST_E_INVALID_ARG;
  if (first_id) *first_id = 0;
  if (n_snapshots) *n_snapshots = 0;
  if (n_lanes == 0) return 0;
  if (!loglikes || !strides || !n_frames) return WFST_E_INVALID_ARG;
  int rc = check_channels(d, channels, n_lanes, true);
  if (rc) return rc;
  for (int32_t i = 0; i < n_lanes; ++i) {
    if (n_frames[i] < 0 || strides[i] < d->dev.g.num_pdfs) return WFST_E_INVALID_ARG;
    if (n_frames[i] > 0 && !loglikes[i]) return WFST_E_INVALID_ARG;
    if (d->frames_fed[channels[i]] + n_frames[i] > d->cfg.max_frames) return WFST_E_HISTORY_OVERFLOW;
  }
  // snapshots of the call: one per snapshot_every frames of its longest lane, at least one
  int32_t n_snaps = 0;
  if (snapshot_every > 0) {
    int32_t longest = 0;
    for (int32_t i = 0; i < n_lanes; ++i) longest = std::max(longest, n_frames[i]);
    n_snaps = std::max(1, (longest + snapshot_every - 1) / snapshot_every);
    if (n_snaps > SNAP_RING || (d->dev.n_blk > 0 && n_snaps > d->dev.n_blk)) return WFST_E_INVALID_ARG;
  }
  const int64_t id0 = d->next_snap_id;
  std::vector<LaneParam> lp((size_t)n_lanes);
  for (int32_t i = 0; i < n_lanes; ++i) {
    lp[i] = LaneParam{loglikes[i], channels[i], n_frames[i], strides[i], snapshot_every, id0, n_snaps, 0};
    d->frames_fed[channels[i]] += n_frames[i];
  }
  // The lanes' scratch and parameter block belong to the decoder, not to the call: a call on
  // another stream than the previous one first waits for that one.
  if (d->have_last_advance && (hipStream_t)stream != d->last_stream)
    HIP_TRY(hipStreamWaitEvent((hipStream_t)stream, d->last_advance, 0));
  d->last_stream = (hipStream_t)stream;
  if (n_snaps > 0 && d->dev.n_blk > 0) {     // the blocks these snapshots will fill start empty
    hipLaunchKernelGGL(k_reset_blocks, dim3((n_snaps + 63) / 64), dim3(64), 0, (hipStream_t)stream, d->dev, (long long)id0, n_snaps);
    HIP_TRY(hipGetLastError());
    for (int32_t j = 0; j < n_snaps; ++j) d->blk_ids[(size_t)((id0 + j) % d->dev.n_blk)] = id0 + j;
  }
  const bool wide = d->cfg.lane_workgroups > 1 && n_snaps == 0 && 2 * n_lanes <= d->num_cus;
  rc = launch_lanes(d, lp, 0, (hipStream_t)stream, wide);
  if (rc) return rc;
  HIP_TRY(hipEventRecord(d->last_advance, (hipStream_t)stream));
  d->have_last_advance = true;
  if (n_snaps > 0) {
    d->next_snap_id += n_snaps;
    d->snap_calls.push_back({id0, n_snaps, n_lanes, (hipStream_t)stream});
    if (d->snap_calls.size() > 64) d->snap_calls.pop_front();
    if (first_id) *first_id = id0;
    if (n_snapshots) *n_snapshots = n_snaps;
  }
  return 0;
}

int wfst_decode_advance(wfst_decoder_t *d, const int32_t *channels, int32_t n_lanes, const float *const *loglikes,
                        const int32_t *strides, const int32_t *n_frames, void *stream) {
  return advance_impl(d, channels, n_lanes, loglikes, strides, n_frames, 0, stream, nullptr, nullptr);
}

int wfst_decode_advance_snapshots(wfst_decoder_t *d, const int32_t *channels, int32_t n_lanes, const float *const *loglikes,
                                  const int32_t *strides, const int32_t *n_frames, int32_t snapshot_every, void *stream,
                                  int64_t *first_id, int32_t *n_snapshots) {
  if (snapshot_every < 1 || !first_id || !n_snapshots) return WFST_E_INVALID_ARG;
  return advance_impl(d, channels, n_lanes, loglikes, strides, n_frames, snapshot_every, stream, first_id, n_snapshots);
}

// Wait on the host until every lane of the call that seals snapshot `id` has sealed it.  The
// lanes publish their progress in pinned host memory; the kernel never waits for anybody, so
// this cannot stall the device.  If the call's stream has drained and the snapshot is still
// missing, something went wrong on the device.
int wfst_decode_snapshot_wait(wfst_decoder_t *d, int64_t id) {
  if (!d || id < 1) return WFST_E_INVALID_ARG;
  const wfst_decoder::SnapCall *call = nullptr;
  for (const auto &c : d->snap_calls) if (id >= c.id0 && id < c.id0 + c.n_snaps) call = &c;
  if (!call) return WFST_E_NOT_INIT;
  bool stream_done = false;
  for (;;) {
    bool all = true;
    for (int32_t i = 0; i < call->n_lanes && all; ++i)
      all = __atomic_load_n(&d->h_sealed[i], __ATOMIC_ACQUIRE) >= id;
    if (all) return 0;
    if (stream_done) return WFST_E_DEVICE;
    const hipError_t q = hipStreamQuery(call->stream);
    if (q == hipSuccess) stream_done = true;            // look at the progress words once more, then give up
    else if (q != hipErrorNotReady) { (void)hipGetLastError(); return WFST_E_DEVICE; }
    else std::this_thread::yield();
  }
}


// Readouts run on the stream of the decoder's last advance call and wait for that stream
// only, so decoders working on different streams do not wait for each other.
static hipError_t copy_sync_on(hipStream_t st, void *dst, const void *src, size_t bytes, hipMemcpyKind kind) {
  hipError_t e = hipMemcpyAsync(dst, src, bytes, kind, st);
  if (e != hipSuccess) return e;
  return hipStreamSynchronize(st);
}
static hipError_t copy_sync(wfst_decoder *d, void *dst, const void *src, size_t bytes, hipMemcpyKind kind) {
  return copy_sync_on(d->last_stream, dst, src, bytes, kind);
}

// Stream a readout runs on.  A snapshot readout runs on the decoder's side stream once all
// lanes have sealed the snapshot; it does not wait for the decoding that goes on behind it.
static int readout_stream(wfst_decoder *d, int64_t snap_id, hipStream_t *st) {
  if (snap_id <= 0) { *st = d->last_stream; return 0; }
  const int rc = wfst_decode_snapshot_wait(d, snap_id);
  if (rc) return rc;
  *st = d->side_stream;
  return 0;
}

// Copy the channel list to the device unless it is the one already there.
static int stage_channels(wfst_decoder *d, hipStream_t st, const int32_t *channels, int32_t n) {
  if ((int32_t)d->staged_chans.size() == n && std::memcmp(d->staged_chans.data(), channels, sizeof(int32_t) * (size_t)n) == 0) return 0;
  HIP_TRY(copy_sync_on(st, d->d_chans, channels, sizeof(int32_t) * (size_t)n, hipMemcpyHostToDevice));
  d->staged_chans.assign(channels, channels + n);
  return 0;
}

static int best_path_batch_impl(wfst_decoder_t *d, int64_t snap, const int32_t *channels, int32_t n, int32_t use_final,
                                int32_t *words, int32_t words_cap, int32_t *n_words, float *total_cost,
                                int32_t *reached_final, int32_t *status) {
  if (!d || n < 0 || words_cap < 0 || (n > 0 && (!n_words || !total_cost || !reached_final || !status))) return WFST_E_INVALID_ARG;
  if (words_cap > 0 && !words && n > 0) return WFST_E_INVALID_ARG;
  if (n == 0) return 0;
  int rc = check_channels(d, channels, n, true);
  if (rc) return rc;
  hipStream_t st = nullptr;
  rc = readout_stream(d, snap, &st);
  if (rc) return rc;
  const long long sn = snap > 0 ? (long long)snap : 0ll;
  if (sizeof(int32_t) * (size_t)n * (size_t)std::max(words_cap, 1) > d->stage_bytes) {
    HIP_TRY(hipStreamSynchronize(st));            // the staging buffer is about to be replaced
    rc = ensure_stage(d, sizeof(int32_t) * (size_t)n * (size_t)std::max(words_cap, 1));
    if (rc) return rc;
  }
  rc = stage_channels(d, st, channels, n);
  if (rc) return rc;
  HIP_TRY(hipMemsetAsync(d->d_cnt, 0, sizeof(unsigned long long), st));
  if (snap > 0)      // beside a running decode kernel: one thread per channel
    hipLaunchKernelGGL(k_best_path_words<1>, dim3((n + 63) / 64), dim3(64), 0, st, d->dev, (const int32_t *)d->d_chans, n,
                       use_final, sn, (int32_t *)d->d_stage, words_cap, d->d_cnt, d->d_pathout);
  else
    hipLaunchKernelGGL(k_best_path_words<64>, dim3(n), dim3(64), 0, st, d->dev, (const int32_t *)d->d_chans, n,
                       use_final, sn, (int32_t *)d->d_stage, words_cap, d->d_cnt, d->d_pathout);
  HIP_TRY(hipGetLastError());
  std::vector<PathOut> po((size_t)n);
  HIP_TRY(copy_sync_on(st, po.data(), d->d_pathout, sizeof(PathOut) * (size_t)n, hipMemcpyDeviceToHost));
  long long used = 0;
  for (int32_t i = 0; i < n; ++i) if (po[i].status == 0) used = std::max(used, po[i].word_off + po[i].n_words);
  std::vector<int32_t> w((size_t)used);
  if (used > 0) HIP_TRY(copy_sync_on(st, w.data(), d->d_stage, sizeof(int32_t) * (size_t)used, hipMemcpyDeviceToHost));
  for (int32_t i = 0; i < n; ++i) {
    if (po[i].status == WFST_E_CAPACITY && po[i].n_words <= words_cap) {
      // the remembered-path scratch was too small for this path: trace it in full instead
      int32_t ch = channels[i];
      HIP_TRY(copy_sync_on(st, d->d_chans, &ch, sizeof(int32_t), hipMemcpyHostToDevice));
      d->staged_chans.clear();
      hipLaunchKernelGGL(k_best_path, dim3(1), dim3(64), 0, st, d->dev, (const int32_t *)d->d_chans, use_final, sn,
                         (int32_t *)d->d_stage, words_cap, (uint32_t *)nullptr, 0, d->d_pathout);
      HIP_TRY(hipGetLastError());
      HIP_TRY(copy_sync_on(st, &po[i], d->d_pathout, sizeof(PathOut), hipMemcpyDeviceToHost));
      if (po[i].status == 0 && po[i].n_words > 0)
        HIP_TRY(copy_sync_on(st, words + (size_t)i * words_cap, (int32_t *)d->d_stage + (words_cap - po[i].n_words),
                          sizeof(int32_t) * (size_t)po[i].n_words, hipMemcpyDeviceToHost));
    } else if (po[i].status == 0 && po[i].n_words > 0) {
      std::memcpy(words + (size_t)i * words_cap, w.data() + po[i].word_off, sizeof(int32_t) * (size_t)po[i].n_words);
    }
    status[i] = po[i].status; n_words[i] = po[i].n_words; total_cost[i] = po[i].total_cost; reached_final[i] = po[i].reached_final;
  }
  return 0;
}

int wfst_decode_best_path_batch(wfst_decoder_t *d, const int32_t *channels, int32_t n, int32_t use_final,
                                int32_t *words, int32_t words_cap, int32_t *n_words, float *total_cost,
                                int32_t *reached_final, int32_t *status) {
  return best_path_batch_impl(d, 0, channels, n, use_final, words, words_cap, n_words, total_cost, reached_final, status);
}

int wfst_decode_snapshot_best_path_batch(wfst_decoder_t *d, int64_t snapshot_id, const int32_t *channels, int32_t n,
                                         int32_t use_final, int32_t *words, int32_t words_cap, int32_t *n_words,
                                         float *total_cost, int32_t *reached_final, int32_t *status) {
  if (snapshot_id < 1) return WFST_E_INVALID_ARG;
  return best_path_batch_impl(d, snapshot_id, channels, n, use_final, words, words_cap, n_words, total_cost, reached_final, status);
}

int wfst_decode_best_path(wfst_decoder_t *d, int32_t channel, int32_t use_final, int32_t *words, int32_t cap,
                          int32_t *n_words, float *total_cost, int32_t *reached_final) {
  if (!n_words || !total_cost || !reached_final) return WFST_E_INVALID_ARG;
  int32_t nw = 0, rf = 0, st = 0; float tc = 0.f;
  int rc = wfst_decode_best_path_batch(d, &channel, 1, use_final, words, cap, &nw, &tc, &rf, &st);
  if (rc) return rc;
  if (st == WFST_E_CAPACITY) { *n_words = nw; return st; }
  if (st) return st;
  *n_words = nw; *total_cost = tc; *reached_final = rf;
  return 0;
}

int wfst_decode_best_path_arcs(wfst_decoder_t *d, int32_t channel, int32_t use_final, uint32_t *arcs, int32_t cap,
                               int32_t *n_arcs, float *total_cost, int32_t *reached_final) {
  if (!d || cap < 0 || !n_arcs || !total_cost || !reached_final || (cap > 0 && !arcs)) return WFST_E_INVALID_ARG;
  int rc = check_channels(d, &channel, 1, true);
  if (rc) return rc;
  HIP_TRY(hipStreamSynchronize(d->last_stream));
  rc = ensure_stage(d, sizeof(uint32_t) * (size_t)std::max(cap, 1));
  if (rc) return rc;
  HIP_TRY(copy_sync(d, d->d_chans, &channel, sizeof(int32_t), hipMemcpyHostToDevice));
  d->staged_chans.clear();
  hipLaunchKernelGGL(k_best_path, dim3(1), dim3(64), 0, d->last_stream, d->dev, (const int32_t *)d->d_chans, use_final, 0,
                     (int32_t *)nullptr, 0, cap > 0 ? (uint32_t *)d->d_stage : nullptr, cap, d->d_pathout);
  HIP_TRY(hipGetLastError());
  PathOut po;
  HIP_TRY(copy_sync(d, &po, d->d_pathout, sizeof(PathOut), hipMemcpyDeviceToHost));
  if (po.status == 0 && po.n_arcs > cap) { *n_arcs = po.n_arcs; return WFST_E_CAPACITY; }
  if (po.status) return po.status;
  if (po.n_arcs > 0)
    HIP_TRY(copy_sync(d, arcs, (uint32_t *)d->d_stage + (cap - po.n_arcs), sizeof(uint32_t) * (size_t)po.n_arcs, hipMemcpyDeviceToHost));
  *n_arcs = po.n_arcs; *total_cost = po.total_cost; *reached_final = po.reached_final;
  return 0;
}

static int read_chan(wfst_decoder *d, int32_t channel, ChanState *cs) {
  HIP_TRY(hipStreamSynchronize(d->last_stream));
  HIP_TRY(copy_sync(d, cs, d->dev.chan + channel, sizeof(ChanState), hipMemcpyDeviceToHost));
  return 0;
}

int wfst_decode_lattice_arcs(wfst_decoder_t *d, int32_t channel, int32_t from_frame, wfst_lat_arc_t *out, int64_t cap,
                             int64_t *n, int32_t out_is_device) {
  if (!d || !n || cap < 0 || (cap > 0 && !out)) return WFST_E_INVALID_ARG;
  int rc = check_channels(d, &channel, 1, true);
  if (rc) return rc;
  ChanState cs;
  rc = read_chan(d, channel, &cs);
  if (rc) return rc;
  if (cs.status != 0 && cs.status != WFST_E_DEAD_CHANNEL && cs.status != WFST_E_NAN_INPUT) return cs.status;
  const long long have = cs.lat_total - cs.lat_head;
  rc = ensure_stage(d, sizeof(LatRec) * (size_t)std::max<long long>(have, 1));
  if (rc) return rc;
  HIP_TRY(hipMemsetAsync(d->d_cnt, 0, sizeof(unsigned long long), d->last_stream));
  if (have > 0) {
    const int blocks = (int)std::min<long long>((have + 255) / 256, 4096);
    hipLaunchKernelGGL(k_export_lattice, dim3(blocks), dim3(256), 0, d->last_stream, d->dev, channel,
                       cs.lat_head % d->dev.lat_cap, have, from_frame, (LatRec *)d->d_stage, have, d->d_cnt);
    HIP_TRY(hipGetLastError());
  }
  unsigned long long cnt = 0;
  HIP_TRY(copy_sync(d, &cnt, d->d_cnt, sizeof(cnt), hipMemcpyDeviceToHost));
  if ((int64_t)cnt > cap) { *n = (int64_t)cnt; return WFST_E_CAPACITY; }
  if (cnt > 0)
    HIP_TRY(copy_sync(d, out, d->d_stage, sizeof(LatRec) * (size_t)cnt, out_is_device ? hipMemcpyDeviceToDevice : hipMemcpyDeviceToHost));
  hipLaunchKernelGGL(k_reset_lattice, dim3(1), dim3(1), 0, d->last_stream, d->dev, channel);
  HIP_TRY(hipGetLastError());
  HIP_TRY(hipStreamSynchronize(d->last_stream));
  *n = (int64_t)cnt;
  return 0;
}

int wfst_decode_lattice_arcs_batch(wfst_decoder_t *d, const int32_t *channels, int32_t n, wfst_lat_arc_t *out,
                                   int64_t cap, int64_t *offsets, int32_t out_is_device) {
  if (!d || n < 0 || cap < 0 || !offsets || (cap > 0 && !out)) return WFST_E_INVALID_ARG;
  offsets[0] = 0;
  if (n == 0) return 0;
  int rc = check_channels(d, channels, n, true);
  if (rc) return rc;
  hipStream_t st = d->last_stream;
  rc = stage_channels(d, st, channels, n);
  if (rc) return rc;
  LatRec *dst = (LatRec *)out;
  if (!out_is_device) {                 // host output goes through device staging of the caller's capacity
    if (sizeof(LatRec) * (size_t)std::max<int64_t>(cap, 1) > d->stage_bytes) HIP_TRY(hipStreamSynchronize(st));
    rc = ensure_stage(d, sizeof(LatRec) * (size_t)std::max<int64_t>(cap, 1));
    if (rc) return rc;
    dst = (LatRec *)d->d_stage;
  }
  // offsets, copy and reset are queued back to back; the copy and the reset check the capacity
  // on the device, so the host waits only once
  hipLaunchKernelGGL(k_lattice_offsets, dim3(1), dim3(1024), 0, st, d->dev, (const int32_t *)d->d_chans, n, d->d_offs);
  hipLaunchKernelGGL(k_export_lattice_batch, dim3(n, 8), dim3(256), 0, st, d->dev, (const int32_t *)d->d_chans, n,
                     (const long long *)d->d_offs, dst, (long long)cap);
  hipLaunchKernelGGL(k_reset_lattice_batch, dim3((n + 255) / 256), dim3(256), 0, st, d->dev, (const int32_t *)d->d_chans, n,
                     (const long long *)d->d_offs, (long long)cap);
  HIP_TRY(hipGetLastError());
  static_assert(sizeof(long long) == sizeof(int64_t), "offset width");
  HIP_TRY(copy_sync_on(st, offsets, d->d_offs, sizeof(long long) * ((size_t)n + 1), hipMemcpyDeviceToHost));
  const long long total = offsets[n];
  if (total > cap) return WFST_E_CAPACITY;
  if (!out_is_device && total > 0) HIP_TRY(copy_sync_on(st, out, dst, sizeof(LatRec) * (size_t)total, hipMemcpyDeviceToHost));
  return 0;
}

int wfst_decode_snapshot_lattice_arcs(wfst_decoder_t *d, int64_t snapshot_id, const int32_t *channels, int32_t n,
                                      int64_t *starts, int64_t *counts, wfst_lat_arc_t *out, int64_t cap,
                                      int32_t out_is_device, int64_t *total, const wfst_lat_arc_t **block) {
  if (!d || snapshot_id < 1 || n < 0 || cap < 0 || !total || (n > 0 && (!starts || !counts))) return WFST_E_INVALID_ARG;
  if (d->dev.n_blk <= 0) return WFST_E_INVALID_ARG;              // the decoder was created without snapshot blocks
  int rc = check_channels(d, channels, n, true);
  if (rc) return rc;
  hipStream_t st = nullptr;
  rc = readout_stream(d, snapshot_id, &st);
  if (rc) return rc;
  const size_t slot = (size_t)(snapshot_id % d->dev.n_blk);
  if (d->blk_ids[slot] != snapshot_id) return WFST_E_NOT_INIT;   // its block has been given to a later snapshot
  if (n > 0) {
    rc = stage_channels(d, st, channels, n);
    if (rc) return rc;
  }
  hipLaunchKernelGGL(k_snapshot_ranges, dim3((std::max(n, 1) + 255) / 256), dim3(256), 0, st, d->dev, (const int32_t *)d->d_chans, n,
                     (long long)snapshot_id, d->d_ranges);
  HIP_TRY(hipGetLastError());
  std::vector<long long> r(2 * (size_t)n + 1);
  HIP_TRY(copy_sync_on(st, r.data(), d->d_ranges, sizeof(long long) * r.size(), hipMemcpyDeviceToHost));
  if (r[2 * (size_t)n] < 0) return WFST_E_NOT_INIT;
  for (int32_t i = 0; i < n; ++i) { starts[i] = r[2 * (size_t)i]; counts[i] = r[2 * (size_t)i + 1]; }
  *total = r[2 * (size_t)n];
  const LatRec *src = d->dev.blk_recs + slot * (size_t)d->dev.blk_cap;
  if (block) *block = (const wfst_lat_arc_t *)src;
  if (out) {
    if (*total > cap) return WFST_E_CAPACITY;
    if (*total > 0)
      HIP_TRY(copy_sync_on(st, out, src, sizeof(LatRec) * (size_t)*total, out_is_device ? hipMemcpyDeviceToDevice : hipMemcpyDeviceToHost));
  }
  return 0;
}

// The final-lattice pass over the staged channel list: extra costs and counts, offsets, emission.
// te / rs / info: the scratch (per channel id with the strides given, or one area with strides 0).
static int final_lattice_launch(wfst_decoder *d, int32_t n, int32_t use_final, uint32_t *te, long long te_stride, long long *rs,
                                long long rs_stride, LatticeInfoDev *info, LatRec *dst, int64_t cap) {
  hipStream_t st = d->last_stream;
  hipLaunchKernelGGL(k_final_lattice_te, dim3(n), dim3(1024), 0, st, d->dev, (const int32_t *)d->d_chans, use_final, te, te_stride,
                     rs, rs_stride, info);
  hipLaunchKernelGGL(k_final_lattice_offsets, dim3(1), dim3(1024), 0, st, (const LatticeInfoDev *)info, n, d->d_offs);
  hipLaunchKernelGGL(k_final_lattice_emit, dim3(n), dim3(1024), 0, st, d->dev, (const int32_t *)d->d_chans, n, (const uint32_t *)te,
                     te_stride, (const long long *)d->d_offs, dst, (long long)cap, (const LatticeInfoDev *)info);
  HIP_TRY(hipGetLastError());
  return 0;
}

static void fill_info(const LatticeInfoDev &li, wfst_lattice_info_t *info) {
  info->arcs_in = li.arcs_in; info->arcs_kept = li.arcs_kept; info->frames = li.frames;
  info->reached_final = li.reached_final; info->best_cost = li.best_cost;
  info->density = (float)((double)li.arcs_kept / (double)std::max(li.frames - 1, 1));
}

int wfst_decode_final_lattice_batch(wfst_decoder_t *d, const int32_t *channels, int32_t n, int32_t use_final, wfst_lat_arc_t *out,
                                    int64_t cap, int64_t *offsets, int32_t out_is_device, wfst_lattice_info_t *info, int32_t *status) {
  if (!d || n < 0 || cap < 0 || !offsets || (cap > 0 && !out) || (n > 0 && (!info || !status))) return WFST_E_INVALID_ARG;
  offsets[0] = 0;
  if (n == 0) return 0;
  if (!d->fl_te) return WFST_E_INVALID_ARG;            // the decoder produces no lattice arcs
  int rc = check_channels(d, channels, n, true);
  if (rc) return rc;
  hipStream_t st = d->last_stream;
  rc = stage_channels(d, st, channels, n);
  if (rc) return rc;
  LatRec *dst = (LatRec *)out;
  if (!out_is_device) {                 // host output goes through device staging of the caller's capacity
    if (sizeof(LatRec) * (size_t)std::max<int64_t>(cap, 1) > d->stage_bytes) HIP_TRY(hipStreamSynchronize(st));
    rc = ensure_stage(d, sizeof(LatRec) * (size_t)std::max<int64_t>(cap, 1));
    if (rc) return rc;
    dst = (LatRec *)d->d_stage;
  }
  rc = final_lattice_launch(d, n, use_final, d->fl_te, (long long)d->dev.hist_cap, d->fl_rs, (long long)d->cfg.max_frames + 3,
                            d->fl_info, dst, cap);
  if (rc) return rc;
  std::vector<LatticeInfoDev> li((size_t)n);
  HIP_TRY(copy_sync_on(st, li.data(), d->fl_info, sizeof(LatticeInfoDev) * (size_t)n, hipMemcpyDeviceToHost));
  static_assert(sizeof(long long) == sizeof(int64_t), "offset width");
  HIP_TRY(copy_sync_on(st, offsets, d->d_offs, sizeof(long long) * ((size_t)n + 1), hipMemcpyDeviceToHost));
  for (int32_t i = 0; i < n; ++i) { status[i] = li[i].status; fill_info(li[i], info + i); }
  if (offsets[n] > cap) return WFST_E_CAPACITY;
  if (!out_is_device && offsets[n] > 0)
    HIP_TRY(copy_sync_on(st, out, dst, sizeof(LatRec) * (size_t)offsets[n], hipMemcpyDeviceToHost));
  return 0;
}

int wfst_decode_final_lattice(wfst_decoder_t *d, int32_t channel, int32_t use_final, wfst_lat_arc_t *out, int64_t cap,
                              int64_t *n, int32_t out_is_device, wfst_lattice_info_t *info) {
  if (!n || !info) return WFST_E_INVALID_ARG;
  int64_t offs[2] = {0, 0};
  int32_t st = 0;
  wfst_lattice_info_t li{};
  const int rc = wfst_decode_final_lattice_batch(d, &channel, 1, use_final, out, cap, offs, out_is_device, &li, &st);
  if (rc == WFST_E_CAPACITY) { *n = offs[1]; return rc; }
  if (rc) return rc;
  if (st) return st;
  *n = offs[1]; *info = li;
  return 0;
}

int wfst_decode_final_lattice_noalloc(wfst_decoder_t *d, int32_t channel, int32_t use_final, wfst_lat_arc_t *out, int64_t cap,
                                      int64_t *n, wfst_lattice_info_t *info) {
  if (!d || !n || !info || cap < 0 || (cap > 0 && !out)) return WFST_E_INVALID_ARG;
  int rc = check_channels(d, &channel, 1, true);
  if (rc) return rc;
  ChanState cs;
  rc = read_chan(d, channel, &cs);
  if (rc) return rc;
  if (cs.status != 0) return cs.status;
  // the pass's scratch inside the fixed array: extra costs, frame offsets, result block
  const size_t te_bytes = sizeof(uint32_t) * (size_t)std::max<long long>(cs.hist_used, 1);
  const size_t rs_off = (te_bytes + 15) & ~(size_t)15;
  const size_t info_off = rs_off + sizeof(long long) * ((size_t)cs.num_frames + 3);
  const size_t need = info_off + sizeof(LatticeInfoDev);
  if (need > NOALLOC_SCRATCH_BYTES) return WFST_E_SCRATCH_LIMIT;
  char *base = (char *)d->noalloc_scratch;          // the looked-up device address, never the array's name
  HIP_TRY(copy_sync(d, d->d_chans, &channel, sizeof(int32_t), hipMemcpyHostToDevice));
  d->staged_chans.clear();
  rc = final_lattice_launch(d, 1, use_final, (uint32_t *)base, 0, (long long *)(base + rs_off), 0, (LatticeInfoDev *)(base + info_off),
                            (LatRec *)out, cap);
  if (rc) return rc;
  LatticeInfoDev li;
  HIP_TRY(copy_sync(d, &li, base + info_off, sizeof(li), hipMemcpyDeviceToHost));
  if (li.status != 0) return li.status;
  *n = li.arcs_kept;
  if (li.arcs_kept > cap) return WFST_E_CAPACITY;
  fill_info(li, info);
  return 0;
}

int wfst_decode_tokens(wfst_decoder_t *d, int32_t channel, int32_t frame, wfst_token_t *out, int32_t cap, int32_t *n) {
  if (!d || !n || cap < 0 || (cap > 0 && !out)) return WFST_E_INVALID_ARG;
  int rc = check_channels(d, &channel, 1, true);
  if (rc) return rc;
  ChanState cs;
  rc = read_chan(d, channel, &cs);
  if (rc) return rc;
  if (frame < 0) frame += cs.num_frames;
  if (frame < 0 || frame >= cs.num_frames) return WFST_E_INVALID_ARG;
  long long off[2];
  HIP_TRY(copy_sync(d, off, d->dev.frame_off + (size_t)channel * (size_t)(d->cfg.max_frames + 2) + frame, sizeof(off), hipMemcpyDeviceToHost));
  const int cnt = (int)(off[1] - off[0]);
  if (cnt > cap) { *n = cnt; return WFST_E_CAPACITY; }
  if (cnt > 0) {
    rc = ensure_stage(d, sizeof(TokOut) * (size_t)cnt);
    if (rc) return rc;
    hipLaunchKernelGGL(k_export_tokens, dim3((cnt + 255) / 256), dim3(256), 0, d->last_stream, d->dev, channel, off[0], cnt, (TokOut *)d->d_stage);
    HIP_TRY(hipGetLastError());
    HIP_TRY(copy_sync(d, out, d->d_stage, sizeof(TokOut) * (size_t)cnt, hipMemcpyDeviceToHost));
  }
  *n = cnt;
  return 0;
}

int wfst_decode_stats(wfst_decoder_t *d, int32_t channel, wfst_stats_t *out) {
  if (!d || !out) return WFST_E_INVALID_ARG;
  int rc = check_channels(d, &channel, 1, true);
  if (rc) return rc;
  ChanState cs;
  rc = read_chan(d, channel, &cs);
  if (rc) return rc;
  out->frames = cs.num_frames; out->arcs_expanded = cs.arcs_expanded; out->lattice_arcs = cs.lat_total; out->tokens = cs.hist_used;
  out->max_tokens_pre_prune = cs.max_pre; out->max_tokens = cs.max_post; out->closure_iters_max = cs.closure_iters_max;
  out->status = cs.status;
  return 0;
}

// ---- channel-to-lane multiplexer (host side; Section 3.1) ---------------------------------------
}  // extern "C"

struct wfst_mux {
  struct Chunk { const float *ll; int32_t stride, n_frames; };
  wfst_decoder *dec = nullptr;
  std::vector<std::deque<Chunk>> queued;   // per channel: chunks submitted, oldest first
  std::deque<int32_t> waiting;             // channels with queued chunks, longest-waiting first; each at most once
  std::vector<uint8_t> is_waiting;
  std::vector<int32_t> lane_chan, lane_stride, lane_frames;   // the batch being bound
  std::vector<const float *> lane_ll;
  int64_t pending = 0, batches = 0, lanes_bound = 0;
};

extern "C" {

int wfst_mux_create(wfst_decoder_t *d, wfst_mux_t **out) {
  if (!d || !out) return WFST_E_INVALID_ARG;
  wfst_mux *m = new (std::nothrow) wfst_mux;
  if (!m) return WFST_E_DEVICE;
  try {
    m->dec = d;
    m->queued.resize((size_t)d->cfg.num_channels);
    m->is_waiting.assign((size_t)d->cfg.num_channels, 0);
    const size_t nl = (size_t)d->cfg.max_lanes;
    m->lane_chan.reserve(nl); m->lane_stride.reserve(nl); m->lane_frames.reserve(nl); m->lane_ll.reserve(nl);
  } catch (const std::bad_alloc &) { delete m; return WFST_E_DEVICE; }
  *out = m;
  return 0;
}

void wfst_mux_destroy(wfst_mux_t *m) { delete m; }

int wfst_mux_submit(wfst_mux_t *m, int32_t channel, const float *loglikes, int32_t stride, int32_t n_frames) {
  if (!m || !loglikes || n_frames < 1) return WFST_E_INVALID_ARG;
  wfst_decoder *d = m->dec;
  if (channel < 0 || channel >= d->cfg.num_channels) return WFST_E_BAD_CHANNEL;
  if (!d->inited[channel]) return WFST_E_NOT_INIT;
  if (stride < d->dev.g.num_pdfs) return WFST_E_INVALID_ARG;
  try {
    m->queued[channel].push_back(wfst_mux::Chunk{loglikes, stride, n_frames});
    if (!m->is_waiting[channel]) { m->waiting.push_back(channel); m->is_waiting[channel] = 1; }
  } catch (const std::bad_alloc &) { return WFST_E_DEVICE; }
  ++m->pending;
  return 0;
}

int wfst_mux_step(wfst_mux_t *m, void *stream, int32_t *n_lanes) {
  if (!m || !n_lanes) return WFST_E_INVALID_ARG;
  wfst_decoder *d = m->dec;
  m->lane_chan.clear(); m->lane_stride.clear(); m->lane_frames.clear(); m->lane_ll.clear();
  // the channels that have waited longest get the lanes; one chunk each
  const size_t first_round = m->waiting.size();
  for (size_t seen = 0; seen < first_round && (int32_t)m->lane_chan.size() < d->cfg.max_lanes; ++seen) {
    const int32_t c = m->waiting.front();
    m->waiting.pop_front();
    std::deque<wfst_mux::Chunk> &q = m->queued[c];
    const wfst_mux::Chunk ck = q.front();
    q.pop_front();
    m->lane_chan.push_back(c); m->lane_ll.push_back(ck.ll); m->lane_stride.push_back(ck.stride); m->lane_frames.push_back(ck.n_frames);
    if (!q.empty()) m->waiting.push_back(c);      // takes its next turn after the others
    else m->is_waiting[c] = 0;
  }
  *n_lanes = (int32_t)m->lane_chan.size();
  if (*n_lanes == 0) return 0;
  // (if the advance call refuses the batch - a channel beyond max_frames, say - the chunks bound
  // here are dropped with it and the error is the caller's to handle)
  m->pending -= *n_lanes;
  ++m->batches; m->lanes_bound += *n_lanes;
  return wfst_decode_advance(d, m->lane_chan.data(), *n_lanes, m->lane_ll.data(), m->lane_stride.data(), m->lane_frames.data(), stream);
}

int64_t wfst_mux_pending(const wfst_mux_t *m) { return m ? m->pending : 0; }

int wfst_mux_stats(const wfst_mux_t *m, int64_t *batches, int64_t *lanes_bound) {
  if (!m) return WFST_E_INVALID_ARG;
  if (batches) *batches = m->batches;
  if (lanes_bound) *lanes_bound = m->lanes_bound;
  return 0;
}

#ifdef WFST_PHASE_TIMING
// Instrumented builds only: summed per-phase wall-clock ticks (100 MHz) of workgroup leaders.
int wfst_debug_phase_times(wfst_decoder_t *d, unsigned long long *out8, int reset) {
  HIP_TRY(hipDeviceSynchronize());
  HIP_TRY(hipMemcpy(out8, d->dev.dbg, 8 * (8 + 16384), hipMemcpyDeviceToHost));
  if (reset) HIP_TRY(hipMemset(d->dev.dbg, 0, 8 * (8 + 16384)));
  return 0;
}
#endif

int wfst_decode_set_profiling(wfst_decoder_t *d, int32_t on) {
  if (!d) return WFST_E_INVALID_ARG;
  d->profiling = on != 0;
  return 0;
}

int wfst_decode_profile(wfst_decoder_t *d, int64_t *launches, double *total_ms) {
  if (!d || !launches || !total_ms) return WFST_E_INVALID_ARG;
  double ms = 0.0;
  for (auto &p : d->prof_events) {
    HIP_TRY(hipEventSynchronize(p.second));
    float t = 0.f;
    HIP_TRY(hipEventElapsedTime(&t, p.first, p.second));
    ms += t;
    (void)hipEventDestroy(p.first); (void)hipEventDestroy(p.second);
  }
  *launches = (int64_t)d->prof_events.size(); *total_ms = ms;
  d->prof_events.clear();
  return 0;
}

}  // extern "C"
