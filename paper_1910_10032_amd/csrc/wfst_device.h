// Device-side data layout shared by the kernels and the host code of the library.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace wfst {

// ---- graph ---------------------------------------------------------------------------
// The graph is one array of 12-byte records (three 32-bit words).  State s owns a header
// record followed by its emitting arcs and then its non-emitting arcs:
//   header        {n_emit, n_eps, final cost bits}
//   emitting arc  {dest handle | HAS_EPS, weight bits, pdf id | degree info of the dest << 16}
//   epsilon arc   {dest handle | HAS_EPS, weight bits,          degree info of the dest << 16}
// The degree info (16 bits: emitting out-degree in the low 12, epsilon out-degree in the high
// 4, all-ones in a field = "does not fit, read the header") lets a token that arrives over an
// arc be expanded in the next step without first fetching its state's header: one dependent
// memory round trip less per frame and per closure round.  It is present when pdf ids fit in
// 16 bits (GraphDev::info_shift == 16); otherwise the third word is the plain pdf id and
// every degree info reads as "read the header".
// A state's "handle" is the index of its header record, an arc's id on the device is the
// index of its record.  Both grow with (state, emitting before epsilon, caller position),
// so comparing record indices is comparing in that canonical arc order.  With the header
// next to the arcs one cache line usually serves a whole state (direct indexing, as in the
// paper's Section 3.2.1; 12 bytes per state and per arc is its Eq. 1 plus 4 bytes per
// epsilon arc).
constexpr uint32_t HAS_EPS = 0x80000000u;   // in a dest word: the destination has epsilon arcs
constexpr uint32_t HMASK = 0x7FFFFFFFu;
constexpr uint32_t NO_ARC = 0xFFFFFFFFu;
constexpr uint32_t EMPTY = 0xFFFFFFFFu;     // empty hash slot
constexpr uint32_t INFO_NE = 0xFFFu;        // degree info: emitting out-degree, INFO_NE itself = escape
constexpr int INFO_NP_SHIFT = 12;           // epsilon out-degree above it, 0xF = escape
constexpr uint32_t INFO_NP = 0xFu;
constexpr uint32_t INFO_UNKNOWN = 0xFFFFu;

struct GraphDev {
  const uint32_t *rec;       // [3 * num_records]
  const int32_t *label;      // [num_records] header: state id; arc: olabel        (readouts)
  const uint32_t *orig;      // [num_records] arc: caller's arc id; header: NO_ARC (readouts)
  uint32_t num_records;
  uint32_t start_handle;
  int32_t num_pdfs;
  uint32_t pdf_mask;         // pdf id = third word & pdf_mask
  int32_t info_shift;        // 16: degree info = third word >> 16; 0: none in the records
  uint32_t start_info;       // degree info of the start state
};
__host__ __device__ inline uint32_t degree_info(uint32_t ne, uint32_t np) {
  return (ne < INFO_NE ? ne : INFO_NE) | ((np < INFO_NP ? np : INFO_NP) << INFO_NP_SHIFT);
}

// ---- per-lane scratch ----------------------------------------------------------------
// One open-addressing table per lane: FST state (handle) -> minimum packed candidate
// (ordered cost bits << 32 | arc record index).
struct __align__(16) Slot {
  unsigned long long val;    // min packed candidate; ~0 when empty
  uint32_t handle;           // EMPTY or the state handle
  uint32_t aux;              // flag bits while the frame is built; after pruning: index of
                             // the kept token in the new frame, or 0xFFFFFFFF
};

// queue entry: slot index | Q_EPS (state has epsilon arcs) | Q_DUP (re-expansion request)
constexpr uint32_t Q_DUP = 0x80000000u;
constexpr uint32_t Q_EPS = 0x40000000u;
constexpr uint32_t Q_SLOT = 0x3FFFFFFFu;

// A candidate arc noted for the lattice stage.  Emitting: {slot of the destination, cost x,
// arc, index of the source token in the previous frame}.  Epsilon (slot has bit 31 set):
// {slot of the source, arc weight, arc, handle of the destination}.
struct __align__(16) Aux {
  uint32_t slot; float x; uint32_t arc; uint32_t src;
};

// ---- per-channel state ---------------------------------------------------------------
struct __align__(16) HTok {  // one kept token of one frame
  uint32_t handle;           // state handle | HAS_EPS
  float cost;
  uint32_t in_arc;           // record index of the best incoming arc, or NO_ARC
  uint32_t prev;             // index of the source token: in the previous frame, or in this
                             // frame when PREV_SAME is set; NO_ARC if unresolved / none
};
constexpr uint32_t PREV_SAME = 0x80000000u;

struct LatRec { int32_t frame; uint32_t arc; float extra; };   // as handed to the caller
// As buffered on the device: also the kept-token indices of both ends, for the final lattice.
// dst: index in frame `frame`; src: index in frame `frame` - 1, or in `frame` if PREV_SAME is set.
struct LatInt { int32_t frame; uint32_t arc; float extra; uint32_t dst; uint32_t src; };

struct ChanState {
  int32_t status;            // sticky error code (WFST_E_*) or 0
  int32_t num_frames;        // token frames written (frame 0 comes from init)
  long long hist_used;       // tokens in the history
  // Lattice records of a channel live in a ring of lat_cap records: record number v (counted
  // from init) sits at v % lat_cap.  Records [lat_head, lat_total) have not been handed out:
  // a live drain hands them to the caller, a lane that seals a snapshot moves them into the
  // snapshot's block.
  long long lat_head;
  long long lat_total;       // lattice records produced since init
  long long arcs_expanded;
  int32_t max_pre, max_post, closure_iters_max;
  int32_t path_nf;           // frames covered by the remembered best path (0 = none)
};

// The state of a channel sealed at a frame boundary, for readouts that run while later
// frames are being decoded.  A channel keeps its last SNAP_RING snapshots; id 0 is none.
constexpr int SNAP_RING = 256;
struct __align__(16) ChanSnap {
  long long id;              // written last
  long long lat_total;       // lattice records produced up to the boundary
  long long hist_used;
  int32_t status, num_frames;
  long long blk_start, blk_count;   // where the lane put the channel's pending lattice records in the snapshot's block
};
// Lattice records of one snapshot, all lanes together, in the form handed to the caller.
// Each lane reserves its range with one compare-and-swap on `used`.
struct SnapBlock { unsigned long long used; long long id; };

struct LaneParam {
  const float *ll;           // device rows of this lane
  int32_t chan, n_frames, stride;
  int32_t snap_every;        // seal a snapshot after every snap_every frames of the call (0: none)
  long long snap_id0;        // id of the call's first snapshot
  int32_t n_snaps, pad;      // snapshots the lane seals in this call (the last ones at its end state)
};

struct DecDev {
  GraphDev g;
  ChanState *chan;
  ChanSnap *snap;            // [num_channels][SNAP_RING]
  long long *lane_sealed;    // [max_lanes] pinned host memory: id of the last snapshot a lane sealed
  SnapBlock *blk;            // [n_blk] snapshot id -> block id % n_blk
  LatRec *blk_recs;          // [n_blk][blk_cap]
  long long blk_cap;
  int32_t n_blk, pad0;
  long long *frame_off;      // [num_channels][max_frames + 2] start of each frame in hist
  HTok *hist;                // [num_channels][hist_cap]
  LatInt *lat;               // [num_channels][lat_cap]
  Slot *slots;               // [max_lanes][H]
  uint32_t *queue;           // [max_lanes][qcap]
  Aux *aux;                  // [max_lanes][auxcap]
  uint32_t *dkey;            // [max_lanes][tokcap] dense cost keys for the selection
  uint32_t *dslot;           // [max_lanes][tokcap]
  int32_t *pc_entry;         // [num_channels][max_frames + 2] remembered best path: token through
                             // which it entered each frame
  int32_t *pc_wcount;        // [num_channels][max_frames + 2] its words up to (and with) that arc
  int32_t *pc_words;         // [num_channels][pc_wcap] its words; the tail is scratch for a trace
  int32_t pc_wcap;
  long long hist_cap, lat_cap;
  uint32_t H;
  int32_t hbits, qcap, auxcap, tokcap, max_frames, max_active, lattice_on;
  float beam, lattice_beam;
  int32_t force_general;         // 1: every frame takes the general form
  int32_t approximate;           // 1: max-active by a single histogram cut (not exact)
  uint32_t wide_spin_limit;      // polls before a lane barrier is given up (lanes shared by several workgroups)
  int32_t pad3;
  unsigned long long *dbg;   // phase timers of instrumented builds, else null
};

// error codes mirrored from the public header (device code cannot include it cleanly)
constexpr int E_TOKEN_OVERFLOW = -6, E_LATTICE_OVERFLOW = -7, E_DEAD_CHANNEL = -8, E_NAN_INPUT = -9,
              E_BROKEN_TRACE = -10, E_DEVICE = -11, E_HISTORY_OVERFLOW = -12, E_CAPACITY = -5, E_NOT_INIT = -4;

}  // namespace wfst
