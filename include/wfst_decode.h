/*
 * wfst_decode — batched, beam-pruned Viterbi token passing over a WFST decoding graph
 * on one AMD MI355X (gfx950) GPU.
 *
 * The calls follow the decoder the paper describes (arXiv 1910.10032): a decoding graph
 * held on the device in compressed-sparse-row form (Section 3.2.1, Eq. 1); many audio
 * streams decoded at once, each owning a "channel" that keeps its state between calls,
 * a call advancing a batch of channels ("lanes") by some frames of acoustic scores
 * (Section 3.1); per frame, emitting arcs, then chains of non-emitting arcs, then
 * pruning with an adaptive beam / max-active limit (Section 3, Fig. 1); and per-frame
 * lattice preprocessing that keeps one representative token per FST state and records
 * every other arc reaching it with its "extra cost" (Section 3.4).  Results come back as
 * a best path and as raw lattice arcs.
 *
 * Conventions
 *  - Every function that returns int returns 0 on success or a negative WFST_E_* code.
 *    Nothing throws or aborts across this boundary.  Out-parameters are written only on
 *    success, except the size reported with WFST_E_CAPACITY.
 *  - HOST pointers are ordinary process memory; DEVICE pointers are GPU global memory on
 *    the device that was current when the graph was loaded.  Each argument says which.
 *  - The library owns all device memory it allocates.  The caller owns every buffer it
 *    passes in and the acoustic-score tensors, which must stay valid until the work of
 *    the advance call has completed on its stream.
 *  - Costs are fp32 in the tropical semiring (smaller is better).  Each addition or
 *    subtraction is rounded on its own (no fused multiply-add).
 *  - Arc ids in results are positions in the caller's arc arrays.  WFST_NO_ARC marks
 *    "no incoming arc" (the start token).
 *  - Errors that concern one channel (token/lattice/history overflow, a channel with no
 *    surviving token, NaN or +inf in the scores it read) are sticky for that channel,
 *    stop that channel at the frame where they occur, and never disturb other channels.
 *  - A graph may be shared by several decoders.  A decoder is not thread-safe.  Its advance
 *    calls are ordered one after the other even when they are given different streams (the
 *    lanes' scratch belongs to the decoder): a call on another stream than the previous one
 *    waits for that one.  Decoders of their own do run side by side.
 */
#ifndef WFST_DECODE_H
#define WFST_DECODE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define WFST_NO_ARC 0xFFFFFFFFu

enum {
  WFST_OK = 0,
  WFST_E_INVALID_ARG = -1,      /* null pointer, negative size, value out of range            */
  WFST_E_BAD_GRAPH = -2,        /* malformed CSR (see wfst_decode_graph_load)                 */
  WFST_E_BAD_CHANNEL = -3,      /* channel id out of range or repeated within one call        */
  WFST_E_NOT_INIT = -4,         /* channel used before wfst_decode_init_channels; a snapshot
                                   that does not exist (any more)                             */
  WFST_E_CAPACITY = -5,         /* caller's buffer too small; the needed size is reported     */
  WFST_E_TOKEN_OVERFLOW = -6,   /* more candidate tokens in a frame than token_capacity       */
  WFST_E_LATTICE_OVERFLOW = -7, /* lattice (or candidate) buffer of the channel, or the
                                   snapshot's block, is full                                  */
  WFST_E_DEAD_CHANNEL = -8,     /* no token survived a frame                                  */
  WFST_E_NAN_INPUT = -9,        /* a score read by the channel was NaN or +inf                */
  WFST_E_BROKEN_TRACE = -10,    /* a best incoming arc starts at a state that holds no token  */
  WFST_E_DEVICE = -11,          /* HIP runtime error (allocation, launch, copy)               */
  WFST_E_HISTORY_OVERFLOW = -12,/* token history of the channel or max_frames exhausted       */
  WFST_E_SCRATCH_LIMIT = -13    /* wfst_decode_final_lattice_noalloc: the channel needs more
                                   than the entry point's fixed scratch                       */
};

typedef struct wfst_graph wfst_graph_t;     /* opaque; device-resident, immutable            */
typedef struct wfst_decoder wfst_decoder_t; /* opaque; owns all channel and lane state       */

/* A decoding graph in CSR form.  All arrays are HOST memory, caller-owned, and copied
 * during wfst_decode_graph_load.  Arcs of state s are [row_offsets[s], row_offsets[s+1]). */
typedef struct {
  int32_t num_states;
  int64_t num_arcs;
  int32_t start_state;
  int32_t num_pdfs;           /* width of one row of acoustic scores                        */
  const int64_t *row_offsets; /* [num_states + 1], non-decreasing, first 0, last num_arcs   */
  const int32_t *ilabel;      /* [num_arcs] 0 = non-emitting (epsilon); else pdf id + 1     */
  const int32_t *olabel;      /* [num_arcs] 0 = none; else word id                          */
  const float *weight;        /* [num_arcs] fp32 cost, finite; >= 0 on non-emitting arcs    */
  const int32_t *nextstate;   /* [num_arcs] destination state                               */
  const float *final_cost;    /* [num_states] +INF = not final; otherwise finite            */
} wfst_csr_t;

/* Decoder hyper-parameters (Section 4: beam, lattice-beam, max-active; Section 3.2.1:
 * number of channels and lanes) and the bounds of the decoder's buffers. */
typedef struct {
  float beam;                /* > 0                                                         */
  float lattice_beam;        /* >= 0                                                        */
  int32_t max_active;        /* >= 1: tokens kept per channel and frame                     */
  int32_t num_channels;      /* streams whose state the decoder can hold                    */
  int32_t max_lanes;         /* channels that one advance/init call can process             */
  int32_t max_frames;        /* frames of scores one channel can consume between inits      */
  int32_t token_capacity;    /* candidate tokens per lane and frame before pruning;
                                0 = 4 * max_active                                          */
  int32_t aux_capacity;      /* candidate arcs per lane and frame kept for lattice and
                                back-pointer resolution; 0 = 2 * token_capacity             */
  int64_t history_capacity;  /* tokens one channel can keep over all its frames;
                                0 = (max_frames + 1) * max_active                           */
  int64_t lattice_capacity;  /* lattice arcs one channel can buffer between readouts;
                                0 = 64 * max_active                                         */
  int32_t lattice_on;        /* 0: no lattice arcs are produced                             */
  int32_t snapshot_blocks;   /* blocks for the lattice arcs of sealed snapshots (see
                                wfst_decode_advance_snapshots); 0 = none: snapshots then
                                cover best paths only                                       */
  int64_t snapshot_block_capacity; /* lattice arcs one block holds, all lanes of a call
                                together; 0 = min(lattice_capacity, 4096 * max_lanes)     */
  int32_t lane_threads;      /* threads of the workgroup that owns a lane: 512, 1024, or 0 =
                                per call: 1024 if the call has no more lanes than the device
                                has compute units, else 512.  Results do not depend on it.  */
  int32_t frame_form;        /* 0 = per frame: the LDS-resident form for frames that fit it
                                (when pdf ids fit in 16 bits), else the general form;
                                1 = always the general form.  Results do not depend on it.  */
  int32_t approximate;       /* 0 = exact max-active: exactly the max_active best tokens by
                                (cost, state id), which is what the CPU checker computes.
                                1 = the paper's histogram-based max-active (Section 4.1: the
                                cut comes from a histogram and is "somewhat arbitrary"): when
                                more than max_active tokens are within the beam, ONE histogram
                                of 1024 equal-width cost bins between the frame's best and
                                worst token places the cut at the upper edge of the bin in
                                which the count reaches max_active.  All tokens up to that edge
                                are kept (max_active plus at most that bin's population), the
                                edge is the frame's effective cutoff, and the refinement passes
                                of the exact selection are saved.  Deterministic, but not the
                                checker's result wherever max-active binds; identical to the
                                exact mode wherever it does not.  The default
                                history_capacity is a quarter larger in this mode.            */
  int32_t lane_workgroups;   /* 0 or 1: one workgroup per lane.  G > 1 (at most 64): a call
                                without snapshots whose lanes are so few that 2 * lanes <= the
                                device's compute units gives every lane min(G, units / lanes)
                                workgroups of 1024 threads that work through each frame
                                together (Section 3.1: small batches leave the device idle and
                                are bound by latency; Section 3.3: the persistent kernel).  For
                                single or few heavy streams; every frame then takes the general
                                form and pays a device-wide barrier per stage, so light streams
                                are slower this way.  Results do not depend on it.  If a
                                barrier is ever given up (a workgroup of the lane not resident
                                for seconds) the channel stops with WFST_E_DEVICE.  (Testing
                                aid: the environment variable WFST_DECODE_WIDE_SPIN_LIMIT,
                                read when a decoder is created, lowers the number of polls
                                after which a barrier is given up.)                           */
} wfst_config_t;

typedef struct { int32_t frame; uint32_t arc; float extra_cost; } wfst_lat_arc_t;
typedef struct { int32_t state; float cost; uint32_t in_arc; } wfst_token_t;

typedef struct {
  int64_t frames;               /* token frames held, including frame 0 written by init     */
  int64_t arcs_expanded;        /* sum over frames of the emitting out-degrees of the tokens
                                   a frame starts from plus the non-emitting out-degrees of
                                   the tokens within the beam after the closure             */
  int64_t lattice_arcs;         /* lattice arcs produced so far (read out or not)           */
  int64_t tokens;               /* tokens kept, summed over all frames                      */
  int32_t max_tokens_pre_prune; /* largest token count after the closure                    */
  int32_t max_tokens;           /* largest token count kept                                 */
  int32_t closure_iters_max;    /* most closure rounds in one frame (diagnostic only)       */
  int32_t status;               /* sticky WFST_E_* of the channel, or 0                     */
} wfst_stats_t;

/* Validate and upload a graph.  WFST_E_BAD_GRAPH if offsets are not monotone, a
 * destination or the start state is out of range, an ilabel is negative or exceeds
 * num_pdfs, a weight is not finite, a non-emitting weight is negative, the non-emitting arcs
 * of weight zero form a cycle (ties around such a cycle would let back-pointers loop), a final
 * cost is NaN or -inf, or num_states + num_arcs >= 2^31 - 1.  On the device the graph takes
 * 12*(num_states + num_arcs) bytes for decoding (the paper's Eq. 1 plus 4 bytes per
 * non-emitting arc) and 8*(num_states + num_arcs) bytes used only by readouts. */
int wfst_decode_graph_load(const wfst_csr_t *csr, wfst_graph_t **out);
void wfst_decode_graph_free(wfst_graph_t *graph);
/* Device bytes of the graph: the part read while decoding, and the readout-only part. */
int wfst_decode_graph_bytes(const wfst_graph_t *graph, int64_t *decode_bytes, int64_t *readout_bytes);

/* Create a decoder and allocate all its device memory (nothing is allocated later
 * except temporary readout staging).  The graph must outlive the decoder. */
int wfst_decode_create(const wfst_graph_t *graph, const wfst_config_t *config, wfst_decoder_t **out);
void wfst_decode_destroy(wfst_decoder_t *decoder);
/* Device bytes held per parked channel, per lane, and in total. */
int wfst_decode_state_bytes(const wfst_decoder_t *decoder, int64_t *per_channel, int64_t *per_lane, int64_t *total);

/* Start (or restart) streams (Section 3.1: a channel holds the state of one audio stream
 * between batches; Section 3, first paragraph: decoding starts from the graph's start state
 * and follows chains of non-emitting arcs before the first frame): each listed channel gets
 * the start token at cost 0 and its non-emitting closure within the beam as frame 0.  channels: HOST [n], distinct, each in [0, num_channels); n may exceed
 * max_lanes (processed in groups).  Synchronises with the device before returning. */
int wfst_decode_init_channels(wfst_decoder_t *decoder, const int32_t *channels, int32_t n);
/* Mark channels unused (Section 3.1: a channel is released when its stream ends); their
 * buffers are reused by the next init. */
int wfst_decode_free_channels(wfst_decoder_t *decoder, const int32_t *channels, int32_t n);

/* Advance n_lanes channels (Section 3.1: a batch works on up to max_lanes channels, one lane
 * each).  Per frame and lane (Section 3, first paragraph; Fig. 1; Section 3.3): every
 * emitting arc out of a token is expanded against the frame's scores, cost = (token cost +
 * arc weight) - loglike[pdf]; candidates above best + beam are dropped and each state keeps
 * its minimum; chains of non-emitting arcs are followed until nothing changes; if more than
 * max_active tokens remain the max_active best are kept and the cost of the last one becomes
 * the frame's cutoff (the adaptive beam); every arc into a kept token within that cutoff and
 * the lattice beam is recorded with its extra cost (Section 3.4).
 * Lane i consumes n_frames[i] rows of scores.
 *   channels  HOST [n_lanes]  distinct initialised channel ids, n_lanes <= max_lanes
 *   loglikes  HOST [n_lanes]  array of DEVICE pointers; lane i's rows are fp32
 *                             [n_frames[i]][strides[i]], already acoustically scaled;
 *                             the decoder reads column pdf of the current row
 *   strides   HOST [n_lanes]  row pitch in floats, >= num_pdfs
 *   n_frames  HOST [n_lanes]  >= 0; lanes may differ (a lane with fewer frames stops early)
 *   stream    hipStream_t on which the work is enqueued, or NULL for the default stream
 * Returns once the work is enqueued.  Per-channel failures are recorded in the channel's
 * sticky status, visible through the readout calls and wfst_decode_stats. */
int wfst_decode_advance(wfst_decoder_t *decoder, const int32_t *channels, int32_t n_lanes,
                        const float *const *loglikes, const int32_t *strides,
                        const int32_t *n_frames, void *stream);

/* Best path of each listed channel over all frames decoded so far (the one-best result of
 * Section 4, Table 2; Section 3.4: each token keeps its best incoming arc, which is what the
 * trace follows back to the start token).
 *   use_final      1: minimise token cost + final cost over final states (falling back
 *                  to 0 when no final state holds a token); 0: minimise token cost
 *   words          HOST [n * words_cap]  channel i's non-zero olabels, in path order, at
 *                  words + i * words_cap
 *   n_words, total_cost, reached_final, status   HOST [n]
 * status[i] receives the channel's own result code (0, its sticky error,
 * WFST_E_BROKEN_TRACE, or WFST_E_CAPACITY with n_words[i] = needed size).  The function
 * itself fails only for invalid arguments or device errors.  Synchronises. */
int wfst_decode_best_path_batch(wfst_decoder_t *decoder, const int32_t *channels, int32_t n,
                                int32_t use_final, int32_t *words, int32_t words_cap,
                                int32_t *n_words, float *total_cost, int32_t *reached_final,
                                int32_t *status);
/* Single-channel form of wfst_decode_best_path_batch (same passages); returns the channel's
 * result code. */
int wfst_decode_best_path(wfst_decoder_t *decoder, int32_t channel, int32_t use_final,
                          int32_t *words, int32_t cap, int32_t *n_words, float *total_cost,
                          int32_t *reached_final);
/* Arcs (caller's ids, path order) of the best path of one channel: the chain of best
 * incoming arcs of Section 3.4 itself, start token first.  arcs: HOST [cap]. */
int wfst_decode_best_path_arcs(wfst_decoder_t *decoder, int32_t channel, int32_t use_final,
                               uint32_t *arcs, int32_t cap, int32_t *n_arcs, float *total_cost,
                               int32_t *reached_final);

/* Drain the lattice arcs buffered for a channel since its last readout (Section 3.4: per
 * frame, one representative token per FST state, and every other arc that reaches the state
 * within the beams kept with its extra cost = its cost minus the state's best; Section 3,
 * Fig. 1: such per-frame results leave the decoder while it goes on).  Records with
 * frame < from_frame are discarded, the others are copied to `out` in no particular
 * order (HOST memory if out_is_device == 0, else DEVICE memory), and the buffer is
 * emptied.  If cap is too small: WFST_E_CAPACITY, *n = needed, nothing is drained.
 * A channel that died or met a bad score still hands out the arcs of its earlier frames;
 * a channel stopped by an overflow returns that error.  Synchronises. */
int wfst_decode_lattice_arcs(wfst_decoder_t *decoder, int32_t channel, int32_t from_frame,
                             wfst_lat_arc_t *out, int64_t cap, int64_t *n, int32_t out_is_device);

/* Drain several channels at once into one buffer (the batch form of
 * wfst_decode_lattice_arcs; Section 3.4): channel i's arcs land at
 * out[offsets[i] .. offsets[i+1]) (offsets: HOST [n + 1]).  A channel stopped by an
 * overflow contributes nothing.  If cap < offsets[n]: WFST_E_CAPACITY, offsets are still
 * filled in, nothing is drained.  Synchronises. */
int wfst_decode_lattice_arcs_batch(wfst_decoder_t *decoder, const int32_t *channels, int32_t n,
                                   wfst_lat_arc_t *out, int64_t cap, int64_t *offsets,
                                   int32_t out_is_device);

/* Readouts beside the decoding.  The paper hides the per-frame device-to-host token copies
 * behind the next frames' kernels with a second stream (Section 3, Fig. 1); here the tokens
 * stay on the device and it is the per-chunk readouts that run beside the decoding.
 *
 * wfst_decode_advance_snapshots is wfst_decode_advance with one addition: after every
 * snapshot_every (>= 1) frames of the call each lane seals a snapshot of its channel - its
 * status and frame count - and goes on decoding.  If the decoder has snapshot blocks, the
 * lane also moves the channel's lattice arcs not handed out yet into the snapshot's block,
 * in the caller's form; without blocks the arcs stay buffered for wfst_decode_lattice_arcs*.
 * The call seals *n_snapshots = max(1, ceil(longest n_frames / snapshot_every)) snapshots
 * (at most 256, and at most snapshot_blocks if there are blocks) with consecutive ids
 * starting at *first_id (ids are positive and grow over the decoder's life); a lane with
 * fewer frames, or one that stops with an error, seals the remaining ones in the state it
 * ends in.  Lanes do not wait for each other at the boundaries, so one call over many
 * chunks keeps the whole GPU busy although the chunks differ from lane to lane.  A channel
 * keeps its last 256 snapshots; snapshot id uses block id % snapshot_blocks, so a block is
 * valid until snapshot_blocks later snapshots have been started.  A block that cannot take
 * a lane's arcs stops that channel with WFST_E_LATTICE_OVERFLOW.
 *
 * wfst_decode_snapshot_wait blocks the calling host thread until every lane of the call has
 * sealed snapshot `id` (WFST_E_NOT_INIT for an id no recent call has produced).  The two
 * readouts below wait likewise, run on a stream of the decoder's own and synchronise with
 * that stream alone, so the lanes go on decoding while they run.  While an advance call is
 * in flight use only these readouts on its channels; every other readout of this header
 * refers to the live state and waits for the decoding.
 *
 * wfst_decode_snapshot_best_path_batch: as wfst_decode_best_path_batch, with paths ending
 * at the snapshot's last frame.  A listed channel without that snapshot reports
 * WFST_E_NOT_INIT in status[i].
 *
 * wfst_decode_snapshot_lattice_arcs: the lattice arcs of the snapshot, i.e. for every lane
 * of the call the arcs produced since its previous hand-over.  The block holds *total arcs,
 * all lanes together, in no particular order; channel i's are at [starts[i], starts[i] +
 * counts[i]) (HOST [n]; 0, 0 for a channel without that snapshot).  If out != NULL the
 * whole block is copied to it (HOST or DEVICE as flagged; WFST_E_CAPACITY with *total set
 * if cap < *total); if block != NULL it receives the DEVICE address of the decoder's own
 * block, for consumers that read the arcs in place.  WFST_E_NOT_INIT if the block has been
 * given to a later snapshot; WFST_E_INVALID_ARG if the decoder has no snapshot blocks. */
int wfst_decode_advance_snapshots(wfst_decoder_t *decoder, const int32_t *channels, int32_t n_lanes,
                                  const float *const *loglikes, const int32_t *strides,
                                  const int32_t *n_frames, int32_t snapshot_every, void *stream,
                                  int64_t *first_id, int32_t *n_snapshots);
int wfst_decode_snapshot_wait(wfst_decoder_t *decoder, int64_t id);
int wfst_decode_snapshot_best_path_batch(wfst_decoder_t *decoder, int64_t snapshot_id,
                                         const int32_t *channels, int32_t n, int32_t use_final,
                                         int32_t *words, int32_t words_cap, int32_t *n_words,
                                         float *total_cost, int32_t *reached_final, int32_t *status);
int wfst_decode_snapshot_lattice_arcs(wfst_decoder_t *decoder, int64_t snapshot_id,
                                      const int32_t *channels, int32_t n, int64_t *starts,
                                      int64_t *counts, wfst_lat_arc_t *out, int64_t cap,
                                      int32_t out_is_device, int64_t *total,
                                      const wfst_lat_arc_t **block);

/* Final lattice of a channel (the step the paper leaves to the end of the utterance, Section
 * 3.4): backward pruning, with the lattice beam, of the lattice arcs currently buffered for
 * the channel (all arcs not handed out yet; nothing is drained).  Every token gets an extra
 * cost te = min over buffered arcs leaving it of (te of the arc's destination + the arc's
 * extra cost); in the last frame te is the token's cost (+ final cost, over final states, if
 * use_final and one holds a token) minus the best such cost.  An arc is kept iff te of its
 * destination + its extra cost <= lattice_beam.  The kept arcs are copied to `out` (HOST or
 * DEVICE as flagged) in no particular order; WFST_E_CAPACITY with *n = needed if cap is too
 * small.  info->density = kept arcs per frame.  Synchronises.  (The single-channel form of
 * wfst_decode_final_lattice_batch.) */
typedef struct {
  int64_t arcs_in;        /* buffered arcs examined                        */
  int64_t arcs_kept;
  int32_t frames;         /* token frames of the channel                   */
  int32_t reached_final;
  float best_cost;        /* cost of the best path the pruning is based on */
  float density;          /* arcs_kept / max(frames - 1, 1)                */
} wfst_lattice_info_t;
int wfst_decode_final_lattice(wfst_decoder_t *decoder, int32_t channel, int32_t use_final,
                              wfst_lat_arc_t *out, int64_t cap, int64_t *n, int32_t out_is_device,
                              wfst_lattice_info_t *info);

/* The final lattices of several channels in one pass (Section 3.4; lattice density as in Section
 * 4.1): one workgroup per channel computes the extra costs, then the surviving arcs of all
 * listed channels are packed into `out` (HOST or DEVICE as flagged): channel i's at
 * out[offsets[i] .. offsets[i+1]) (offsets: HOST [n + 1]).  info, status: HOST [n]; status[i] is
 * the channel's own result (0, its sticky error, or WFST_E_DEAD_CHANNEL); a channel with an
 * error contributes no arcs.  The scratch of the pass (4 bytes per token of history capacity and
 * 8 bytes per frame, for every channel) is allocated when the decoder is created with
 * lattice_on, so the call itself allocates nothing on the device when `out` is device memory.
 * If cap < offsets[n]: WFST_E_CAPACITY, offsets / info / status are still filled in, no arc is
 * written.  Nothing is drained.  Synchronises. */
int wfst_decode_final_lattice_batch(wfst_decoder_t *decoder, const int32_t *channels, int32_t n,
                                    int32_t use_final, wfst_lat_arc_t *out, int64_t cap,
                                    int64_t *offsets, int32_t out_is_device,
                                    wfst_lattice_info_t *info, int32_t *status);

/* wfst_decode_final_lattice for callers that cannot allocate device memory (code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc): the same result, but the
 * pass's scratch - one 32-bit word per kept token of the channel, one 64-bit offset per frame
 * and a small result block - lives in a fixed 8 MiB array inside the library's device image
 * instead of being allocated per call, and `out` must be DEVICE memory (no staging buffer).
 * The call allocates nothing, on the device or through any allocating routine.  A channel that
 * needs more scratch (4 * tokens kept + 8 * (frames + 3) + 64 bytes > 8 MiB, i.e. beyond about
 * two million kept tokens) is rejected with WFST_E_SCRATCH_LIMIT and nothing is launched.  All
 * calls on one GPU share that GPU's array: calls that overlap in time on one GPU (two host
 * threads, two decoders on different streams) race, so issue them one at a time; the array
 * keeps the previous call's contents and every call initialises the part it uses.
 * WFST_E_CAPACITY with *n = needed if cap is too small.  Synchronises with the decoder's
 * stream. */
int wfst_decode_final_lattice_noalloc(wfst_decoder_t *decoder, int32_t channel, int32_t use_final,
                                      wfst_lat_arc_t *out, int64_t cap, int64_t *n,
                                      wfst_lattice_info_t *info);

/* Tokens kept for one frame of a channel (frame -1 = last), in no particular order (Section
 * 3.3: what survives the contraction of a frame - state, cost, best incoming arc).
 * out: HOST [cap].  A parity hook: the token history is what best_path walks. */
int wfst_decode_tokens(wfst_decoder_t *decoder, int32_t channel, int32_t frame,
                       wfst_token_t *out, int32_t cap, int32_t *n);

/* Counters of a channel (Section 4.1 discusses the decoder in terms of active tokens and
 * expanded arcs; arcs_expanded is the numerator of the arcs-per-second figure). */
int wfst_decode_stats(wfst_decoder_t *decoder, int32_t channel, wfst_stats_t *out);

/* Per-kernel timing with HIP events on the stream of each call (off by default).  While
 * on, every advance call is bracketed by an event pair; wfst_decode_profile waits for
 * the recorded work and returns the number of advance launches and their summed
 * duration since profiling was switched on or last read. */
int wfst_decode_set_profiling(wfst_decoder_t *decoder, int32_t on);
int wfst_decode_profile(wfst_decoder_t *decoder, int64_t *launches, double *total_ms);

/* Channel-to-lane multiplexer (Section 3.1: the decoder keeps many channels and works on at
 * most max_lanes of them per batch; host threads feed the lanes from the channels that have
 * audio waiting, and switching a lane to another channel costs a few microseconds per batch).
 * The multiplexer is a host-side queue over one decoder: chunks of scores are submitted per
 * channel as they arrive, and every wfst_mux_step binds the channels that have waited longest
 * (at most max_lanes, at most one chunk per channel and step) to the lanes of one
 * wfst_decode_advance call.  A channel with further chunks queued goes to the back of the
 * queue, so channels take turns.  Here a channel's state is addressed by its id and never
 * copied, so the switch itself moves no data; what a step costs beyond the decoding is the
 * host-side binding and the upload of the lanes' parameters.
 *   wfst_mux_create   decoder: must outlive the multiplexer; its channels are initialised and
 *                     read out by the caller through the decoder's own calls
 *   wfst_mux_submit   loglikes: DEVICE rows [n_frames][stride] (n_frames >= 1), valid until the
 *                     step that consumes them has completed on its stream
 *   wfst_mux_step     issues one advance call on `stream` (NULL: default stream) for the waiting
 *                     channels; *n_lanes = how many it bound (0: nothing was waiting, no call).
 *                     If the advance call fails (a channel beyond max_frames, say) its error is
 *                     returned and the chunks bound in this step are dropped
 *   wfst_mux_pending  chunks submitted and not yet bound to a lane
 *   wfst_mux_stats    batches issued and lanes bound so far
 * Not thread-safe (one feeding thread per multiplexer). */
typedef struct wfst_mux wfst_mux_t;
int wfst_mux_create(wfst_decoder_t *decoder, wfst_mux_t **out);
void wfst_mux_destroy(wfst_mux_t *mux);
int wfst_mux_submit(wfst_mux_t *mux, int32_t channel, const float *loglikes, int32_t stride, int32_t n_frames);
int wfst_mux_step(wfst_mux_t *mux, void *stream, int32_t *n_lanes);
int64_t wfst_mux_pending(const wfst_mux_t *mux);
int wfst_mux_stats(const wfst_mux_t *mux, int64_t *batches, int64_t *lanes_bound);

const char *wfst_decode_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* WFST_DECODE_H */
