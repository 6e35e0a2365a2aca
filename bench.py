#!/usr/bin/env python3
"""Benchmark of the decoding hot path on one MI355X.

Workload: benchmark configs[3] — the 8M-state / 23M-arc synthetic decoding graph,
500 concurrent channels fed 50-frame chunks, beam 13, max-active 7000, lattice beam 6,
with a best-path and a lattice-arc readout for every channel after every chunk.

A "step" is one pass of the whole hot path over one batch: all 500 lanes advance by one
50-frame chunk (emitting expansion, closure, pruning, lattice records), and the per-chunk
readouts of that chunk (best path and lattice arcs of every channel).  The lanes are
persistent workgroups: one advance call covers --chunks-per-call chunks (default: all timed
ones), every lane seals a snapshot of its channel at each chunk boundary and goes on, and the
readouts of each boundary run on a second stream beside the decoding (the paper's second
stream, Section 3) as soon as all lanes have passed it.  Every chunk boundary of every
channel is read out inside the timed region.  --sync-readout gives the lock-step variant:
one call per chunk, read out before the next one is queued.  Scores are generated on the
device beforehand and are resident in HBM when the timed region starts.  value = seconds of
audio decoded per wall second at 10 ms per frame (RTFx), whole job.

Beside `value` the JSON line carries: the roofline object of the advance kernel (HIP events on
its stream), two measured ceilings of the same device in the same process (a plain streaming
copy; random 12-byte record gathers in the benchmark's launch shape), the same chunks decoded
lock-step and with the lattice arcs copied to pinned host memory (PCIe-inclusive: never
`value`), the cost of switching the lanes to other channels in every batch, and the CPU
checker timed on one host core and on all of them.

Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import subprocess
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

FRAME_SHIFT_S = 0.010
HBM_PEAK_GBS = 8000.0
# Algorithmic HBM bytes - what the method itself must move per unit of work, whatever the
# implementation fetches on top (cache-line granularity, re-reads):
BYTES_PER_ARC = 16.0      # 12-byte arc record + 4-byte score
BYTES_PER_TOKEN = 44.0    # 12-byte state record + 16-byte token read when expanded + 16-byte token written
BYTES_PER_LAT = 12.0      # one lattice record


def cpu_worker(spec: str) -> int:
    """Child process of the all-cores CPU leg: decode streams first..first+count-1 of the workload
    with the CPU checker (one thread) and print what it did.  Touches no GPU."""
    first, count, n_frames, beam = spec.split(",")
    first, count, n_frames, beam = int(first), int(count), int(n_frames), float(beam)
    import oracle
    import synth
    if not sys.stdin.readline():                 # idle until the GPU legs are over
        return 1
    cfg = synth.configs()[3]
    g = synth.make_graph(cfg.graph)
    og = oracle.OracleGraph(g)
    rows = [cfg.loglikes(s, 0, n_frames) for s in range(first, first + count)]
    print(json.dumps({"ready": 1}), flush=True)
    if not sys.stdin.readline():                 # all workers start decoding together
        return 1
    t0 = time.perf_counter()
    arcs = 0
    for r in rows:
        od = oracle.OracleDecoder(og, beam, cfg.lattice_beam, cfg.max_active)
        od.advance(r)
        arcs += od.arcs_expanded
    print(json.dumps({"seconds": time.perf_counter() - t0, "frames": count * n_frames, "arcs": arcs}), flush=True)
    return 0


def cpu_model() -> str:
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--channels", type=int, default=0, help="override the number of channels (default: the config's 500)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-readout", action="store_true", help="time the advance calls only")
    ap.add_argument("--cpu-streams", type=int, default=100, help="streams the one-core CPU leg decodes")
    ap.add_argument("--cpu-frames", type=int, default=1000, help="frames per stream of the CPU legs")
    ap.add_argument("--sync-readout", action="store_true",
                    help="one call per chunk, read out before the next one is queued (no overlap with decoding)")
    ap.add_argument("--copy-lattice", action="store_true",
                    help="also copy each snapshot's lattice block from the decoder's memory into a buffer of the caller "
                         "(default: the block is handed over in place, by address and per-channel ranges)")
    ap.add_argument("--lattice-to-host", action="store_true",
                    help="copy each snapshot's lattice block to pinned host memory (the PCIe-inclusive variant; never the benchmark)")
    ap.add_argument("--no-extras", action="store_true", help="skip the lock-step, lattice-to-host and rotation legs and the ceilings")
    ap.add_argument("--chunks-per-call", type=int, default=0,
                    help="chunks one advance call covers (0: all chunks of the warm-up / of the timed region)")
    ap.add_argument("--beam", type=float, default=0.0,
                    help="decode with another beam than the config's 13 (a sweep point, not the benchmark: the JSON says so)")
    ap.add_argument("--lane-threads", type=int, default=0, help="threads of a lane's workgroup (0: the library's choice)")
    ap.add_argument("--copy-probe", action="store_true",
                    help="run only a plain 1 GiB device copy (calibrates the HBM byte counters under rocprofv3)")
    ap.add_argument("--cpu-worker", default="", help=argparse.SUPPRESS)
    args = ap.parse_args()
    if args.cpu_worker:
        return cpu_worker(args.cpu_worker)
    if args.copy_probe:
        import torch
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(4):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_probe_bytes_read": src.numel() * 4, "copy_probe_bytes_written": src.numel() * 4, "copies": 4}))
        return 0
    if args.gpus != 1:
        print("bench.py: this build decodes on one GPU only (streams are independent; more GPUs would each "
              "run their own decoder on a share of the channels) — run with --gpus 1", file=sys.stderr)
        return 2

    # The processes of the all-cores CPU leg are started now, before this process touches the GPU,
    # and sit idle until the GPU legs are over.
    ncore, per_worker = max(1, min(16, os.cpu_count() or 1)), 30
    cpu_frames = min(args.cpu_frames, (args.steps + args.warmup) * 50)
    procs = []
    if not args.no_cpu_baseline:
        beam_arg = args.beam or 13.0
        procs = [subprocess.Popen([sys.executable, os.path.abspath(__file__), "--cpu-worker",
                                   f"{i * per_worker},{per_worker},{cpu_frames},{beam_arg}"],
                                  stdin=subprocess.PIPE, stdout=subprocess.PIPE, text=True) for i in range(ncore)]

    import numpy as np
    import torch

    import synth
    from paper_1910_10032_amd import binding as B

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    torch.cuda.set_device(0)
    cfg = synth.configs()[3]
    n_ch = args.channels or cfg.n_streams
    beam = args.beam or cfg.beam
    chunk = cfg.chunk
    K, W = args.steps, args.warmup
    n_frames = (K + W) * chunk
    assert n_frames <= cfg.len_hi, f"steps + warmup must be <= {cfg.len_hi // chunk} chunks of {chunk} frames"
    P = cfg.graph.num_pdfs
    extras = not args.no_extras and not args.no_readout and not args.sync_readout and not args.lattice_to_host

    t_setup = time.perf_counter()
    g = synth.make_graph(cfg.graph)
    graph = B.WfstGraph(g)
    scores = torch.empty((n_ch, n_frames, P), dtype=torch.float32, device="cuda")
    for s in range(n_ch):
        synth.device_loglikes(scores[s], cfg.ll_seed, s, 0, cfg.ll_mu, cfg.ll_sigma, cfg.ll_boost)
    torch.cuda.synchronize()
    # buffer sizes for the benchmark's beam; a wider beam of a sweep keeps many more tokens per frame
    scale = 1 if beam <= cfg.beam else 8
    dec = B.WfstDecoder(graph, beam, cfg.lattice_beam, cfg.max_active, num_channels=n_ch, max_lanes=n_ch,
                        max_frames=n_frames, token_capacity=16384 * (4 if scale > 1 else 1),
                        history_capacity=1250 * scale * n_frames, lattice_capacity=400_000 * scale,
                        snapshot_blocks=max(K, W, 1),
                        snapshot_block_capacity=16_000 * (scale if beam <= cfg.beam + 3 else 64) * n_ch,
                        lane_threads=args.lane_threads)
    ch_np = np.arange(n_ch, dtype=np.int32)
    dec.init_channels(ch_np)
    stream = torch.cuda.Stream().cuda_stream
    strides, nfr = np.full(n_ch, P, np.int32), np.full(n_ch, chunk, np.int32)
    row0 = scores.data_ptr() + np.arange(n_ch, dtype=np.uint64) * np.uint64(n_frames * P * 4)
    lat_buf = torch.empty(n_ch * 80_000 * 12, dtype=torch.uint8, device="cuda")
    host_buf = torch.empty(lat_buf.numel(), dtype=torch.uint8, pin_memory=True) if (args.lattice_to_host or extras) else None
    chans = list(range(n_ch))
    readout = not args.no_readout

    def launch(i: int, n_chunks: int = 1, snapshot_every: int = 0, channels=ch_np):
        return dec.advance_ptrs(channels, row0 + np.uint64(i * chunk * P * 4), strides, nfr * np.int32(n_chunks), stream,
                                snapshot_every)

    def read(snapshot: int = 0, to_host: bool = False, channels=ch_np):
        """Best path of every channel and its lattice arcs since the last readout, in device
        memory in the caller's form (or copied to pinned host memory): returns (paths, number of arcs)."""
        paths = dec.best_path_batch(channels, use_final=False, words_cap=1024, raw=True, snapshot=snapshot)
        if snapshot:
            r = dec.snapshot_lattice_arcs(snapshot, channels, out_device=None if to_host else lat_buf,
                                          out_host=host_buf if to_host else None, copy=args.copy_lattice or to_host)
            return paths, int(r["total"])
        return paths, int(dec.lattice_arcs_batch(channels, out_device=lat_buf)[-1])

    def all_stats():
        return [dec.stats(int(c)) for c in ch_np]

    def run(first: int, count: int, overlap: bool, to_host: bool = False):
        """Steps (chunks) [first, first + count), each decoded and read out."""
        last = None
        if not overlap:
            for i in range(first, first + count):
                launch(i)
                if readout:
                    last = read()
            torch.cuda.synchronize()
            return last
        per_call = args.chunks_per_call or count
        calls = [(i, min(per_call, first + count - i)) for i in range(first, first + count, per_call)]
        ids = launch(*calls[0], snapshot_every=chunk)
        for k, (i, m) in enumerate(calls):
            nxt = launch(*calls[k + 1], snapshot_every=chunk) if k + 1 < len(calls) else None   # queued behind this call
            assert ids[1] == m
            for j in range(m):
                last = read(ids[0] + j, to_host)   # waits until all lanes have sealed this boundary
            ids = nxt
        torch.cuda.synchronize()
        return last

    def timed(overlap: bool, to_host: bool = False):
        if W:
            run(0, W, overlap, to_host)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        last = run(W, K, overlap, to_host)
        return time.perf_counter() - t0, last

    overlap = readout and not args.sync_readout
    if W:
        run(0, W, overlap, args.lattice_to_host)
    stats0 = all_stats()
    arcs0 = sum(s["arcs_expanded"] for s in stats0)
    dec.set_profiling(True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    last = run(W, K, overlap, args.lattice_to_host)
    t1 = time.perf_counter()
    launches, kernel_ms = dec.profile()
    dec.set_profiling(False)
    stats = all_stats()
    bad = [(c, s["status"]) for c, s in zip(chans, stats) if s["status"] != 0]
    assert not bad, f"channels stopped with an error: {bad[:5]}"
    arcs = sum(s["arcs_expanded"] for s in stats) - arcs0
    wall = t1 - t0
    audio_s = K * n_ch * chunk * FRAME_SHIFT_S
    rtfx = audio_s / wall
    tokens = sum(s["tokens"] for s in stats) - sum(s["tokens"] for s in stats0)
    lat_recs = sum(s["lattice_arcs"] for s in stats) - sum(s["lattice_arcs"] for s in stats0)
    avg_launch_s = kernel_ms / 1e3 / max(launches, 1)
    algo_bytes = BYTES_PER_ARC * arcs + BYTES_PER_TOKEN * tokens + BYTES_PER_LAT * lat_recs
    achieved = algo_bytes / max(launches, 1) / avg_launch_s / 1e9

    # HBM bytes per launch from the committed rocprofv3 counter runs (FETCH_SIZE / WRITE_SIZE,
    # scaled by a plain copy of known size); not measurable from inside this process
    traffic, traffic_note = None, None
    tpath = os.path.join(ROOT, "profiles", "k_advance_config3_traffic.json")
    if os.path.exists(tpath) and n_ch == cfg.n_streams and beam == cfg.beam:
        with open(tpath) as f:
            tj = json.load(f)
        per_chunk = tj["fetch_bytes_per_chunk"] + tj["write_bytes_per_chunk"]
        traffic = round(per_chunk * (K / max(launches, 1)))
        traffic_note = ("rocprofv3 FETCH_SIZE + WRITE_SIZE of a %d-chunk launch (profiles/k_advance_config3.md), per chunk x the "
                        "%d chunks of this launch" % (tj.get("chunks_per_launch_measured", 0), K // max(launches, 1)))

    result = {
        "metric": "decode RTFx (audio s / wall s) + arcs expanded/s, batched streams, 1 GPU",
        "value": round(rtfx, 1), "unit": "x real time (10 ms frames)", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": round(wall / K * 1e3, 3), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "configs[3]: 8M-state/23M-arc synthetic graph, %d channels x %d-frame chunks, beam %g, "
                               "max-active %d, lattice-beam %g, per-chunk best-path + lattice readout%s"
                               % (n_ch, chunk, beam, cfg.max_active, cfg.lattice_beam, (("" if overlap else " (lock-step)") + (" + lattice copied to host" if args.lattice_to_host else "")) if readout else " (readout off)"),
                   "channels": n_ch, "chunk_frames": chunk, "stream_frames_timed": K * n_ch * chunk,
                   "chunks_per_advance_call": (args.chunks_per_call or K) if overlap else 1},
        "arcs_expanded_per_s": round(arcs / wall, 1),
        "stream_frames_per_s": round(K * n_ch * chunk / wall, 1),
        "arcs_per_stream_frame": round(arcs / (K * n_ch * chunk), 1),
        "advance_kernel_ms_per_launch": round(kernel_ms / max(launches, 1), 3), "readout_overlapped": bool(overlap),
        "max_tokens_pre_prune": max(s["max_tokens_pre_prune"] for s in stats),
        "max_tokens": max(s["max_tokens"] for s in stats),
        "roofline": {"bound": "hbm", "kernel": "k_advance", "achieved": round(achieved, 2), "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 5), "traffic": traffic,
                     "traffic_source": traffic_note,
                     "algorithmic_bytes_per_launch": round(algo_bytes / max(launches, 1)),
                     "arcs_per_launch": round(arcs / max(launches, 1)), "launches": launches,
                     "avg_launch_ms": round(avg_launch_s * 1e3, 4)},
        "setup_s": round(t0 - t_setup, 1),
    }
    if readout:
        result["lattice_arcs_last_chunk"] = int(last[1])
    if extras:
        # the same device's ceilings, measured in this process with trivial kernels
        copy_gbs = synth.probe_copy_gbs()
        gth = synth.probe_gather(12 * (g.num_states + g.num_arcs), n_ch, 512, inflight=4)
        result["copy_ceiling_gbs"] = round(copy_gbs, 1)
        result["gather_ceiling"] = {"records_per_s": round(gth["records_per_s"], 1), "gbs_in_64_byte_lines": round(gth["line_gbs"], 1),
                                    "note": "random 12-byte records from a table of the graph's size, %d x 512 threads, 4 loads in flight each" % n_ch}
        result["roofline"]["frac_of_copy_ceiling"] = round(achieved / copy_gbs, 5)
        # the same chunks again, lock-step: one call per chunk, read out before the next is queued
        dec.init_channels(ch_np)
        dt, _ = timed(False)
        result["lock_step"] = {"value": round(audio_s / dt, 1), "ms_per_step": round(dt / K * 1e3, 3),
                               "note": "one advance call per chunk, its readouts before the next call"}
        # ... and with every snapshot's lattice arcs copied to pinned host memory (PCIe-inclusive)
        dec.init_channels(ch_np)
        dt, _ = timed(True, True)
        result["lattice_to_host"] = {"value": round(audio_s / dt, 1), "ms_per_step": round(dt / K * 1e3, 3),
                                     "note": "as value, plus each chunk's lattice arcs copied to pinned host memory beside the decoding"}
        # ... and four times as many channels taking turns on the lanes (Section 3.1: channels are
        # multiplexed onto lanes; the paper quotes about 5 us per batch for the context switch)
        from paper_1910_10032_amd.multiplex import rotation_cost_us
        result["context_switch"] = rotation_cost_us(graph, beam, cfg.lattice_beam, cfg.max_active, n_ch, 5, chunk, row0, P, stream,
                                                    token_capacity=16384, history_capacity=1250 * 7 * chunk, lattice_capacity=200_000)

    if not args.no_cpu_baseline:
        import oracle
        og = oracle.OracleGraph(g)
        ns, nf_cpu = args.cpu_streams, cpu_frames
        rows = [cfg.loglikes(s, 0, nf_cpu) for s in range(ns)]
        t_c = time.perf_counter()
        c_arcs = 0
        for s in range(ns):
            od = oracle.OracleDecoder(og, beam, cfg.lattice_beam, cfg.max_active)
            od.advance(rows[s])
            c_arcs += od.arcs_expanded
        cpu_wall = time.perf_counter() - t_c
        del rows
        result["cpu_baseline"] = {"value": round(ns * nf_cpu * FRAME_SHIFT_S / cpu_wall, 2), "unit": "x real time (10 ms frames)",
                                  "cores": 1, "kind": "oracle",
                                  "sample": f"streams 0..{ns - 1} of the same workload, first {nf_cpu} frames each, one thread, {cpu_wall:.1f} s",
                                  "arcs_expanded_per_s": round(c_arcs / cpu_wall, 1), "cpu": cpu_model()}
        # all host cores: one process per core, each decoding its own streams
        for p in procs:
            p.stdin.write("prepare\n"); p.stdin.flush()
        ok = all(p.stdout.readline().strip() for p in procs)          # every worker has its inputs ready
        for p in procs:
            p.stdin.write("go\n"); p.stdin.flush()
        outs = [json.loads(p.stdout.readline()) for p in procs] if ok else []
        for p in procs:
            p.wait()
        if outs:
            slowest = max(o["seconds"] for o in outs)
            result["cpu_baseline_all_cores"] = {
                "value": round(sum(o["frames"] for o in outs) * FRAME_SHIFT_S / slowest, 2), "unit": "x real time (10 ms frames)",
                "cores": ncore, "kind": "oracle", "cpu": cpu_model(),
                "sample": f"{ncore} processes x {per_worker} streams x {cpu_frames} frames of the same workload, {slowest:.1f} s",
                "arcs_expanded_per_s": round(sum(o["arcs"] for o in outs) / slowest, 1)}
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
