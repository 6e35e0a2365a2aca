"""GPU parity at the full sizes of configs 1-4, in the launch configuration the benchmark times
(all channels of the config in every call).  EVERY channel is compared with the CPU checker:
status, frame count, canonical arc count, token high-water marks, the token set of the last
frame (states, cost bits, best incoming arcs), an order-independent digest of its whole lattice
record set {frame, arc, extra-cost bits}, and its best paths (words, cost bits, final flag) with
and without final costs.  A sample of channels is compared frame by frame on top of that, with
the per-chunk partial results and the final lattices.  Streams are independent, so the checker
decodes them one by one (on a pool of host threads: the checker's C code runs without the
interpreter lock)."""
import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest

import oracle
import synth
from gpu_compare import range_digests, record_hashes, set_digest, sorted_tokens

pytestmark = pytest.mark.gpu
WORKERS = max(1, min(16, os.cpu_count() or 1))


def checker_summary(og, cfg, s, length, beam, max_active, keep=False, final_lattice=False):
    """Decode stream s with the CPU checker; return what is compared for every channel (and the
    decoder itself if keep)."""
    od = oracle.OracleDecoder(og, beam, cfg.lattice_beam, max_active)
    od.advance(cfg.loglikes(s, 0, length))
    fr, ar, ex = od.lattice()
    out = dict(status=od.status, frames=od.num_frames, arcs=od.arcs_expanded, max_pre=od.max_tokens_pre_prune,
               max_post=od.max_tokens, last=od.tokens(-1), lattice=set_digest(record_hashes(fr, ar, ex)),
               paths=[od.best_path(u) for u in (True, False)] if od.status == 0 else None)
    if final_lattice and od.status == 0:
        out["final"] = []
        for u in (True, False):
            fl = od.final_lattice(u)
            out["final"].append((set_digest(record_hashes(fl["frame"], fl["arc"], fl["extra"])), fl["best_cost"], fl["reached_final"]))
    if keep:
        out["od"] = od
    return out


def decode_and_compare(cfg, sample, token_capacity, history_capacity, lattice_capacity, frame_step=1, channels=None,
                       beam=None, max_active=None, n_frames=None, check=None, **kw):
    """channels: how many of the config's streams take part (default: all); check: which of them
    are compared with the checker (default: all)."""
    import torch

    from paper_1910_10032_amd import binding as B
    assert torch.cuda.is_available()
    beam = beam or cfg.beam
    max_active = max_active or cfg.max_active
    g = synth.make_graph(cfg.graph)
    graph = B.WfstGraph(g)
    n_ch, P = channels or cfg.n_streams, cfg.graph.num_pdfs
    lens = np.array([n_frames or cfg.length(s) for s in range(n_ch)], np.int64)
    T = int(lens.max())
    check = list(range(n_ch)) if check is None else sorted(set(check) | set(sample))
    dec = B.WfstDecoder(graph, beam, cfg.lattice_beam, max_active, num_channels=n_ch, max_lanes=n_ch,
                        max_frames=T, token_capacity=token_capacity, history_capacity=history_capacity,
                        lattice_capacity=lattice_capacity, **kw)
    # the checker starts on the host threads while the GPU decodes
    og = oracle.OracleGraph(g)
    pool = ThreadPoolExecutor(WORKERS)
    offline = not cfg.chunk
    futures = {s: pool.submit(checker_summary, og, cfg, s, int(lens[s]), beam, max_active, s in sample, offline and s in check)
               for s in check}
    # scores of all streams, ragged, in one device buffer
    starts = np.concatenate([[0], np.cumsum(lens)])
    scores = torch.empty((int(starts[-1]), P), dtype=torch.float32, device="cuda")
    for s in range(n_ch):
        synth.device_loglikes(scores[starts[s]:starts[s + 1]], cfg.ll_seed, s, 0, cfg.ll_mu, cfg.ll_sigma, cfg.ll_boost)
    torch.cuda.synchronize()
    chans = np.arange(n_ch, dtype=np.int32)
    dec.init_channels(chans)
    chunk = cfg.chunk or T
    stream = torch.cuda.current_stream().cuda_stream
    lat = {s: [] for s in sample}
    partial = {s: [] for s in sample}
    dig = [np.zeros(n_ch, np.int64), np.zeros(n_ch, np.uint64), np.zeros(n_ch, np.uint64)]   # lattice digests of all channels
    base = scores.data_ptr()
    strides = np.full(n_ch, P, np.int32)
    if cfg.chunk:
        # online, as the benchmark runs it: one call over all chunks, every lane seals a snapshot
        # at each chunk boundary, and every boundary of every channel is read out from its
        # snapshot while the lanes go on decoding
        first, count = dec.advance_ptrs(chans, (base + starts[:-1] * P * 4).astype(np.uint64), strides,
                                        lens.astype(np.int32), stream, snapshot_every=chunk)
        assert count == (T + chunk - 1) // chunk
        for j in range(count):
            paths = dec.best_path_batch(chans, use_final=False, words_cap=1024, raw=True, snapshot=first + j)
            assert (paths[4] == 0).all()
            r = dec.snapshot_lattice_arcs(first + j, chans)
            assert r["counts"].sum() == r["total"]
            rec = r["records"]
            c, sm, xr = range_digests(record_hashes(rec["frame"], rec["arc"], rec["extra_cost"]), r["starts"], r["counts"])
            with np.errstate(over="ignore"):
                dig[0] += c; dig[1] += sm; dig[2] ^= xr
            last_paths = paths
            for s in sample:
                lat[s].append(rec[r["starts"][s]:r["starts"][s] + r["counts"][s]].copy())
                partial[s].append(paths[0][s, :paths[1][s]].copy())
    else:
        dec.advance_ptrs(chans, (base + starts[:-1] * P * 4).astype(np.uint64), strides, lens.astype(np.int32), stream)
    final = {}
    if offline:                                        # offline: one readout per channel at the end
        import time
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        batch = [dec.final_lattice_batch(check, u, cap=1 << 22) for u in (True, False)]     # all final lattices in one pass each
        dt = (time.perf_counter() - t0) / 2
        assert all((b[3] == 0).all() for b in batch)
        print(f"\n{cfg.name}: final lattices of {len(check)} channels in one batch call: {dt * 1e3:.1f} ms, "
              f"{int(batch[0][1][-1])} of {sum(i['arcs_in'] for i in batch[0][2])} arcs kept, mean density "
              f"{np.mean([i['density'] for i in batch[0][2]]):.2f} arcs/frame")
        for k, s in enumerate(check):
            final[s] = tuple((b[0][b[1][k]:b[1][k + 1]], b[2][k]) for b in batch)
            if s in sample:                            # the single-channel call gives the same records
                for u, (got, info) in zip((True, False), final[s]):
                    one, oinfo = dec.final_lattice(s, u)
                    assert set_digest(record_hashes(one["frame"], one["arc"], one["extra_cost"])) == \
                        set_digest(record_hashes(got["frame"], got["arc"], got["extra_cost"])) and oinfo == info
            rec = dec.lattice_arcs(s)
            dig[0][s], dig[1][s], dig[2][s] = set_digest(record_hashes(rec["frame"], rec["arc"], rec["extra_cost"]))
            if s in sample:
                lat[s].append(rec)
    torch.cuda.synchronize()
    stats = [dec.stats(int(c)) for c in chans]
    if cfg.chunk:
        # all lattice arcs were handed over through the snapshots, and the last snapshot's best path is the live one
        assert np.array_equal(dig[0], np.array([st["lattice_arcs"] for st in stats]))
        live = dec.best_path_batch(chans, use_final=False, words_cap=1024, raw=True)
        assert np.array_equal(live[1], last_paths[1]) and np.array_equal(live[2].view(np.uint32), last_paths[2].view(np.uint32))
        for c in range(n_ch):
            assert np.array_equal(live[0][c, :live[1][c]], last_paths[0][c, :last_paths[1][c]])
    assert all(st["status"] == 0 for st in stats), f"channels with errors: {[(i, st['status']) for i, st in enumerate(stats) if st['status']][:5]}"
    gpu_paths = {u: dec.best_path_batch(chans, use_final=u, words_cap=4096, raw=True) for u in (True, False)}

    # ---- every checked channel against the checker -------------------------------------------
    for s in check:
        want = futures[s].result()
        st, label = stats[s], f"{cfg.name}/ch{s}"
        assert want["status"] == 0, label
        assert st["frames"] == want["frames"] == lens[s] + 1, label
        assert st["arcs_expanded"] == want["arcs"], f"{label} arcs_expanded {st['arcs_expanded']} != {want['arcs']}"
        assert st["max_tokens_pre_prune"] == want["max_pre"] and st["max_tokens"] == want["max_post"], label
        gs, gc, ga = sorted_tokens(dec.tokens(s, -1))
        os_, oc, oa = want["last"]
        assert np.array_equal(gs, os_) and np.array_equal(gc.view(np.uint32), oc.view(np.uint32)) and np.array_equal(ga, oa), f"{label} last frame"
        assert (int(dig[0][s]), int(dig[1][s]), int(dig[2][s])) == want["lattice"], f"{label} lattice record set"
        assert st["lattice_arcs"] == want["lattice"][0], label
        for k, u in enumerate((True, False)):
            bp, gp = want["paths"][k], gpu_paths[u]
            assert gp[4][s] == 0 and np.array_equal(gp[0][s, :gp[1][s]], bp["words"]), f"{label} best-path words"
            assert np.float32(gp[2][s]).view(np.uint32) == np.float32(bp["total_cost"]).view(np.uint32), label
            assert bool(gp[3][s]) == bp["reached_final"], label
        if offline:
            for k in (0, 1):
                got, info = final[s][k]
                d, best, rf = want["final"][k]
                assert set_digest(record_hashes(got["frame"], got["arc"], got["extra_cost"])) == d, f"{label} final lattice"
                assert np.float32(info["best_cost"]).view(np.uint32) == np.float32(best).view(np.uint32) and bool(info["reached_final"]) == rf, label

    # ---- the sampled channels frame by frame --------------------------------------------------
    for s in sample:
        od = futures[s].result()["od"]
        label = f"{cfg.name}/ch{s}"
        for f in list(range(0, od.num_frames, frame_step)) + [od.num_frames - 1]:
            gs, gc, ga = sorted_tokens(dec.tokens(s, f))
            os_, oc, oa = od.tokens(f)
            assert np.array_equal(gs, os_), f"{label} frame {f}: states"
            assert np.array_equal(gc.view(np.uint32), oc.view(np.uint32)), f"{label} frame {f}: costs"
            assert np.array_equal(ga, oa), f"{label} frame {f}: arcs"
        got = np.concatenate(lat[s])
        o = np.lexsort((got["arc"], got["frame"]))
        fr, ar, ex = od.lattice()
        assert len(got) == len(fr) == stats[s]["lattice_arcs"], label
        assert np.array_equal(got["frame"][o], fr) and np.array_equal(got["arc"][o], ar), label
        assert np.array_equal(got["extra_cost"][o].view(np.uint32), ex.view(np.uint32)), label
        if offline:
            for use_final, (got, info) in ((True, final[s][0]), (False, final[s][1])):
                want = od.final_lattice(use_final)
                o2 = np.lexsort((got["arc"], got["frame"]))
                assert len(got) == len(want["frame"]), f"{label} final lattice size"
                assert np.array_equal(got["frame"][o2], want["frame"]) and np.array_equal(got["arc"][o2], want["arc"]), label
                assert np.array_equal(got["extra_cost"][o2].view(np.uint32), want["extra"].view(np.uint32)), label
        if cfg.chunk:                                  # the per-chunk partial results, against a second checker run
            od2 = oracle.OracleDecoder(og, beam, cfg.lattice_beam, max_active)
            rows = cfg.loglikes(s, 0, int(lens[s]))
            for k, f0 in enumerate(range(0, T, chunk)):
                if len(rows[f0:f0 + chunk]):
                    od2.advance(rows[f0:f0 + chunk])
                if k % 5 == 0 or f0 + chunk >= T:
                    assert np.array_equal(partial[s][k], od2.best_path(False)["words"]), f"{label} partial path after chunk {k}"
        for use_final in (True, False):
            bp = od.best_path(use_final)
            assert np.array_equal(dec.best_path_arcs(s, use_final)["arcs"].astype(np.int64), bp["arcs"]), label
    pool.shutdown()
    return dec


def test_config3_online_500_channels():
    cfg = synth.configs()[3]
    decode_and_compare(cfg, sample=[0, 137, 499], token_capacity=16384, history_capacity=2_500_000,
                       lattice_capacity=400_000, snapshot_blocks=40, snapshot_block_capacity=16_000 * cfg.n_streams)


@pytest.mark.parametrize("lane_threads", [0, 512])      # 0: the library's choice (1024 threads for 100 lanes)
def test_config2_offline_ragged_batch(lane_threads):
    cfg = synth.configs()[2]
    decode_and_compare(cfg, sample=[0, 41, 99] if lane_threads == 0 else [7, 58], token_capacity=32768,
                       history_capacity=4_000_000, lattice_capacity=6_000_000, lane_threads=lane_threads,
                       check=None if lane_threads == 0 else range(0, 100, 4))


def test_config4_large_graph():
    cfg = synth.configs()[4]
    decode_and_compare(cfg, sample=[3, 150], token_capacity=60000, history_capacity=12_000_000,
                       lattice_capacity=14_000_000, frame_step=3, check=range(0, 200, 6))


@pytest.mark.parametrize("lane_threads,max_active,n_frames", [(512, 7000, 200), (1024, 7000, 200), (256, 2000, 120),
                                                             (512, 2000, 120), (1024, 2000, 120)])
def test_max_active_binds_on_the_8m_state_graph(lane_threads, max_active, n_frames):
    """The graph of configs 2-3 with beam 18: thousands of tokens within the beam (peaks of 8 000 -
    15 000), so the exact max-active selection binds on the large graph - at the peaks with the
    config's limit of 7000, in most frames with a limit of 2000 - for every lane size.  All 16
    channels are compared with the checker."""
    cfg = synth.configs()[2]
    dec = decode_and_compare(cfg, sample=[0, 9], token_capacity=1 << 16, history_capacity=2_000_000, lattice_capacity=8_000_000,
                             channels=16, beam=18.0, max_active=max_active, n_frames=n_frames, lane_threads=lane_threads,
                             frame_step=7)
    st = [dec.stats(c) for c in range(16)]
    binding = [s for s in st if s["max_tokens_pre_prune"] > max_active]
    assert len(binding) >= 12 and all(s["max_tokens"] == max_active for s in binding)


@pytest.mark.parametrize("lane_workgroups", [0, 16])
def test_config1_whole_stream_with_max_active_binding(lane_workgroups):
    """Config 1: one stream of 1000 frames on the 200k-state graph, ~26k tokens before and 7000
    after pruning in nearly every frame, so the exact max-active selection runs a thousand
    times at different places of the cost range; every frame is compared.  Once with one
    workgroup on the lane, once with sixteen working through every frame together."""
    cfg = synth.configs()[1]
    decode_and_compare(cfg, sample=[0], token_capacity=1 << 16, history_capacity=8_000_000, lattice_capacity=8_000_000,
                       lane_workgroups=lane_workgroups)
