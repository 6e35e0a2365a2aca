"""GPU parity under randomly mixed use: random small graphs (with epsilon chains), ragged
streams, a random sequence of plain and snapshot-sealing advance calls of random lengths over
random subsets of the channels, small lattice rings that wrap, few snapshot blocks that are
reused, both lane sizes, integer and real costs, tight and loose max-active.  Every snapshot
that is read and the final state of every channel must be the CPU checker's, bit for bit."""
import numpy as np
import pytest

import oracle
from gpu_compare import compare_channel
from helpers import random_graph

pytestmark = pytest.mark.gpu
F32 = np.float32


def _records_of(od, lo, hi):
    fr, ar, ex = od.lattice()
    m = (fr >= lo) & (fr < hi)
    return fr[m], ar[m], ex[m]


def _same_records(got, want, label):
    o = np.lexsort((got["arc"], got["frame"]))
    fr, ar, ex = want
    assert len(got) == len(fr), f"{label}: {len(got)} records, expected {len(fr)}"
    assert np.array_equal(got["frame"][o], fr) and np.array_equal(got["arc"][o], ar), label
    assert np.array_equal(got["extra_cost"][o].view(np.uint32), ex.view(np.uint32)), label


@pytest.mark.parametrize("seed", range(48))
def test_random_call_patterns(seed):
    import torch

    from paper_1910_10032_amd import binding as B
    assert torch.cuda.is_available()
    rng = np.random.default_rng(4200 + seed)
    integer = bool(seed % 3 == 0)
    num_pdfs = int(rng.integers(4, 16))
    g = random_graph(rng, num_states=int(rng.integers(20, 160)), n_emit_per_state=(1, int(rng.integers(2, 7))),
                     eps_prob=float(rng.choice([0.0, 0.01, 0.04])), num_pdfs=num_pdfs, wmax=4, integer=integer,
                     eps_first=bool(seed % 2), n_final=4)
    n_ch = int(rng.integers(2, 7))
    lens = [int(rng.integers(5, 70)) for _ in range(n_ch)]
    rows = [(-rng.integers(0, 5, size=(T, num_pdfs)).astype(F32)) if integer else rng.normal(-4, 2, size=(T, num_pdfs)).astype(F32)
            for T in lens]
    if seed % 7 == 5:                             # positive log-likelihoods: path costs go negative
        rows = [r + F32(7.0) for r in rows]
    if seed % 5 == 3:                             # one stream dies: a frame whose scores are all -inf
        rows[0][len(rows[0]) // 2, :] = -np.inf
    if seed % 5 == 4:                             # one stream meets a NaN score
        rows[-1][len(rows[-1]) // 3, :] = np.nan
    beam, lbeam = float(rng.choice([4.0, 7.0, 10.0])), float(rng.choice([0.0, 2.0, 5.0]))
    alpha = int(rng.choice([3, 12, 50, 5000]))
    og = oracle.OracleGraph(g)
    full = []
    for r in rows:
        od = oracle.OracleDecoder(og, beam, lbeam, alpha)
        od.advance(r)
        full.append(od)
    most = max(len(od.lattice()[0]) for od in full) + 16
    use_blocks = bool(seed % 4 != 1)
    n_blocks = int(rng.integers(2, 6)) if use_blocks else 0
    # with blocks the ring only has to hold what a channel produces between two seals; without, everything
    dec = B.WfstDecoder(B.WfstGraph(g), beam, lbeam, alpha, num_channels=n_ch, max_lanes=n_ch, max_frames=max(lens),
                        token_capacity=4096, lattice_capacity=most, snapshot_blocks=n_blocks, snapshot_block_capacity=most * n_ch,
                        lane_threads=int(rng.choice([0, 256, 512, 1024])), frame_form=int(rng.integers(0, 4) == 0))
    dec.init_channels(list(range(n_ch)))
    dev = [torch.from_numpy(r).cuda() for r in rows]
    fed = [0] * n_ch                              # frames given to each channel so far
    handed = [0] * n_ch                           # first frame whose lattice records have not been handed over
    step = [oracle.OracleDecoder(og, beam, lbeam, alpha) for _ in range(n_ch)]
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        while any(fed[c] < lens[c] for c in range(n_ch)):
            chans = [c for c in range(n_ch) if fed[c] < lens[c] and rng.uniform() < 0.8]
            if not chans:
                continue
            take = [int(min(lens[c] - fed[c], rng.integers(0, 25))) for c in chans]
            every = int(rng.integers(1, 12)) if rng.uniform() < 0.7 else 0
            if every and n_blocks and (max(take) + every - 1) // every > n_blocks:
                every = (max(take) + n_blocks - 1) // n_blocks          # no more snapshots than blocks
            tens = [dev[c][fed[c]:fed[c] + t] for c, t in zip(chans, take)]
            ids = dec.advance(chans, tens, snapshot_every=every)
            if every:
                first, count = ids
                assert count == max(1, (max(take) + every - 1) // every)
                for j in range(count):
                    ends = [fed[c] + min(t, (j + 1) * every) for c, t in zip(chans, take)]   # frames fed at this boundary
                    for c, e in zip(chans, ends):
                        if e > step[c].num_frames - 1:
                            step[c].advance(rows[c][step[c].num_frames - 1:e])
                    use_final = bool(rng.integers(0, 2))
                    got = dec.best_path_batch(chans, use_final=use_final, snapshot=first + j)
                    for c, r in zip(chans, got):
                        want_status = {0: 0, 1: B.WFST_E_DEAD_CHANNEL, 2: B.WFST_E_NAN_INPUT}[step[c].status]
                        assert r["status"] == want_status, f"seed {seed} snapshot {j} ch {c}: status {r['status']}"
                        if want_status == 0:
                            want = step[c].best_path(use_final)
                            assert np.array_equal(r["words"], want["words"]), f"seed {seed} snapshot {j} ch {c}"
                            assert np.float32(r["total_cost"]).view(np.uint32) == np.float32(want["total_cost"]).view(np.uint32)
                    if n_blocks:
                        lat = dec.snapshot_lattice_arcs(first + j, chans)
                        for i, (c, e) in enumerate(zip(chans, ends)):
                            a, n = int(lat["starts"][i]), int(lat["counts"][i])
                            _same_records(lat["records"][a:a + n], _records_of(full[c], handed[c], e + 1), f"seed {seed} snapshot {j} ch {c}")
                            handed[c] = e + 1
            for c, t in zip(chans, take):
                fed[c] += t
    torch.cuda.synchronize()
    # whatever has not been handed over through snapshots is still buffered, and everything else agrees
    recs, offs = dec.lattice_arcs_batch(list(range(n_ch)))
    for c in range(n_ch):
        if full[c].status == 0:
            _same_records(recs[offs[c]:offs[c + 1]], _records_of(full[c], handed[c], lens[c] + 1), f"seed {seed} rest ch {c}")
        compare_channel(dec, c, full[c], lattice=False, label=f"seed {seed} ch {c}")


@pytest.mark.parametrize("seed", range(12))
def test_random_heavy_frames(seed):
    """Frames of thousands of tokens on the 200k-state synthetic graph with random beams,
    max-active limits and score seeds: the max-active cut falls at many different places in
    the cost range (every call of the exact selection bins a different key range), frames
    start in the LDS table and outgrow it, or run on the global table from the start, with
    both lane sizes and with chunked calls."""
    import torch

    import synth
    from paper_1910_10032_amd import binding as B
    assert torch.cuda.is_available()
    rng = np.random.default_rng(9100 + seed)
    c = synth.configs()[1]
    g = synth.make_graph(c.graph)
    beam = float(c.beam - rng.choice([0.0, 1.0, 2.0, 3.0]))
    alpha = int(rng.choice([300, 1500, 4000, 7000]))
    lbeam = float(rng.choice([1.0, 4.0]))
    T = int(rng.integers(24, 40))
    stream_id = int(rng.integers(0, 1000))
    rows = synth.host_loglikes(c.ll_seed + seed, stream_id, 0, T, c.graph.num_pdfs, c.ll_mu, c.ll_sigma, c.ll_boost)
    od = oracle.OracleDecoder(oracle.OracleGraph(g), beam, lbeam, alpha)
    od.advance(rows)
    dec = B.WfstDecoder(B.WfstGraph(g), beam, lbeam, alpha, num_channels=1, max_lanes=1, max_frames=T, token_capacity=1 << 16,
                        lattice_capacity=len(od.lattice()[0]) + 16, lane_threads=int(rng.choice([256, 512, 1024])))
    dec.init_channels([0])
    t = torch.from_numpy(rows).cuda()
    pos = 0
    while pos < T:
        n = int(rng.integers(1, 9))
        dec.advance([0], [t[pos:pos + n]])
        pos += n
    torch.cuda.synchronize()
    assert od.max_tokens_pre_prune > 1500, "the case is meant to be heavy"
    compare_channel(dec, 0, od, label=f"heavy seed {seed} beam {beam} alpha {alpha}")
