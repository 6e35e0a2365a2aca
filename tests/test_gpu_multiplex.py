"""The channel-to-lane multiplexer (Section 3.1): four times more channels than lanes take turns
on the lanes, chunk by chunk, in the order their audio arrives.  Every channel is compared with
the CPU checker, which decodes each stream on its own in one go: multiplexing must not change
a single bit."""
import numpy as np
import pytest

import oracle
import synth
from gpu_compare import compare_channel

pytestmark = pytest.mark.gpu
F32 = np.float32


@pytest.mark.parametrize("seed", [0, 1])
def test_channels_rotate_through_fewer_lanes(seed):
    import torch

    from paper_1910_10032_amd import binding as B
    assert torch.cuda.is_available()
    c = synth.configs()[0]
    g = synth.make_graph(c.graph)
    rng = np.random.default_rng(seed)
    n_ch, n_lanes, chunk = 32, 8, 25
    lens = rng.integers(60, 151, size=n_ch)                 # ragged streams, last chunks shorter
    rows = [c.loglikes(s, 0, int(lens[s])) for s in range(n_ch)]
    dev = [torch.from_numpy(r).cuda() for r in rows]
    dec = B.WfstDecoder(B.WfstGraph(g), c.beam, c.lattice_beam, c.max_active, num_channels=n_ch, max_lanes=n_lanes,
                        max_frames=int(lens.max()), lattice_capacity=1 << 19, lane_threads=int(rng.choice([0, 256, 512, 1024])))
    dec.init_channels(list(range(n_ch)))
    mux = B.WfstMux(dec)
    P = g.num_pdfs
    fed = [0] * n_ch
    batches = 0
    # audio "arrives" for random channels, a chunk at a time; a step is taken now and then, so the
    # queue holds from a few to many waiting channels, and some channels queue several chunks
    order = [s for s in range(n_ch) for _ in range((int(lens[s]) + chunk - 1) // chunk)]
    rng.shuffle(order)
    bound = 0
    for k, s in enumerate(order):
        n = min(chunk, int(lens[s]) - fed[s])
        mux.submit(s, dev[s].data_ptr() + fed[s] * P * 4, P, n)
        fed[s] += n
        if rng.integers(0, 3) == 0 or k == len(order) - 1:
            while mux.pending() > (0 if k == len(order) - 1 else int(rng.integers(0, 12))):
                got = mux.step()
                assert 1 <= got <= n_lanes
                bound += got
                batches += 1
    torch.cuda.synchronize()
    assert mux.pending() == 0 and mux.step() == 0
    assert mux.stats() == (batches, bound) and bound == len(order)
    assert batches > len(order) // n_lanes                  # lanes were shared: far fewer lanes than channels
    og = oracle.OracleGraph(g)
    for s in range(n_ch):
        od = oracle.OracleDecoder(og, c.beam, c.lattice_beam, c.max_active)
        od.advance(rows[s])
        compare_channel(dec, s, od, label=f"mux/ch{s}")
    # argument errors
    with pytest.raises(B.WfstError) as e:
        mux.submit(n_ch, dev[0].data_ptr(), P, 1)
    assert e.value.code == B.WFST_E_BAD_CHANNEL
    with pytest.raises(B.WfstError) as e:
        mux.submit(0, dev[0].data_ptr(), P - 1, 1)
    assert e.value.code == B.WFST_E_INVALID_ARG
    mux.destroy()
