"""The allocation-free entry point (wfst_decode_final_lattice_noalloc) against the entry point it
is a variant of (wfst_decode_final_lattice), through the C ABI: same kept arcs, same extra costs
(as bits), same summary - on two calls in a row, the second on a smaller channel, so that what
the first call left in the shared scratch cannot leak into the second."""
import numpy as np
import pytest

import synth

pytestmark = pytest.mark.gpu
F32 = np.float32


def _lattice(dec, B, torch, ch, use_final, noalloc, cap):
    out = torch.zeros(cap * 12, dtype=torch.uint8, device="cuda")
    n, info = dec.final_lattice_device(ch, use_final, out.data_ptr(), cap, noalloc=noalloc)
    rec = np.frombuffer(out.cpu().numpy().tobytes(), dtype=B.LAT_DTYPE)[:n]
    o = np.lexsort((rec["arc"], rec["frame"]))
    return rec[o], info


def test_noalloc_final_lattice_matches_the_allocating_entry_point():
    import torch
    from paper_1910_10032_amd import binding as B
    assert torch.cuda.is_available()
    B.lib()
    c = synth.configs()[0]
    g = synth.make_graph(c.graph)
    lens = [300, 120]                              # channel 1 is the smaller input
    rows = [c.loglikes(s, 0, n) for s, n in enumerate(lens)]
    dec = B.WfstDecoder(B.WfstGraph(g), c.beam, c.lattice_beam, c.max_active, num_channels=2, max_lanes=2,
                        max_frames=max(lens), lattice_capacity=1 << 20)
    dec.init_channels([0, 1])
    dec.advance([0, 1], [torch.from_numpy(r).cuda() for r in rows])
    torch.cuda.synchronize()
    cap = 1 << 18
    for ch in (0, 1):                              # two calls in a row, the second smaller
        for use_final in (True, False):
            want, winfo = _lattice(dec, B, torch, ch, use_final, False, cap)
            got, ginfo = _lattice(dec, B, torch, ch, use_final, True, cap)
            assert len(want) > 0 and len(got) == len(want)
            assert np.array_equal(got["frame"], want["frame"]) and np.array_equal(got["arc"], want["arc"])
            assert np.array_equal(got["extra_cost"].view(np.uint32), want["extra_cost"].view(np.uint32))
            assert ginfo["arcs_in"] == winfo["arcs_in"] and ginfo["arcs_kept"] == winfo["arcs_kept"] == len(want)
            assert ginfo["frames"] == winfo["frames"] == lens[ch] + 1
            assert ginfo["reached_final"] == winfo["reached_final"]
            assert F32(ginfo["best_cost"]).view(np.uint32) == F32(winfo["best_cost"]).view(np.uint32)
    # a buffer that is too small reports the needed size and writes nothing beyond it
    with pytest.raises(B.WfstError) as e:
        dec.final_lattice_device(0, True, torch.zeros(12, dtype=torch.uint8, device="cuda").data_ptr(), 1, noalloc=True)
    assert e.value.code == B.WFST_E_CAPACITY
