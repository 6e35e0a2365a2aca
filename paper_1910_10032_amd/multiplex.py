"""Measurement of what it costs to rotate more channels than lanes through the decoder (the
context switch of the paper's Section 3.1), on top of the multiplexer binding.  Argument
marshalling and timing only: the binding and the decoding are the library's."""
from __future__ import annotations

import time

import numpy as np

from . import binding as B


def rotation_cost_us(graph: "B.WfstGraph", beam: float, lattice_beam: float, max_active: int, n_lanes: int, steps: int,
                     chunk: int, row0: np.ndarray, stride: int, stream: int, **decoder_args) -> dict:
    """Two timed sequences of `steps` multiplexer steps (one chunk per lane and step, no readouts)
    that decode exactly the same rows from exactly the same states:
      (a) one group of n_lanes channels takes all the steps (chunks 2 .. 2 + steps - 1 of its streams);
      (b) `steps` other groups take one step each: group k was brought to chunk 2 + k beforehand and
          decodes that chunk, so every step binds n_lanes channels the previous step did not touch.
    Channel g * n_lanes + l reads the score rows of lane l (row0[l]: device address of its first
    row), so step k of (b) does the same work as step k of (a); the difference per step is what
    switching the lanes to other channels costs."""
    import torch
    groups = steps + 1
    total = groups * n_lanes
    frames = (2 + steps) * chunk
    dec = B.WfstDecoder(graph, beam, lattice_beam, max_active, num_channels=total, max_lanes=n_lanes, max_frames=frames,
                        **decoder_args)
    dec.init_channels(np.arange(total, dtype=np.int32))
    mux = B.WfstMux(dec)
    row_bytes = stride * 4
    depth = [0] * groups                                     # chunks each group has consumed

    def submit_group(g: int) -> None:
        for lane in range(n_lanes):
            mux.submit(g * n_lanes + lane, int(row0[lane]) + depth[g] * chunk * row_bytes, stride, chunk)
        depth[g] += 1

    for g in range(groups):                                  # untimed: group 0 to chunk 2, group k >= 1 to chunk 2 + k - 1
        for _ in range(2 if g == 0 else 2 + g - 1):
            submit_group(g)
            assert mux.step(stream) == n_lanes
    torch.cuda.synchronize()

    def timed(order) -> float:
        for g in order:                                      # queued before the clock starts: the steps alone are timed
            submit_group(g)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in order:
            assert mux.step(stream) == n_lanes
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / len(order) * 1e6

    rotating = timed(list(range(1, groups)))                 # group k decodes chunk 2 + k - 1
    same = timed([0] * steps)                                # group 0 decodes chunks 2 .. 2 + steps - 1
    assert mux.pending() == 0
    arcs_same = sum(dec.stats(c)["arcs_expanded"] for c in range(0, n_lanes, max(1, n_lanes // 16)))
    mux.destroy()
    dec.destroy()
    return {"us_per_batch": round(rotating - same, 1), "same_channels_us_per_step": round(same, 1),
            "rotating_channels_us_per_step": round(rotating, 1), "channels": total, "lanes": n_lanes, "steps": steps,
            "note": "one %d-frame chunk per lane and step, no readouts; the same rows decoded from the same states by one group "
                    "of %d channels in all steps vs a different group in every step; a channel's state is addressed by its id "
                    "and never copied" % (chunk, n_lanes)}
