"""Element-by-element comparison of one GPU channel against one CPU-checker stream."""
from __future__ import annotations

import numpy as np


def sorted_tokens(tok):
    o = np.argsort(tok["state"], kind="stable")
    return tok["state"][o], tok["cost"][o], tok["in_arc"][o]


def compare_channel(dec, ch, od, frames=None, lattice=True, label=""):
    """dec: WfstDecoder, ch: channel id, od: OracleDecoder fed the same rows.
    frames: iterable of frame indices to compare (default: all).  Bit-exact everywhere."""
    st = dec.stats(ch)
    want_status = {0: 0, 1: -8, 2: -9}[od.status]
    assert st["status"] == want_status, f"{label} status {st['status']} != {want_status}"
    assert st["frames"] == od.num_frames, f"{label} frames {st['frames']} != {od.num_frames}"
    assert st["arcs_expanded"] == od.arcs_expanded, f"{label} arcs_expanded {st['arcs_expanded']} != {od.arcs_expanded}"
    assert st["max_tokens_pre_prune"] == od.max_tokens_pre_prune, label
    assert st["max_tokens"] == od.max_tokens, label
    if frames is None:
        frames = range(od.num_frames)
    for f in frames:
        gs, gc, ga = sorted_tokens(dec.tokens(ch, f))
        os_, oc, oa = od.tokens(f)
        assert np.array_equal(gs, os_), f"{label} frame {f}: token states differ ({len(gs)} vs {len(os_)})"
        assert np.array_equal(gc.view(np.uint32), oc.view(np.uint32)), f"{label} frame {f}: costs differ"
        assert np.array_equal(ga, oa), f"{label} frame {f}: best incoming arcs differ"
    if lattice and od.status == 0:
        check_final_lattice(dec, ch, od, label)
    if lattice:
        lat = dec.lattice_arcs(ch)
        o = np.lexsort((lat["arc"], lat["frame"]))
        fr, ar, ex = od.lattice()
        assert len(lat) == len(fr), f"{label} lattice size {len(lat)} != {len(fr)}"
        assert np.array_equal(lat["frame"][o], fr) and np.array_equal(lat["arc"][o], ar), f"{label} lattice arcs differ"
        assert np.array_equal(lat["extra_cost"][o].view(np.uint32), ex.view(np.uint32)), f"{label} extra costs differ"
        assert st["lattice_arcs"] == len(fr)
    if od.status == 0:
        for use_final in (True, False):
            bp = od.best_path(use_final)
            g = dec.best_path(ch, use_final)
            assert np.array_equal(g["words"], bp["words"]), f"{label} best-path words differ"
            assert np.float32(g["total_cost"]).view(np.uint32) == np.float32(bp["total_cost"]).view(np.uint32), label
            assert g["reached_final"] == bp["reached_final"], label
            ga = dec.best_path_arcs(ch, use_final)
            assert np.array_equal(ga["arcs"].astype(np.int64), bp["arcs"]), f"{label} best-path arcs differ"


def check_final_lattice(dec, ch, od, label=""):
    """Backward-pruned lattice of the arcs still buffered on the device (nothing drained yet)
    against the checker's, for both kinds of end condition."""
    for use_final in (True, False):
        got, info = dec.final_lattice(ch, use_final)
        want = od.final_lattice(use_final)
        o = np.lexsort((got["arc"], got["frame"]))
        assert len(got) == len(want["frame"]) == info["arcs_kept"], f"{label} final lattice size {len(got)} != {len(want['frame'])}"
        assert np.array_equal(got["frame"][o], want["frame"]) and np.array_equal(got["arc"][o], want["arc"]), f"{label} final lattice arcs"
        assert np.array_equal(got["extra_cost"][o].view(np.uint32), want["extra"].view(np.uint32)), label
        assert np.float32(info["best_cost"]).view(np.uint32) == np.float32(want["best_cost"]).view(np.uint32), label
        assert bool(info["reached_final"]) == want["reached_final"], label
        assert info["frames"] == od.num_frames


# ---- order-independent digests, for comparing every channel of a full-size workload ----------

_M1, _M2, _G = np.uint64(0xBF58476D1CE4E5B9), np.uint64(0x94D049BB133111EB), np.uint64(0x9E3779B97F4A7C15)


def _mix(x):
    x = (x ^ (x >> np.uint64(30))) * _M1
    x = (x ^ (x >> np.uint64(27))) * _M2
    return x ^ (x >> np.uint64(31))


def record_hashes(frame, arc, extra):
    """One 64-bit hash per lattice record {frame, arc, extra cost bits}."""
    with np.errstate(over="ignore"):
        x = (frame.astype(np.uint64) << np.uint64(32)) | arc.astype(np.uint64)
        x = _mix(x + _G)
        return _mix(x ^ (np.ascontiguousarray(extra, np.float32).view(np.uint32).astype(np.uint64) * _G))


def set_digest(hashes):
    """(count, wrapping sum, xor) of a multiset of record hashes: equal multisets give equal digests,
    whatever the order; different ones collide with negligible probability."""
    with np.errstate(over="ignore"):
        return (int(len(hashes)), int(hashes.sum(dtype=np.uint64)) if len(hashes) else 0,
                int(np.bitwise_xor.reduce(hashes)) if len(hashes) else 0)


def range_digests(hashes, starts, counts):
    """set_digest of hashes[starts[i] : starts[i] + counts[i]] for every i, in one pass."""
    with np.errstate(over="ignore"):
        ps = np.concatenate([np.zeros(1, np.uint64), np.cumsum(hashes, dtype=np.uint64)])
        px = np.concatenate([np.zeros(1, np.uint64), np.bitwise_xor.accumulate(hashes)]) if len(hashes) else np.zeros(1, np.uint64)
        a, b = np.asarray(starts, np.int64), np.asarray(starts, np.int64) + np.asarray(counts, np.int64)
        return np.asarray(counts, np.int64), ps[b] - ps[a], px[b] ^ px[a]
