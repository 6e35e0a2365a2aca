"""The paper's closed-form memory budgets, used to compare this library's actual device
footprint against them (host arithmetic only)."""


def paper_fst_bytes(num_states: int, num_arcs: int, num_emitting_arcs: int) -> int:
    """Device bytes of the decoding graph by the paper's Eq. 1 (Section 3.2.1)."""
    return 12 * num_states + 8 * num_arcs + 4 * num_emitting_arcs


def paper_state_bytes(max_active: int, num_channels: int, num_lanes: int) -> int:
    """Device bytes of the full decoder state by the paper's Eq. 2 (Section 3.2.1)."""
    return 64 * max_active * num_channels + 544 * max_active * num_lanes + 1024 * num_lanes


def graph_decode_bytes(num_states: int, num_arcs: int) -> int:
    """Bytes this library reads while decoding: one 12-byte record per state (out-degrees
    and final cost) and per arc; Eq. 1 plus 4 bytes for every non-emitting arc."""
    return 12 * (num_states + num_arcs)
