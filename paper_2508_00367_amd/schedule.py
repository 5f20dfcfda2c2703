"""Host logic: pruning schedules (percentages -> per-block keep counts) and FLOP accounting.

Schedule rule (Sec. 4.1 "Settings", Sec. 4.2): block l (counted from 1) is scored around
its MLP and pruned after the block is complete; a percentage refers to the tokens outside
the protected prefix and the number dropped is rounded down.
"""
from __future__ import annotations


def keep_counts(N: int, n_prefix: int, blocks: int, prune: dict | None):
    """Per block: (tokens entering, non-prefix tokens kept after it).

    prune: {"kind": "drop_pct", "pct": p, "after": [l, ...]} or
           {"kind": "drop_count", "r": r, "after": [l, ...]} or None.
    """
    out = []
    n_in = N
    after = set(prune["after"]) if prune else ()
    for l in range(1, blocks + 1):
        cand = n_in - n_prefix
        drop = 0
        if l in after:
            if prune["kind"] == "drop_pct":
                drop = cand * int(prune["pct"]) // 100
            elif prune["kind"] == "drop_count":
                drop = min(int(prune["r"]), cand)
            else:
                raise ValueError(prune["kind"])
        out.append((n_in, cand - drop))
        n_in -= drop
    return out


def block_flops(N: int, D: int, Dm: int) -> tuple[int, int]:
    """(linear, attention) FLOPs of one block on N tokens of one image: 2 x the
    multiply-accumulates of QKV + proj + fc1 + fc2 and of QK^T + PV (Sec. 3.1 cost terms)."""
    return 2 * N * (4 * D * D + 2 * D * Dm), 4 * N * N * D


def forward_flops(N: int, n_prefix: int, D: int, Dm: int, blocks: int, prune: dict | None):
    lin = att = 0
    for n_in, _ in keep_counts(N, n_prefix, blocks, prune):
        a, b = block_flops(n_in, D, Dm)
        lin += a
        att += b
    return lin, att
