"""TEST INFRASTRUCTURE ONLY: pruning schedule and cost accounting of the checker.

Reading of the schedule (the paper gives percentages and layer lists, Sec. 4.1
"Settings" and Sec. 4.2): the score comes from block l's MLP, tokens are dropped
after the complete block l (l counted from 1), percentages apply to the tokens
outside the protected prefix, and the dropped count is rounded down.  This is
the reading under which the multiply-accumulate counts below reproduce the
GFLOPs rows of Tables 2, 4 and 5 (pinned in tests/test_oracle_schedule.py).
"""
from __future__ import annotations


def drop_count(n_nonprefix: int, drop_pct: int) -> int:
    """Tokens dropped when `drop_pct` percent of n non-prefix tokens go: floor."""
    return (n_nonprefix * drop_pct) // 100


def tokens_per_block(N: int, n_prefix: int, blocks: int, prune: dict | None) -> list[int]:
    """Token count entering each of `blocks` blocks (index 0 = block 1)."""
    out = []
    n = N
    after = set(prune["after"]) if prune else set()
    for l in range(1, blocks + 1):
        out.append(n)
        if l in after:
            if prune["kind"] == "drop_pct":
                r = drop_count(n - n_prefix, prune["pct"])
            else:
                r = min(prune["r"], n - n_prefix)
            n -= r
    return out


def block_macs(N: int, D: int, Dm: int | None = None) -> int:
    """Multiply-accumulates of one block on N tokens: the four linear layers
    (D*3D + D*D + 2*D*Dm per token) plus QK^T and PV (2*N*D per token); the
    O(N^2 C + N C^2) cost of Sec. 3.1 with its constants."""
    Dm = 4 * D if Dm is None else Dm
    return N * (4 * D * D + 2 * D * Dm) + 2 * N * N * D


def model_macs(N: int, n_prefix: int, D: int, blocks: int, prune: dict | None,
               patch_tokens: int = 0, patch_in: int = 0) -> int:
    """Encoder MACs under a schedule, plus a linear patch embedding of
    `patch_tokens` tokens with `patch_in` inputs each."""
    total = patch_tokens * patch_in * D
    for n in tokens_per_block(N, n_prefix, blocks, prune):
        total += block_macs(n, D)
    return total
