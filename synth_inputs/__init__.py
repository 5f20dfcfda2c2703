"""Seeded synthetic inputs for the representation-shift hot path.

This module only *produces arrays*: token tensors, weight tensors, and the
bf16 storage conversion of those arrays.  It holds none of the method's
arithmetic (no attention, no normalisation, no scoring, no selection, no
schedule rule) so that both the HIP path and the CPU checker can consume the
very same numbers without sharing any computation.

Generator: numpy's Philox counter-based bit generator keyed by
``(seed, stream)``; every tensor draws from a stream id of its own, so a tensor's
values do not depend on which other tensors were drawn before it.

Value distributions follow the workload recipe: tokens ~ N(0, 1), every linear
weight and bias ~ N(0, 0.02^2), LayerNorm gamma = 1 and beta = 0.
"""
from __future__ import annotations

import numpy as np

# Stream ids.  One per tensor kind; block index is folded in by `_stream`.
_TOKENS = 1
_TOKEN_SCALE = 2
_W_QKV, _B_QKV, _W_PROJ, _B_PROJ, _W_FC1, _B_FC1, _W_FC2, _B_FC2 = range(10, 18)
_GENERIC = 100


def _stream(kind: int, block: int = 0) -> int:
    return kind + 1000 * block


def normal(seed: int, stream: int, shape, std: float = 1.0) -> np.ndarray:
    """fp32 array of N(0, std^2) draws from stream `stream` of seed `seed`."""
    g = np.random.Generator(np.random.Philox(key=[int(seed), int(stream)]))
    a = g.standard_normal(int(np.prod(shape)), dtype=np.float32).reshape(shape)
    if std != 1.0:
        a *= np.float32(std)
    return a


# --------------------------------------------------------------------------
# bf16 storage format helpers (round-to-nearest-even on the host).
# --------------------------------------------------------------------------
def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round an fp32 array to bf16 (RNE); returns the uint16 bit patterns."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    nan = np.isnan(a)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    r = ((u + bias) >> np.uint32(16)).astype(np.uint16)
    if nan.any():
        r = np.where(nan, np.uint16(0x7FC0), r)
    return r


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns (uint16) to fp32 exactly."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """fp32 array whose every value is representable in bf16 (RNE rounded)."""
    return bf16_bits_to_f32(f32_to_bf16_bits(a))


# --------------------------------------------------------------------------
# Tensors of one encoder block.
# --------------------------------------------------------------------------
def tokens(seed: int, B: int, N: int, D: int, spread: float = 0.0) -> np.ndarray:
    """Token tensor [B, N, D] ~ N(0,1).

    `spread` > 0 multiplies token i of image b by exp(z), z ~ N(0, spread^2), a
    per-token magnitude so that per-token scores are well separated (the way
    foreground/background tokens differ); 0 leaves the plain i.i.d. recipe.
    """
    x = normal(seed, _stream(_TOKENS), (B, N, D))
    if spread > 0.0:
        z = normal(seed, _stream(_TOKEN_SCALE), (B, N, 1), std=spread)
        x = x * np.exp(z, dtype=np.float32)
    return x


WEIGHT_NAMES = ("ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_proj", "b_proj",
                "ln2_g", "ln2_b", "w_fc1", "b_fc1", "w_fc2", "b_fc2")


def block_weights(seed: int, block: int, D: int, Dm: int, std: float = 0.02) -> dict:
    """fp32 weights of encoder block `block`; matrices are [in, out] row-major."""
    return {
        "ln1_g": np.ones(D, np.float32), "ln1_b": np.zeros(D, np.float32),
        "w_qkv": normal(seed, _stream(_W_QKV, block), (D, 3 * D), std),
        "b_qkv": normal(seed, _stream(_B_QKV, block), (3 * D,), std),
        "w_proj": normal(seed, _stream(_W_PROJ, block), (D, D), std),
        "b_proj": normal(seed, _stream(_B_PROJ, block), (D,), std),
        "ln2_g": np.ones(D, np.float32), "ln2_b": np.zeros(D, np.float32),
        "w_fc1": normal(seed, _stream(_W_FC1, block), (D, Dm), std),
        "b_fc1": normal(seed, _stream(_B_FC1, block), (Dm,), std),
        "w_fc2": normal(seed, _stream(_W_FC2, block), (Dm, D), std),
        "b_fc2": normal(seed, _stream(_B_FC2, block), (D,), std),
    }


def generic(seed: int, tag: int, shape, std: float = 1.0) -> np.ndarray:
    """A free-standing tensor (q/k/v for attention-only cases, f_out/f_in ...)."""
    return normal(seed, _stream(_GENERIC + tag), shape, std)


# --------------------------------------------------------------------------
# Workload shapes (data only).  `prune` lists, per workload, after which
# 1-indexed blocks tokens are dropped and how the amount is specified; turning
# a percentage into a count is the consumer's job.
# --------------------------------------------------------------------------
WORKLOADS = {
    "vit_block_fp32": dict(dtype="f32", B=4, N=197, D=192, H=3, Dm=768, blocks=1,
                           prune=dict(kind="drop_pct", pct=30, after=[1])),
    "vit_s16": dict(dtype="bf16", B=64, N=197, D=384, H=6, Dm=1536, blocks=12,
                    prune=dict(kind="drop_count", r=16, after=list(range(1, 12)))),
    "vit_b16": dict(dtype="bf16", B=256, N=197, D=768, H=12, Dm=3072, blocks=12,
                    prune=dict(kind="drop_pct", pct=10, after=list(range(4, 12)))),
    "video_vit_b16": dict(dtype="bf16", B=8, N=1569, D=768, H=12, Dm=3072, blocks=12,
                          prune=dict(kind="drop_pct", pct=50, after=[2, 5, 8])),
    "video_vit_l14": dict(dtype="bf16", B=4, N=4097, D=1024, H=16, Dm=4096, blocks=24,
                          prune=dict(kind="drop_pct", pct=30, after=[4, 8, 12, 16])),
    # --- the shapes and schedules of the paper's own runs (Sec. 4.1, 4.2, 3.2), synthetic data ---
    # image classification, Sec. 4.2: batch 512, 20 % of the patch tokens dropped after blocks 1, 4, 7
    "deit_t": dict(dtype="bf16", B=512, N=197, D=192, H=3, Dm=768, blocks=12,
                   prune=dict(kind="drop_pct", pct=20, after=[1, 4, 7])),
    "deit_s": dict(dtype="bf16", B=512, N=197, D=384, H=6, Dm=1536, blocks=12,
                   prune=dict(kind="drop_pct", pct=20, after=[1, 4, 7])),
    "deit_b": dict(dtype="bf16", B=512, N=197, D=768, H=12, Dm=3072, blocks=12,
                   prune=dict(kind="drop_pct", pct=20, after=[1, 4, 7])),
    # video-text retrieval / video QA, Sec. 4.1: batch 20, 12 frames x 196 patches, no class token,
    # 20 % (retrieval) or 10 % (QA) dropped in each of the first three blocks
    "umt_b_ret": dict(dtype="bf16", B=20, N=2352, n_prefix=0, D=768, H=12, Dm=3072, blocks=12,
                      prune=dict(kind="drop_pct", pct=20, after=[1, 2, 3])),
    "umt_b_qa": dict(dtype="bf16", B=20, N=2352, n_prefix=0, D=768, H=12, Dm=3072, blocks=12,
                     prune=dict(kind="drop_pct", pct=10, after=[1, 2, 3])),
    "umt_l_ret": dict(dtype="bf16", B=20, N=2352, n_prefix=0, D=1024, H=16, Dm=4096, blocks=24,
                      prune=dict(kind="drop_pct", pct=20, after=[1, 2, 3])),
    "umt_l_qa": dict(dtype="bf16", B=20, N=2352, n_prefix=0, D=1024, H=16, Dm=4096, blocks=24,
                     prune=dict(kind="drop_pct", pct=10, after=[1, 2, 3])),
    # toy study of Sec. 3.2: the k lowest-score tokens dropped at ONE layer (here layer index 4 of
    # [0, 2, 4, 6, 8], i.e. after block 5), shift taken around the attention layer
    "deit_s_toy": dict(dtype="bf16", B=512, N=197, D=384, H=6, Dm=1536, blocks=12, op="attn",
                       prune=dict(kind="drop_count", r=40, after=[5])),
    "umt_b_toy": dict(dtype="bf16", B=20, N=2352, n_prefix=0, D=768, H=12, Dm=3072, blocks=12, op="attn",
                      prune=dict(kind="drop_count", r=1100, after=[5])),
}
