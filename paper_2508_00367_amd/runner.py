"""Launch sequence of a whole encoder stack: block after block through rs_block_fwd, ping-ponging two
activation buffers, optionally with the batch cut into parts that run on HIP streams of their own.

Argument marshalling and buffer management only: every step of the computation runs inside the
HIP library.  bench.py times `EncoderStack.step`, and the full-depth parity tests run the very same
object (same configurations, buffers and streams) with a `capture` callback between blocks.
"""
from __future__ import annotations

import torch

from . import binding as rs
from .schedule import keep_counts

_OPS = {"mlp": rs.RS_SHIFT_MLP, "attn": rs.RS_SHIFT_ATTN, "block": rs.RS_SHIFT_BLOCK}


class EncoderStack:
    """`wl`: a workload description (B, N, D, H, Dm, blocks, prune, optional n_prefix / op);
    `x0`: device tensor [B, N, D] (bf16); `block_weights[l]`: dict name -> device tensor.

    streams = S > 1 cuts the batch into S nearly equal parts, each with its own workspace, buffers
    and HIP stream: images are independent, the kernels are the same and so are the results."""

    def __init__(self, wl: dict, x0: torch.Tensor, block_weights: list, streams: int = 1, unpruned: bool = False):
        self.B, self.N, self.D, self.H, self.Dm, self.L = wl["B"], wl["N"], wl["D"], wl["H"], wl["Dm"], wl["blocks"]
        self.P = wl.get("n_prefix", 1)
        self.op = _OPS[wl.get("op", "mlp")]
        self.sched = keep_counts(self.N, self.P, self.L, None if unpruned else wl["prune"])
        self.x0 = x0
        self.dtype = x0.dtype
        dev = x0.device
        assert x0.shape == (self.B, self.N, self.D) and len(block_weights) == self.L
        self._keep_alive = []
        self.weights = []
        cfg0 = rs.make_cfg(self.B, self.N, self.D, self.H, self.Dm, self.P, self.N - self.P, self.dtype)
        for w in block_weights:                      # one-off re-layout, outside any timed region
            packed = torch.empty(max(rs.rs_packed_weights_size(cfg0), 16), dtype=torch.uint8, device=dev)
            rs.rs_pack_weights(cfg0, rs.make_weights(w), packed)
            self._keep_alive.append((w, packed))
            self.weights.append(rs.make_weights(w, packed))
        self.gemm_variant = 0            # tile-variant switch of the bf16 GEMMs (0 = chosen by shape)
        self.chain = True                # hand row statistics from block to block (same results either way)
        self.set_streams(streams)

    def tune(self, candidates=((1, 0), (2, 0), (2, 1)), steps: int = 8, rounds: int = 2):
        """Times a few launch configurations (streams, GEMM tile variant) and keeps the fastest.
        Every configuration computes the same bits (images are independent, the tile variants add
        products and shift sums in one fixed order), so this is a choice of speed only: parts on
        several streams overlap well when every kernel is of one kind (the persistent 256 x 256 GEMM
        everywhere), a single stream gains most from the shape-dependent mix of kernels.
        Returns {(streams, variant): seconds per step}."""
        import time
        seen = {}
        for _ in range(rounds):                      # every candidate `rounds` times, the best time counts
            for S, v in candidates:
                if S > self.B:
                    continue
                self.set_streams(S)
                self.gemm_variant = v
                for _ in range(2):
                    self.step()
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                for _ in range(steps):
                    self.step()
                torch.cuda.synchronize()
                key = (len(self.parts), v)
                seen[key] = min(seen.get(key, 1e30), (time.perf_counter() - t0) / steps)
        (S, v) = min(seen, key=seen.get)
        self.set_streams(S)
        self.gemm_variant = v
        return seen

    def set_streams(self, streams: int) -> None:
        S = max(1, min(int(streams), self.B))
        dev = self.x0.device
        self.parts, first = [], 0
        for i in range(S):
            Bp = self.B // S + (1 if i < self.B % S else 0)
            cfgs = [rs.make_cfg(Bp, n_in, self.D, self.H, self.Dm, self.P, n_keep, self.dtype, op=self.op)
                    for n_in, n_keep in self.sched]
            self.parts.append(dict(
                first=first, B=Bp, x=self.x0[first:first + Bp], cfgs=cfgs,
                ws=torch.empty(max(rs.rs_block_workspace_size(c) for c in cfgs), dtype=torch.uint8, device=dev),
                bufs=[torch.empty((Bp, self.N, self.D), device=dev, dtype=self.dtype) for _ in range(2)],
                kept=torch.empty((Bp, self.N), device=dev, dtype=torch.int32),
                stats=torch.empty((Bp * self.N, 2), device=dev, dtype=torch.float32),
                stream=torch.cuda.Stream() if S > 1 else None))
            first += Bp

    def step(self, capture=None, scores=None):
        """One forward of the stack.  Parts with a stream of their own are enqueued there, a single
        part on the current stream (the capture stream while a HIP graph is recorded).
        capture(l, part, src, dst) is called after block l of a part has been enqueued;
        scores: optional per-part list of float32 [Bp, N] tensors the blocks write their scores to.
        Returns the per-part output tensors (views of the ping-pong buffers, [Bp, K_last, D])."""
        rs.rs_tune_gemm_variant(self.gemm_variant)     # process-wide switch: set on every step
        src = [p["x"] for p in self.parts]
        for l in range(self.L):
            for i, p in enumerate(self.parts):
                stream = p["stream"] if p["stream"] is not None else torch.cuda.current_stream()
                dst = p["bufs"][l & 1]
                # every block but the last leaves the row statistics of its output for the next
                # block's first LayerNorm (written by the gather as it copies the surviving rows)
                rs.rs_block_fwd_chained(p["cfgs"][l], self.weights[l], src[i], p["stats"] if l > 0 and self.chain else None,
                                        dst, p["stats"] if l + 1 < self.L and self.chain else None, p["kept"],
                                        None if scores is None else scores[i], p["ws"], stream)
                if capture is not None:
                    capture(l, p, src[i], dst)
                src[i] = dst
        K = self.P + self.sched[-1][1]
        return [s.view(-1)[:p["B"] * K * self.D].view(p["B"], K, self.D) for s, p in zip(src, self.parts)]
