#!/usr/bin/env python3
"""Throughput of the representation-shift hot path on one MI355X.

A step = one full forward of the encoder stack (every block: LayerNorm, QKV, fused
attention, projection, MLP with the shift epilogue; after the scheduled blocks: score,
top-k selection, gather) over one batch of seeded synthetic tokens that already sit in
HBM.  Patch embedding, positional embedding, final norm and classifier head are not
part of the path.

Prints ONE JSON line (see the keys below).  `roofline` is measured live: after the timed
region the same steps are replayed with the library's per-kernel HIP-event timing on the
launch stream; `cpu_baseline` times the fp64 CPU checker on a bounded sample of the same
workload on this machine's host cores.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 matrix peak
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E peak


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="vit_b16",
                    help="a key of synth_inputs.WORKLOADS: vit_b16 (default) | vit_s16 | video_vit_b16 | "
                         "video_vit_l14 | deit_t/s/b | umt_b_ret/qa | umt_l_ret/qa | deit_s_toy | umt_b_toy")
    ap.add_argument("--unpruned", action="store_true", help="run the same stack without pruning")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample", type=int, default=0, help="images for the CPU baseline (0 = auto)")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the two side measurements: rs_shift_topk alone on an HBM-resident shape (B=4096, "
                         "N=197, D=768) and rs_attention_fwd alone at the long video shape (4 x 4097 tokens x 16 heads)")
    ap.add_argument("--streams", type=int, default=2,
                    help="the batch is cut into this many equal parts, each run block by block on a HIP stream of "
                         "its own: images are independent, and the parts' kernels fill each other's idle CUs "
                         "(last rounds of the GEMMs, small kernels).  1 = the whole batch on one stream")
    ap.add_argument("--graph", action="store_true",
                    help="capture one step into a HIP graph and time its replays (for the small, launch-bound "
                         "workloads; the per-kernel replay stays eager)")
    ap.add_argument("--calib-copy-mb", type=int, default=0,
                    help="after the run, copy this many MiB device-to-device three times: a kernel of known "
                         "traffic to scale rocprofv3 FETCH_SIZE / WRITE_SIZE readings with")
    return ap.parse_args()


# HBM bytes per launch (fetch + write) from the rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this
# script, scaled by what the same counters read for a 1 GiB device copy (fetch x2.000, write x1.000);
# the runs and their per-kernel table are profiles/vit_b16_forward_hbm_traffic.md.  Counters cannot
# be read from inside the process, so the figure is carried here; None where no run was made.
MEASURED_HBM_BYTES_PER_LAUNCH = {
    ("vit_b16", False, "gemm_fc2"): 556.4e6,   # the 8 of 12 launches that carry the shift epilogue
    ("vit_b16", False, "gemm_fc1"): 574.5e6,
    ("vit_b16", False, "gemm_qkv"): 445.0e6,
}


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
              "--gpus %d is not supported" % a.gpus, file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2508_00367_amd as rs
    import synth_inputs as si

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    wl = dict(si.WORKLOADS[a.workload])
    assert wl["dtype"] == "bf16"
    B, N, D, H, Dm, L = wl["B"], wl["N"], wl["D"], wl["H"], wl["Dm"], wl["blocks"]
    P = wl.get("n_prefix", 1)                        # protected prefix (class token), 0 for the video models
    op = {"mlp": rs.RS_SHIFT_MLP, "attn": rs.RS_SHIFT_ATTN, "block": rs.RS_SHIFT_BLOCK}[wl.get("op", "mlp")]
    prune = None if a.unpruned else wl["prune"]
    sched = rs.keep_counts(N, P, L, prune)           # per block: (tokens in, non-prefix kept)
    tdt = torch.bfloat16
    dev = "cuda"

    # ---- inputs and weights: seeded, rounded to bf16 on the host, resident in HBM ----
    def up(arr):
        return torch.from_numpy(si.round_to_bf16(arr)).to(dev, tdt)

    x0 = up(si.tokens(0, B, N, D))
    weights, keep_alive = [], []
    for l in range(L):
        w = {k: up(v) for k, v in si.block_weights(0, l, D, Dm).items()}
        cfg0 = rs.make_cfg(B, N, D, H, Dm, P, N - P, tdt)
        packed = torch.empty(rs.rs_packed_weights_size(cfg0), dtype=torch.uint8, device=dev)
        rs.rs_pack_weights(cfg0, rs.make_weights(w), packed)      # one-off, untimed
        keep_alive.append((w, packed))
        weights.append(rs.make_weights(w, packed))
    cfgs = [rs.make_cfg(B, n_in, D, H, Dm, P, n_keep, tdt, op=op) for n_in, n_keep in sched]
    ws = torch.empty(max(rs.rs_block_workspace_size(c) for c in cfgs), dtype=torch.uint8, device=dev)
    bufs = [torch.empty((B, N, D), device=dev, dtype=tdt) for _ in range(2)]
    kept = torch.empty((B, N), device=dev, dtype=torch.int32)

    def step():
        stream = torch.cuda.current_stream()   # the capture stream while a graph is recorded
        src = x0
        for l in range(L):
            dst = bufs[l & 1]
            rs.rs_block_fwd(cfgs[l], weights[l], src, dst, kept, None, ws, stream)
            src = dst
        return src

    # the timed configuration: S parts of the batch on S streams (same kernels, same results)
    S = min(a.streams, B) if (a.streams > 1 and not a.graph) else 1
    run = step
    if S > 1:
        parts, first = [], 0
        for i in range(S):
            Bp = B // S + (1 if i < B % S else 0)
            cfgs_p = [rs.make_cfg(Bp, n_in, D, H, Dm, P, n_keep, tdt, op=op) for n_in, n_keep in sched]
            parts.append(dict(x=x0[first:first + Bp], cfgs=cfgs_p,
                              ws=torch.empty(max(rs.rs_block_workspace_size(c) for c in cfgs_p), dtype=torch.uint8, device=dev),
                              bufs=[torch.empty((Bp, N, D), device=dev, dtype=tdt) for _ in range(2)],
                              kept=torch.empty((Bp, N), device=dev, dtype=torch.int32), stream=torch.cuda.Stream()))
            first += Bp

        def step_parts():
            src = [p["x"] for p in parts]
            for l in range(L):
                for i, p in enumerate(parts):
                    dst = p["bufs"][l & 1]
                    rs.rs_block_fwd(p["cfgs"][l], weights[l], src[i], dst, p["kept"], None, p["ws"], p["stream"])
                    src[i] = dst
        run = step_parts
    if a.graph:
        # the library neither allocates nor synchronises, so a whole step records as is
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
        run = graph.replay

    torch.cuda.synchronize()
    for _ in range(a.warmup):
        run()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(a.steps):
        run()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / a.steps * 1e3
    images_s = B * a.steps / dt
    tokens_s = images_s * N

    # ---- per-kernel durations: replay the same steps with event timing on ----
    rs.rs_profile_enable(True)
    t0 = time.perf_counter()
    for _ in range(a.steps):
        step()
    prof = rs.rs_profile_read()
    instr_ms_per_step = (time.perf_counter() - t0) / a.steps * 1e3
    rs.rs_profile_enable(False)

    # algorithmic work per step, per kernel class
    e = 2
    fl = {k: 0.0 for k in ("gemm_qkv", "gemm_proj", "gemm_fc1", "gemm_fc2", "attention")}
    by = {k: 0.0 for k in ("attention", "layernorm", "prune")}
    for (n_in, n_keep) in sched:
        M = B * n_in
        fl["gemm_qkv"] += 2.0 * M * D * 3 * D
        fl["gemm_proj"] += 2.0 * M * D * D
        fl["gemm_fc1"] += 2.0 * M * D * Dm
        fl["gemm_fc2"] += 2.0 * M * Dm * D
        fl["attention"] += 4.0 * B * n_in * n_in * D
        by["attention"] += 4.0 * M * D * e            # read q, k, v once, write o
        by["layernorm"] += 2 * 2.0 * M * D * e
        if n_keep < n_in - P:                          # score finalise + select + gather of K rows
            K = P + n_keep
            by["prune"] += B * (8.0 * n_in + 4.0 * K + 2.0 * K * D * e)
    total_flops = sum(fl.values())

    def kern(name):
        ms, n = prof[name]
        return (ms / n * 1e-3, n // a.steps) if n else (0.0, 0)

    kernels = {}
    for name in ("gemm_qkv", "gemm_proj", "gemm_fc1", "gemm_fc2", "attention"):
        avg_s, per_step = kern(name)
        if per_step:
            tf = fl[name] / per_step / avg_s / 1e12
            kernels[name] = {"avg_us": round(avg_s * 1e6, 2), "launches_per_step": per_step,
                             "TFLOP/s": round(tf, 1), "frac_mfma": round(tf / PEAK_BF16_TFLOPS, 4)}
    avg_s, per_step = kern("attention")
    if per_step:
        kernels["attention"]["GB/s"] = round(by["attention"] / per_step / avg_s / 1e9, 1)
    avg_s, per_step = kern("layernorm")
    if per_step:
        kernels["layernorm"] = {"avg_us": round(avg_s * 1e6, 2), "launches_per_step": per_step,
                                "GB/s": round(by["layernorm"] / per_step / avg_s / 1e9, 1)}
    prune_ms = sum(prof[k][0] for k in ("shift_score", "select", "gather")) / a.steps
    n_prune = sum(1 for (n_in, n_keep) in sched if n_keep < n_in - P)
    if n_prune:
        kernels["prune_pass"] = {"ms_per_step": round(prune_ms, 4), "passes_per_step": n_prune,
                                 "GB/s": round(by["prune"] / (prune_ms * 1e-3) / 1e9, 1),
                                 "note": "score finalise + select + gather inside rs_block_fwd"}

    # the dominant kernel by time
    dom = max(("gemm_qkv", "gemm_proj", "gemm_fc1", "gemm_fc2", "attention"), key=lambda k: prof[k][0])
    avg_s, per_step = kern(dom)
    achieved = fl[dom] / per_step / avg_s / 1e12
    roofline = {"kernel": dom, "bound": "mfma", "achieved": round(achieved, 2), "peak": PEAK_BF16_TFLOPS,
                "unit": "TFLOP/s", "frac": round(achieved / PEAK_BF16_TFLOPS, 4),
                "traffic": MEASURED_HBM_BYTES_PER_LAUNCH.get((a.workload, a.unpruned, dom)),
                "avg_launch_us": round(avg_s * 1e6, 2), "launches_per_step": per_step,
                "whole_step_frac_of_mfma_peak": round(total_flops / (ms_per_step * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4)}

    out = {
        "metric": "images/s ViT-B fwd w/ rep-shift pruning" if a.workload == "vit_b16" else
                  "images/s encoder fwd w/ rep-shift pruning", "value": round(images_s, 1), "unit": "images/s",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic (seeded N(0,1) tokens, N(0,0.02) weights, resident in HBM)",
        "config": {"workload": a.workload + ("_unpruned" if a.unpruned else ""), "batch": B, "tokens": N,
                   "D": D, "heads": H, "mlp": Dm, "blocks": L,
                   "tokens_per_block": [n for n, _ in sched],
                   "excluded": "patch/pos embedding, final norm, head"},
        "tokens_per_s": round(tokens_s, 1),
        "gflop_per_image": round(total_flops / B / 1e9, 3),
        "roofline": roofline,
        "kernels": kernels,
        "instrumented_ms_per_step": round(instr_ms_per_step, 4),
        "launch": "hip graph replay" if a.graph else "eager",
        "streams": S,
    }
    if S > 1:
        out["roofline"]["measured_on"] = ("instrumented replay of the whole batch on one stream (a launch has the "
                                          "chip to itself); the timed steps run %d parts of the batch on %d streams" % (S, S))

    # ---- optional: the prune pass alone on an HBM-resident shape ----
    if not a.no_extras:
        Bs, Ns, Ds, Ks = 4096, 197, 768, 177
        f_in = torch.randn((Bs, Ns, Ds), device=dev, dtype=tdt)
        f_out = f_in + 0.1 * torch.randn((Bs, Ns, Ds), device=dev, dtype=tdt)
        sc = torch.empty((Bs, Ns), device=dev, dtype=torch.float32)
        kp = torch.empty((Bs, 1 + Ks), device=dev, dtype=torch.int32)
        g = torch.empty((Bs, 1 + Ks, Ds), device=dev, dtype=tdt)
        for _ in range(3):
            rs.rs_shift_topk(f_out, f_in, None, 1, Ks, sc, kp, g)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        reps = 10
        for _ in range(reps):
            rs.rs_shift_topk(f_out, f_in, None, 1, Ks, sc, kp, g)
        torch.cuda.synchronize()
        ts = (time.perf_counter() - t0) / reps
        alg = Bs * (2.0 * Ns * Ds * e + 8.0 * Ns + 4.0 * (1 + Ks) + (1 + Ks) * Ds * e)
        out["prune_stress"] = {"shape": [Bs, Ns, Ds, Ks], "ms": round(ts * 1e3, 4),
                               "GB/s": round(alg / ts / 1e9, 1), "frac_hbm": round(alg / ts / 1e9 / PEAK_HBM_GBS, 4)}
        del f_in, f_out, g
        # fused attention alone at the long-sequence video shape (matrix-core utilisation of the core step)
        Ba, Na, Ha = 4, 4097, 16
        qkv = torch.randn((Ba, Na, 3, Ha, 64), device=dev, dtype=tdt)
        oa = torch.empty((Ba, Na, Ha, 64), device=dev, dtype=tdt)
        for _ in range(3):
            rs.rs_attention_fwd(qkv[:, :, 0], qkv[:, :, 1], qkv[:, :, 2], oa, 0.125)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(20):
            rs.rs_attention_fwd(qkv[:, :, 0], qkv[:, :, 1], qkv[:, :, 2], oa, 0.125)
        torch.cuda.synchronize()
        ta = (time.perf_counter() - t0) / 20
        fa = 4.0 * Ba * Ha * Na * Na * 64
        out["attention_long"] = {"shape": [Ba, Na, Ha, 64], "us": round(ta * 1e6, 1),
                                 "TFLOP/s": round(fa / ta / 1e12, 1), "frac_mfma": round(fa / ta / 1e12 / PEAK_BF16_TFLOPS, 4)}
        del qkv, oa

    if a.calib_copy_mb:
        src_c = torch.empty(a.calib_copy_mb << 20, dtype=torch.uint8, device=dev).fill_(1)
        dst_c = torch.empty_like(src_c)
        for _ in range(3):
            dst_c.copy_(src_c)
        torch.cuda.synchronize()
        out["calib_copy_bytes"] = int(src_c.numel())
        del src_c, dst_c

    # ---- CPU baseline: the fp64 checker on a bounded sample of the same workload ----
    if not a.no_cpu_baseline:
        import oracle
        per_img_gflop = total_flops / B / 1e9
        ns = a.cpu_sample or max(1, min(B, int(round(64 * 26.6 / per_img_gflop)) or 1))
        xs = si.round_to_bf16(si.tokens(0, B, N, D)[:ns]).astype(np.float64)
        wts = [{k: si.round_to_bf16(v) for k, v in si.block_weights(0, l, D, Dm).items()} for l in range(L)]
        t0 = time.perf_counter()
        for l, (n_in, n_keep) in enumerate(sched):
            r = oracle.block_pruned(xs, wts[l], H, P, n_keep, op=op)   # the op codes are the same on both sides
            xs = r["y"]
        tc = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": round(ns / tc, 3), "unit": "images/s", "cores": oracle.num_threads(),
                               "kind": "oracle",
                               "sample": "%d of %d images, all %d blocks, same schedule, fp64, gcc -O2 -fopenmp, %.1f s"
                                         % (ns, B, L, tc)}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
