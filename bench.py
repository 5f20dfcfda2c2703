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
workload on this machine's host cores.  Unless --no-extras is given the line also carries
the unpruned run of the same stack, the other BASELINE workloads (a few steps each), the
prune pass alone on an HBM-resident shape and the fused attention alone at the long video shape.
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
                    help="skip the side measurements: the unpruned stack, the other BASELINE workloads, "
                         "rs_shift_topk alone on an HBM-resident shape (B=4096, N=197, D=768) and "
                         "rs_attention_fwd alone at the long video shape (4 x 4097 tokens x 16 heads)")
    ap.add_argument("--streams", type=int, default=0,
                    help="the batch is cut into this many equal parts, each run block by block on a HIP stream of "
                         "its own: images are independent, and the parts' kernels fill each other's idle CUs "
                         "(last rounds of the GEMMs, small kernels).  1 = the whole batch on one stream; 0 (default) = "
                         "a short timing of (1 stream, GEMM tiles by shape), (2 streams, by shape) and (2 streams, "
                         "persistent GEMM only) before the timed region picks the fastest (same results in all)")
    ap.add_argument("--gemm-variant", type=int, default=0,
                    help="with --streams N > 0: tile variant of the bf16 GEMMs (0 = by shape, 1..4 = one kernel only)")
    ap.add_argument("--graph", action="store_true",
                    help="capture one step into a HIP graph and time its replays (for the small, launch-bound "
                         "workloads; the per-kernel replay stays eager)")
    ap.add_argument("--calib-copy-mb", type=int, default=0,
                    help="after the run, copy this many MiB device-to-device three times: a kernel of known "
                         "traffic to scale rocprofv3 FETCH_SIZE / WRITE_SIZE readings with")
    return ap.parse_args()


# HBM bytes per launch (fetch + write) of the dominant kernel from the rocprofv3 --pmc FETCH_SIZE /
# WRITE_SIZE runs of this script (profiles/vit_b16_forward_hbm_traffic.md gives the commands and the
# scaling by a device copy of known size).  Counters cannot be read from inside the process, so the
# figure is carried here together with the build string it was measured under; a library built with
# other tile configurations gets no carried figure.
_MEASURED_BUILD = ("bf16 gemm: persistent tiles (BM,BN,BK,stages,waves m,waves n) 256, 256, 64, 2, 2, 4, three activation stages "
                   "when K >= 2048; ring tiles 128x256x32 and 128x128x32, 3 stages, 4 waves, 2 workgroups per CU, up to 0.5 rounds "
                   "(1.5 if K <= 512); rows behind whole rounds go to a ring kernel when K >= 2048 and the last round is under "
                   "0.5 full")
MEASURED_HBM_BYTES_PER_LAUNCH = {
    # (workload, unpruned, kernel class): (bytes per layer launch, rs_build_info() of the measured build)
    ("vit_b16", False, "gemm_fc1"): (575.0e6, _MEASURED_BUILD),
    ("vit_b16", False, "gemm_fc2"): (576.2e6, _MEASURED_BUILD),   # persistent kernel + ring kernel of the layer
    ("vit_b16", False, "gemm_qkv"): (448.6e6, _MEASURED_BUILD),
    ("vit_b16", False, "gemm_proj"): (235.8e6, _MEASURED_BUILD),
}


def build_stack(rs, si, torch, name, streams, unpruned=False):
    wl = dict(si.WORKLOADS[name])
    assert wl["dtype"] == "bf16"
    tdt = torch.bfloat16

    def up(arr):
        return torch.from_numpy(si.round_to_bf16(arr)).to("cuda", tdt)

    x0 = up(si.tokens(0, wl["B"], wl["N"], wl["D"]))
    ws = [{k: up(v) for k, v in si.block_weights(0, l, wl["D"], wl["Dm"]).items()} for l in range(wl["blocks"])]
    return wl, rs.EncoderStack(wl, x0, ws, streams=streams, unpruned=unpruned)


def time_steps(torch, run, steps, warmup):
    torch.cuda.synchronize()
    for _ in range(warmup):
        run()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        run()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / steps


def stack_flops(stack):
    B, D, Dm = stack.B, stack.D, stack.Dm
    fl = {k: 0.0 for k in ("gemm_qkv", "gemm_proj", "gemm_fc1", "gemm_fc2", "attention")}
    for (n_in, _) in stack.sched:
        M = B * n_in
        fl["gemm_qkv"] += 2.0 * M * D * 3 * D
        fl["gemm_proj"] += 2.0 * M * D * D
        fl["gemm_fc1"] += 2.0 * M * D * Dm
        fl["gemm_fc2"] += 2.0 * M * Dm * D
        fl["attention"] += 4.0 * B * n_in * n_in * D
    return fl


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
    dev, tdt, e = "cuda", torch.bfloat16, 2

    # ---- the timed configuration: S parts of the batch on S streams (same kernels, same results) ----
    S = 1 if a.graph else max(a.streams, 1)
    wl, stack = build_stack(rs, si, torch, a.workload, S, a.unpruned)
    tuned = None
    if a.streams == 0 and not a.graph:
        tuned = stack.tune()
    else:
        stack.gemm_variant = a.gemm_variant
    B, N, D, H, Dm, L, P = stack.B, stack.N, stack.D, stack.H, stack.Dm, stack.L, stack.P
    sched = stack.sched
    S = len(stack.parts)
    run = stack.step
    if a.graph:
        # the library neither allocates nor synchronises, so a whole step records as is
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            stack.step()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            stack.step()
        run = graph.replay

    sec = time_steps(torch, run, a.steps, a.warmup)
    ms_per_step = sec * 1e3
    images_s = B / sec
    tokens_s = images_s * N

    # ---- per-kernel durations: the same steps, whole batch on one stream, event timing on ----
    timed_variant = stack.gemm_variant
    stack.set_streams(1)
    stack.step()
    torch.cuda.synchronize()
    rs.rs_profile_enable(True)
    t0 = time.perf_counter()
    for _ in range(a.steps):
        stack.step()
    prof = rs.rs_profile_read()
    instr_ms_per_step = (time.perf_counter() - t0) / a.steps * 1e3
    rs.rs_profile_enable(False)

    # algorithmic work per step, per kernel class
    fl = stack_flops(stack)
    by = {k: 0.0 for k in ("attention", "layernorm", "prune")}
    slots = D // 64                                    # score partial sums per row left by the GEMM epilogue
    for l, (n_in, n_keep) in enumerate(sched):
        M = B * n_in
        by["attention"] += 4.0 * M * D * e            # read q, k, v once, write o
        # row-statistics passes (read the rows, write (mean, rstd)): always the one in front of the MLP;
        # the one in front of the attention only in the first block, later blocks get the statistics the
        # block before them left for its output: from its gather when it prunes, else from a pass over y
        prunes = n_keep < n_in - P
        n_stat = M * (2 if l == 0 else 1) + (B * (P + n_keep) if (not prunes and l + 1 < L) else 0)
        by["layernorm"] += n_stat * (D * e + 8.0)
        if prunes:                                     # partial sums in, scores + kept_idx out, gather of K rows (+ their statistics)
            K = P + n_keep
            by["prune"] += B * (12.0 * slots * n_in + 8.0 * n_in + 4.0 * K + 2.0 * K * D * e + (8.0 * K if l + 1 < L else 0.0))
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
        kernels["attention"]["frac_hbm"] = round(by["attention"] / per_step / avg_s / 1e9 / PEAK_HBM_GBS, 4)
    avg_s, per_step = kern("layernorm")
    if per_step:
        kernels["row_statistics"] = {"avg_us": round(avg_s * 1e6, 2), "launches_per_step": per_step,
                                     "GB/s": round(by["layernorm"] / per_step / avg_s / 1e9, 1),
                                     "note": "the LayerNorms are folded into the GEMMs behind them; this pass reads "
                                             "the rows once and writes (mean, rstd) per row; after a pruning block "
                                             "the gather leaves the statistics of the rows it writes instead"}
    prune_ms = sum(prof[k][0] for k in ("shift_score", "select", "gather")) / a.steps
    n_prune = sum(1 for (n_in, n_keep) in sched if n_keep < n_in - P)
    if n_prune:
        kernels["prune_pass"] = {"ms_per_step": round(prune_ms, 4), "passes_per_step": n_prune,
                                 "select_ms_per_step": round(prof["select"][0] / a.steps, 4),
                                 "gather_ms_per_step": round(prof["gather"][0] / a.steps, 4),
                                 "GB/s": round(by["prune"] / (prune_ms * 1e-3) / 1e9, 1),
                                 "note": "scores from the epilogue's partial sums + select + gather inside rs_block_fwd "
                                         "(tensors of 40-80 MB just written by the fc2 GEMM)"}

    # the dominant kernel by time
    dom = max(("gemm_qkv", "gemm_proj", "gemm_fc1", "gemm_fc2", "attention"), key=lambda k: prof[k][0])
    avg_s, per_step = kern(dom)
    achieved = fl[dom] / per_step / avg_s / 1e12
    # algorithmic bytes of that kernel per launch (mean over the step's launches): operands read once,
    # result written once, plus the residual read and the score partial sums where the epilogue has them
    Ms = [B * n for n, _ in sched]
    Mmean = sum(Ms) / len(Ms)
    shapes = {"gemm_qkv": (D, 3 * D, 0, 0), "gemm_proj": (D, D, 1, 0), "gemm_fc1": (D, Dm, 0, 0),
              "gemm_fc2": (Dm, D, 1, 1)}
    alg_bytes = None
    if dom in shapes:
        Kd, Nd, res, part = shapes[dom]
        alg_bytes = (Mmean * Kd + Nd * Kd + Mmean * Nd * (1 + res)) * e + part * Mmean * slots * 4.0 * n_prune / L
    elif dom == "attention":
        alg_bytes = by["attention"] / per_step
    carried = MEASURED_HBM_BYTES_PER_LAUNCH.get((a.workload, a.unpruned, dom))
    traffic = carried[0] if carried and carried[1] == rs.rs_build_info() else None
    roofline = {"kernel": dom, "bound": "mfma", "achieved": round(achieved, 2), "peak": PEAK_BF16_TFLOPS,
                "unit": "TFLOP/s", "frac": round(achieved / PEAK_BF16_TFLOPS, 4),
                "traffic": traffic,
                "algorithmic_bytes": None if alg_bytes is None else round(alg_bytes),
                "traffic_ratio": None if (traffic is None or not alg_bytes) else round(traffic / alg_bytes, 3),
                "avg_launch_us": round(avg_s * 1e6, 2), "launches_per_step": per_step,
                "whole_step_frac_of_mfma_peak": round(total_flops / (ms_per_step * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4),
                "build": rs.rs_build_info()}
    if traffic is None:
        roofline["traffic_note"] = ("no rocprofv3 FETCH_SIZE / WRITE_SIZE run is on record for this kernel under this "
                                    "build string" if not carried else
                                    "the figure on record was measured under another build string: " + carried[1])

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
        "streams": S, "gemm_variant": timed_variant,
    }
    if tuned is not None:
        out["launch_tuning"] = {"ms_per_step by (streams, gemm variant)": {"%d,%d" % k: round(v * 1e3, 4) for k, v in tuned.items()},
                                "note": "timed once before the timed region; the fastest configuration is the one timed; "
                                        "all configurations give bit-identical outputs"}
    if S > 1:
        out["roofline"]["measured_on"] = ("instrumented replay of the whole batch on one stream (a launch has the "
                                          "chip to itself); the timed steps run %d parts of the batch on %d streams" % (S, S))
    del stack
    torch.cuda.empty_cache()

    if not a.no_extras:
        # ---- the same stack without pruning, and the other BASELINE workloads (a few steps each) ----
        def side_run(name, unpruned, steps=5, warmup=2):
            _, st = build_stack(rs, si, torch, name, max(a.streams, 1), unpruned)
            if a.streams == 0:
                st.tune()
            else:
                st.gemm_variant = a.gemm_variant
            s_ = time_steps(torch, st.step, steps, warmup)
            f_ = sum(stack_flops(st).values())
            r_ = {"images_per_s": round(st.B / s_, 1), "ms_per_step": round(s_ * 1e3, 4), "steps": steps,
                  "streams": len(st.parts), "gemm_variant": st.gemm_variant,
                  "batch": st.B, "tokens_per_block": sorted(set(n for n, _ in st.sched), reverse=True),
                  "gflop_per_image": round(f_ / st.B / 1e9, 2),
                  "frac_of_mfma_peak": round(f_ / s_ / 1e12 / PEAK_BF16_TFLOPS, 4)}
            del st
            torch.cuda.empty_cache()
            return r_

        if not a.unpruned:
            u = side_run(a.workload, True)
            out["unpruned"] = dict(u, speedup_from_pruning=round(images_s / u["images_per_s"], 3))
        out["workloads"] = {n: side_run(n, False) for n in ("vit_s16", "video_vit_b16", "video_vit_l14")
                            if n != a.workload}

        # ---- the prune pass alone on an HBM-resident shape ----
        Bs, Ns, Ds, Ks = 4096, 197, 768, 177
        f_in = torch.randn((Bs, Ns, Ds), device=dev, dtype=tdt)
        f_out = f_in + 0.1 * torch.randn((Bs, Ns, Ds), device=dev, dtype=tdt)
        sc = torch.empty((Bs, Ns), device=dev, dtype=torch.float32)
        kp = torch.empty((Bs, 1 + Ks), device=dev, dtype=torch.int32)
        g = torch.empty((Bs, 1 + Ks, Ds), device=dev, dtype=tdt)
        ts = time_steps(torch, lambda: rs.rs_shift_topk(f_out, f_in, None, 1, Ks, sc, kp, g), 10, 3)
        alg = Bs * (2.0 * Ns * Ds * e + 8.0 * Ns + 4.0 * (1 + Ks) + (1 + Ks) * Ds * e)
        alg_reread = alg + Bs * (1.0 + Ks) * Ds * e
        out["prune_stress"] = {"shape": [Bs, Ns, Ds, Ks], "ms": round(ts * 1e3, 4),
                               "GB/s": round(alg / ts / 1e9, 1), "frac_hbm": round(alg / ts / 1e9 / PEAK_HBM_GBS, 4),
                               "GB/s_incl_gather_read": round(alg_reread / ts / 1e9, 1),
                               "note": "GB/s counts every tensor once (read f_out, f_in; write scores, kept_idx, gathered "
                                       "rows); _incl_gather_read adds a second read of the kept rows, which the one-pass "
                                       "kernel used for this shape does not perform (they stay in registers)"}
        # the same pass when the rows to gather come from a third tensor (three launches: score, select, gather)
        src3 = torch.randn((Bs, Ns, Ds), device=dev, dtype=tdt)
        t3 = time_steps(torch, lambda: rs.rs_shift_topk(f_out, f_in, src3, 1, Ks, sc, kp, g), 10, 3)
        out["prune_stress_three_launch"] = {"ms": round(t3 * 1e3, 4), "GB/s": round(alg_reread / t3 / 1e9, 1),
                                            "frac_hbm": round(alg_reread / t3 / 1e9 / PEAK_HBM_GBS, 4),
                                            "note": "rows gathered from a separate tensor: its read is algorithmic here"}
        del f_in, f_out, g, src3
        # ---- fused attention alone at the long-sequence video shape ----
        Ba, Na, Ha = 4, 4097, 16
        qkv = torch.randn((Ba, Na, 3, Ha, 64), device=dev, dtype=tdt)
        oa = torch.empty((Ba, Na, Ha, 64), device=dev, dtype=tdt)
        ta = time_steps(torch, lambda: rs.rs_attention_fwd(qkv[:, :, 0], qkv[:, :, 1], qkv[:, :, 2], oa, 0.125), 20, 3)
        fa = 4.0 * Ba * Ha * Na * Na * 64
        out["attention_long"] = {"shape": [Ba, Na, Ha, 64], "us": round(ta * 1e6, 1),
                                 "TFLOP/s": round(fa / ta / 1e12, 1), "frac_mfma": round(fa / ta / 1e12 / PEAK_BF16_TFLOPS, 4)}
        del qkv, oa
        # ---- and at the image shape (batch 256 x 197 tokens x 12 heads: HBM-bound) ----
        Bi, Ni, Hi = 256, 197, 12
        qkv = torch.randn((Bi, Ni, 3, Hi, 64), device=dev, dtype=tdt)
        oa = torch.empty((Bi, Ni, Hi, 64), device=dev, dtype=tdt)
        ti = time_steps(torch, lambda: rs.rs_attention_fwd(qkv[:, :, 0], qkv[:, :, 1], qkv[:, :, 2], oa, 0.125), 20, 3)
        bi = 4.0 * Bi * Ni * Hi * 64 * e
        out["attention_short"] = {"shape": [Bi, Ni, Hi, 64], "us": round(ti * 1e6, 1), "GB/s": round(bi / ti / 1e9, 1),
                                  "frac_hbm": round(bi / ti / 1e9 / PEAK_HBM_GBS, 4),
                                  "frac_mfma": round(4.0 * Bi * Hi * Ni * Ni * 64 / ti / 1e12 / PEAK_BF16_TFLOPS, 4)}
        del qkv, oa

    if not a.no_extras:
        # ---- context: standard attention with the map written out (rs_attention_map_fwd) against the fused kernel,
        # and the cost of the attention-based scores against the representation-shift score of the block ----
        cmp_ = {}
        for tag, (Bc, Nc, Hc) in {"image_256x197x12": (256, 197, 12), "video_8x1569x12": (8, 1569, 12)}.items():
            qkv = torch.randn((Bc, Nc, 3, Hc, 64), device=dev, dtype=tdt)
            oa = torch.empty((Bc, Nc, Hc, 64), device=dev, dtype=tdt)
            amap = torch.empty(rs.rs_attention_map_size(Bc, Hc, Nc), dtype=torch.uint8, device=dev)
            wsa = torch.empty(rs.rs_attention_map_workspace_size(Bc, Hc, Nc), dtype=torch.uint8, device=dev)
            sm = torch.empty((Bc, Nc), device=dev, dtype=torch.float32)
            t_f = time_steps(torch, lambda: rs.rs_attention_fwd(qkv[:, :, 0], qkv[:, :, 1], qkv[:, :, 2], oa, 0.125), 10, 2)
            t_u = time_steps(torch, lambda: rs.rs_attention_map_fwd(qkv[:, :, 0], qkv[:, :, 1], qkv[:, :, 2], oa, 0.125,
                                                                    amap, None, None, wsa), 10, 2)
            t_s = time_steps(torch, lambda: rs.rs_attention_map_fwd(qkv[:, :, 0], qkv[:, :, 1], qkv[:, :, 2], oa, 0.125,
                                                                    amap, sm, sm, wsa), 10, 2)
            cmp_[tag] = {"fused_us": round(t_f * 1e6, 1), "map_written_us": round(t_u * 1e6, 1),
                         "map_written_with_scores_us": round(t_s * 1e6, 1), "fused_speedup": round(t_u / t_f, 2),
                         "map_MB": round(amap.numel() / 1e6, 1)}
            del qkv, oa, amap, wsa
        out["attention_fused_vs_map_written"] = dict(cmp_, note="context only (Sec. 3.1, Table 1): the comparison system "
                                                     "with Eq. (2)/(3) scores; the representation-shift score costs no pass "
                                                     "of its own (it falls out of the fc2 epilogue)")

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
        op = {"mlp": 0, "attn": 1, "block": 2}[wl.get("op", "mlp")]   # the op codes are the same on both sides
        t0 = time.perf_counter()
        for l, (n_in, n_keep) in enumerate(sched):
            r = oracle.block_pruned(xs, wts[l], H, P, n_keep, op=op)
            xs = r["y"]
        tc = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": round(ns / tc, 3), "unit": "images/s", "cores": oracle.num_threads(),
                               "kind": "oracle",
                               "sample": "%d of %d images, all %d blocks, same schedule, fp64, gcc -O2 -fopenmp, %.1f s"
                                         % (ns, B, L, tc)}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
