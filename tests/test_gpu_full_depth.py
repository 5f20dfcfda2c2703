"""GPU parity, part 3: whole forwards of the BASELINE workloads in the very configuration bench.py
times (paper_2508_00367_amd.EncoderStack: packed weights, ping-pong buffers, one shared kept_idx
buffer, the batch as two parts on two HIP streams), checked block by block against the fp64 checker
in teacher-forced mode: the checker recomputes each checked block from the GPU's own block input
and is compared on the GPU's kept set (kept sets may differ legitimately inside the rounding band,
after which the two forwards would no longer see the same tokens).

With RS_PARITY_OUT=<folder> in the environment every check appends one JSON line of statistics to
<folder>/parity_summary.jsonl: score / output errors, per-element relative error with a floor, whether kept_idx
matched exactly, how many tokens differ, and the width of the admissible band (2 tau) relative to
the median gap between neighbouring scores."""
import json
import os
import sys

import numpy as np
import pytest
import torch

import oracle
import paper_2508_00367_amd as rs
import synth_inputs as si
from rs_testlib import TOL, check_kept_admissible, host_round, norm_err, rel_err_floor, to_dev, to_host

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def _record(rec):
    d = os.environ.get("RS_PARITY_OUT")
    if not d:
        return
    d = d if os.path.isabs(d) else os.path.join(ROOT, d)
    try:
        os.makedirs(d, exist_ok=True)
        with open(os.path.join(d, "parity_summary.jsonl"), "a") as f:
            f.write(json.dumps(rec) + "\n")
    except OSError:
        pass


def _forward_checked(name, check_blocks, sample, streams=2):
    """Runs the stack once with scores written per block, copying the sampled images' block inputs,
    outputs, kept indices and scores to the host after every checked block; then once more exactly as
    bench.py does (no scores) and checks that the final outputs agree bit for bit."""
    wl = dict(si.WORKLOADS[name])
    B, N, D, H, Dm, L = wl["B"], wl["N"], wl["D"], wl["H"], wl["Dm"], wl["blocks"]
    x0 = to_dev(host_round(si.tokens(0, B, N, D), "bf16"), "bf16")
    w_host = [{k: host_round(v, "bf16") for k, v in si.block_weights(0, l, D, Dm).items()} for l in range(L)]
    w_dev = [{k: to_dev(v, "bf16") for k, v in w.items()} for w in w_host]
    stack = rs.EncoderStack(wl, x0, w_dev, streams=streams)
    P, sched = stack.P, stack.sched
    scores = [torch.empty((p["B"], N), device="cuda", dtype=torch.float32) for p in stack.parts]
    seen = {}

    def capture(l, part, src, dst):
        if (l + 1) not in check_blocks:
            return
        n_in, n_keep = sched[l]
        K = P + n_keep
        for b in sample:
            lb = b - part["first"]
            if not (0 <= lb < part["B"]):
                continue
            (part["stream"] or torch.cuda.current_stream()).synchronize()
            i = stack.parts.index(part)
            seen[(l + 1, b)] = dict(
                x=to_host(src.view(-1)[:part["B"] * n_in * D].view(part["B"], n_in, D)[lb]),
                y=to_host(dst.view(-1)[:part["B"] * K * D].view(part["B"], K, D)[lb]),
                kept=part["kept"].view(-1)[:part["B"] * K].view(part["B"], K)[lb].cpu().numpy(),
                s=to_host(scores[i].view(-1)[:part["B"] * n_in].view(part["B"], n_in)[lb]))

    outs = stack.step(capture=capture, scores=scores)
    torch.cuda.synchronize()
    final = [o.clone() for o in outs]
    outs2 = stack.step()                      # bench.py's call: no scores, nothing between the blocks
    torch.cuda.synchronize()
    for o, f in zip(outs2, final):
        assert torch.equal(o.view(torch.int16), f.view(torch.int16))
        assert torch.isfinite(o.float()).all()

    op = {"mlp": oracle.OP_MLP, "attn": oracle.OP_ATTN, "block": oracle.OP_BLOCK}[wl.get("op", "mlp")]
    for (blk, b), g in sorted(seen.items()):
        n_in, n_keep = sched[blk - 1]
        ref = oracle.block(g["x"][None], w_host[blk - 1], H, op=op)
        s_ref, s = ref["scores"], g["s"][None]
        kept = g["kept"][None]
        e_s = norm_err(s, s_ref)
        y_ref = oracle.gather(ref["xhat"], kept)
        e_y = norm_err(g["y"][None], y_ref)
        e_rel = rel_err_floor(g["y"][None], y_ref)
        np.testing.assert_array_equal(kept, oracle.topk(s, P, n_keep))       # exact on the GPU's own scores
        exact = check_kept_admissible(kept, s, s_ref, P, n_keep) if n_keep > 0 else 1.0
        kept_ref = oracle.topk(s_ref, P, n_keep)
        n_diff = len(set(kept[0].tolist()) ^ set(kept_ref[0].tolist())) // 2
        tau = float(np.abs(s - s_ref).max())
        cand = np.sort(s_ref[0, P:])
        gap = float(np.median(np.diff(cand))) if cand.size > 1 else 0.0
        rec = dict(workload=name, block=blk, image=b, tokens_in=n_in, kept=P + n_keep, streams=streams,
                   score_err=e_s, y_err=e_y, y_rel_err_floored=e_rel, kept_exact=bool(exact == 1.0),
                   tokens_differing=n_diff, tau=tau, band_2tau_over_median_gap=(2 * tau / gap if gap > 0 else None))
        _record(rec)
        _say("  %s block %d image %d: N %d -> %d, score err %.2e, y err %.2e (rel/floor %.2e), kept %s (%d differ), "
             "2tau/gap %.2f" % (name, blk, b, n_in, P + n_keep, e_s, e_y, e_rel, "exact" if exact == 1.0 else "in band",
                                n_diff, rec["band_2tau_over_median_gap"] or 0.0))
        assert e_s < TOL["bf16"] and e_y < TOL["bf16"]
    return seen


def test_full_depth_vit_b16_two_streams():
    """BASELINE config 3: 256 images, 12 blocks, 10 % of the patch tokens dropped after blocks 4-11;
    four images (two per stream part) checked at every block."""
    seen = _forward_checked("vit_b16", set(range(1, 13)), [0, 127, 128, 255])
    assert len(seen) == 48


def test_full_depth_vit_s16_two_streams():
    """BASELINE config 2: 64 images, 12 blocks, 16 tokens dropped after blocks 1-11 (197 -> 21)."""
    seen = _forward_checked("vit_s16", set(range(1, 13)), [0, 31, 32, 63])
    assert len(seen) == 48


def test_full_depth_video_vit_b16():
    """BASELINE config 4: 8 clips of 1569 tokens, half dropped after blocks 2, 5, 8: one clip at every
    sequence length of the schedule (1569, 785, 393, 197)."""
    _forward_checked("video_vit_b16", {2, 5, 8, 12}, [5])


def test_full_depth_video_vit_l14():
    """BASELINE config 5: 4 clips of 4097 tokens, 24 blocks, 30 % dropped after blocks 4, 8, 12, 16:
    one clip at every sequence length of the schedule (4097, 2869, 2009, 1407, 986)."""
    _forward_checked("video_vit_l14", {4, 8, 12, 16, 24}, [2])
