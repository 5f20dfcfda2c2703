"""GPU parity, part 2: the linear-layer entry point, and full-size checks in the launch
configuration bench.py times (sampled outputs the fp64 checker can compute one by one)."""
import math
import sys

import numpy as np
import pytest
import torch

import oracle
import paper_2508_00367_amd as rs
import synth_inputs as si
from rs_testlib import TOL, check_kept_admissible, host_round, norm_err, to_dev, to_host

pytestmark = pytest.mark.gpu


def _say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def _gelu64(x):
    return oracle.gelu(x)


LIN_SHAPES = [(1, 64, 64), (37, 128, 192), (300, 256, 64), (513, 384, 1152), (1000, 768, 768),
              (259, 192, 768), (64, 1024, 320)]


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("epi", [rs.RS_EPI_BIAS, rs.RS_EPI_BIAS_GELU, rs.RS_EPI_BIAS_RES])
@pytest.mark.parametrize("M,K,N", LIN_SHAPES)
def test_linear(dtype, epi, M, K, N):
    """out = epilogue(a W + b) against the checker's linear (ascending-k fp64 sums), ragged M,
    K from one to 16 slices, N below and above one tile."""
    _say("linear", dtype, epi, M, K, N)
    a = host_round(si.generic(3, 30, (M, K)), dtype)
    w = host_round(si.generic(3, 31, (K, N), std=0.05), dtype)
    b = host_round(si.generic(3, 32, (N,), std=0.5), dtype)
    res = host_round(si.generic(3, 33, (M, N)), dtype)
    ref = oracle.linear(a, w, b)
    if epi == rs.RS_EPI_BIAS_GELU:
        ref = _gelu64(ref)
    elif epi == rs.RS_EPI_BIAS_RES:
        ref = ref + res
    da, dw, db, dres = (to_dev(t, dtype) for t in (a, w, b, res))
    wt = torch.empty((N, K), device="cuda", dtype=da.dtype) if dtype == "bf16" else dw
    if dtype == "bf16":
        rs.rs_pack_linear(dw, wt)
    out = torch.full((M, N), float("nan"), device="cuda", dtype=da.dtype)
    rs.rs_linear_fwd(da, wt, db, dres if epi == rs.RS_EPI_BIAS_RES else None, out, epi)
    torch.cuda.synchronize()
    err = norm_err(to_host(out), ref)
    _say("  err %.3e" % err)
    assert err < (5e-3 if dtype == "bf16" else 1e-5)


def test_linear_without_bias_and_empty():
    M, K, N = 70, 128, 128
    a = host_round(si.generic(4, 30, (M, K)), "bf16")
    w = host_round(si.generic(4, 31, (K, N), std=0.05), "bf16")
    da, dw = to_dev(a, "bf16"), to_dev(w, "bf16")
    wt = torch.empty((N, K), device="cuda", dtype=torch.bfloat16)
    rs.rs_pack_linear(dw, wt)
    out = torch.empty((M, N), device="cuda", dtype=torch.bfloat16)
    rs.rs_linear_fwd(da, wt, None, None, out, rs.RS_EPI_BIAS)
    torch.cuda.synchronize()
    assert norm_err(to_host(out), oracle.linear(a, w)) < 5e-3
    rs.rs_linear_fwd(da[:0], wt, None, None, out[:0], rs.RS_EPI_BIAS)  # M = 0: no launch


def test_fullsize_vit_b_block_sampled_images():
    """The bench workload's first pruning block at full size (batch 256, 197 tokens, D 768, 12
    heads, MLP 3072, keep 177 of 196), packed weights, scores not requested (as bench.py calls
    it): the checker recomputes a sample of the images; the others are covered by invariants."""
    wl = si.WORKLOADS["vit_b16"]
    B, N, D, H, Dm = wl["B"], wl["N"], wl["D"], wl["H"], wl["Dm"]
    n_keep = rs.keep_counts(N, 1, wl["blocks"], wl["prune"])[3][1]
    assert n_keep == 177
    x = host_round(si.tokens(0, B, N, D), "bf16")
    w = {k: host_round(v, "bf16") for k, v in si.block_weights(0, 3, D, Dm).items()}
    dw = {k: to_dev(v, "bf16") for k, v in w.items()}
    dx = to_dev(x, "bf16")
    cfg = rs.make_cfg(B, N, D, H, Dm, 1, n_keep, torch.bfloat16)
    packed = torch.empty(rs.rs_packed_weights_size(cfg), dtype=torch.uint8, device="cuda")
    rs.rs_pack_weights(cfg, rs.make_weights(dw), packed)
    ws = torch.empty(rs.rs_block_workspace_size(cfg), dtype=torch.uint8, device="cuda")
    y = torch.full((B, 1 + n_keep, D), float("nan"), device="cuda", dtype=torch.bfloat16)
    kept = torch.full((B, 1 + n_keep), -1, device="cuda", dtype=torch.int32)
    rs.rs_block_fwd(cfg, rs.make_weights(dw, packed), dx, y, kept, None, ws)
    # second run with scores, to check the selection on them
    scores = torch.empty((B, N), device="cuda", dtype=torch.float32)
    y2 = torch.empty_like(y)
    kept2 = torch.empty_like(kept)
    rs.rs_block_fwd(cfg, rs.make_weights(dw, packed), dx, y2, kept2, scores, ws)
    torch.cuda.synchronize()
    assert torch.equal(y, y2) and torch.equal(kept, kept2)          # bit-reproducible
    kept_h, s = kept.cpu().numpy(), to_host(scores)
    # properties that hold for every image
    assert np.isfinite(to_host(y)).all() and np.isfinite(s).all()
    assert (kept_h[:, 0] == 0).all() and (np.diff(kept_h, axis=1) > 0).all() and kept_h.max() < N
    np.testing.assert_array_equal(kept_h, oracle.topk(s, 1, n_keep))   # exact on the GPU's scores
    # sampled images against the checker
    sample = [0, 1, 97, 255]
    ref = oracle.block(x[sample], w, H)
    assert norm_err(s[sample], ref["scores"]) < TOL["bf16"]
    exact = check_kept_admissible(kept_h[sample], s[sample], ref["scores"], 1, n_keep)
    e_y = norm_err(to_host(y)[sample], oracle.gather(ref["xhat"], kept_h[sample]))
    _say("  full-size block: y err %.3e, kept exact on %.0f%% of sampled images" % (e_y, 100 * exact))
    assert e_y < TOL["bf16"]


@pytest.mark.parametrize("name,block,sample", [("video_vit_b16", 2, [0, 7]), ("video_vit_l14", 4, [3]),
                                               ("umt_b_ret", 1, [19]), ("umt_b_ret", 3, [4]), ("umt_b_qa", 3, [11]),
                                               ("deit_t", 1, [0, 300, 511])])
def test_fullsize_video_block_sampled_clips(name, block, sample):
    """Pruning blocks of the video workloads at full size, with the sequence length the block sees
    in the schedule (8 x 1569 x 768 keep half; 4 x 4097 x 1024 keep 70 %; 20 x 2352 x 768 without
    class token keep 80 %; the third UMT blocks at 1506 -> 1205 and 1906 -> 1716 tokens), and the
    narrowest image model (512 x 197 x 192): long-sequence attention plans, LayerNorm-folded GEMMs
    and the prune pass together.  The checker recomputes the sampled clips; invariants cover the rest."""
    wl = si.WORKLOADS[name]
    B, D, H, Dm, P = wl["B"], wl["D"], wl["H"], wl["Dm"], wl.get("n_prefix", 1)
    n_in, n_keep = rs.keep_counts(wl["N"], P, wl["blocks"], wl["prune"])[block - 1]
    N = n_in
    assert n_keep < N - P
    _say("full-size block", name, B, N, D, "keep", n_keep)
    x = host_round(si.tokens(0, B, N, D, 0.3), "bf16")
    w = {k: host_round(v, "bf16") for k, v in si.block_weights(0, block - 1, D, Dm).items()}
    dw = {k: to_dev(v, "bf16") for k, v in w.items()}
    dx = to_dev(x, "bf16")
    cfg = rs.make_cfg(B, N, D, H, Dm, P, n_keep, torch.bfloat16)
    packed = torch.empty(rs.rs_packed_weights_size(cfg), dtype=torch.uint8, device="cuda")
    rs.rs_pack_weights(cfg, rs.make_weights(dw), packed)
    ws = torch.empty(rs.rs_block_workspace_size(cfg), dtype=torch.uint8, device="cuda")
    y = torch.full((B, P + n_keep, D), float("nan"), device="cuda", dtype=torch.bfloat16)
    kept = torch.full((B, P + n_keep), -1, device="cuda", dtype=torch.int32)
    scores = torch.empty((B, N), device="cuda", dtype=torch.float32)
    rs.rs_block_fwd(cfg, rs.make_weights(dw, packed), dx, y, kept, scores, ws)
    torch.cuda.synchronize()
    kept_h, s = kept.cpu().numpy(), to_host(scores)
    assert np.isfinite(to_host(y)).all() and np.isfinite(s).all()
    assert (np.diff(kept_h, axis=1) > 0).all() and kept_h.max() < N and kept_h.min() >= 0
    if P:
        assert (kept_h[:, 0] == 0).all()
    np.testing.assert_array_equal(kept_h, oracle.topk(s, P, n_keep))   # exact on the GPU's scores
    ref = oracle.block(x[sample], w, H)
    e_s = norm_err(s[sample], ref["scores"])
    exact = check_kept_admissible(kept_h[sample], s[sample], ref["scores"], P, n_keep)
    e_y = norm_err(to_host(y)[sample], oracle.gather(ref["xhat"], kept_h[sample]))
    _say("  score err %.3e, y err %.3e, kept exact on %.0f%% of sampled clips" % (e_s, e_y, 100 * exact))
    assert e_s < TOL["bf16"] and e_y < TOL["bf16"]


@pytest.mark.parametrize("B,N,H", [(4, 4097, 16), (8, 1569, 12)])
def test_fullsize_video_attention_sampled_rows(B, N, H):
    """Joint space-time attention at the video workloads' sizes: the checker recomputes sampled
    (image, head) pairs in full; every output row must be finite and inside the hull of V."""
    qkv = host_round(si.generic(5, 1, (B, N, 3, H, 64)), "bf16")
    d = to_dev(qkv, "bf16")
    o = torch.full((B, N, H, 64), float("nan"), device="cuda", dtype=torch.bfloat16)
    rs.rs_attention_fwd(d[:, :, 0], d[:, :, 1], d[:, :, 2], o, 0.125)
    torch.cuda.synchronize()
    got = to_host(o)
    assert np.isfinite(got).all()
    v = qkv[:, :, 2].astype(np.float64)
    assert (got <= v.max(axis=1, keepdims=True) + 1e-2).all() and (got >= v.min(axis=1, keepdims=True) - 1e-2).all()
    for (b, h) in [(0, 0), (B - 1, H - 1)]:
        sl = qkv[b:b + 1, :, :, h:h + 1]
        ref = oracle.attention(sl[:, :, 0], sl[:, :, 1], sl[:, :, 2], 0.125)
        err = norm_err(got[b:b + 1, :, h:h + 1], ref)
        _say("  attention N=%d (b=%d,h=%d) err %.3e" % (N, b, h, err))
        assert err < TOL["bf16"]
