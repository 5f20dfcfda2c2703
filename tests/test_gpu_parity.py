"""GPU parity: the HIP path (through the C ABI) against the fp64 CPU checker, element by
element, on the same seeded inputs.  Tolerances: tensor-normalised max error 1e-4 (fp32),
2e-2 (bf16); indices bit-exact, with the tie-band rule where scores differ by rounding."""
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


# ----------------------------------------------------------------------------
# fused attention
# ----------------------------------------------------------------------------
ATT_SHAPES = [(1, 1, 1), (1, 2, 1), (2, 17, 3), (1, 64, 2), (1, 65, 1), (2, 197, 3), (1, 198, 2),
              (1, 300, 2), (1, 1569, 1)]


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("B,N,H", ATT_SHAPES)
def test_attention_packed_qkv(dtype, B, N, H):
    """q, k, v as strided views of one [B, N, 3, H, 64] buffer (the block's layout)."""
    _say("attention", dtype, B, N, H)
    qkv = host_round(si.generic(0, 1, (B, N, 3, H, 64)), dtype)
    scale = 0.125
    ref = oracle.attention(qkv[:, :, 0], qkv[:, :, 1], qkv[:, :, 2], scale)
    d = to_dev(qkv, dtype)
    o = torch.full((B, N, H, 64), float("nan"), device="cuda", dtype=d.dtype)
    rs.rs_attention_fwd(d[:, :, 0], d[:, :, 1], d[:, :, 2], o, scale)
    torch.cuda.synchronize()
    err = norm_err(to_host(o), ref)
    _say("  err", err)
    assert err < TOL[dtype]


# (B, N, H) chosen so that the launcher takes each of its long-sequence plans (a round is 512
# workgroups of 256 rows): every row in the tiled kernel, the last workgroup of a head holding one
# row and seven idle waves (128 heads x 3 tiles fit one round); the one row beyond the last full
# tile in the tail kernel (128 x 5 tiles would start a second round); 36 tail rows with a padded
# last key tile; no rows left over.
@pytest.mark.parametrize("B,N,H", [(8, 513, 16), (8, 1025, 16), (8, 1060, 16), (8, 1024, 12)])
def test_attention_long_sequence_plans(B, N, H):
    _say("attention plans", B, N, H)
    qkv = host_round(si.generic(7, 1, (B, N, 3, H, 64)), "bf16")
    ref = oracle.attention(qkv[:, :, 0], qkv[:, :, 1], qkv[:, :, 2], 0.125)
    d = to_dev(qkv, "bf16")
    o = torch.full((B, N, H, 64), float("nan"), device="cuda", dtype=torch.bfloat16)
    rs.rs_attention_fwd(d[:, :, 0], d[:, :, 1], d[:, :, 2], o, 0.125)
    torch.cuda.synchronize()
    got = to_host(o)
    assert np.isfinite(got).all()
    err = norm_err(got, ref)
    err_tail = norm_err(got[:, -40:], ref[:, -40:])
    _say("  err %.3e, last 40 rows %.3e" % (err, err_tail))
    assert err < TOL["bf16"] and err_tail < TOL["bf16"]
    again = torch.empty_like(o)
    rs.rs_attention_fwd(d[:, :, 0], d[:, :, 1], d[:, :, 2], again, 0.125)
    torch.cuda.synchronize()
    assert torch.equal(o.view(torch.int16), again.view(torch.int16))  # merge order is fixed


# The short-sequence kernel copies up to four key tiles of 64 into LDS and starts on the first two
# while the others are still in flight: every tile count, full and padded last tiles, the idle
# eighth wave (N <= 224), and enough (image, head) pairs that workgroups share CUs.
@pytest.mark.parametrize("N", [31, 63, 64, 65, 127, 128, 129, 161, 192, 193, 224, 225, 255, 256, 257])
def test_attention_short_sequence_tile_boundaries(N):
    B, H = 48, 12
    _say("attention short", B, N, H)
    qkv = host_round(si.generic(11, 1, (B, N, 3, H, 64)), "bf16")
    d = to_dev(qkv, "bf16")
    o = torch.full((B, N, H, 64), float("nan"), device="cuda", dtype=torch.bfloat16)
    rs.rs_attention_fwd(d[:, :, 0], d[:, :, 1], d[:, :, 2], o, 0.125)
    torch.cuda.synchronize()
    got = to_host(o)
    assert np.isfinite(got).all()
    for b in (0, 17, B - 1):   # the oracle on three of the images, the rest by repetition below
        ref = oracle.attention(qkv[b:b + 1, :, 0], qkv[b:b + 1, :, 1], qkv[b:b + 1, :, 2], 0.125)
        err = norm_err(got[b:b + 1], ref)
        _say("  image %d err %.3e" % (b, err))
        assert err < TOL["bf16"]
    # images with equal inputs give equal bits wherever they ran
    d2 = d.clone()
    d2[1:] = d[:1]
    o2 = torch.empty_like(o)
    rs.rs_attention_fwd(d2[:, :, 0], d2[:, :, 1], d2[:, :, 2], o2, 0.125)
    torch.cuda.synchronize()
    assert torch.equal(o2[0].view(torch.int16), o[0].view(torch.int16))
    assert all(torch.equal(o2[b].view(torch.int16), o2[0].view(torch.int16)) for b in range(1, B))


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_attention_large_logits_and_separate_tensors(dtype):
    B, N, H = 1, 130, 2
    q = host_round(si.generic(1, 2, (B, N, H, 64), std=6.0), dtype)
    k = host_round(si.generic(1, 3, (B, N, H, 64), std=6.0), dtype)
    v = host_round(si.generic(1, 4, (B, N, H, 64)), dtype)
    scale = 1.0 / math.sqrt(64.0)
    ref = oracle.attention(q, k, v, scale)
    o = torch.empty((B, N, H, 64), device="cuda", dtype=to_dev(q, dtype).dtype)
    rs.rs_attention_fwd(to_dev(q, dtype), to_dev(k, dtype), to_dev(v, dtype), o, scale)
    torch.cuda.synchronize()
    got = to_host(o)
    assert np.isfinite(got).all()
    assert norm_err(got, ref) < TOL[dtype]


@pytest.mark.parametrize("N", [65, 197, 300, 1060])
def test_attention_rows_behind_the_last_key_are_never_used(N):
    """The bf16 kernels copy whole 64-key tiles and rely on rows past N arriving as zeros (a padded V
    row holding NaN or Inf would poison the output through 0 x NaN).  Here q, k, v are the first N
    tokens of a longer NaN-filled allocation, for the last image too, so a bound that is off by a
    row shows up as a non-finite output."""
    B, H, PAD = 3, 4, 80
    _say("attention nan-padded", N)
    qkv = host_round(si.generic(13, 1, (B, N, 3, H, 64)), "bf16")
    big = torch.full((B, N + PAD, 3, H, 64), float("nan"), device="cuda", dtype=torch.bfloat16)
    big[:, :N] = to_dev(qkv, "bf16")
    o = torch.full((B, N, H, 64), float("nan"), device="cuda", dtype=torch.bfloat16)
    d = big[:, :N]
    rs.rs_attention_fwd(d[:, :, 0], d[:, :, 1], d[:, :, 2], o, 0.125)
    torch.cuda.synchronize()
    got = to_host(o)
    assert np.isfinite(got).all()
    ref = oracle.attention(qkv[:, :, 0], qkv[:, :, 1], qkv[:, :, 2], 0.125)
    assert norm_err(got, ref) < TOL["bf16"]


@pytest.mark.parametrize("N", [65, 197, 300])
def test_block_with_poisoned_workspace(N):
    """The workspace arrives full of 0xFF bytes (NaN in every float format): every scratch tensor
    must be written before it is read, and rows past the last token of the last image (which, in
    the packed QKV buffer, are whatever the workspace held) must not reach any output."""
    B, D, H, Dm, P, K = 2, 128, 2, 256, 1, N // 2
    _say("block poisoned workspace", N)
    x, w = _block_inputs(14, B, N, D, Dm, "bf16", std=0.05, spread=0.3)
    dw = {k: to_dev(v, "bf16") for k, v in w.items()}
    dx = to_dev(x, "bf16")
    cfg = rs.make_cfg(B, N, D, H, Dm, P, K, torch.bfloat16)
    ws = torch.full((rs.rs_block_workspace_size(cfg) + 4096,), 0xFF, dtype=torch.uint8, device="cuda")
    y = torch.full((B, P + K, D), float("nan"), device="cuda", dtype=torch.bfloat16)
    kept = torch.full((B, P + K), -1, device="cuda", dtype=torch.int32)
    scores = torch.full((B, N), float("nan"), device="cuda", dtype=torch.float32)
    rs.rs_block_fwd(cfg, rs.make_weights(dw), dx, y, kept, scores, ws)
    torch.cuda.synchronize()
    assert (ws[-4096:] == 0xFF).all()                      # nothing written past the stated size
    ref = oracle.block(x, w, H)
    s, kept_h = to_host(scores), kept.cpu().numpy()
    assert np.isfinite(s).all() and np.isfinite(to_host(y)).all()
    assert norm_err(s, ref["scores"]) < TOL["bf16"]
    check_kept_admissible(kept_h, s, ref["scores"], P, K)
    assert norm_err(to_host(y), oracle.gather(ref["xhat"], kept_h)) < TOL["bf16"]


@pytest.mark.parametrize("B,N,H,cls", [(2, 17, 3, 0), (1, 64, 2, 5), (2, 197, 3, 0), (1, 300, 2, 299), (1, 1060, 1, 0)])
def test_attention_map_and_attention_scores(B, N, H, cls):
    """The comparison system of Sec. 3.1: attention with the map written to memory, and the
    importance scores of Eqs. (2), (3) taken from it, against the checker; its output must also
    agree with the fused kernel's."""
    _say("attention map", B, N, H, cls)
    qkv = host_round(si.generic(15, 1, (B, N, 3, H, 64)), "bf16")
    o_ref, A_ref = oracle.attention_map(qkv[:, :, 0], qkv[:, :, 1], qkv[:, :, 2], 0.125)
    s_cls_ref, s_mean_ref = oracle.attention_scores(A_ref, cls)
    d = to_dev(qkv, "bf16")
    Np = (N + 63) // 64 * 64
    o = torch.full((B, N, H, 64), float("nan"), device="cuda", dtype=torch.bfloat16)
    amap = torch.full((B, H, N, Np), float("nan"), device="cuda", dtype=torch.bfloat16)
    assert amap.numel() * 2 == rs.rs_attention_map_size(B, H, N)
    s_cls = torch.full((B, N), float("nan"), device="cuda", dtype=torch.float32)
    s_mean = torch.full((B, N), float("nan"), device="cuda", dtype=torch.float32)
    ws = torch.full((rs.rs_attention_map_workspace_size(B, H, N),), 0xFF, dtype=torch.uint8, device="cuda")
    rs.rs_attention_map_fwd(d[:, :, 0], d[:, :, 1], d[:, :, 2], o, 0.125, amap, s_cls, s_mean, ws, cls_index=cls)
    o_fused = torch.empty_like(o)
    rs.rs_attention_fwd(d[:, :, 0], d[:, :, 1], d[:, :, 2], o_fused, 0.125)
    torch.cuda.synchronize()
    A = to_host(amap)
    assert np.isfinite(A).all() and (A[..., N:] == 0).all()
    e_map = np.abs(A[..., :N] - A_ref).max() / A_ref.max()
    e_o, e_f = norm_err(to_host(o), o_ref), norm_err(to_host(o_fused), o_ref)
    e_c, e_m = norm_err(to_host(s_cls), s_cls_ref), norm_err(to_host(s_mean), s_mean_ref)
    _say("  map err %.2e, o err %.2e (fused %.2e), s_cls err %.2e, s_mean err %.2e" % (e_map, e_o, e_f, e_c, e_m))
    assert e_map < TOL["bf16"] and e_o < TOL["bf16"] and e_c < TOL["bf16"] and e_m < TOL["bf16"]
    # the scores are the stated sums of the map the GPU wrote (fp32 sums of bf16 entries)
    np.testing.assert_allclose(to_host(s_cls), A[:, :, cls, :N].mean(1), rtol=1e-5, atol=1e-8)
    np.testing.assert_allclose(to_host(s_mean), A[..., :N].mean(axis=(1, 2)), rtol=1e-4, atol=1e-8)
    # a selection by either score is exact on the GPU's scores (the prune pass takes any score vector)
    kept = oracle.topk(to_host(s_mean), 1, N // 2)
    check_kept_admissible(kept, to_host(s_mean), s_mean_ref, 1, N // 2)


def test_attention_closed_forms_on_gpu():
    # identical keys -> mean of V; V = 1 -> 1
    B, N, H = 1, 100, 1
    q = host_round(si.generic(2, 5, (B, N, H, 64)), "bf16")
    k = np.broadcast_to(host_round(si.generic(2, 6, (B, 1, H, 64)), "bf16"), q.shape).copy()
    v = host_round(si.generic(2, 7, (B, N, H, 64)), "bf16")
    o = torch.empty((B, N, H, 64), device="cuda", dtype=torch.bfloat16)
    rs.rs_attention_fwd(to_dev(q, "bf16"), to_dev(k, "bf16"), to_dev(v, "bf16"), o, 0.125)
    torch.cuda.synchronize()
    assert norm_err(to_host(o), np.broadcast_to(v.astype(np.float64).mean(1, keepdims=True), v.shape)) < 1e-2
    ones = torch.ones((B, N, H, 64), device="cuda", dtype=torch.bfloat16)
    rs.rs_attention_fwd(to_dev(q, "bf16"), to_dev(k, "bf16"), ones, o, 0.125)
    torch.cuda.synchronize()
    assert np.abs(to_host(o) - 1.0).max() < 1e-2


# ----------------------------------------------------------------------------
# shift score + selection + gather
# ----------------------------------------------------------------------------
def _run_shift_topk(f_out, f_in, src, P, K, dist, dtype):
    B, N, D = f_in.shape
    d_out, d_in = to_dev(f_out, dtype), to_dev(f_in, dtype)
    d_src = None if src is None else to_dev(src, dtype)
    scores = torch.full((B, N), float("nan"), device="cuda", dtype=torch.float32)
    kept = torch.full((B, P + K), -1, device="cuda", dtype=torch.int32)
    gathered = torch.full((B, P + K, D), float("nan"), device="cuda", dtype=d_in.dtype)
    rs.rs_shift_topk(d_out, d_in, d_src, P, K, scores, kept, gathered, dist=dist)
    torch.cuda.synchronize()
    return to_host(scores), kept.cpu().numpy(), to_host(gathered)


SHIFT_CASES = [  # B, N, D, n_prefix, n_keep
    (3, 17, 64, 1, 7), (2, 197, 192, 1, 138), (4, 197, 768, 1, 177), (1, 4097, 1024, 1, 2868),
    (2, 1, 64, 1, 0), (2, 5, 72, 0, 5), (2, 300, 384, 2, 1), (1, 1000, 8, 0, 0), (5, 263, 2056, 3, 100)]


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("dist", [rs.RS_DIST_L2, rs.RS_DIST_L1, rs.RS_DIST_COS])
@pytest.mark.parametrize("B,N,D,P,K", SHIFT_CASES)
def test_shift_topk(dtype, dist, B, N, D, P, K):
    _say("shift_topk", dtype, dist, B, N, D, P, K)
    f_in = host_round(si.tokens(0, B, N, D, spread=0.5), dtype)
    f_out = host_round(f_in + si.generic(0, 8, (B, N, D), std=0.3) * np.exp(si.generic(0, 9, (B, N, 1), std=0.7)), dtype)
    src = host_round(si.generic(0, 10, (B, N, D)), dtype)
    s_ref, kept_ref, g_ref = oracle.shift_topk(f_out, f_in, src, P, K, dist)
    s, kept, g = _run_shift_topk(f_out, f_in, src, P, K, dist, dtype)
    assert norm_err(s, s_ref) < 1e-5  # inputs identical on both sides, fp32 accumulation
    # selection is exact on the GPU's own scores (integer work: bit-exact) ...
    np.testing.assert_array_equal(kept, oracle.topk(s, P, K))
    # ... and agrees with the checker's selection outside the rounding band
    check_kept_admissible(kept, s, s_ref, P, K)
    # gather is a copy of the selected rows
    np.testing.assert_array_equal(g, oracle.gather(src, kept))


# Images whose rows fit a compute unit's registers take the one-pass kernel when the rows to gather
# are f_in's own (src NULL): rows per wave from 1 to 13, row chunks of 1, 2 and 3 x 512 bytes with
# ragged ends, more images than workgroups (the grid is persistent), prefix-only and keep-all.
RESIDENT_CASES = [  # B, N, D, n_prefix, n_keep
    (3, 17, 64, 1, 7), (4, 197, 768, 1, 177), (2, 208, 384, 0, 100), (300, 33, 192, 1, 20), (2, 1, 8, 1, 0),
    (2, 197, 192, 1, 196), (3, 100, 520, 2, 0), (2, 16, 256, 0, 16), (1, 207, 760, 1, 1)]


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("dist", [rs.RS_DIST_L2, rs.RS_DIST_L1, rs.RS_DIST_COS])
@pytest.mark.parametrize("B,N,D,P,K", RESIDENT_CASES)
def test_shift_topk_one_pass(dtype, dist, B, N, D, P, K):
    if dtype == "f32" and D * 4 > 1536:
        pytest.skip("fp32 rows beyond 1536 bytes take the three-launch path (covered by test_shift_topk)")
    _say("shift_topk one pass", dtype, dist, B, N, D, P, K)
    f_in = host_round(si.tokens(3, B, N, D, spread=0.5), dtype)
    f_out = host_round(f_in + si.generic(3, 8, (B, N, D), std=0.3) * np.exp(si.generic(3, 9, (B, N, 1), std=0.7)), dtype)
    sample = sorted(set([0, B // 2, B - 1]))      # the checker on a few images when the batch is large
    s_ref, kept_ref, g_ref = oracle.shift_topk(f_out[sample], f_in[sample], None, P, K, dist)
    s, kept, g = _run_shift_topk(f_out, f_in, None, P, K, dist, dtype)
    # fp32 sums of identical inputs; 1 - cos cancels, so the cosine score carries an absolute error of
    # a few ulps of 1 whatever its size
    assert (np.abs(s[sample] - s_ref).max() < 2e-6) if dist == rs.RS_DIST_COS else (norm_err(s[sample], s_ref) < 1e-5)
    np.testing.assert_array_equal(kept, oracle.topk(s, P, K))           # exact on the GPU's own scores, every image
    check_kept_admissible(kept[sample], s[sample], s_ref, P, K)
    np.testing.assert_array_equal(g, oracle.gather(f_in, kept))         # every image: a copy of the kept rows
    # the three-launch path (taken when the rows come from another tensor) agrees
    s3, kept3, g3 = _run_shift_topk(f_out, f_in, f_in.copy(), P, K, dist, dtype)
    assert np.abs(s3 - s).max() <= 1e-6 * max(np.abs(s).max(), 1.0)
    same = (kept3 == kept).all(axis=1)
    assert same.mean() > 0.9
    np.testing.assert_array_equal(g3[same], g[same])


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_shift_topk_exact_ties(dtype):
    """Small-integer data: scores are exact in fp32 and heavily tied, so kept_idx must
    equal the checker's bit for bit (lower index wins a tie)."""
    B, N, D, P, K = 4, 197, 64, 1, 100
    rng = np.random.default_rng(7)
    f_in = rng.integers(-3, 4, size=(B, N, D)).astype(np.float32)
    delta = np.zeros((B, N, D), np.float32)
    delta[:, :, :4] = rng.integers(0, 3, size=(B, N, 4))
    f_out = f_in + delta
    for dist in (rs.RS_DIST_L2, rs.RS_DIST_L1):
        s_ref, kept_ref, g_ref = oracle.shift_topk(f_out, f_in, None, P, K, dist)
        s, kept, g = _run_shift_topk(f_out, f_in, None, P, K, dist, dtype)
        np.testing.assert_allclose(s, s_ref, rtol=1e-6)
        np.testing.assert_array_equal(kept, kept_ref)
        np.testing.assert_array_equal(g, g_ref)
    # all-equal scores: lowest indices
    s, kept, g = _run_shift_topk(f_in + 1.0, f_in, None, 1, 10, rs.RS_DIST_L2, dtype)
    np.testing.assert_array_equal(kept, np.tile(np.arange(11), (B, 1)))
    # identity sub-layer: zero shift
    s, kept, g = _run_shift_topk(f_in, f_in, None, 1, 10, rs.RS_DIST_L2, dtype)
    assert (s == 0).all()


# ----------------------------------------------------------------------------
# whole block
# ----------------------------------------------------------------------------
def _block_inputs(seed, B, N, D, Dm, dtype, block=0, std=0.02, spread=0.0, affine_ln=False):
    x = host_round(si.tokens(seed, B, N, D, spread), dtype)
    w = {k: host_round(v, dtype) for k, v in si.block_weights(seed, block, D, Dm, std).items()}
    if affine_ln:
        for i, k in enumerate(("ln1_g", "ln1_b", "ln2_g", "ln2_b")):
            base = 1.0 if k.endswith("_g") else 0.0
            w[k] = host_round(base + si.generic(seed, 20 + i, (D,), std=0.2), dtype)
    return x, w


def _run_block(x, w, H, P, K, dtype, dist=rs.RS_DIST_L2, want_scores=True, pack=False, ln_eps=1e-6,
               op=rs.RS_SHIFT_MLP):
    B, N, D = x.shape
    Dm = w["w_fc1"].shape[1]
    dw = {k: to_dev(v, dtype) for k, v in w.items()}
    dx = to_dev(x, dtype)
    cfg = rs.make_cfg(B, N, D, H, Dm, P, K, dx.dtype, ln_eps=ln_eps, dist=dist, op=op)
    packed = None
    if pack and dtype == "bf16":
        packed = torch.empty(rs.rs_packed_weights_size(cfg), dtype=torch.uint8, device="cuda")
        rs.rs_pack_weights(cfg, rs.make_weights(dw), packed)
    ws = torch.empty(rs.rs_block_workspace_size(cfg), dtype=torch.uint8, device="cuda")
    y = torch.full((B, P + K, D), float("nan"), device="cuda", dtype=dx.dtype)
    kept = torch.full((B, P + K), -1, device="cuda", dtype=torch.int32)
    scores = torch.full((B, N), float("nan"), device="cuda", dtype=torch.float32) if want_scores else None
    rs.rs_block_fwd(cfg, rs.make_weights(dw, packed), dx, y, kept, scores, ws)
    torch.cuda.synchronize()
    return y, kept, scores


def _check_block(x, w, H, P, K, dtype, dist=rs.RS_DIST_L2, **kw):
    y, kept, scores = _run_block(x, w, H, P, K, dtype, dist=dist, **kw)
    ref = oracle.block(x, w, H, ln_eps=kw.get("ln_eps", 1e-6), dist=dist, op=kw.get("op", 0))
    s, kept_h = to_host(scores), kept.cpu().numpy()
    e_s = norm_err(s, ref["scores"])
    exact = check_kept_admissible(kept_h, s, ref["scores"], P, K)
    # teacher forcing: compare the compacted rows on the GPU's own kept set
    e_y = norm_err(to_host(y), oracle.gather(ref["xhat"], kept_h))
    _say("  score err %.3e  y err %.3e  kept exact on %.0f%% of images" % (e_s, e_y, 100 * exact))
    assert e_s < TOL[dtype] and e_y < TOL[dtype]
    np.testing.assert_array_equal(kept_h, oracle.topk(s, P, K))  # selection exact on the GPU's scores
    return exact


def test_block_fp32_config1():
    """Single ViT block, fp32: batch 4, 197 tokens, D 192, 3 heads, MLP 768, drop 30% of the
    non-class tokens (196 -> 138)."""
    wl = si.WORKLOADS["vit_block_fp32"]
    (n_in, n_keep), = rs.keep_counts(wl["N"], 1, 1, wl["prune"])
    assert n_keep == 138
    x, w = _block_inputs(0, wl["B"], wl["N"], wl["D"], wl["Dm"], "f32")
    _say("block fp32 config 1")
    exact = _check_block(x, w, wl["H"], 1, n_keep, "f32")
    assert exact == 1.0  # fp32 scores are close enough that the kept sets agree exactly here


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("B,N,D,H,Dm,P,K", [(2, 197, 384, 6, 1536, 1, 180), (1, 50, 128, 2, 192, 0, 20),
                                             (3, 300, 192, 3, 768, 2, 100), (1, 129, 64, 1, 64, 1, 1)])
def test_block_shapes(dtype, B, N, D, H, Dm, P, K):
    _say("block", dtype, B, N, D, H, Dm, P, K)
    x, w = _block_inputs(1, B, N, D, Dm, dtype, std=0.05, spread=0.3, affine_ln=True)
    _check_block(x, w, H, P, K, dtype, ln_eps=1e-5)


@pytest.mark.parametrize("dist", [rs.RS_DIST_L2, rs.RS_DIST_COS])
@pytest.mark.parametrize("B,N,K", [(63, 257, 100), (64, 257, 100), (66, 300, 299), (2, 1024, 400), (2, 1025, 1),
                                   (1, 1300, 650), (64, 256, 128)])
def test_block_selection_switch_over_points(B, N, K, dist):
    """The selection inside the bf16 block on both sides of its switch-over points: by counting
    up to 256 tokens and by radix passes beyond; scores formed by the selection kernel itself
    (64 images or more) or by a grid over all rows before it (fewer, longer sequences); 256 or
    1024 threads per image around 1024 tokens.  Kept indices exact on the GPU's own scores."""
    _say("block selection", B, N, K, dist)
    x, w = _block_inputs(14, B, N, 64, 128, "bf16", std=0.1, spread=0.3)
    _check_block(x, w, 1, 1, K, "bf16", dist=dist)


@pytest.mark.parametrize("dist", [rs.RS_DIST_L1, rs.RS_DIST_COS])
def test_block_other_distances(dist):
    x, w = _block_inputs(2, 2, 100, 128, 256, "bf16", std=0.1, spread=0.3)
    _say("block dist", dist)
    _check_block(x, w, 2, 1, 40, "bf16", dist=dist)
    _check_block(x.astype(np.float32), w, 2, 1, 40, "f32", dist=dist)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("dist", [rs.RS_DIST_L2, rs.RS_DIST_L1, rs.RS_DIST_COS])
@pytest.mark.parametrize("op", [rs.RS_SHIFT_ATTN, rs.RS_SHIFT_BLOCK, rs.RS_SHIFT_MLP_STREAM, rs.RS_SHIFT_MLP_NORMED])
def test_block_operation_choice(op, dist, dtype):
    """The shift around the attention layer, around the whole block, and the two other readings
    of the MLP case (Sec. 3.3, "Operation choice"), each with every distance; ragged row and
    column tiles (300 tokens x 3 images, D 192)."""
    assert (rs.RS_SHIFT_MLP, rs.RS_SHIFT_ATTN, rs.RS_SHIFT_BLOCK, rs.RS_SHIFT_MLP_STREAM, rs.RS_SHIFT_MLP_NORMED) == \
        (oracle.OP_MLP, oracle.OP_ATTN, oracle.OP_BLOCK, oracle.OP_MLP_STREAM, oracle.OP_MLP_NORMED)
    _say("block op", op, "dist", dist, dtype)
    x, w = _block_inputs(6, 3, 300, 192, 768, dtype, std=0.1, spread=0.3, affine_ln=True)
    _check_block(x, w, 3, 1, 120, dtype, dist=dist, op=op)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_block_widest_supported_rows(dtype):
    """D = 4096 (the library's limit), 64 heads: the wide-row paths of the row-statistics /
    LayerNorm kernels, 16 column tiles in the projection, 64 score slots per row."""
    _say("block D=4096", dtype)
    x, w = _block_inputs(13, 1, 40, 4096, 128, dtype, std=0.02, spread=0.3)
    _check_block(x, w, 64, 1, 17, dtype)


@pytest.mark.parametrize("pack", [False, True])
def test_block_offset_rows_and_outlier_channels(pack):
    """Rows far from zero mean (offset 6 standard deviations) with two channels 30 times larger
    than the rest and affine LayerNorm parameters: the bf16 path applies the LayerNorm inside
    the GEMM epilogue as rstd * (x W' - mean * colsum) + bias', which must not lose the signal
    next to the mean's share of the accumulator."""
    B, N, D, H, Dm = 2, 197, 384, 6, 1536
    x, w = _block_inputs(8, B, N, D, Dm, "bf16", std=0.05, spread=0.3, affine_ln=True)
    x = x.astype(np.float64)
    x[..., 7] *= 30.0
    x[..., 300] *= 30.0
    x = host_round(x + 6.0, "bf16")
    _say("block offset rows, packed", pack)
    _check_block(x, w, H, 1, 150, "bf16", ln_eps=1e-5, pack=pack)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_block_without_pruning_and_null_biases(dtype):
    B, N, D, H, Dm = 2, 70, 128, 2, 256
    x, w = _block_inputs(3, B, N, D, Dm, dtype, std=0.05)
    for k in ("b_qkv", "b_proj", "b_fc1", "b_fc2", "ln1_b", "ln2_b", "ln1_g"):
        w[k] = None
    ref = oracle.block(x, w, H)
    for want_scores in (False, True):
        y, kept, scores = _run_block(x, w, H, 1, N - 1, dtype, want_scores=want_scores)
        assert norm_err(to_host(y), ref["xhat"]) < TOL[dtype]
        np.testing.assert_array_equal(kept.cpu().numpy(), np.tile(np.arange(N), (B, 1)))
        if want_scores:
            assert norm_err(to_host(scores), ref["scores"]) < TOL[dtype]
    # prefix only: everything but the class token is dropped
    y, kept, scores = _run_block(x, w, H, 1, 0, dtype)
    np.testing.assert_array_equal(kept.cpu().numpy(), np.zeros((B, 1), np.int32))
    assert norm_err(to_host(y), ref["xhat"][:, :1]) < TOL[dtype]


@pytest.mark.parametrize("seed", [11, 12])
def test_block_seeded_random_shapes(seed):
    """Forty seeded random configurations per seed around the kernels' switch-over points: sequence
    lengths at tile boundaries, MLP widths that take the long-K GEMM path with and without padded
    trips, every distance, operation choice and GEMM tile variant, prefix 0-2, any keep count."""
    import random
    rnd = random.Random(seed)
    for c in range(40):
        H = rnd.choice([1, 2, 3, 6, 12])
        D = 64 * H
        Dm = rnd.choice([64, 192, 768, 1536, 2048, 2560, 3072, 4096])
        N = rnd.choice([1, 2, 31, 64, 65, 127, 197, 256, 257, 300, 513, 785])
        B = rnd.choice([1, 2, 3, 5])
        if B * N * (D + Dm) > 4_000_000:
            B = 1
        P = rnd.choice([0, 1, 2]) if N > 2 else 0
        K = rnd.randint(0 if P else 1, N - P)
        dist = rnd.choice([rs.RS_DIST_L2, rs.RS_DIST_L1, rs.RS_DIST_COS])
        op = rnd.choice([rs.RS_SHIFT_MLP, rs.RS_SHIFT_ATTN, rs.RS_SHIFT_BLOCK, rs.RS_SHIFT_MLP_STREAM])
        variant = rnd.choice([0, 0, 0, 1, 2, 3, 4])
        _say("random case %d.%d: B %d N %d D %d Dm %d P %d K %d dist %d op %d variant %d"
             % (seed, c, B, N, D, Dm, P, K, dist, op, variant))
        x, w = _block_inputs(1000 * seed + c, B, N, D, Dm, "bf16", std=0.05, spread=0.3, affine_ln=bool(c & 1))
        try:
            rs.rs_tune_gemm_variant(variant)
            _check_block(x, w, H, P, K, "bf16", dist=dist, op=op, pack=bool(c & 2))
        finally:
            rs.rs_tune_gemm_variant(0)


def test_block_packed_weights_and_determinism():
    x, w = _block_inputs(4, 2, 197, 384, 1536, "bf16")
    a = _run_block(x, w, 6, 1, 150, "bf16", pack=False)
    b = _run_block(x, w, 6, 1, 150, "bf16", pack=True)
    c = _run_block(x, w, 6, 1, 150, "bf16", pack=True)
    for t0, t1, t2 in zip(a, b, c):
        assert torch.equal(t0, t1) and torch.equal(t1, t2)


@pytest.mark.parametrize("dist", [rs.RS_DIST_L2, rs.RS_DIST_COS])
def test_gemm_tile_variants_give_the_same_bits(dist):
    """The bf16 GEMMs pick a tile variant by shape (256 x 256 persistent workgroups, 256 x 128 or
    128 x 128 ring kernels, or the first for whole rounds and a ring kernel for the rows behind them).
    Products are accumulated in the same order in all of them and the shift sums are added in one
    fixed order, so outputs, scores and kept indices must not depend on the variant: 700 rows x 3
    images (ragged row tiles in every variant), D 192 (one and a half 128-wide column tiles)."""
    x, w = _block_inputs(17, 3, 700, 192, 768, "bf16", std=0.1, spread=0.3, affine_ln=True)
    outs = []
    try:
        for variant in (0, 1, 2, 3):
            rs.rs_tune_gemm_variant(variant)
            outs.append(_run_block(x, w, 3, 1, 300, "bf16", dist=dist, op=rs.RS_SHIFT_BLOCK))
    finally:
        rs.rs_tune_gemm_variant(0)
    for y, kept, scores in outs[1:]:
        assert torch.equal(scores.view(torch.int32), outs[0][2].view(torch.int32))
        assert torch.equal(kept, outs[0][1])
        assert torch.equal(y.view(torch.int16), outs[0][0].view(torch.int16))


def test_gemm_rows_split_between_two_kernels():
    """A GEMM whose 256 x 256 tiles make one whole round of the chip and a small second one: the rows
    of the whole round go to the persistent kernel, the rest to a ring kernel in a second launch.
    Both halves against the checker (sampled rows), and the result against the one-kernel variants."""
    M, K, N = 256 * 90 + 77, 256, 768      # 91 row panels x 3 column tiles = 273 tiles on 256 CUs
    a = host_round(si.generic(19, 30, (M, K)), "bf16")
    wgt = host_round(si.generic(19, 31, (K, N), std=0.05), "bf16")
    b = host_round(si.generic(19, 32, (N,), std=0.5), "bf16")
    res = host_round(si.generic(19, 33, (M, N)), "bf16")
    da, dw, db, dres = (to_dev(t, "bf16") for t in (a, wgt, b, res))
    wt = torch.empty((N, K), device="cuda", dtype=torch.bfloat16)
    rs.rs_pack_linear(dw, wt)
    outs = []
    try:
        for variant in (0, 1, 2):
            rs.rs_tune_gemm_variant(variant)
            out = torch.full((M, N), float("nan"), device="cuda", dtype=torch.bfloat16)
            rs.rs_linear_fwd(da, wt, db, dres, out, rs.RS_EPI_BIAS_RES)
            torch.cuda.synchronize()
            outs.append(out)
    finally:
        rs.rs_tune_gemm_variant(0)
    assert torch.equal(outs[0].view(torch.int16), outs[1].view(torch.int16))
    assert torch.equal(outs[0].view(torch.int16), outs[2].view(torch.int16))
    rows = np.r_[0:40, 21700:21800, M - 150:M]     # first tile, around the split (row 21760), ragged end
    ref = oracle.linear(a[rows], wgt, b) + res[rows]
    assert norm_err(to_host(outs[0])[rows], ref) < 5e-3


@pytest.mark.parametrize("M,K,N", [(300, 3072, 256), (777, 2560, 320), (513, 4096, 128), (260, 2048, 64)])
def test_persistent_gemm_long_k(M, K, N):
    """The persistent GEMM keeps three LDS stages for the activation rows when K is long (trip of six
    slices: 3072 fits, 2560 and 4096 are padded with zero slices, 2048 would be padded by too much and
    keeps two stages): forced on small ragged problems, against the checker and bit for bit against
    the 128 x 128 ring kernel, with the residual epilogue."""
    a = host_round(si.generic(23, 30, (M, K)), "bf16")
    wgt = host_round(si.generic(23, 31, (K, N), std=0.03), "bf16")
    b = host_round(si.generic(23, 32, (N,), std=0.5), "bf16")
    res = host_round(si.generic(23, 33, (M, N)), "bf16")
    da, dw, db, dres = (to_dev(t, "bf16") for t in (a, wgt, b, res))
    wt = torch.empty((N, K), device="cuda", dtype=torch.bfloat16)
    rs.rs_pack_linear(dw, wt)
    outs = []
    try:
        for variant in (1, 3):
            rs.rs_tune_gemm_variant(variant)
            out = torch.full((M, N), float("nan"), device="cuda", dtype=torch.bfloat16)
            rs.rs_linear_fwd(da, wt, db, dres, out, rs.RS_EPI_BIAS_RES)
            torch.cuda.synchronize()
            outs.append(out)
    finally:
        rs.rs_tune_gemm_variant(0)
    assert torch.equal(outs[0].view(torch.int16), outs[1].view(torch.int16))
    assert norm_err(to_host(outs[0]), oracle.linear(a, wgt, b) + res) < 5e-3


def test_multi_block_teacher_forced():
    """Four blocks of a ViT-S-like stack with 16 tokens dropped after each: the checker follows
    the GPU's kept set block by block (kept sets may legitimately differ inside the rounding band)."""
    B, N, D, H, Dm, dtype = 2, 197, 384, 6, 1536, "bf16"
    x = host_round(si.tokens(5, B, N, D), dtype)
    dx = to_dev(x, dtype)
    for blk in range(4):
        w = {k: host_round(v, dtype) for k, v in si.block_weights(5, blk, D, Dm).items()}
        n = dx.shape[1]
        K = n - 1 - 16
        dw = {k: to_dev(v, dtype) for k, v in w.items()}
        cfg = rs.make_cfg(B, n, D, H, Dm, 1, K, dx.dtype)
        ws = torch.empty(rs.rs_block_workspace_size(cfg), dtype=torch.uint8, device="cuda")
        y = torch.empty((B, 1 + K, D), device="cuda", dtype=dx.dtype)
        kept = torch.empty((B, 1 + K), device="cuda", dtype=torch.int32)
        scores = torch.empty((B, n), device="cuda", dtype=torch.float32)
        rs.rs_block_fwd(cfg, rs.make_weights(dw), dx, y, kept, scores, ws)
        torch.cuda.synchronize()
        # checker continues from the GPU's block input (teacher forcing), so each block is
        # compared like with like
        ref = oracle.block(to_host(dx), w, H)
        s, kept_h = to_host(scores), kept.cpu().numpy()
        assert norm_err(s, ref["scores"]) < TOL[dtype]
        exact = check_kept_admissible(kept_h, s, ref["scores"], 1, K)
        assert norm_err(to_host(y), oracle.gather(ref["xhat"], kept_h)) < TOL[dtype]
        _say("  block %d: kept exact on %.0f%% of images" % (blk + 1, 100 * exact))
        dx = y


def test_block_stack_replays_from_a_hip_graph():
    """Three blocks with pruning recorded into one HIP graph (the library neither allocates nor
    synchronises); every replay, with eager work and synchronisations in between, must equal
    the eager result bit for bit."""
    B, N, D, H, Dm = 4, 197, 192, 3, 768
    sched = rs.keep_counts(N, 1, 3, dict(kind="drop_pct", pct=25, after=[1, 2]))
    x0 = to_dev(host_round(si.tokens(9, B, N, D, 0.3), "bf16"), "bf16")
    ws_list, cfgs, keep = [], [], []
    for l, (n_in, n_keep) in enumerate(sched):
        w = {k: to_dev(host_round(v, "bf16"), "bf16") for k, v in si.block_weights(9, l, D, Dm, 0.05).items()}
        cfg = rs.make_cfg(B, n_in, D, H, Dm, 1, n_keep, torch.bfloat16)
        packed = torch.empty(rs.rs_packed_weights_size(cfg), dtype=torch.uint8, device="cuda")
        rs.rs_pack_weights(cfg, rs.make_weights(w), packed)
        keep.append((w, packed))
        ws_list.append(rs.make_weights(w, packed))
        cfgs.append(cfg)
    ws = torch.empty(max(rs.rs_block_workspace_size(c) for c in cfgs), dtype=torch.uint8, device="cuda")
    bufs = [torch.zeros((B, N, D), device="cuda", dtype=torch.bfloat16) for _ in range(2)]
    kept = torch.zeros((B, N), device="cuda", dtype=torch.int32)

    def step():
        stream = torch.cuda.current_stream()
        src = x0
        for l in range(3):
            rs.rs_block_fwd(cfgs[l], ws_list[l], src, bufs[l & 1], kept, None, ws, stream)
            src = bufs[l & 1]
        return src

    K_last = 1 + sched[-1][1]
    step()
    torch.cuda.synchronize()
    n_y, n_k = B * K_last * D, B * K_last     # y and kept_idx are compact [B, K, D] / [B, K] at the buffer start
    want = step().view(-1)[:n_y].clone()
    want_kept = kept.view(-1)[:n_k].clone()
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        out = step()
    for rep in range(4):
        for b_ in bufs:
            b_.fill_(float(rep))      # eager work between replays; stale data must not survive
        kept.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out.view(-1)[:n_y].view(torch.int16), want.view(torch.int16)), rep
        assert torch.equal(kept.view(-1)[:n_k], want_kept), rep


def test_encoder_stack_replays_from_a_hip_graph():
    """The launch sequence bench.py times (EncoderStack.step: chained blocks, ping-pong buffers) recorded
    into one HIP graph: every replay, with eager work in between, equals the eager step bit for bit."""
    wl = dict(B=6, N=65, D=192, H=3, Dm=384, blocks=4, n_prefix=1, prune=dict(kind="drop_pct", pct=20, after=[1, 3]))
    x0 = to_dev(host_round(si.tokens(31, wl["B"], wl["N"], wl["D"], 0.3), "bf16"), "bf16")
    w_dev = [{k: to_dev(host_round(v, "bf16"), "bf16") for k, v in si.block_weights(31, l, wl["D"], wl["Dm"], 0.05).items()}
             for l in range(wl["blocks"])]
    stack = rs.EncoderStack(wl, x0, w_dev, streams=1)
    want = stack.step()[0].clone()
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        stack.step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        out = stack.step()[0]
    for rep in range(3):
        for p in stack.parts:
            for b_ in p["bufs"]:
                b_.fill_(float(rep + 1))
            p["stats"].fill_(float("nan"))
            p["kept"].zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out.view(torch.int16), want.view(torch.int16)), rep
    # the unchained sequence gives the same bits
    stack.chain = False
    assert torch.equal(stack.step()[0].view(torch.int16), want.view(torch.int16))


@pytest.mark.parametrize("D,H,Dm", [(192, 3, 768), (384, 6, 1536), (1152, 18, 1152)])
def test_chained_blocks_equal_unchained_blocks(D, H, Dm):
    """rs_block_fwd_chained hands the row statistics of a block's output to the next block (written by
    the gather in pruning blocks, by a pass over y otherwise): outputs, kept indices and scores of a
    pruning / non-pruning / pruning stack must equal rs_block_fwd's bit for bit, y_stats must be the
    statistics of y, and a block that keeps every token must leave kept_idx[b, j] = j."""
    B, N, P = 3, 77, 1
    sched = [(77, 60), (61, 60), (61, 33)]
    x0 = to_dev(host_round(si.tokens(21, B, N, D, 0.4), "bf16"), "bf16")
    cfgs, wl = [], []
    for l, (n_in, n_keep) in enumerate(sched):
        w = {k: to_dev(host_round(v, "bf16"), "bf16") for k, v in si.block_weights(21, l, D, Dm, 0.05).items()}
        cfgs.append(rs.make_cfg(B, n_in, D, H, Dm, P, n_keep, torch.bfloat16))
        wl.append((w, rs.make_weights(w)))
    ws = torch.empty(max(rs.rs_block_workspace_size(c) for c in cfgs), dtype=torch.uint8, device="cuda")

    def run(chained):
        bufs = [torch.zeros((B, N, D), device="cuda", dtype=torch.bfloat16) for _ in range(2)]
        stats = torch.full((B * N, 2), float("nan"), device="cuda", dtype=torch.float32)
        outs, src = [], x0
        for l, (n_in, n_keep) in enumerate(sched):
            K = P + n_keep
            kept = torch.full((B, K), -1, device="cuda", dtype=torch.int32)
            sc = torch.empty((B, n_in), device="cuda", dtype=torch.float32)
            dst = bufs[l & 1]
            if chained:
                rs.rs_block_fwd_chained(cfgs[l], wl[l][1], src, stats if l > 0 else None, dst, stats, kept, sc, ws)
            else:
                rs.rs_block_fwd(cfgs[l], wl[l][1], src, dst, kept, sc, ws)
            torch.cuda.synchronize()
            y = dst.view(-1)[:B * K * D].view(B, K, D).clone()
            outs.append((y, kept.clone(), sc.clone(), stats[:B * K].clone() if chained else None))
            src = dst
        return outs

    plain, chain = run(False), run(True)
    for l, ((y0, k0, s0, _), (y1, k1, s1, st)) in enumerate(zip(plain, chain)):
        assert torch.equal(y0.view(torch.int16), y1.view(torch.int16)), l
        assert torch.equal(k0, k1), l
        assert torch.equal(s0, s1), l
        yh = y1.float().cpu().numpy().astype(np.float64).reshape(-1, D)
        mean, var = yh.mean(-1), yh.var(-1)
        np.testing.assert_allclose(st[:, 0].cpu().numpy(), mean, rtol=0, atol=2e-6 * np.abs(yh).max())
        np.testing.assert_allclose(st[:, 1].cpu().numpy(), 1.0 / np.sqrt(var + 1e-6), rtol=2e-5)
    K1 = P + sched[1][1]
    assert torch.equal(chain[1][1], torch.arange(K1, device="cuda", dtype=torch.int32).expand(B, K1))


def test_chained_block_fp32_leaves_statistics_of_y():
    """The fp32 parity configuration ignores x_stats and still fills y_stats."""
    B, N, D, H, Dm, P, n_keep = 2, 50, 128, 2, 256, 1, 30
    x = si.tokens(22, B, N, D)
    w = si.block_weights(22, 0, D, Dm)
    cfg = rs.make_cfg(B, N, D, H, Dm, P, n_keep, torch.float32)
    dw = {k: to_dev(v, "f32") for k, v in w.items()}
    ws = torch.empty(rs.rs_block_workspace_size(cfg), dtype=torch.uint8, device="cuda")
    K = P + n_keep
    y0, y1 = (torch.empty((B, K, D), device="cuda", dtype=torch.float32) for _ in range(2))
    k0, k1 = (torch.empty((B, K), device="cuda", dtype=torch.int32) for _ in range(2))
    stats = torch.empty((B * K, 2), device="cuda", dtype=torch.float32)
    bogus = torch.full((B * N, 2), float("nan"), device="cuda", dtype=torch.float32)
    rs.rs_block_fwd(cfg, rs.make_weights(dw), to_dev(x, "f32"), y0, k0, None, ws)
    rs.rs_block_fwd_chained(cfg, rs.make_weights(dw), to_dev(x, "f32"), bogus, y1, stats, k1, None, ws)
    torch.cuda.synchronize()
    assert torch.equal(y0, y1) and torch.equal(k0, k1)
    yh = y1.cpu().numpy().astype(np.float64).reshape(-1, D)
    np.testing.assert_allclose(stats[:, 0].cpu().numpy(), yh.mean(-1), atol=1e-6 * np.abs(yh).max())
    np.testing.assert_allclose(stats[:, 1].cpu().numpy(), 1.0 / np.sqrt(yh.var(-1) + 1e-6), rtol=1e-5)


# ----------------------------------------------------------------------------
# line-wise pruning of a 2-D grid
# ----------------------------------------------------------------------------
GRID_CASES = [  # B, H, W, C, keep_rows, keep_cols  (ResNet stage shapes: 56x56x64 -> 48x48, 28x28x128 -> 24x24)
    (2, 56, 56, 64, 48, 48), (3, 28, 28, 128, 24, 24), (1, 7, 5, 8, 7, 5), (2, 9, 300, 16, 0, 3), (1, 1, 1, 2048, 1, 1)]


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("dist", [rs.RS_DIST_L2, rs.RS_DIST_COS])
@pytest.mark.parametrize("B,H,W,C,R,Q", GRID_CASES)
def test_grid_line_prune(dtype, dist, B, H, W, C, R, Q):
    _say("grid", dtype, dist, B, H, W, C, R, Q)
    f_in = host_round(si.generic(11, 1, (B, H, W, C)), dtype)
    f_out = host_round(f_in + si.generic(11, 2, (B, H, W, C), std=0.3) * np.exp(si.generic(11, 3, (B, H, W, 1), std=0.7)), dtype)
    src = host_round(si.generic(11, 4, (B, H, W, C)), dtype)
    s_ref, r_ref, c_ref, kr_ref, kc_ref, g_ref = oracle.grid_line_prune(f_out, f_in, src, R, Q, dist)
    d_out, d_in, d_src = (to_dev(t, dtype) for t in (f_out, f_in, src))
    scores = torch.full((B, H, W), float("nan"), device="cuda", dtype=torch.float32)
    rsc = torch.full((B, H), float("nan"), device="cuda", dtype=torch.float32)
    csc = torch.full((B, W), float("nan"), device="cuda", dtype=torch.float32)
    kr = torch.full((B, R), -1, device="cuda", dtype=torch.int32)
    kc = torch.full((B, Q), -1, device="cuda", dtype=torch.int32)
    g = torch.full((B, R, Q, C), float("nan"), device="cuda", dtype=d_in.dtype)
    rs.rs_grid_line_prune(d_out, d_in, d_src, R, Q, scores, rsc, csc, kr, kc, g, dist=dist)
    torch.cuda.synchronize()
    s, r_, c_ = to_host(scores), to_host(rsc), to_host(csc)
    assert norm_err(s, s_ref) < 1e-5 and norm_err(r_, r_ref) < 1e-5 and norm_err(c_, c_ref) < 1e-5
    kr_h, kc_h = kr.cpu().numpy(), kc.cpu().numpy()
    # selection is exact on the GPU's own line scores, and admissible against the checker's
    np.testing.assert_array_equal(kr_h, oracle.topk(r_, 0, R))
    np.testing.assert_array_equal(kc_h, oracle.topk(c_, 0, Q))
    check_kept_admissible(kr_h, r_, r_ref, 0, R)
    check_kept_admissible(kc_h, c_, c_ref, 0, Q)
    np.testing.assert_array_equal(to_host(g), oracle.grid_gather(src, kr_h, kc_h))


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("dist", [rs.RS_DIST_L2, rs.RS_DIST_L1])
@pytest.mark.parametrize("B,H,W,C,R,Q", GRID_CASES + [(2, 300, 9, 16, 280, 9), (1, 6, 7, 8, 0, 3)])
def test_grid_token_prune(dtype, dist, B, H, W, C, R, Q):
    """Token-wise pruning of a grid (rows lose their lowest positions, then the compacted columns)."""
    _say("grid token-wise", dtype, dist, B, H, W, C, R, Q)
    f_in = host_round(si.generic(12, 1, (B, H, W, C)), dtype)
    f_out = host_round(f_in + si.generic(12, 2, (B, H, W, C), std=0.3) * np.exp(si.generic(12, 3, (B, H, W, 1), std=0.7)), dtype)
    src = host_round(si.generic(12, 4, (B, H, W, C)), dtype)
    s_ref, kc_ref, cs_ref, kr_ref, g_ref = oracle.grid_token_prune(f_out, f_in, src, R, Q, dist)
    d_out, d_in, d_src = (to_dev(t, dtype) for t in (f_out, f_in, src))
    scores = torch.full((B, H, W), float("nan"), device="cuda", dtype=torch.float32)
    kc = torch.full((B, H, Q), -1, device="cuda", dtype=torch.int32)
    cs = torch.full((B, Q, H), float("nan"), device="cuda", dtype=torch.float32)
    kr = torch.full((B, Q, R), -1, device="cuda", dtype=torch.int32)
    g = torch.full((B, R, Q, C), float("nan"), device="cuda", dtype=d_in.dtype)
    rs.rs_grid_token_prune(d_out, d_in, d_src, R, Q, scores, kc, cs, kr, g, dist=dist)
    torch.cuda.synchronize()
    s, kc_h, cs_h, kr_h = to_host(scores), kc.cpu().numpy(), to_host(cs), kr.cpu().numpy()
    assert norm_err(s, s_ref) < 1e-5
    # step 1: exact on the GPU's own scores, admissible against the checker's
    np.testing.assert_array_equal(kc_h.reshape(B * H, Q), oracle.topk(s.reshape(B * H, W), 0, Q))
    check_kept_admissible(kc_h.reshape(B * H, Q), s.reshape(B * H, W), s_ref.reshape(B * H, W), 0, Q)
    if Q == 0 or R == 0:
        return
    # step 2 on the GPU's compacted grid: the scores are the selected ones, the selection is exact
    want_cs = np.take_along_axis(s, kc_h.astype(np.int64), axis=2).transpose(0, 2, 1)
    np.testing.assert_array_equal(cs_h, want_cs)
    np.testing.assert_array_equal(kr_h.reshape(B * Q, R), oracle.topk(cs_h.reshape(B * Q, H), 0, R))
    # gathered rows are copies of src at the selected positions
    got = to_host(g)
    for b in range(B):
        for j in range(Q):
            rows = kr_h[b, j]
            np.testing.assert_array_equal(got[b, :, j], src[b, rows, kc_h[b, rows, j]].astype(np.float64))
    # where both selections agree with the checker's, so does everything
    if np.array_equal(kc_h, kc_ref) and np.array_equal(kr_h, kr_ref):
        np.testing.assert_array_equal(got, g_ref)


def test_batch_parts_on_streams_equal_the_whole_batch():
    """bench.py runs the batch as parts on separate HIP streams.  Images are independent and every
    kernel's arithmetic per row is the same whatever the batch size, so the parts must reproduce
    the whole-batch result bit for bit (two pruning blocks, 8 images as 2 x 4)."""
    B, N, D, H, Dm, S = 8, 197, 192, 3, 768, 2
    sched = rs.keep_counts(N, 1, 2, dict(kind="drop_pct", pct=20, after=[1, 2]))
    x0 = to_dev(host_round(si.tokens(21, B, N, D, 0.3), "bf16"), "bf16")
    blocks, keep = [], []
    for l in range(2):
        w = {k: to_dev(host_round(v, "bf16"), "bf16") for k, v in si.block_weights(21, l, D, Dm, 0.05).items()}
        cfg = rs.make_cfg(B, N, D, H, Dm, 1, N - 1, torch.bfloat16)
        packed = torch.empty(rs.rs_packed_weights_size(cfg), dtype=torch.uint8, device="cuda")
        rs.rs_pack_weights(cfg, rs.make_weights(w), packed)
        keep.append((w, packed))
        blocks.append(rs.make_weights(w, packed))

    def forward(x, stream):
        Bx = x.shape[0]
        cfgs = [rs.make_cfg(Bx, n_in, D, H, Dm, 1, n_keep, torch.bfloat16) for n_in, n_keep in sched]
        ws = torch.empty(max(rs.rs_block_workspace_size(c) for c in cfgs), dtype=torch.uint8, device="cuda")
        bufs = [torch.zeros((Bx, N, D), device="cuda", dtype=torch.bfloat16) for _ in range(2)]
        kepts = [torch.zeros((Bx, N), device="cuda", dtype=torch.int32) for _ in range(2)]
        src = x
        for l in range(2):
            rs.rs_block_fwd(cfgs[l], blocks[l], src, bufs[l], kepts[l], None, ws, stream)
            src = bufs[l]
        return bufs, kepts, ws

    torch.cuda.synchronize()
    whole_b, whole_k, _ws = forward(x0, torch.cuda.current_stream())
    streams = [torch.cuda.Stream() for _ in range(S)]
    Bp = B // S
    outs = [forward(x0[i * Bp:(i + 1) * Bp], streams[i]) for i in range(S)]
    torch.cuda.synchronize()
    for l, (n_in, n_keep) in enumerate(sched):
        K = 1 + n_keep
        for i in range(S):
            part_y = outs[i][0][l].view(-1)[:Bp * K * D].view(Bp, K, D)
            part_k = outs[i][1][l].view(-1)[:Bp * K].view(Bp, K)
            whole_y = whole_b[l].view(-1)[:B * K * D].view(B, K, D)[i * Bp:(i + 1) * Bp]
            whole_kk = whole_k[l].view(-1)[:B * K].view(B, K)[i * Bp:(i + 1) * Bp]
            assert torch.equal(part_k, whole_kk), (l, i)
            assert torch.equal(part_y.view(torch.int16), whole_y.view(torch.int16)), (l, i)
