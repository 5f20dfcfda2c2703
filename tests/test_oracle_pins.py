"""Pins of the fp64 CPU checker (oracle/) against what the paper and the mathematics fix.

None of these tests touches the HIP path.  Each pins one part of the checker to
something other than itself: a hand-worked value, a closed form, an invariant,
a brute-force enumeration, or a library routine of another code base
(numpy / scipy / torch CPU in fp64) on a case that reduces to it.
"""
import itertools
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle
import synth_inputs as si

RNG = np.random.default_rng(1234)


# ----------------------------------------------------------------------------
# Attention, Eq. (1) of Sec. 3.1
# ----------------------------------------------------------------------------
def test_attention_hand_worked_two_keys():
    # scale 1; logits row0 = [0, ln 3] -> P = [1/4, 3/4]; row1 = [0, 0] -> P = [1/2, 1/2]
    q = np.array([[1.0, 0.0], [0.0, 0.0]]).reshape(1, 2, 1, 2)
    k = np.array([[0.0, 5.0], [math.log(3.0), -7.0]]).reshape(1, 2, 1, 2)
    v = np.array([[1.0, 10.0], [5.0, -2.0]]).reshape(1, 2, 1, 2)
    o = oracle.attention(q, k, v, 1.0)[0, :, 0, :]
    np.testing.assert_allclose(o[0], [0.25 * 1 + 0.75 * 5, 0.25 * 10 + 0.75 * -2], rtol=1e-14)
    np.testing.assert_allclose(o[1], [3.0, 4.0], rtol=1e-14)


def test_attention_scale_enters_logits():
    # one query, two keys, logits = scale * [0, 2 ln 3]; scale = 1/2 -> P = [1/4, 3/4]
    q = np.array([[2.0]]).reshape(1, 1, 1, 1)
    q = np.concatenate([q, np.zeros_like(q)], axis=1)
    k = np.array([0.0, math.log(3.0)]).reshape(1, 2, 1, 1)
    v = np.array([0.0, 1.0]).reshape(1, 2, 1, 1)
    o = oracle.attention(q, k, v, 0.5)
    assert abs(o[0, 0, 0, 0] - 0.75) < 1e-14
    assert abs(o[0, 1, 0, 0] - 0.5) < 1e-14


def test_attention_closed_forms():
    B, N, H, dh = 2, 7, 3, 4
    q = RNG.standard_normal((B, N, H, dh))
    k = RNG.standard_normal((B, N, H, dh))
    v = RNG.standard_normal((B, N, H, dh))
    # identical keys -> uniform weights -> mean of V
    k_same = np.broadcast_to(k[:, :1], k.shape).copy()
    o = oracle.attention(q, k_same, v, 0.5)
    np.testing.assert_allclose(o, np.broadcast_to(v.mean(axis=1, keepdims=True), v.shape), atol=1e-14)
    # V = 1 -> rows of the map sum to one
    o = oracle.attention(q, k, np.ones_like(v), 0.5)
    np.testing.assert_allclose(o, 1.0, atol=1e-14)
    # N = 1 -> O = V
    o = oracle.attention(q[:, :1], k[:, :1], v[:, :1], 0.5)
    np.testing.assert_allclose(o, v[:, :1], atol=1e-15)
    # adding one vector c to every key shifts each row of logits by a constant
    c = RNG.standard_normal((1, 1, H, dh))
    np.testing.assert_allclose(oracle.attention(q, k + c, v, 0.5), oracle.attention(q, k, v, 0.5),
                               atol=1e-12)


def test_attention_no_overflow_on_huge_logits():
    q = np.array([[1e4, 0.0]]).reshape(1, 1, 1, 2)
    q = np.concatenate([q, -q], axis=1)
    k = np.array([[1.0, 0.0], [-1.0, 0.0]]).reshape(1, 2, 1, 2)
    v = np.array([[1.0, 2.0], [3.0, 4.0]]).reshape(1, 2, 1, 2)
    o = oracle.attention(q, k, v, 1.0)
    np.testing.assert_allclose(o[0, 0, 0], [1.0, 2.0], atol=1e-14)  # all mass on key 0
    np.testing.assert_allclose(o[0, 1, 0], [3.0, 4.0], atol=1e-14)  # all mass on key 1
    assert np.isfinite(o).all()


@pytest.mark.parametrize("shape", [(1, 5, 1, 3), (2, 9, 4, 8), (1, 33, 2, 64)])
def test_attention_against_torch_library(shape):
    B, N, H, dh = shape
    q, k, v = (RNG.standard_normal(shape) for _ in range(3))
    scale = 1.0 / math.sqrt(dh)
    o = oracle.attention(q, k, v, scale)
    tq, tk, tv = (torch.from_numpy(a).permute(0, 2, 1, 3) for a in (q, k, v))
    ref = F.scaled_dot_product_attention(tq, tk, tv, scale=scale).permute(0, 2, 1, 3).numpy()
    np.testing.assert_allclose(o, ref, rtol=1e-11, atol=1e-12)


def test_attention_heads_are_independent_slices():
    # head h of the multi-head call equals a single-head call on slice h (numpy softmax)
    B, N, H, dh = 1, 6, 3, 4
    q, k, v = (RNG.standard_normal((B, N, H, dh)) for _ in range(3))
    o = oracle.attention(q, k, v, 0.3)
    for h in range(H):
        s = 0.3 * q[0, :, h] @ k[0, :, h].T
        p = np.exp(s - s.max(axis=1, keepdims=True))
        p /= p.sum(axis=1, keepdims=True)
        np.testing.assert_allclose(o[0, :, h], p @ v[0, :, h], rtol=1e-12, atol=1e-13)


# ----------------------------------------------------------------------------
# LayerNorm and GELU
# ----------------------------------------------------------------------------
def test_layernorm_hand_worked():
    # [1,2,3,4]: mean 2.5, population variance 1.25
    x = np.array([[1.0, 2.0, 3.0, 4.0]])
    eps = 1e-6
    inv = 1.0 / math.sqrt(1.25 + eps)
    np.testing.assert_allclose(oracle.layernorm(x, eps=eps)[0],
                               [-1.5 * inv, -0.5 * inv, 0.5 * inv, 1.5 * inv], rtol=1e-15)
    g = np.array([2.0, 0.0, -1.0, 1.0])
    b = np.array([0.5, 7.0, 0.0, -1.0])
    np.testing.assert_allclose(oracle.layernorm(x, g, b, eps)[0],
                               [-3.0 * inv + 0.5, 7.0, -0.5 * inv, 1.5 * inv - 1.0], rtol=1e-15)


def test_layernorm_moments_and_library():
    x = RNG.standard_normal((5, 48)) * 3.0 + 1.7
    eps = 1e-6
    y = oracle.layernorm(x, eps=eps)
    np.testing.assert_allclose(y.mean(axis=1), 0.0, atol=1e-14)
    var = x.var(axis=1)
    np.testing.assert_allclose(y.var(axis=1), var / (var + eps), rtol=1e-12)
    g, b = RNG.standard_normal(48), RNG.standard_normal(48)
    ref = F.layer_norm(torch.from_numpy(x), (48,), torch.from_numpy(g), torch.from_numpy(b), eps).numpy()
    np.testing.assert_allclose(oracle.layernorm(x, g, b, eps), ref, rtol=1e-12, atol=1e-13)


def test_gelu_values():
    # x * Phi(x) with the standard normal CDF: Phi(1) = 0.8413447460685429, Phi(2) = 0.9772498680518208
    g = oracle.gelu(np.array([0.0, 1.0, -1.0, 2.0, -2.0, 10.0, -10.0]))
    np.testing.assert_allclose(g[:5], [0.0, 0.8413447460685429, -0.15865525393145707,
                                       1.9544997361036416, -0.045500263896358417], rtol=1e-14, atol=1e-16)
    assert abs(g[5] - 10.0) < 1e-12 and abs(g[6]) < 1e-12
    x = RNG.standard_normal(100) * 3
    np.testing.assert_allclose(oracle.gelu(x) - oracle.gelu(-x), x, atol=1e-14)  # odd part is x/2 * 2
    np.testing.assert_allclose(oracle.gelu(x), F.gelu(torch.from_numpy(x)).numpy(), rtol=1e-13, atol=1e-15)


def test_linear_orientation_in_by_out():
    # [Q,K,V] = xW with W in R^{C x 3C}: row vector times [in, out] matrix
    a = np.array([[1.0, 2.0]])
    w = np.array([[1.0, 10.0, 100.0], [2.0, 20.0, 200.0]])
    np.testing.assert_allclose(oracle.linear(a, w, np.array([0.5, 0.0, -1.0]))[0], [5.5, 50.0, 499.0])
    a = RNG.standard_normal((7, 5))
    w = RNG.standard_normal((5, 3))
    b = RNG.standard_normal(3)
    np.testing.assert_allclose(oracle.linear(a, w, b), a @ w + b, rtol=1e-13, atol=1e-14)


# ----------------------------------------------------------------------------
# Block wiring, Eqs. (5), (6)
# ----------------------------------------------------------------------------
def _weights(D, Dm, seed=0, std=0.2):
    return {k: v.astype(np.float64) for k, v in si.block_weights(seed, 0, D, Dm, std).items()}


def test_block_zero_projection_leaves_residual():
    B, N, D, H, Dm = 2, 5, 8, 2, 16
    x = RNG.standard_normal((B, N, D))
    w = _weights(D, Dm)
    w["w_proj"][:] = 0
    w["b_proj"][:] = 0
    r = oracle.block(x, w, H)
    np.testing.assert_array_equal(r["x1"], x)


def test_block_zero_fc2_score_is_norm_of_residual():
    B, N, D, H, Dm = 2, 5, 8, 2, 16
    x = RNG.standard_normal((B, N, D))
    w = _weights(D, Dm)
    w["w_fc2"][:] = 0
    w["b_fc2"][:] = 0
    r = oracle.block(x, w, H)
    np.testing.assert_array_equal(r["xhat"], r["x1"])
    np.testing.assert_array_equal(r["mlp"], 0.0)
    np.testing.assert_allclose(r["scores"], np.linalg.norm(r["x1"], axis=-1), rtol=1e-14)
    # constant MLP output c: score is ||c - x1|| (sign of the difference does not matter, offset does)
    c = RNG.standard_normal(D)
    w["b_fc2"][:] = c
    r = oracle.block(x, w, H)
    np.testing.assert_allclose(r["scores"], np.linalg.norm(c - r["x1"], axis=-1), rtol=1e-13)
    np.testing.assert_allclose(r["xhat"], r["x1"] + c, rtol=1e-14)


def test_block_uniform_attention_closed_form():
    # W_q = W_k = 0 and zero q/k bias: every attention row is uniform, so
    # SA(u)_i = (mean_n u_n W_v + b_v) W_proj + b_proj for every token i.
    B, N, D, H, Dm = 2, 6, 8, 2, 16
    x = RNG.standard_normal((B, N, D))
    w = _weights(D, Dm)
    w["w_qkv"][:, :2 * D] = 0
    w["b_qkv"][:2 * D] = 0
    w["ln1_g"] = RNG.standard_normal(D)
    w["ln1_b"] = RNG.standard_normal(D)
    r = oracle.block(x, w, H)
    u = F.layer_norm(torch.from_numpy(x), (D,), torch.from_numpy(w["ln1_g"]),
                     torch.from_numpy(w["ln1_b"]), 1e-6).numpy()
    vbar = u.mean(axis=1, keepdims=True) @ w["w_qkv"][:, 2 * D:] + w["b_qkv"][2 * D:]
    np.testing.assert_allclose(r["x1"], x + vbar @ w["w_proj"] + w["b_proj"], rtol=1e-12, atol=1e-13)


@pytest.mark.parametrize("dims", [(1, 4, 8, 1, 12), (2, 9, 16, 2, 40), (1, 17, 128, 2, 96)])
def test_block_against_torch_library(dims):
    """Whole block composed of torch CPU library ops in fp64 (layer_norm, linear,
    scaled_dot_product_attention, gelu)."""
    B, N, D, H, Dm = dims
    x = RNG.standard_normal((B, N, D))
    w = _weights(D, Dm, seed=3)
    w["ln1_g"], w["ln1_b"] = RNG.standard_normal(D), RNG.standard_normal(D)
    w["ln2_g"], w["ln2_b"] = RNG.standard_normal(D), RNG.standard_normal(D)
    r = oracle.block(x, w, H, ln_eps=1e-5)
    t = {k: torch.from_numpy(v) for k, v in w.items()}
    tx = torch.from_numpy(x)
    u = F.layer_norm(tx, (D,), t["ln1_g"], t["ln1_b"], 1e-5)
    qkv = F.linear(u, t["w_qkv"].T, t["b_qkv"]).reshape(B, N, 3, H, D // H).permute(2, 0, 3, 1, 4)
    att = F.scaled_dot_product_attention(qkv[0], qkv[1], qkv[2]).permute(0, 2, 1, 3).reshape(B, N, D)
    x1 = tx + F.linear(att, t["w_proj"].T, t["b_proj"])
    v = F.layer_norm(x1, (D,), t["ln2_g"], t["ln2_b"], 1e-5)
    mlp = F.linear(F.gelu(F.linear(v, t["w_fc1"].T, t["b_fc1"])), t["w_fc2"].T, t["b_fc2"])
    np.testing.assert_allclose(r["x1"], x1.numpy(), rtol=1e-10, atol=1e-11)
    np.testing.assert_allclose(r["mlp"], mlp.numpy(), rtol=1e-10, atol=1e-11)
    np.testing.assert_allclose(r["xhat"], (x1 + mlp).numpy(), rtol=1e-10, atol=1e-11)
    np.testing.assert_allclose(r["scores"], torch.linalg.vector_norm(mlp - x1, dim=-1).numpy(), rtol=1e-10)


def test_block_null_biases_mean_zero():
    B, N, D, H, Dm = 1, 5, 8, 2, 16
    x = RNG.standard_normal((B, N, D))
    w = _weights(D, Dm)
    w0 = dict(w)
    for k in ("b_qkv", "b_proj", "b_fc1", "b_fc2", "ln1_b", "ln2_b"):
        w0[k] = np.zeros_like(w[k])
    wn = dict(w0)
    for k in ("b_qkv", "b_proj", "b_fc1", "b_fc2", "ln1_b", "ln2_b"):
        wn[k] = None
    a, b = oracle.block(x, w0, H), oracle.block(x, wn, H)
    for k in a:
        np.testing.assert_array_equal(a[k], b[k])


def test_block_scores_permutation_equivariant():
    # no positional term inside a block: permuting tokens permutes scores and outputs
    B, N, D, H, Dm = 2, 11, 16, 2, 32
    x = RNG.standard_normal((B, N, D))
    w = _weights(D, Dm, seed=5)
    perm = np.concatenate([[0], 1 + RNG.permutation(N - 1)])
    r, rp = oracle.block(x, w, H), oracle.block(x[:, perm], w, H)
    np.testing.assert_allclose(rp["scores"], r["scores"][:, perm], rtol=1e-11)
    np.testing.assert_allclose(rp["xhat"], r["xhat"][:, perm], rtol=1e-10, atol=1e-11)
    # kept sets map through the permutation
    k0 = oracle.topk(r["scores"], 1, 6)
    kp = oracle.topk(rp["scores"], 1, 6)
    for b in range(B):
        assert set(perm[kp[b]]) == set(k0[b])


# ----------------------------------------------------------------------------
# Operation choice (Sec. 3.3, cases (i)-(iii)) and the other readings of the MLP case
# ----------------------------------------------------------------------------
def test_operation_choice_closed_forms():
    B, N, D, H, Dm = 2, 5, 8, 2, 16
    x = RNG.standard_normal((B, N, D))
    c = RNG.standard_normal(D)
    # (i) attention: SA == c (zero projection, bias c)  =>  s_i = ||c - x_i||
    w = _weights(D, Dm)
    w["w_proj"][:] = 0
    w["b_proj"][:] = c
    r = oracle.block(x, w, H, op=oracle.OP_ATTN)
    np.testing.assert_allclose(r["sa"], np.broadcast_to(c, x.shape), rtol=0, atol=0)
    np.testing.assert_allclose(r["scores"], np.linalg.norm(c - x, axis=-1), rtol=1e-13)
    # (iii) whole block: both branches constant  =>  xhat - x = c + d for every token
    d = RNG.standard_normal(D)
    w["w_fc2"][:] = 0
    w["b_fc2"][:] = d
    r = oracle.block(x, w, H, op=oracle.OP_BLOCK)
    np.testing.assert_allclose(r["scores"], np.full((B, N), np.linalg.norm(c + d)), rtol=1e-12)
    r = oracle.block(x, w, H, op=oracle.OP_BLOCK, dist=oracle.DIST_L1)
    np.testing.assert_allclose(r["scores"], np.full((B, N), np.abs(c + d).sum()), rtol=1e-12)
    # residual stream before/after the MLP: xhat - x1 = d
    r = oracle.block(x, w, H, op=oracle.OP_MLP_STREAM)
    np.testing.assert_allclose(r["scores"], np.full((B, N), np.linalg.norm(d)), rtol=1e-12)
    # the MLP's own input and output with MLP == 0: s = ||LN(x1)|| = sqrt(D var / (var + eps)), gamma 1, beta 0
    w["b_fc2"][:] = 0
    w["ln2_g"][:] = 1
    w["ln2_b"][:] = 0
    r = oracle.block(x, w, H, op=oracle.OP_MLP_NORMED, ln_eps=1e-3)
    var = r["x1"].var(axis=-1)
    np.testing.assert_allclose(r["scores"], np.sqrt(D * var / (var + 1e-3)), rtol=1e-12)
    # identity-like block: nothing added on either branch  =>  case (iii) is exactly 0
    w["b_proj"][:] = 0
    r = oracle.block(x, w, H, op=oracle.OP_BLOCK)
    np.testing.assert_array_equal(r["scores"], 0.0)
    with pytest.raises(ValueError):
        oracle.block(x, w, H, op=7)


@pytest.mark.parametrize("dist", [0, 1, 2])
def test_operation_choice_against_torch_library(dist):
    """Every pair (f_out, f_in) rebuilt from torch CPU library ops in fp64, every distance from
    torch's own norm / cosine_similarity."""
    B, N, D, H, Dm = 2, 9, 16, 2, 40
    x = RNG.standard_normal((B, N, D))
    w = _weights(D, Dm, seed=11)
    w["ln2_g"], w["ln2_b"] = RNG.standard_normal(D), RNG.standard_normal(D)
    t = {k: torch.from_numpy(v) for k, v in w.items()}
    tx = torch.from_numpy(x)
    u = F.layer_norm(tx, (D,), t["ln1_g"], t["ln1_b"], 1e-6)
    qkv = F.linear(u, t["w_qkv"].T, t["b_qkv"]).reshape(B, N, 3, H, D // H).permute(2, 0, 3, 1, 4)
    att = F.scaled_dot_product_attention(qkv[0], qkv[1], qkv[2]).permute(0, 2, 1, 3).reshape(B, N, D)
    sa = F.linear(att, t["w_proj"].T, t["b_proj"])
    x1 = tx + sa
    v = F.layer_norm(x1, (D,), t["ln2_g"], t["ln2_b"], 1e-6)
    mlp = F.linear(F.gelu(F.linear(v, t["w_fc1"].T, t["b_fc1"])), t["w_fc2"].T, t["b_fc2"])
    xhat = x1 + mlp
    pairs = {oracle.OP_MLP: (mlp, x1), oracle.OP_ATTN: (sa, tx), oracle.OP_BLOCK: (xhat, tx),
             oracle.OP_MLP_STREAM: (xhat, x1), oracle.OP_MLP_NORMED: (mlp, v)}
    for op, (fo, fi) in pairs.items():
        if dist == 0:
            want = torch.linalg.vector_norm(fo - fi, dim=-1)
        elif dist == 1:
            want = torch.linalg.vector_norm(fo - fi, ord=1, dim=-1)
        else:
            want = 1.0 - F.cosine_similarity(fo, fi, dim=-1, eps=0.0)
        r = oracle.block(x, w, H, dist=dist, op=op)
        np.testing.assert_allclose(r["scores"], want.numpy(), rtol=1e-9, atol=1e-12, err_msg="op %d" % op)


# ----------------------------------------------------------------------------
# Representation shift, Eq. (4), and the three distances of Sec. 3.3
# ----------------------------------------------------------------------------
def test_shift_identity_is_zero():
    x = RNG.standard_normal((3, 7, 20))
    for d in (oracle.DIST_L2, oracle.DIST_L1):
        np.testing.assert_array_equal(oracle.shift_scores(x, x, d), 0.0)
    np.testing.assert_allclose(oracle.shift_scores(x, x, oracle.DIST_COS), 0.0, atol=1e-15)


def test_shift_closed_forms():
    x = RNG.standard_normal((2, 5, 12))
    nrm = np.sqrt((x * x).sum(-1))
    np.testing.assert_allclose(oracle.shift_scores(2 * x, x), nrm, rtol=1e-14)       # F(x) = 2x
    np.testing.assert_allclose(oracle.shift_scores(-x, x), 2 * nrm, rtol=1e-14)
    e = np.zeros(12)
    e[3] = -2.5
    np.testing.assert_allclose(oracle.shift_scores(x + e, x), 2.5, rtol=1e-13)       # one coordinate moved
    np.testing.assert_allclose(oracle.shift_scores(x + e, x, oracle.DIST_L1), 2.5, rtol=1e-13)
    y = RNG.standard_normal(x.shape)
    np.testing.assert_allclose(oracle.shift_scores(-3 * y, -3 * x), 3 * oracle.shift_scores(y, x), rtol=1e-13)
    np.testing.assert_allclose(oracle.shift_scores(y, x), oracle.shift_scores(x, y), rtol=1e-15)
    # 3-4-5 triangle: L2 = 5, L1 = 7
    a = np.array([[3.0, 0.0, 4.0]])
    z = np.zeros((1, 3))
    assert oracle.shift_scores(a, z)[0] == 5.0
    assert oracle.shift_scores(a, z, oracle.DIST_L1)[0] == 7.0
    # cosine distance: parallel 0, orthogonal 1, opposite 2, scale invariant
    u = np.array([[1.0, 0.0], [1.0, 0.0], [1.0, 0.0], [1.0, 1.0]])
    w = np.array([[5.0, 0.0], [0.0, 3.0], [-2.0, 0.0], [1.0, 0.0]])
    np.testing.assert_allclose(oracle.shift_scores(u, w, oracle.DIST_COS),
                               [0.0, 1.0, 2.0, 1.0 - 1.0 / math.sqrt(2.0)], atol=1e-15)


# ----------------------------------------------------------------------------
# Selection and gather (Sec. 3.1: x~ in R^{(N-r) x C}; Sec. 3.2: drop the lowest k)
# ----------------------------------------------------------------------------
def _brute_force_keep(s, n_prefix, n_keep):
    """Enumerate every n_keep-subset; the right one maximises the score sum and,
    among equals, prefers lower indices (lexicographically smallest)."""
    N = len(s)
    best = None
    for comb in itertools.combinations(range(n_prefix, N), n_keep):
        key = (-sum(s[i] for i in comb), comb)
        if best is None or key < best[0]:
            best = (key, comb)
    return list(range(n_prefix)) + list(best[1])


@pytest.mark.parametrize("n_prefix,n_keep", [(1, 3), (0, 4), (2, 1), (1, 0), (1, 7)])
def test_topk_brute_force(n_prefix, n_keep):
    for trial in range(6):
        N = 8
        s = RNG.integers(0, 4, size=N).astype(float) if trial % 2 else RNG.standard_normal(N)
        got = oracle.topk(s[None], n_prefix, n_keep)[0]
        assert list(got) == _brute_force_keep(list(s), n_prefix, n_keep)


def test_topk_against_sorted_list():
    B, N, P, K = 3, 50, 1, 20
    s = np.round(RNG.standard_normal((B, N)), 1)  # many exact ties
    got = oracle.topk(s, P, K)
    for b in range(B):
        order = sorted(range(P, N), key=lambda i: (-s[b, i], i))
        assert list(got[b]) == sorted(list(range(P)) + order[:K])


def test_topk_special_cases():
    s = RNG.standard_normal((2, 9))
    np.testing.assert_array_equal(oracle.topk(s, 1, 8), np.tile(np.arange(9), (2, 1)))   # keep all
    np.testing.assert_array_equal(oracle.topk(s, 2, 0), np.tile(np.arange(2), (2, 1)))   # prefix only
    flat = np.ones((1, 9))
    np.testing.assert_array_equal(oracle.topk(flat, 1, 3)[0], [0, 1, 2, 3])            # ties: lowest index
    # the class token is kept even with the lowest score, and is not counted in n_keep
    s2 = np.array([[-100.0, 1.0, 5.0, 3.0, 4.0]])
    np.testing.assert_array_equal(oracle.topk(s2, 1, 2)[0], [0, 2, 4])
    # duplicated score at the threshold
    s3 = np.array([[9.0, 2.0, 7.0, 2.0, 2.0, 8.0]])
    np.testing.assert_array_equal(oracle.topk(s3, 0, 4)[0], [0, 1, 2, 5])


def test_gather_rows():
    src = RNG.standard_normal((2, 6, 3))
    kept = np.array([[0, 2, 5], [1, 3, 4]], np.int32)
    out = oracle.gather(src, kept)
    for b in range(2):
        for j in range(3):
            np.testing.assert_array_equal(out[b, j], src[b, kept[b, j]])


def test_shift_topk_composition_drops_lowest_shift():
    # tokens 1..N-1 move by a known amount each: the smallest movers are dropped
    B, N, D = 1, 8, 4
    x = RNG.standard_normal((B, N, D))
    amount = np.array([0.0, 0.3, 0.9, 0.1, 0.7, 0.5, 0.2, 0.8])
    f = x.copy()
    f[0, :, 1] += amount
    s, kept, y = oracle.shift_topk(f, x, None, 1, 4)
    np.testing.assert_allclose(s[0], amount, atol=1e-15)
    np.testing.assert_array_equal(kept[0], [0, 2, 4, 5, 7])
    np.testing.assert_array_equal(y[0], x[0, [0, 2, 4, 5, 7]])
    s, kept, y = oracle.shift_topk(f, x, f, 1, 4)
    np.testing.assert_array_equal(y[0], f[0, [0, 2, 4, 5, 7]])


# ----------------------------------------------------------------------------
# Line-wise pruning of a 2-D grid (Sec. 4.2, "CNN and SSM", variant (ii))
# ----------------------------------------------------------------------------
def test_grid_line_prune_closed_forms():
    B, H, W, C = 2, 5, 4, 8
    f_in = RNG.standard_normal((B, H, W, C))
    # the shift depends on the row only: row h moves by amp[h] along one channel
    amp = np.array([0.5, 3.0, 1.0, 2.0, 0.25])
    f_out = f_in.copy()
    f_out[..., 0] += amp[None, :, None]
    s, rs_, cs_, kr, kc, g = oracle.grid_line_prune(f_out, f_in, None, 3, 2)
    np.testing.assert_allclose(s, np.broadcast_to(amp[None, :, None], (B, H, W)), rtol=1e-12)
    np.testing.assert_allclose(rs_, np.broadcast_to(amp, (B, H)), rtol=1e-12)
    np.testing.assert_allclose(cs_, np.full((B, W), amp.mean()), rtol=1e-12)
    np.testing.assert_array_equal(kr, np.tile([1, 2, 3], (B, 1)))     # the three largest rows, ascending
    np.testing.assert_array_equal(kc, np.tile([0, 1], (B, 1)))        # all columns tie: lowest indices
    np.testing.assert_array_equal(g, f_out[:, [1, 2, 3]][:, :, [0, 1]])
    # keep everything: identity
    s, rs_, cs_, kr, kc, g = oracle.grid_line_prune(f_out, f_in, f_in, H, W)
    np.testing.assert_array_equal(g, f_in)


def test_grid_line_prune_against_numpy_sort():
    B, H, W, C = 3, 7, 6, 16
    f_in = RNG.standard_normal((B, H, W, C))
    f_out = f_in + RNG.standard_normal((B, H, W, C)) * np.exp(RNG.standard_normal((B, H, W, 1)))
    src = RNG.standard_normal((B, H, W, C))
    for dist in (0, 1, 2):
        s, rs_, cs_, kr, kc, g = oracle.grid_line_prune(f_out, f_in, src, 4, 3, dist)
        if dist == 0:
            want = np.linalg.norm(f_out - f_in, axis=-1)
        elif dist == 1:
            want = np.abs(f_out - f_in).sum(-1)
        else:
            want = 1 - (f_out * f_in).sum(-1) / (np.linalg.norm(f_out, axis=-1) * np.linalg.norm(f_in, axis=-1))
        np.testing.assert_allclose(s, want, rtol=1e-10)
        np.testing.assert_allclose(rs_, want.mean(axis=2), rtol=1e-12)
        np.testing.assert_allclose(cs_, want.mean(axis=1), rtol=1e-12)
        for b in range(B):
            np.testing.assert_array_equal(kr[b], np.sort(np.argsort(-want.mean(axis=2)[b], kind="stable")[:4]))
            np.testing.assert_array_equal(kc[b], np.sort(np.argsort(-want.mean(axis=1)[b], kind="stable")[:3]))
            np.testing.assert_array_equal(g[b], src[b][kr[b]][:, kc[b]])


# ----------------------------------------------------------------------------
# token-wise pruning of a 2-D grid (Sec. 4.2, CNN variant (i))
# ----------------------------------------------------------------------------
def _grid_case(seed, B, H, W, C):
    rng = np.random.default_rng(seed)
    f_in = rng.standard_normal((B, H, W, C))
    f_out = f_in + rng.standard_normal((B, H, W, C)) * np.exp(rng.standard_normal((B, H, W, 1)))
    return f_out, f_in


def test_grid_token_prune_against_sorting_by_hand():
    """Brute force with Python's sort on (-score, index) keys, written without the checker's own
    selection routine: per row keep the Q highest, then per compacted column the R highest."""
    B, H, W, C, R, Q = 2, 6, 7, 5, 4, 3
    f_out, f_in = _grid_case(1, B, H, W, C)
    s, kc, cs, kr, g = oracle.grid_token_prune(f_out, f_in, None, R, Q)
    for b in range(B):
        sc = np.sqrt(((f_out[b] - f_in[b]) ** 2).sum(-1))
        np.testing.assert_allclose(s[b], sc, rtol=1e-12)
        cols = [sorted(sorted(range(W), key=lambda w: (-sc[h, w], w))[:Q]) for h in range(H)]
        np.testing.assert_array_equal(kc[b], np.array(cols))
        for j in range(Q):
            col = [sc[h, cols[h][j]] for h in range(H)]
            np.testing.assert_allclose(cs[b, j], col, rtol=1e-12)
            rows = sorted(sorted(range(H), key=lambda h: (-col[h], h))[:R])
            np.testing.assert_array_equal(kr[b, j], rows)
            for i, r in enumerate(rows):
                np.testing.assert_array_equal(g[b, i, j], f_out[b, r, cols[r][j]])


def test_grid_token_prune_closed_forms():
    B, H, W, C = 1, 5, 6, 4
    f_in = np.zeros((B, H, W, C))
    # shift that depends on the column only: every row keeps the same columns (the Q largest
    # amplitudes), every compacted column then ties over the rows -> the first R rows survive
    amp = np.array([3.0, 1.0, 5.0, 2.0, 6.0, 4.0])
    f_out = np.zeros((B, H, W, C))
    f_out[..., 0] = amp[None, None, :]
    s, kc, cs, kr, g = oracle.grid_token_prune(f_out, f_in, None, 3, 4)
    np.testing.assert_array_equal(kc[0], np.tile([0, 2, 4, 5], (H, 1)))
    np.testing.assert_array_equal(kr[0], np.tile([0, 1, 2], (4, 1)))
    np.testing.assert_array_equal(g[0, :, :, 0], np.tile(amp[[0, 2, 4, 5]], (3, 1)))
    # shift that depends on the row only: rows tie inside -> the first Q columns; then the R largest rows
    ramp = np.array([2.0, 9.0, 1.0, 7.0, 3.0])
    f_out = np.zeros((B, H, W, C))
    f_out[..., 1] = ramp[None, :, None]
    s, kc, cs, kr, g = oracle.grid_token_prune(f_out, f_in, None, 2, 3)
    np.testing.assert_array_equal(kc[0], np.tile([0, 1, 2], (H, 1)))
    np.testing.assert_array_equal(kr[0], np.tile([1, 3], (3, 1)))
    # the same answer as the line-wise variant in these two separable cases
    s2, r2, c2, kr2, kc2, g2 = oracle.grid_line_prune(f_out, f_in, None, 2, 3)
    np.testing.assert_array_equal(g, g2)
    # keep everything: identity
    f_out, f_in = _grid_case(2, 2, 4, 3, 8)
    s, kc, cs, kr, g = oracle.grid_token_prune(f_out, f_in, None, 4, 3)
    np.testing.assert_array_equal(g, f_out)
    np.testing.assert_array_equal(kc, np.tile(np.arange(3), (2, 4, 1)))
    # a position with a large shift in an otherwise weak row survives step 1 and step 2, which
    # line-wise pruning would have dropped with its row
    f_in = np.zeros((1, 4, 4, 2))
    f_out = np.zeros((1, 4, 4, 2))
    f_out[0, :, :, 0] = np.array([[5, 5, 5, 5], [5, 5, 5, 5], [0.1, 0.1, 9.0, 0.1], [5, 5, 5, 5]])
    s, kc, cs, kr, g = oracle.grid_token_prune(f_out, f_in, None, 3, 3)
    assert 9.0 in g[0, :, :, 0]
    s2, r2, c2, kr2, kc2, g2 = oracle.grid_line_prune(f_out, f_in, None, 3, 3)
    assert 9.0 not in g2[0, :, :, 0]


# ----------------------------------------------------------------------------
# materialised attention map and attention-based scores (Sec. 3.1, Eqs. (2), (3))
# ----------------------------------------------------------------------------
def test_attention_map_and_scores():
    rng = np.random.default_rng(5)
    B, N, H, dh = 2, 9, 3, 8
    q, k, v = (rng.standard_normal((B, N, H, dh)) for _ in range(3))
    o, A = oracle.attention_map(q, k, v, 0.3)
    # the output is the fused definition's (the C routine, written independently of the numpy one)
    np.testing.assert_allclose(o, oracle.attention(q, k, v, 0.3), rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(A.sum(-1), 1.0, rtol=1e-13)
    s_cls, s_mean = oracle.attention_scores(A, cls_index=0)
    # each row of A is a distribution over keys, so both scores are distributions over tokens
    np.testing.assert_allclose(s_cls.sum(-1), 1.0, rtol=1e-13)
    np.testing.assert_allclose(s_mean.sum(-1), 1.0, rtol=1e-13)
    # written out by hand for one token
    b, j = 1, 4
    want_cls = np.mean([A[b, h, 0, j] for h in range(H)])
    want_mean = np.mean([A[b, h, i, j] for h in range(H) for i in range(N)])
    assert abs(s_cls[b, j] - want_cls) < 1e-15 and abs(s_mean[b, j] - want_mean) < 1e-15
    # another class-token position
    s_cls3, _ = oracle.attention_scores(A, cls_index=3)
    np.testing.assert_allclose(s_cls3, A[:, :, 3, :].mean(1), rtol=1e-15)


def test_attention_scores_closed_forms():
    B, N, H, dh = 1, 6, 2, 4
    rng = np.random.default_rng(6)
    q = rng.standard_normal((B, N, H, dh))
    v = rng.standard_normal((B, N, H, dh))
    # identical keys: uniform attention, every token scores 1/N under both definitions
    k = np.broadcast_to(rng.standard_normal((B, 1, H, dh)), (B, N, H, dh)).copy()
    _, A = oracle.attention_map(q, k, v, 0.5)
    s_cls, s_mean = oracle.attention_scores(A)
    np.testing.assert_allclose(s_cls, 1.0 / N, rtol=1e-12)
    np.testing.assert_allclose(s_mean, 1.0 / N, rtol=1e-12)
    # hand-worked two-key case: logits ln 1 and ln 3 for every query -> P = [1/4, 3/4]
    q2 = np.zeros((1, 2, 1, 2)); q2[..., 0] = 1.0
    k2 = np.zeros((1, 2, 1, 2)); k2[0, 0, 0, 0] = np.log(1.0); k2[0, 1, 0, 0] = np.log(3.0)
    _, A2 = oracle.attention_map(q2, k2, np.ones((1, 2, 1, 2)), 1.0)
    s_cls, s_mean = oracle.attention_scores(A2)
    np.testing.assert_allclose(s_cls[0], [0.25, 0.75], rtol=1e-13)
    np.testing.assert_allclose(s_mean[0], [0.25, 0.75], rtol=1e-13)
    # one key that every query prefers by a wide margin takes (almost) all of both scores
    k3 = rng.standard_normal((B, N, H, dh)) * 0.01
    q3 = np.ones((B, N, H, dh))
    k3[0, 2] = 50.0
    _, A3 = oracle.attention_map(q3, k3, v, 1.0)
    s_cls, s_mean = oracle.attention_scores(A3)
    assert s_cls[0, 2] > 1 - 1e-9 and s_mean[0, 2] > 1 - 1e-9
