"""TEST INFRASTRUCTURE ONLY: numpy front end of the fp64 CPU checker (rs_oracle.c).

Only tests, the smoke check and the bench's cpu_baseline leg may import this
package.  It shares no code with the HIP path and never imports it.

Every function takes numpy arrays (any float dtype, widened to fp64 here) and
returns fp64 / int32 numpy arrays.

Every function is pinned in tests/test_oracle_pins.py / test_oracle_schedule.py against closed
forms, hand-worked cases, brute force or library routines.  Two READINGS of the paper have no
worked example to pin them against (the arithmetic of each reading is pinned, the choice is
not): which pair of tensors "the MLP shift" compares (OP_MLP is the printed formula of
"Operation choice"; OP_MLP_STREAM and OP_MLP_NORMED are the other two) -- parity unpinned --
and how token-wise grid pruning (Sec. 4.2, variant (i)) keeps the grid rectangular
(grid_token_prune) -- parity unpinned.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "rs_oracle.c")
_LIB = os.path.join(_HERE, "librs_oracle.so")

DIST_L2, DIST_L1, DIST_COS = 0, 1, 2
# which pair (f_out, f_in) the shift is taken over ("Operation choice", Sec. 3.3, and the two other
# readings of the MLP case): (MLP(LN(x1)), x1), (SA(LN(x)), x), (xhat, x), (xhat, x1), (MLP(v), v = LN(x1))
OP_MLP, OP_ATTN, OP_BLOCK, OP_MLP_STREAM, OP_MLP_NORMED = 0, 1, 2, 3, 4


def build(force: bool = False) -> str:
    """Compile rs_oracle.c with gcc -O2 -fopenmp into oracle/librs_oracle.so."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared",
                               _SRC, "-o", tmp, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None
_pd = ctypes.POINTER(ctypes.c_double)
_pi = ctypes.POINTER(ctypes.c_int32)
_i64 = ctypes.c_int64


def lib():
    global _lib
    if _lib is None:
        L = ctypes.CDLL(build())
        L.rs_oracle_num_threads.restype = ctypes.c_int
        L.rs_oracle_set_num_threads.argtypes = [ctypes.c_int]
        L.rs_oracle_layernorm.argtypes = [_pd, _pd, _pd, ctypes.c_double, _i64, _i64, _pd]
        L.rs_oracle_gelu.argtypes = [ctypes.c_double]
        L.rs_oracle_gelu.restype = ctypes.c_double
        L.rs_oracle_linear.argtypes = [_pd, _pd, _pd, _i64, _i64, _i64, _pd]
        L.rs_oracle_attention.argtypes = [_pd, _pd, _pd, _pd] + [_i64] * 10 + [ctypes.c_double]
        L.rs_oracle_shift_scores.argtypes = [_pd, _pd, _i64, _i64, ctypes.c_int, _pd]
        L.rs_oracle_topk.argtypes = [_pd, _i64, _i64, _i64, _i64, _pi]
        L.rs_oracle_gather.argtypes = [_pd, _pi, _i64, _i64, _i64, _i64, _pd]
        L.rs_oracle_block.argtypes = ([_i64] * 5 + [ctypes.c_double, ctypes.c_double, ctypes.c_int, ctypes.c_int]
                                      + [_pd] * 13 + [_pd] * 5)
        L.rs_oracle_block.restype = ctypes.c_int
        _lib = L
    return _lib


def num_threads() -> int:
    return int(lib().rs_oracle_num_threads())


def set_num_threads(n: int) -> None:
    lib().rs_oracle_set_num_threads(int(n))


def _d(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.float64)


def _p(a):
    return None if a is None else a.ctypes.data_as(_pd)


def layernorm(x, gamma=None, beta=None, eps=1e-6):
    x = _d(x)
    D = x.shape[-1]
    g, b = _d(gamma), _d(beta)
    out = np.empty_like(x)
    lib().rs_oracle_layernorm(_p(x), _p(g), _p(b), float(eps), x.size // D, D, _p(out))
    return out


def gelu(x):
    x = _d(x)
    f = lib().rs_oracle_gelu
    return np.array([f(float(t)) for t in x.ravel()]).reshape(x.shape)


def linear(a, w, bias=None):
    a, w, bias = _d(a), _d(w), _d(bias)
    K, N = w.shape
    M = a.size // K
    out = np.empty(a.shape[:-1] + (N,), np.float64)
    lib().rs_oracle_linear(_p(a), _p(w), _p(bias), M, K, N, _p(out))
    return out


def attention(q, k, v, scale):
    """q, k, v: [B, N, H, dh] -> o [B, N, H, dh]."""
    q, k, v = _d(q), _d(k), _d(v)
    B, N, H, dh = q.shape
    o = np.empty_like(q)
    lib().rs_oracle_attention(_p(q), _p(k), _p(v), _p(o), B, H, N, dh,
                              N * H * dh, H * dh, dh, N * H * dh, H * dh, dh, float(scale))
    return o


def attention_map(q, k, v, scale):
    """Standard (unfused) attention with the attention map written out, Sec. 3.1:
    A = Softmax(Q K^T * scale) per image and head, O = A V.
    q, k, v: [B, N, H, dh] -> (o [B, N, H, dh], A [B, H, N, N]).  numpy matmuls in fp64."""
    q, k, v = _d(q), _d(k), _d(v)
    S = np.einsum("bnhd,bmhd->bhnm", q, k) * float(scale)
    S = S - S.max(axis=-1, keepdims=True)
    P = np.exp(S)
    A = P / P.sum(axis=-1, keepdims=True)
    return np.einsum("bhnm,bmhd->bnhd", A, v), A


def attention_scores(A, cls_index=0):
    """Attention-based token importance from the map A [B, H, N, N] (Sec. 3.1):
    Eq. (2): the class token's attention row, s_j = A[cls, j];
    Eq. (3): the attentiveness summed over all queries, s_j = (1/N) sum_i A[i, j].
    The paper writes both for one head; with H heads the mean over heads is taken.
    Returns (s_cls [B, N], s_mean [B, N])."""
    A = _d(A)
    return A[:, :, cls_index, :].mean(axis=1), A.mean(axis=(1, 2))


def shift_scores(f_out, f_in, dist=DIST_L2):
    """f_out, f_in: [..., D] -> scores [...]."""
    a, b = _d(f_out), _d(f_in)
    D = a.shape[-1]
    s = np.empty(a.shape[:-1], np.float64)
    lib().rs_oracle_shift_scores(_p(a), _p(b), a.size // D, D, int(dist), _p(s))
    return s


def topk(scores, n_prefix, n_keep):
    """scores [B, N] -> kept_idx int32 [B, n_prefix + n_keep], ascending per image."""
    s = _d(scores)
    B, N = s.shape
    assert 0 <= n_prefix <= N and 0 <= n_keep <= N - n_prefix
    kept = np.empty((B, n_prefix + n_keep), np.int32)
    lib().rs_oracle_topk(_p(s), B, N, n_prefix, n_keep, kept.ctypes.data_as(_pi))
    return kept


def gather(src, kept_idx):
    """src [B, N, D], kept_idx [B, K] -> [B, K, D]."""
    src = _d(src)
    kept = np.ascontiguousarray(kept_idx, dtype=np.int32)
    B, N, D = src.shape
    K = kept.shape[1]
    out = np.empty((B, K, D), np.float64)
    lib().rs_oracle_gather(_p(src), kept.ctypes.data_as(_pi), B, N, K, D, _p(out))
    return out


def shift_topk(f_out, f_in, src, n_prefix, n_keep, dist=DIST_L2):
    """Scores, kept indices and gathered rows of `src` (f_in when src is None)."""
    s = shift_scores(f_out, f_in, dist)
    kept = topk(s, n_prefix, n_keep)
    return s, kept, gather(f_in if src is None else src, kept)


def grid_line_scores(scores):
    """Line-wise scores of a 2-D token grid (Sec. 4.2, "CNN and SSM", variant (ii)): the shift
    averaged along each row and along each column.  scores [B, H, W] -> ([B, H], [B, W]).
    Plain sequential sums in index order."""
    s = _d(scores)
    B, H, W = s.shape
    rows = np.zeros((B, H), np.float64)
    cols = np.zeros((B, W), np.float64)
    for w in range(W):
        rows += s[:, :, w]
    for h in range(H):
        cols += s[:, h, :]
    return rows / W, cols / H


def grid_line_prune(f_out, f_in, src, keep_rows, keep_cols, dist=DIST_L2):
    """Line-wise pruning of a [B, H, W, C] grid: per-position shift D(f_out, f_in) over the
    channels, averaged per row and per column; the keep_rows rows and keep_cols columns with
    the highest averages survive (ties: lower index; survivors in ascending order), and `src`
    (f_out when None: the stage output is what gets pruned) is cut down to them.

    Returns scores [B,H,W], row_scores [B,H], col_scores [B,W], kept_rows [B,keep_rows],
    kept_cols [B,keep_cols], gathered [B,keep_rows,keep_cols,C]."""
    a, b = _d(f_out), _d(f_in)
    B, H, W, C = a.shape
    s = shift_scores(a, b, dist)
    rs_, cs_ = grid_line_scores(s)
    kr = topk(rs_, 0, keep_rows)
    kc = topk(cs_, 0, keep_cols)
    g = grid_gather(a if src is None else src, kr, kc)
    return s, rs_, cs_, kr, kc, g


def grid_gather(src, kept_rows, kept_cols):
    """src [B, H, W, C] -> [B, R, Q, C] with out[b, i, j] = src[b, kept_rows[b, i], kept_cols[b, j]]."""
    src = _d(src)
    B = src.shape[0]
    out = np.empty((B, kept_rows.shape[1], kept_cols.shape[1], src.shape[3]), np.float64)
    for b_ in range(B):
        for i, r in enumerate(kept_rows[b_]):
            for j, c in enumerate(kept_cols[b_]):
                out[b_, i, j] = src[b_, r, c]
    return out


def grid_token_prune(f_out, f_in, src, keep_rows, keep_cols, dist=DIST_L2):
    """Token-wise pruning of a [B, H, W, C] grid (Sec. 4.2, "CNN and SSM", variant (i): the least
    important tokens are removed from each row and column).  Reading taken: first every ROW loses
    its W - keep_cols lowest-shift positions and closes up to the left (the grid becomes H x
    keep_cols, position j of row h being that row's j-th survivor); then every COLUMN of that
    compacted grid loses its H - keep_rows lowest-shift positions and closes up upwards.  Ties: the
    lower index survives; survivors keep their order.  `src` (f_out when None) is cut down the same way.

    Returns scores [B,H,W], kept_cols [B,H,Q] (per row, original column indices), col_scores [B,Q,H]
    (shift of the row-compacted grid, column by column), kept_rows [B,Q,R] (per compacted column, row
    indices), gathered [B,R,Q,C] with gathered[b,i,j] = src[b, r, kept_cols[b,r,j]], r = kept_rows[b,j,i]."""
    a, b = _d(f_out), _d(f_in)
    B, H, W, C = a.shape
    R, Q = int(keep_rows), int(keep_cols)
    s = shift_scores(a, b, dist)                                        # [B, H, W]
    kc = topk(s.reshape(B * H, W), 0, Q).reshape(B, H, Q)               # step 1: per row
    cs = np.empty((B, Q, H), np.float64)
    for b_ in range(B):
        for h in range(H):
            for j in range(Q):
                cs[b_, j, h] = s[b_, h, kc[b_, h, j]]
    kr = topk(cs.reshape(B * Q, H), 0, R).reshape(B, Q, R)              # step 2: per compacted column
    g = np.empty((B, R, Q, C), np.float64)
    sr = a if src is None else _d(src)
    for b_ in range(B):
        for i in range(R):
            for j in range(Q):
                r = kr[b_, j, i]
                g[b_, i, j] = sr[b_, r, kc[b_, r, j]]
    return s, kc, cs, kr, g


def block(x, w, H, ln_eps=1e-6, attn_scale=None, dist=DIST_L2, op=OP_MLP):
    """One encoder block on x [B, N, D] with weight dict `w` (missing/None bias = 0).

    Returns dict(sa, x1, mlp, xhat [B,N,D], scores [B,N]); `op` picks the pair the shift is taken over."""
    x = _d(x)
    B, N, D = x.shape
    Dm = w["w_fc1"].shape[1]
    if attn_scale is None:
        attn_scale = 1.0 / np.sqrt(D // H)
    ws = {k: _d(w.get(k)) for k in ("ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_proj", "b_proj",
                                     "ln2_g", "ln2_b", "w_fc1", "b_fc1", "w_fc2", "b_fc2")}
    assert ws["w_qkv"].shape == (D, 3 * D) and ws["w_proj"].shape == (D, D)
    assert ws["w_fc1"].shape == (D, Dm) and ws["w_fc2"].shape == (Dm, D)
    sa = np.empty_like(x)
    x1 = np.empty_like(x)
    mlp = np.empty_like(x)
    xhat = np.empty_like(x)
    s = np.empty((B, N), np.float64)
    rc = lib().rs_oracle_block(B, N, D, H, Dm, float(ln_eps), float(attn_scale), int(dist), int(op),
                               _p(x), *[_p(ws[k]) for k in
                                        ("ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_proj", "b_proj",
                                         "ln2_g", "ln2_b", "w_fc1", "b_fc1", "w_fc2", "b_fc2")],
                               _p(sa), _p(x1), _p(mlp), _p(xhat), _p(s))
    if rc == -2:
        raise ValueError("unknown shift operation %r" % (op,))
    if rc != 0:
        raise MemoryError("rs_oracle_block")
    return dict(sa=sa, x1=x1, mlp=mlp, xhat=xhat, scores=s)


def block_pruned(x, w, H, n_prefix, n_keep, **kw):
    """Block followed by selection and gather: adds kept_idx [B,K] and y [B,K,D]."""
    r = block(x, w, H, **kw)
    r["kept_idx"] = topk(r["scores"], n_prefix, n_keep)
    r["y"] = gather(r["xhat"], r["kept_idx"])
    return r
