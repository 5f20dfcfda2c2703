"""ctypes binding of librs_hip.so: same names as include/rs.h, argument marshalling only.

PyTorch is used for device memory (tensor.data_ptr()) and the current stream; every step of
the computation runs inside the HIP library.  There is no CPU or PyTorch fallback: if the
library is missing or fails to load, importing the calls raises.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "librs_hip.so")

RS_OK, RS_ERR_INVALID_ARG, RS_ERR_UNSUPPORTED, RS_ERR_WORKSPACE_TOO_SMALL, RS_ERR_DEVICE = range(5)
RS_F32, RS_BF16 = 0, 1
RS_DIST_L2, RS_DIST_L1, RS_DIST_COS = 0, 1, 2
RS_SHIFT_MLP, RS_SHIFT_ATTN, RS_SHIFT_BLOCK, RS_SHIFT_MLP_STREAM, RS_SHIFT_MLP_NORMED = 0, 1, 2, 3, 4

RS_PROFILE_CLASSES = 11
RS_EPI_BIAS, RS_EPI_BIAS_GELU, RS_EPI_BIAS_RES = 0, 1, 2

EXPORTS = ("rs_last_error", "rs_version", "rs_build_info", "rs_tune_gemm_variant", "rs_profile_enable", "rs_profile_read",
           "rs_profile_class_name", "rs_attention_fwd", "rs_attention_map_size",
           "rs_attention_map_workspace_size", "rs_attention_map_fwd", "rs_shift_topk_workspace_size",
           "rs_shift_topk", "rs_grid_line_prune", "rs_grid_token_prune", "rs_pack_linear", "rs_linear_fwd", "rs_packed_weights_size", "rs_pack_weights", "rs_block_workspace_size",
           "rs_block_fwd", "rs_block_fwd_chained", "rs_block_static_scratch_size", "rs_block_fwd_static")

_vp = ctypes.c_void_p
_i32 = ctypes.c_int32
_i64 = ctypes.c_int64


class RsBlockWeights(ctypes.Structure):
    _fields_ = [(n, _vp) for n in ("ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_proj", "b_proj",
                                   "ln2_g", "ln2_b", "w_fc1", "b_fc1", "w_fc2", "b_fc2", "packed")]


class RsBlockCfg(ctypes.Structure):
    _fields_ = [("B", _i32), ("N", _i32), ("D", _i32), ("H", _i32), ("Dm", _i32),
                ("n_prefix", _i32), ("n_keep", _i32), ("ln_eps", ctypes.c_float),
                ("attn_scale", ctypes.c_float), ("dtype", ctypes.c_int), ("dist", ctypes.c_int),
                ("op", ctypes.c_int)]


class RsError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__("rs status %d: %s" % (status, message))
        self.status = status


_lib = None


def lib():
    """Load librs_hip.so (built in-tree by build.py); loud failure if absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError("%s not found: run `python -m paper_2508_00367_amd.build` "
                              "(the HIP library has no fallback)" % LIB_PATH)
        L = ctypes.CDLL(LIB_PATH)
        L.rs_last_error.restype = ctypes.c_char_p
        L.rs_version.restype = _i32
        L.rs_build_info.restype = ctypes.c_char_p
        L.rs_tune_gemm_variant.argtypes = [_i32]
        L.rs_tune_gemm_variant.restype = ctypes.c_int
        L.rs_profile_enable.argtypes = [_i32]
        L.rs_profile_enable.restype = ctypes.c_int
        L.rs_profile_read.argtypes = [ctypes.POINTER(ctypes.c_double), ctypes.POINTER(_i64)]
        L.rs_profile_read.restype = ctypes.c_int
        L.rs_profile_class_name.argtypes = [_i32]
        L.rs_profile_class_name.restype = ctypes.c_char_p
        L.rs_attention_fwd.argtypes = [_vp, _vp, _vp, _vp, _i32, _i32, _i32, _i32] + [_i64] * 6 + \
            [ctypes.c_float, ctypes.c_int, _vp]
        L.rs_attention_fwd.restype = ctypes.c_int
        L.rs_attention_map_size.argtypes = [_i32, _i32, _i32]
        L.rs_attention_map_size.restype = ctypes.c_size_t
        L.rs_attention_map_workspace_size.argtypes = [_i32, _i32, _i32]
        L.rs_attention_map_workspace_size.restype = ctypes.c_size_t
        L.rs_attention_map_fwd.argtypes = [_vp, _vp, _vp, _vp, _i32, _i32, _i32, _i32] + [_i64] * 6 + \
            [ctypes.c_float, ctypes.c_int, _i32, _vp, _vp, _vp, _vp, ctypes.c_size_t, _vp]
        L.rs_attention_map_fwd.restype = ctypes.c_int
        L.rs_shift_topk_workspace_size.argtypes = [_i32, _i32, _i32, ctypes.c_int]
        L.rs_shift_topk_workspace_size.restype = ctypes.c_size_t
        L.rs_shift_topk.argtypes = [_vp, _vp, _vp, _i32, _i32, _i32, _i32, _i32, ctypes.c_int,
                                    ctypes.c_int, _vp, _vp, _vp, _vp, ctypes.c_size_t, _vp]
        L.rs_shift_topk.restype = ctypes.c_int
        L.rs_pack_linear.argtypes = [_vp, _vp, _i32, _i32, ctypes.c_int, _vp]
        L.rs_pack_linear.restype = ctypes.c_int
        L.rs_grid_line_prune.argtypes = [_vp, _vp, _vp, _i32, _i32, _i32, _i32, _i32, _i32, ctypes.c_int, ctypes.c_int,
                                         _vp, _vp, _vp, _vp, _vp, _vp, _vp]
        L.rs_grid_line_prune.restype = ctypes.c_int
        L.rs_grid_token_prune.argtypes = [_vp, _vp, _vp, _i32, _i32, _i32, _i32, _i32, _i32, ctypes.c_int, ctypes.c_int,
                                          _vp, _vp, _vp, _vp, _vp, _vp]
        L.rs_grid_token_prune.restype = ctypes.c_int
        L.rs_linear_fwd.argtypes = [_vp, _vp, _vp, _vp, _vp, _i64, _i32, _i32, ctypes.c_int, ctypes.c_int, _vp]
        L.rs_linear_fwd.restype = ctypes.c_int
        L.rs_packed_weights_size.argtypes = [ctypes.POINTER(RsBlockCfg)]
        L.rs_packed_weights_size.restype = ctypes.c_size_t
        L.rs_pack_weights.argtypes = [ctypes.POINTER(RsBlockCfg), ctypes.POINTER(RsBlockWeights), _vp, _vp]
        L.rs_pack_weights.restype = ctypes.c_int
        L.rs_block_workspace_size.argtypes = [ctypes.POINTER(RsBlockCfg)]
        L.rs_block_workspace_size.restype = ctypes.c_size_t
        L.rs_block_fwd.argtypes = [ctypes.POINTER(RsBlockCfg), ctypes.POINTER(RsBlockWeights),
                                   _vp, _vp, _vp, _vp, _vp, ctypes.c_size_t, _vp]
        L.rs_block_fwd.restype = ctypes.c_int
        L.rs_block_fwd_chained.argtypes = [ctypes.POINTER(RsBlockCfg), ctypes.POINTER(RsBlockWeights),
                                           _vp, _vp, _vp, _vp, _vp, _vp, _vp, ctypes.c_size_t, _vp]
        L.rs_block_fwd_chained.restype = ctypes.c_int
        L.rs_block_static_scratch_size.argtypes = []
        L.rs_block_static_scratch_size.restype = ctypes.c_size_t
        L.rs_block_fwd_static.argtypes = [ctypes.POINTER(RsBlockCfg), ctypes.POINTER(RsBlockWeights),
                                          _vp, _vp, _vp, _vp, _vp]
        L.rs_block_fwd_static.restype = ctypes.c_int
        _lib = L
    return _lib


def rs_last_error() -> str:
    return lib().rs_last_error().decode()


def _check(status: int) -> None:
    if status != RS_OK:
        raise RsError(status, rs_last_error())


def _ptr(t):
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream=None):
    if stream is None:
        return torch.cuda.current_stream().cuda_stream if torch.cuda.is_available() else None
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else stream


def dtype_code(t: torch.dtype) -> int:
    if t == torch.float32:
        return RS_F32
    if t == torch.bfloat16:
        return RS_BF16
    raise TypeError("unsupported dtype %s" % t)


def make_cfg(B, N, D, H, Dm, n_prefix, n_keep, dtype, ln_eps=1e-6, attn_scale=0.0,
             dist=RS_DIST_L2, op=RS_SHIFT_MLP) -> RsBlockCfg:
    code = dtype if isinstance(dtype, int) else dtype_code(dtype)
    return RsBlockCfg(B, N, D, H, Dm, n_prefix, n_keep, ln_eps, attn_scale, code, dist, op)


def make_weights(w: dict, packed=None) -> RsBlockWeights:
    """w: name -> device tensor (or None) for the twelve block tensors."""
    s = RsBlockWeights()
    for name, _ in RsBlockWeights._fields_:
        setattr(s, name, _ptr(packed if name == "packed" else w.get(name)))
    return s


# ---- the calls of include/rs.h ------------------------------------------------
def rs_version() -> int:
    return int(lib().rs_version())


def rs_build_info() -> str:
    return lib().rs_build_info().decode()


def rs_tune_gemm_variant(variant: int) -> None:
    _check(lib().rs_tune_gemm_variant(int(variant)))


def rs_profile_enable(enable: bool) -> None:
    _check(lib().rs_profile_enable(1 if enable else 0))


def rs_profile_read() -> dict:
    """{class name: (milliseconds, launches)} since the last read; waits for the events."""
    ms = (ctypes.c_double * RS_PROFILE_CLASSES)()
    n = (_i64 * RS_PROFILE_CLASSES)()
    _check(lib().rs_profile_read(ms, n))
    return {lib().rs_profile_class_name(i).decode(): (ms[i], n[i]) for i in range(RS_PROFILE_CLASSES)}


def rs_attention_fwd(q, k, v, o, scale, stream=None) -> None:
    """q, k, v, o: [B, N, H, dh] tensors (any strides with contiguous dh; q, k, v share strides)."""
    B, N, H, dh = q.shape
    assert k.shape == q.shape and v.shape == q.shape and o.shape == q.shape
    assert q.stride() == k.stride() == v.stride() and q.stride(3) == 1 and o.stride(3) == 1
    _check(lib().rs_attention_fwd(_ptr(q), _ptr(k), _ptr(v), _ptr(o), B, H, N, dh,
                                  q.stride(0), q.stride(1), q.stride(2),
                                  o.stride(0), o.stride(1), o.stride(2),
                                  float(scale), dtype_code(q.dtype), _stream(stream)))


def rs_attention_map_size(B, H, N) -> int:
    return int(lib().rs_attention_map_size(B, H, N))


def rs_attention_map_workspace_size(B, H, N) -> int:
    return int(lib().rs_attention_map_workspace_size(B, H, N))


def rs_attention_map_fwd(q, k, v, o, scale, attn_map, s_cls, s_mean, workspace, cls_index=0, stream=None) -> None:
    """Standard attention with the map written out: q, k, v, o as in rs_attention_fwd; attn_map bf16
    [B, H, N, Np]; s_cls / s_mean float [B, N] or None."""
    B, N, H, dh = q.shape
    assert q.stride() == k.stride() == v.stride() and q.stride(3) == 1 and o.stride(3) == 1
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().rs_attention_map_fwd(_ptr(q), _ptr(k), _ptr(v), _ptr(o), B, H, N, dh,
                                      q.stride(0), q.stride(1), q.stride(2), o.stride(0), o.stride(1), o.stride(2),
                                      float(scale), dtype_code(q.dtype), cls_index, _ptr(attn_map), _ptr(s_cls),
                                      _ptr(s_mean), _ptr(workspace), ws_bytes, _stream(stream)))


def rs_shift_topk_workspace_size(B, N, D, dtype) -> int:
    return int(lib().rs_shift_topk_workspace_size(B, N, D, dtype if isinstance(dtype, int) else dtype_code(dtype)))


def rs_shift_topk(f_out, f_in, src, n_prefix, n_keep, scores, kept_idx, gathered,
                  dist=RS_DIST_L2, workspace=None, stream=None) -> None:
    B, N, D = f_in.shape
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().rs_shift_topk(_ptr(f_out), _ptr(f_in), _ptr(src), B, N, D, n_prefix, n_keep, dist,
                               dtype_code(f_in.dtype), _ptr(scores), _ptr(kept_idx), _ptr(gathered),
                               _ptr(workspace), ws_bytes, _stream(stream)))


def rs_grid_line_prune(f_out, f_in, src, keep_rows, keep_cols, scores, row_scores, col_scores, kept_rows,
                       kept_cols, gathered, dist=RS_DIST_L2, stream=None) -> None:
    """Line-wise pruning of a [B, H, W, C] grid: keep the rows / columns with the highest mean shift."""
    B, H, W, C = f_in.shape
    _check(lib().rs_grid_line_prune(_ptr(f_out), _ptr(f_in), _ptr(src), B, H, W, C, keep_rows, keep_cols, dist,
                                    dtype_code(f_in.dtype), _ptr(scores), _ptr(row_scores), _ptr(col_scores),
                                    _ptr(kept_rows), _ptr(kept_cols), _ptr(gathered), _stream(stream)))


def rs_grid_token_prune(f_out, f_in, src, keep_rows, keep_cols, scores, kept_cols, col_scores, kept_rows, gathered,
                        dist=RS_DIST_L2, stream=None) -> None:
    """Token-wise pruning of a [B, H, W, C] grid: rows lose their lowest positions, then the compacted columns."""
    B, H, W, C = f_in.shape
    _check(lib().rs_grid_token_prune(_ptr(f_out), _ptr(f_in), _ptr(src), B, H, W, C, keep_rows, keep_cols, dist,
                                     dtype_code(f_in.dtype), _ptr(scores), _ptr(kept_cols), _ptr(col_scores),
                                     _ptr(kept_rows), _ptr(gathered), _stream(stream)))


def rs_pack_linear(w, wt, stream=None) -> None:
    """w [K, N] -> wt [N, K] (bf16; a no-op for fp32, whose GEMM reads w directly)."""
    K, N = w.shape
    _check(lib().rs_pack_linear(_ptr(w), _ptr(wt), K, N, dtype_code(w.dtype), _stream(stream)))


def rs_linear_fwd(a, w, bias, res, out, epi=RS_EPI_BIAS, stream=None) -> None:
    """out [M, N] = epilogue(a [M, K] @ W + bias); w is the packed [N, K] tensor for bf16, [K, N] for fp32."""
    M, K = a.shape
    N = out.shape[1]
    _check(lib().rs_linear_fwd(_ptr(a), _ptr(w), _ptr(bias), _ptr(res), _ptr(out), M, N, K, epi,
                               dtype_code(a.dtype), _stream(stream)))


def rs_packed_weights_size(cfg: RsBlockCfg) -> int:
    return int(lib().rs_packed_weights_size(ctypes.byref(cfg)))


def rs_pack_weights(cfg: RsBlockCfg, weights: RsBlockWeights, packed_out, stream=None) -> None:
    _check(lib().rs_pack_weights(ctypes.byref(cfg), ctypes.byref(weights), _ptr(packed_out), _stream(stream)))


def rs_block_workspace_size(cfg: RsBlockCfg) -> int:
    return int(lib().rs_block_workspace_size(ctypes.byref(cfg)))


def rs_block_fwd(cfg: RsBlockCfg, weights: RsBlockWeights, x, y, kept_idx, scores, workspace,
                 stream=None) -> None:
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().rs_block_fwd(ctypes.byref(cfg), ctypes.byref(weights), _ptr(x), _ptr(y), _ptr(kept_idx),
                              _ptr(scores), _ptr(workspace), ws_bytes, _stream(stream)))


def rs_block_fwd_chained(cfg: RsBlockCfg, weights: RsBlockWeights, x, x_stats, y, y_stats, kept_idx, scores,
                         workspace, stream=None) -> None:
    """rs_block_fwd that takes the row statistics of x from x_stats (float [B*N, 2] or None) and leaves
    those of y in y_stats (float [B*K, 2] or None)."""
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().rs_block_fwd_chained(ctypes.byref(cfg), ctypes.byref(weights), _ptr(x), _ptr(x_stats), _ptr(y),
                                      _ptr(y_stats), _ptr(kept_idx), _ptr(scores), _ptr(workspace), ws_bytes,
                                      _stream(stream)))


def rs_block_static_scratch_size() -> int:
    return int(lib().rs_block_static_scratch_size())


def rs_block_fwd_static(cfg: RsBlockCfg, weights: RsBlockWeights, x, y, kept_idx, scores, stream=None) -> None:
    """rs_block_fwd on the library's own static scratch buffer (no workspace, no allocation)."""
    _check(lib().rs_block_fwd_static(ctypes.byref(cfg), ctypes.byref(weights), _ptr(x), _ptr(y), _ptr(kept_idx),
                                     _ptr(scores), _stream(stream)))
