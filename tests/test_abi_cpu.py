"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol
the header declares, and rejects bad arguments before touching a device."""
import ctypes
import os
import re

import paper_2508_00367_amd as rs
from paper_2508_00367_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "rs.h")).read()
    return sorted(set(re.findall(r"RS_API[^;(]*?\b(rs_\w+)\s*\(", text)))


def test_header_symbols_exported():
    names = _declared()
    assert len(names) >= 9
    L = rs.lib()
    for n in names:
        assert hasattr(L, n), n
    assert set(names) == set(binding.EXPORTS)
    assert rs.rs_version() >= 100


def test_struct_layouts_match_header():
    # 13 pointers; 7 int32 + 2 float + 3 enums
    assert ctypes.sizeof(binding.RsBlockWeights) == 13 * 8
    assert ctypes.sizeof(binding.RsBlockCfg) == 12 * 4


def _cfg(**kw):
    base = dict(B=2, N=10, D=128, H=2, Dm=256, n_prefix=1, n_keep=4, dtype=rs.RS_BF16)
    base.update(kw)
    return rs.make_cfg(**base)


FAKE = 0x1000  # aligned, never dereferenced: every check below fails before any launch


def _weights(**kw):
    w = binding.RsBlockWeights()
    for name, _ in binding.RsBlockWeights._fields_:
        setattr(w, name, FAKE)
    for k, v in kw.items():
        setattr(w, k, v)
    return w


def test_block_rejects_bad_config():
    w = _weights()
    for kw, want in [(dict(H=3), rs.RS_ERR_INVALID_ARG),           # D not divisible by H
                     (dict(D=256, H=2), rs.RS_ERR_UNSUPPORTED),    # head width 128
                     (dict(Dm=100), rs.RS_ERR_UNSUPPORTED),
                     (dict(B=1, N=100000, D=4096, H=64, n_keep=0), rs.RS_ERR_UNSUPPORTED),  # QKV rows beyond 32-bit byte offsets
                     (dict(n_keep=10), rs.RS_ERR_INVALID_ARG),     # prefix + keep > N
                     (dict(n_prefix=-1), rs.RS_ERR_INVALID_ARG),
                     (dict(ln_eps=0.0), rs.RS_ERR_INVALID_ARG),
                     (dict(dtype=7), rs.RS_ERR_INVALID_ARG),
                     (dict(dist=9), rs.RS_ERR_INVALID_ARG),
                     (dict(op=5), rs.RS_ERR_INVALID_ARG),           # beyond the five shift operations
                     (dict(op=-1), rs.RS_ERR_INVALID_ARG),
                     (dict(B=70000, N=2, n_keep=1), rs.RS_ERR_UNSUPPORTED),   # beyond one launch-grid axis
                     (dict(Dm=1 << 21), rs.RS_ERR_UNSUPPORTED),      # fc2's K beyond a tile's 32-bit byte offsets
                     (dict(B=-1), rs.RS_ERR_INVALID_ARG)]:
        cfg = _cfg(**kw)
        st = rs.lib().rs_block_fwd(ctypes.byref(cfg), ctypes.byref(w), FAKE, FAKE * 2, FAKE * 3, None,
                                   FAKE * 16, 1 << 40, None)
        assert st == want, (kw, rs.rs_last_error())
        assert rs.rs_last_error() != ""
        assert rs.rs_block_workspace_size(cfg) == 0


def test_block_rejects_bad_pointers_and_workspace():
    cfg = _cfg()
    need = rs.rs_block_workspace_size(cfg)
    assert need > 0
    L = rs.lib()

    def call(w, x, y, kept, ws, ws_bytes):
        return L.rs_block_fwd(ctypes.byref(cfg), ctypes.byref(w), x, y, kept, None, ws, ws_bytes, None)

    w = _weights()
    assert call(w, FAKE, 2 * FAKE, 3 * FAKE, 16 * FAKE, need - 1) == rs.RS_ERR_WORKSPACE_TOO_SMALL
    assert "workspace" in rs.rs_last_error()
    assert call(w, None, 2 * FAKE, 3 * FAKE, 16 * FAKE, need) == rs.RS_ERR_INVALID_ARG
    assert call(w, FAKE, None, 3 * FAKE, 16 * FAKE, need) == rs.RS_ERR_INVALID_ARG
    assert call(w, FAKE, 2 * FAKE, None, 16 * FAKE, need) == rs.RS_ERR_INVALID_ARG
    assert call(w, FAKE, FAKE, 3 * FAKE, 16 * FAKE, need) == rs.RS_ERR_INVALID_ARG       # y aliases x
    assert call(w, FAKE + 4, 2 * FAKE, 3 * FAKE, 16 * FAKE, need) == rs.RS_ERR_INVALID_ARG  # misaligned
    assert call(w, FAKE, 2 * FAKE, 3 * FAKE, None, need) == rs.RS_ERR_INVALID_ARG
    assert call(w, FAKE, 2 * FAKE, 3 * FAKE, 16 * FAKE + 16, need) == rs.RS_ERR_INVALID_ARG  # ws alignment
    assert call(_weights(w_fc1=None), FAKE, 2 * FAKE, 3 * FAKE, 16 * FAKE, need) == rs.RS_ERR_INVALID_ARG
    assert L.rs_block_fwd(None, ctypes.byref(w), FAKE, FAKE, FAKE, None, FAKE, need, None) == rs.RS_ERR_INVALID_ARG
    assert L.rs_block_fwd(ctypes.byref(cfg), None, FAKE, 2 * FAKE, FAKE, None, FAKE, need, None) == rs.RS_ERR_INVALID_ARG
    # outputs (or the input) inside the workspace: the kernels would overwrite tensors still in use
    ws0 = 1 << 30
    assert call(w, FAKE, ws0 + 256, 3 * FAKE, ws0, need) == rs.RS_ERR_INVALID_ARG
    assert "outside the workspace" in rs.rs_last_error()
    assert call(w, FAKE, 2 * FAKE, ws0 + need - 16, ws0, need) == rs.RS_ERR_INVALID_ARG
    assert call(w, ws0 + 1024, 2 * FAKE, 3 * FAKE, ws0, need) == rs.RS_ERR_INVALID_ARG
    assert L.rs_block_fwd(ctypes.byref(cfg), ctypes.byref(w), FAKE, 2 * FAKE, 3 * FAKE, ws0 + 4096, ws0, need,
                          None) == rs.RS_ERR_INVALID_ARG      # scores
    # empty batch is a successful no-op that never reaches the device
    cfg0 = _cfg(B=0)
    assert L.rs_block_fwd(ctypes.byref(cfg0), ctypes.byref(w), None, None, None, None, None, 0, None) == rs.RS_OK


def test_chained_block_entry_validates_its_statistics_buffers():
    """rs_block_fwd_chained: x_stats / y_stats are checked like the other tensors, before any launch."""
    cfg = _cfg()
    need = rs.rs_block_workspace_size(cfg)
    L = rs.lib()
    w = _weights()
    ws0 = 1 << 30

    def call(xs, ys, y=2 * FAKE, kept=3 * FAKE):
        return L.rs_block_fwd_chained(ctypes.byref(cfg), ctypes.byref(w), FAKE, xs, y, ys, kept, None, ws0, need, None)

    assert call(ws0 + 512, None) == rs.RS_ERR_INVALID_ARG          # x_stats inside the workspace
    assert "outside the workspace" in rs.rs_last_error()
    assert call(None, ws0 + need - 8) == rs.RS_ERR_INVALID_ARG     # y_stats inside the workspace
    assert call(None, 2 * FAKE + 64) == rs.RS_ERR_INVALID_ARG      # y_stats overlaps y
    assert "y_stats" in rs.rs_last_error()
    assert call(None, 3 * FAKE) == rs.RS_ERR_INVALID_ARG           # y_stats overlaps kept_idx
    assert call(None, FAKE + 16) == rs.RS_ERR_INVALID_ARG          # y_stats overlaps x
    assert call(5 * FAKE + 4, None) == rs.RS_ERR_INVALID_ARG       # misaligned
    assert call(None, 5 * FAKE + 4) == rs.RS_ERR_INVALID_ARG
    cfg0 = _cfg(B=0)
    assert L.rs_block_fwd_chained(ctypes.byref(cfg0), ctypes.byref(w), None, None, None, None, None, None, None, 0,
                                  None) == rs.RS_OK


def test_attention_rejects_bad_arguments():
    L = rs.lib()

    def call(q=FAKE, k=2 * FAKE, v=3 * FAKE, o=4 * FAKE, B=1, H=1, N=4, dh=64, sn=64, scale=0.125, dt=rs.RS_BF16):
        return L.rs_attention_fwd(q, k, v, o, B, H, N, dh, N * sn, sn, 64, N * sn, sn, 64, scale, dt, None)

    assert call(dh=128) == rs.RS_ERR_UNSUPPORTED
    assert call(dh=0) == rs.RS_ERR_INVALID_ARG
    assert call(q=None) == rs.RS_ERR_INVALID_ARG
    assert call(o=FAKE) == rs.RS_ERR_INVALID_ARG          # aliases q
    assert call(q=FAKE + 2) == rs.RS_ERR_INVALID_ARG
    assert call(sn=60) == rs.RS_ERR_INVALID_ARG
    assert call(scale=0.0) == rs.RS_ERR_INVALID_ARG
    assert call(dt=5) == rs.RS_ERR_INVALID_ARG
    assert call(B=-2) == rs.RS_ERR_INVALID_ARG
    assert call(N=0) == rs.RS_OK and call(B=0, q=None) == rs.RS_OK
    assert call(N=1 << 20, sn=1024) == rs.RS_ERR_UNSUPPORTED    # K/V rows of a head beyond 32-bit byte offsets
    assert "2 GiB" in rs.rs_last_error()
    assert call(sn=60) == rs.RS_ERR_INVALID_ARG
    assert "stride" in rs.rs_last_error() or rs.rs_last_error() != ""


def test_attention_map_rejects_bad_arguments():
    L = rs.lib()
    need = rs.rs_attention_map_workspace_size(1, 2, 70)
    assert need > 0 and rs.rs_attention_map_size(1, 2, 70) == 1 * 2 * 70 * 128 * 2

    def call(q=FAKE, k=2 * FAKE, v=3 * FAKE, o=4 * FAKE, B=1, H=2, N=70, dh=64, sn=128, scale=0.125, dt=rs.RS_BF16,
             cls=0, amap=5 * FAKE, ws=16 * FAKE, wsb=None):
        return L.rs_attention_map_fwd(q, k, v, o, B, H, N, dh, N * sn, sn, 64, N * sn, sn, 64, scale, dt, cls, amap,
                                      None, None, ws, need if wsb is None else wsb, None)

    assert call(dt=rs.RS_F32) == rs.RS_ERR_UNSUPPORTED
    assert call(dh=32) == rs.RS_ERR_UNSUPPORTED
    assert call(B=300, H=300) == rs.RS_ERR_UNSUPPORTED       # B * H beyond one grid axis
    assert call(cls=70) == rs.RS_ERR_INVALID_ARG
    assert call(amap=None) == rs.RS_ERR_INVALID_ARG
    assert call(o=FAKE) == rs.RS_ERR_INVALID_ARG
    assert call(sn=60) == rs.RS_ERR_INVALID_ARG
    assert call(scale=-1.0) == rs.RS_ERR_INVALID_ARG
    assert call(wsb=need - 1) == rs.RS_ERR_WORKSPACE_TOO_SMALL
    assert call(ws=None) == rs.RS_ERR_INVALID_ARG
    assert call(N=0, q=None) == rs.RS_OK


def test_shift_topk_rejects_bad_arguments():
    L = rs.lib()

    def call(fo=FAKE, fi=2 * FAKE, src=None, B=2, N=8, D=64, P=1, K=3, dist=0, dt=rs.RS_BF16,
             sc=3 * FAKE, kept=4 * FAKE, g=5 * FAKE):
        return L.rs_shift_topk(fo, fi, src, B, N, D, P, K, dist, dt, sc, kept, g, None, 0, None)

    assert call(D=60) == rs.RS_ERR_INVALID_ARG
    assert call(P=5, K=4) == rs.RS_ERR_INVALID_ARG
    assert call(K=-1) == rs.RS_ERR_INVALID_ARG
    assert call(fo=None) == rs.RS_ERR_INVALID_ARG
    assert call(sc=None) == rs.RS_ERR_INVALID_ARG
    assert call(kept=None) == rs.RS_ERR_INVALID_ARG
    assert call(g=2 * FAKE) == rs.RS_ERR_INVALID_ARG       # gathered aliases src (= f_in)
    assert call(dist=4) == rs.RS_ERR_INVALID_ARG
    assert call(B=0, fo=None) == rs.RS_OK


def test_grid_line_prune_rejects_bad_arguments():
    L = rs.lib()

    def call(fo=FAKE, fi=2 * FAKE, src=None, B=2, H=6, W=5, C=16, R=4, Q=3, dist=0, dt=rs.RS_BF16,
             sc=3 * FAKE, rsc=4 * FAKE, csc=5 * FAKE, kr=6 * FAKE, kc=7 * FAKE, g=8 * FAKE):
        return L.rs_grid_line_prune(fo, fi, src, B, H, W, C, R, Q, dist, dt, sc, rsc, csc, kr, kc, g, None)

    assert call(C=12) == rs.RS_ERR_INVALID_ARG
    assert call(R=7) == rs.RS_ERR_INVALID_ARG              # more rows kept than there are
    assert call(Q=-1) == rs.RS_ERR_INVALID_ARG
    assert call(fi=None) == rs.RS_ERR_INVALID_ARG
    assert call(rsc=None) == rs.RS_ERR_INVALID_ARG
    assert call(kr=None) == rs.RS_ERR_INVALID_ARG
    assert call(g=FAKE) == rs.RS_ERR_INVALID_ARG           # gathered aliases src (= f_out)
    assert call(dist=3) == rs.RS_ERR_INVALID_ARG
    assert call(dt=5) == rs.RS_ERR_INVALID_ARG
    assert call(B=0, fo=None) == rs.RS_OK
    assert "keep_rows" in rs.rs_last_error() or rs.rs_last_error() != ""


def test_linear_rejects_bad_arguments():
    L = rs.lib()

    def call(a=FAKE, w=2 * FAKE, bias=None, res=None, out=3 * FAKE, M=10, N=128, K=128, epi=rs.RS_EPI_BIAS,
             dt=rs.RS_BF16):
        return L.rs_linear_fwd(a, w, bias, res, out, M, N, K, epi, dt, None)

    assert call(N=100) == rs.RS_ERR_UNSUPPORTED
    assert call(K=96) == rs.RS_ERR_UNSUPPORTED
    assert call(K=1 << 21) == rs.RS_ERR_UNSUPPORTED        # a tile's rows beyond 32-bit byte offsets
    assert call(M=1 << 31) == rs.RS_ERR_INVALID_ARG
    assert call(epi=rs.RS_EPI_BIAS_RES) == rs.RS_ERR_INVALID_ARG   # residual missing
    assert call(out=FAKE) == rs.RS_ERR_INVALID_ARG          # aliases a
    assert call(a=None) == rs.RS_ERR_INVALID_ARG
    assert call(epi=7) == rs.RS_ERR_INVALID_ARG
    assert call(M=0, a=None) == rs.RS_OK


def test_static_scratch_entry_validates_before_any_device_call():
    """rs_block_fwd_static: the size check and the configuration checks come before the first HIP call."""
    L = rs.lib()
    w = _weights()
    assert rs.rs_block_static_scratch_size() == 64 << 20
    big = _cfg(B=64, N=197, D=768, H=12, Dm=3072, n_keep=100)
    assert rs.rs_block_workspace_size(big) > rs.rs_block_static_scratch_size()
    assert L.rs_block_fwd_static(ctypes.byref(big), ctypes.byref(w), FAKE, 2 * FAKE, 3 * FAKE, None, None) == \
        rs.RS_ERR_UNSUPPORTED
    assert "static buffer" in rs.rs_last_error()
    bad = _cfg(H=3)
    assert L.rs_block_fwd_static(ctypes.byref(bad), ctypes.byref(w), FAKE, 2 * FAKE, 3 * FAKE, None, None) == \
        rs.RS_ERR_INVALID_ARG
    assert L.rs_block_fwd_static(None, ctypes.byref(w), FAKE, 2 * FAKE, 3 * FAKE, None, None) == rs.RS_ERR_INVALID_ARG
    empty = _cfg(B=0)
    assert L.rs_block_fwd_static(ctypes.byref(empty), ctypes.byref(w), None, None, None, None, None) == rs.RS_OK


def test_grid_token_prune_rejects_bad_arguments():
    L = rs.lib()

    def call(fo=FAKE, fi=2 * FAKE, src=None, B=2, H=6, W=5, C=16, R=4, Q=3, dist=0, dt=rs.RS_BF16,
             sc=3 * FAKE, kc=4 * FAKE, cs=5 * FAKE, kr=6 * FAKE, g=8 * FAKE):
        return L.rs_grid_token_prune(fo, fi, src, B, H, W, C, R, Q, dist, dt, sc, kc, cs, kr, g, None)

    assert call(C=20) == rs.RS_ERR_INVALID_ARG
    assert call(R=7) == rs.RS_ERR_INVALID_ARG
    assert call(Q=6) == rs.RS_ERR_INVALID_ARG
    assert call(fo=None) == rs.RS_ERR_INVALID_ARG
    assert call(sc=None) == rs.RS_ERR_INVALID_ARG
    assert call(kc=None) == rs.RS_ERR_INVALID_ARG
    assert call(cs=None) == rs.RS_ERR_INVALID_ARG
    assert call(kr=None) == rs.RS_ERR_INVALID_ARG
    assert call(g=FAKE) == rs.RS_ERR_INVALID_ARG           # gathered aliases src (= f_out)
    assert call(dist=5) == rs.RS_ERR_INVALID_ARG
    assert call(B=0, fo=None) == rs.RS_OK


def test_pack_weights_validation():
    cfg = _cfg()
    # four bf16 matrices plus, for the two LayerNorms folded into W_qkv and W_fc1, an fp32 column-sum
    # and bias vector each (every piece a multiple of 256 bytes here)
    assert rs.rs_packed_weights_size(cfg) == (3 * 128 * 128 + 128 * 128 + 2 * 128 * 256) * 2 + \
        2 * (3 * 128 + 256) * 4
    L = rs.lib()
    w = _weights()
    assert L.rs_pack_weights(ctypes.byref(cfg), ctypes.byref(w), None, None) == rs.RS_ERR_INVALID_ARG
    assert L.rs_pack_weights(ctypes.byref(cfg), None, FAKE, None) == rs.RS_ERR_INVALID_ARG
    cfg32 = _cfg(dtype=rs.RS_F32)
    assert rs.rs_packed_weights_size(cfg32) == 0
    assert L.rs_pack_weights(ctypes.byref(cfg32), ctypes.byref(w), None, None) == rs.RS_OK


def test_schedule_matches_workload_statement():
    import synth_inputs as si
    kc = rs.keep_counts(197, 1, 12, si.WORKLOADS["vit_b16"]["prune"])
    assert [n for n, _ in kc] == [197, 197, 197, 197, 178, 161, 145, 131, 118, 107, 97, 88]
    assert kc[3] == (197, 177) and kc[11] == (88, 87)
    kc = rs.keep_counts(197, 1, 1, si.WORKLOADS["vit_block_fp32"]["prune"])
    assert kc == [(197, 138)]
    lin, att = rs.forward_flops(197, 1, 768, 3072, 12, si.WORKLOADS["vit_b16"]["prune"])
    assert abs(lin / 1e9 - 25.664) < 1e-3 and abs(att / 1e9 - 0.902) < 1e-3
    # the product's schedule and the checker's agree (two independent implementations)
    from oracle import schedule as osch
    for name, wl in si.WORKLOADS.items():
        ours = [n for n, _ in rs.keep_counts(wl["N"], 1, wl["blocks"], wl["prune"])]
        assert ours == osch.tokens_per_block(wl["N"], 1, wl["blocks"], wl["prune"]), name


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    """No CPU or PyTorch fallback: without the built library every call raises."""
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "librs_hip.so"))
    import pytest
    with pytest.raises(ImportError, match="no fallback"):
        binding.lib()
    with pytest.raises(ImportError):
        rs.rs_version()
