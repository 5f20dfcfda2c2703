"""The entry point that allocates nothing (rs_block_fwd_static: scratch in a static device buffer of
the library) against rs_block_fwd with a caller workspace, through the C ABI: same kernels, so the
outputs must agree bit for bit, on two calls in a row, the second with a smaller input that
leaves most of the buffer holding the first call's data."""
import ctypes
import sys

import numpy as np
import pytest
import torch

import oracle
import paper_2508_00367_amd as rs
import synth_inputs as si
from rs_testlib import TOL, host_round, norm_err, to_dev, to_host

pytestmark = pytest.mark.gpu


def _case(seed, B, N, D, H, Dm, P, K, dtype):
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    x = host_round(si.tokens(seed, B, N, D, 0.3), dtype)
    w = {k: host_round(v, dtype) for k, v in si.block_weights(seed, 0, D, Dm, 0.05).items()}
    dw = {k: to_dev(v, dtype) for k, v in w.items()}
    dx = to_dev(x, dtype)
    cfg = rs.make_cfg(B, N, D, H, Dm, P, K, tdt)
    outs = []
    for _ in range(2):
        outs.append((torch.full((B, P + K, D), float("nan"), device="cuda", dtype=tdt),
                     torch.full((B, P + K), -1, device="cuda", dtype=torch.int32),
                     torch.full((B, N), float("nan"), device="cuda", dtype=torch.float32)))
    return x, w, dx, dw, cfg, outs


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_static_scratch_entry_matches_workspace_entry(dtype):
    L = rs.lib()
    cap = rs.rs_block_static_scratch_size()
    assert cap == 64 << 20
    stream = torch.cuda.current_stream().cuda_stream
    # first a batch that uses a large part of the buffer, then a smaller one
    for (seed, B, N, D, H, Dm, P, K) in [(31, 6, 197, 384, 6, 1536, 1, 150), (32, 2, 70, 128, 2, 256, 1, 30)]:
        print("static scratch", dtype, B, N, D, flush=True)
        sys.stdout.flush()
        x, w, dx, dw, cfg, outs = _case(seed, B, N, D, H, Dm, P, K, dtype)
        need = rs.rs_block_workspace_size(cfg)
        assert 0 < need <= cap
        wts = rs.make_weights(dw)
        ws = torch.empty(need, dtype=torch.uint8, device="cuda")
        (y0, k0, s0), (y1, k1, s1) = outs
        st = L.rs_block_fwd(ctypes.byref(cfg), ctypes.byref(wts), dx.data_ptr(), y0.data_ptr(), k0.data_ptr(),
                            s0.data_ptr(), ws.data_ptr(), need, stream)
        assert st == rs.RS_OK, rs.rs_last_error()
        st = L.rs_block_fwd_static(ctypes.byref(cfg), ctypes.byref(wts), dx.data_ptr(), y1.data_ptr(), k1.data_ptr(),
                                   s1.data_ptr(), stream)
        assert st == rs.RS_OK, rs.rs_last_error()
        torch.cuda.synchronize()
        assert torch.equal(k0, k1)
        assert torch.equal(s0.view(torch.int32), s1.view(torch.int32))
        assert torch.equal(y0.view(torch.int16 if dtype == "bf16" else torch.int32),
                           y1.view(torch.int16 if dtype == "bf16" else torch.int32))
        # and the shared result is the checker's
        ref = oracle.block(x, w, H)
        kept_h = k1.cpu().numpy()
        assert norm_err(to_host(s1), ref["scores"]) < TOL[dtype]
        assert norm_err(to_host(y1), oracle.gather(ref["xhat"], kept_h)) < TOL[dtype]
        np.testing.assert_array_equal(kept_h, oracle.topk(to_host(s1), P, K))


def test_static_scratch_entry_rejects_what_does_not_fit():
    L = rs.lib()
    cfg = rs.make_cfg(64, 197, 768, 12, 3072, 1, 177, torch.bfloat16)
    assert rs.rs_block_workspace_size(cfg) > rs.rs_block_static_scratch_size()
    w = rs.binding.RsBlockWeights()
    st = L.rs_block_fwd_static(ctypes.byref(cfg), ctypes.byref(w), 0x1000, 0x2000, 0x3000, None, None)
    assert st == rs.RS_ERR_UNSUPPORTED and "static buffer" in rs.rs_last_error()
