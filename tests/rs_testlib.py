"""Helpers shared by the GPU parity tests: host<->device marshalling, error metric,
and the admissibility rule for kept indices."""
import numpy as np
import torch

import synth_inputs as si

TOL = {"f32": 1e-4, "bf16": 2e-2}   # tensor-normalised max error allowed vs the fp64 checker


def host_round(a, dtype):
    """The fp32 host array as the device will hold it (bf16: RNE rounded)."""
    a = np.ascontiguousarray(a, np.float32)
    return si.round_to_bf16(a) if dtype == "bf16" else a


def to_dev(a, dtype):
    """Host array (already representable in `dtype`) -> device tensor of that dtype."""
    if a is None:
        return None
    t = torch.from_numpy(np.ascontiguousarray(a, np.float32))
    return t.to("cuda", torch.bfloat16 if dtype == "bf16" else torch.float32)


def to_host(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def norm_err(got, ref):
    """max |got - ref| / max |ref| over the tensor."""
    ref = np.asarray(ref, np.float64)
    got = np.asarray(got, np.float64)
    den = np.abs(ref).max()
    return float(np.abs(got - ref).max() / (den if den > 0 else 1.0))


def rel_err_floor(got, ref, floor=1e-3):
    """max over elements of |got - ref| / max(|ref|, floor * max|ref|): per-element relative error
    with an absolute floor (reported next to norm_err, not bounded by the tolerance: an element
    much smaller than the tensor's largest carries the same absolute rounding error)."""
    ref = np.asarray(ref, np.float64)
    got = np.asarray(got, np.float64)
    den = np.maximum(np.abs(ref), floor * max(np.abs(ref).max(), 1e-300))
    return float((np.abs(got - ref) / den).max())


def check_kept_admissible(kept_gpu, scores_gpu, scores_ref, n_prefix, n_keep):
    """kept_idx must equal the checker's selection except for tokens whose checker score
    lies within 2*tau of the checker's threshold score, tau = max |s_gpu - s_ref| of the image.
    Returns the fraction of images whose kept_idx matches exactly."""
    import oracle
    kept_ref = oracle.topk(scores_ref, n_prefix, n_keep)
    B = kept_ref.shape[0]
    exact = 0
    for b in range(B):
        g, r = kept_gpu[b], kept_ref[b]
        assert list(g) == sorted(set(g.tolist())), "kept_idx not strictly ascending"
        assert list(g[:n_prefix]) == list(range(n_prefix))
        if np.array_equal(g, r):
            exact += 1
            continue
        tau = np.abs(scores_gpu[b] - scores_ref[b]).max()
        cand = np.sort(scores_ref[b, n_prefix:])[::-1]
        thr = cand[n_keep - 1]
        diff = set(g.tolist()) ^ set(r.tolist())
        for i in diff:
            assert abs(scores_ref[b, i] - thr) <= 2 * tau + 1e-30, \
                "image %d token %d: score gap %.3e > 2*tau %.3e" % (b, i, abs(scores_ref[b, i] - thr), 2 * tau)
    return exact / max(B, 1)
