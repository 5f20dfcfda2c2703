"""The checker's schedule reading and cost accounting against the paper's printed
multiply-accumulate counts (tests/golden/paper_gmacs.txt: Tables 2, 4 and 5)."""
import os

from oracle import schedule as sch


def _rows(golden_dir):
    for line in open(os.path.join(golden_dir, "paper_gmacs.txt")):
        if line.startswith("#") or not line.strip():
            continue
        f = line.split()
        after = [] if f[6] == "-" else [int(t) for t in f[6].split(",")]
        yield f[0], int(f[1]), int(f[2]), int(f[3]), int(f[4]), int(f[5]), after, float(f[7])


def _gmacs(N, P, D, blocks, pct, after):
    prune = dict(kind="drop_pct", pct=pct, after=after) if after else None
    patch_tokens = N - P
    return sch.model_macs(N, P, D, blocks, prune, patch_tokens, 16 * 16 * 3) / 1e9


def test_printed_gmacs_reproduced(golden_dir):
    n = 0
    for name, N, P, D, blocks, pct, after, printed in _rows(golden_dir):
        ours = _gmacs(N, P, D, blocks, pct, after)
        if name.startswith("deit"):
            # one printed decimal
            assert abs(ours - printed) <= 0.05 + 1e-9, (name, ours, printed)
        else:
            assert abs(ours - printed) / printed < 1.0e-3, (name, ours, printed)
        n += 1
    assert n == 12


def test_other_schedule_readings_miss(golden_dir):
    """Pruning one block later, or before the block instead of after it, does not
    reproduce the printed numbers: the pin discriminates."""
    rows = {r[0]: r for r in _rows(golden_dir)}
    _, N, P, D, blocks, pct, after, printed = rows["deit_b_ours"]
    later = _gmacs(N, P, D, blocks, pct, [a + 1 for a in after])
    assert abs(later - printed) > 0.3
    _, N, P, D, blocks, pct, after, printed = rows["umt_b_ret"]
    # pruning before blocks 1, 2, 3 = entering block 1 already pruned, then after blocks 1, 2
    n1 = N - sch.drop_count(N, pct)
    before = sch.model_macs(n1, P, D, blocks, dict(kind="drop_pct", pct=pct, after=[1, 2]), N, 768) / 1e9
    assert abs(before - printed) / printed > 0.05


def test_token_counts_of_the_workloads():
    import synth_inputs as si
    w = si.WORKLOADS
    assert sch.tokens_per_block(197, 1, 1, w["vit_block_fp32"]["prune"]) == [197]
    assert 196 - sch.drop_count(196, 30) == 138
    assert sch.tokens_per_block(197, 1, 12, w["vit_s16"]["prune"]) == \
        [197, 181, 165, 149, 133, 117, 101, 85, 69, 53, 37, 21]
    assert sch.tokens_per_block(197, 1, 12, w["vit_b16"]["prune"]) == \
        [197, 197, 197, 197, 178, 161, 145, 131, 118, 107, 97, 88]
    assert sch.tokens_per_block(1569, 1, 12, w["video_vit_b16"]["prune"]) == \
        [1569, 1569, 785, 785, 785, 393, 393, 393, 197, 197, 197, 197]
    assert sch.tokens_per_block(4097, 1, 24, w["video_vit_l14"]["prune"]) == \
        [4097] * 4 + [2869] * 4 + [2009] * 4 + [1407] * 4 + [986] * 8


def test_paper_workloads_match_the_printed_rows(golden_dir):
    """The bench workloads named after the paper's runs carry exactly the shape and schedule of
    the fixture row whose printed cost they reproduce."""
    import synth_inputs as si
    rows = {r[0]: r for r in _rows(golden_dir)}
    for wl_name, row in (("deit_t", "deit_t_ours"), ("deit_s", "deit_s_ours"), ("deit_b", "deit_b_ours"),
                         ("umt_b_ret", "umt_b_ret"), ("umt_b_qa", "umt_b_qa"),
                         ("umt_l_ret", "umt_l_ret"), ("umt_l_qa", "umt_l_qa")):
        w = si.WORKLOADS[wl_name]
        _, N, P, D, blocks, pct, after, _ = rows[row]
        assert (w["N"], w.get("n_prefix", 1), w["D"], w["blocks"]) == (N, P, D, blocks), wl_name
        assert w["prune"] == dict(kind="drop_pct", pct=pct, after=after), wl_name
        assert w["Dm"] == 4 * D and w["D"] // w["H"] == 64
    # the product's schedule helper agrees with the checker's on every workload
    from paper_2508_00367_amd import schedule as psch
    for name, w in si.WORKLOADS.items():
        P = w.get("n_prefix", 1)
        assert [n for n, _ in psch.keep_counts(w["N"], P, w["blocks"], w["prune"])] == \
            sch.tokens_per_block(w["N"], P, w["blocks"], w["prune"]), name
    assert sch.tokens_per_block(2352, 0, 12, si.WORKLOADS["umt_b_ret"]["prune"])[:5] == [2352, 1882, 1506, 1205, 1205]
    assert sch.tokens_per_block(197, 1, 12, si.WORKLOADS["deit_b"]["prune"]) == \
        [197, 158, 158, 158, 127, 127, 127, 102, 102, 102, 102, 102]
