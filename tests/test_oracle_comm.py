"""The communication model against what the paper prints and against the host library."""
import numpy as np
import pytest

from oracle import comm as ocomm
from paper_2408_12596_amd import binding as pb


def test_feed_forward_block_at_stage_3_is_24_d_h_squared():
    # Appendix "Analysis of Experiments": Comm_Volume = 24 d h^2 for the block of (h x 4h) + (4h x h) parameters
    for h, d in ((768, 8), (4096, 16), (64, 3)):
        P = h * 4 * h + 4 * h * h
        m = ocomm.comm_model(P, d, 3, 2, 2, 1.0)
        assert m["total_micro_elements"] == 24 * d * h * h
        # forward all-gather + backward all-gather + reduce-scatter, the block's parameters each
        assert ocomm.comm_elements(P, d, 3) == (2 * P, P, 0, 0)


def test_elements_per_stage_follow_from_the_appendix_list_of_collectives():
    # tests/golden/zero_collectives.json lists, stage by stage, the collectives Appendix "Details about ZeRO" names;
    # every one moves the whole flat vector (P elements per device, the count of Appendix "Analysis of Experiments")
    import json, os
    with open(os.path.join(os.path.dirname(__file__), "golden", "zero_collectives.json")) as f:
        gold = json.load(f)["stages"]
    P, d = 12345, 6
    for stage in range(4):
        want = {("micro_step", "parameters"): 0, ("micro_step", "gradients"): 0, ("optimizer_step", "parameters"): 0, ("optimizer_step", "gradients"): 0}
        for c in gold[str(stage)]:
            assert c["collective"] in ("reduce_scatter", "all_gather")
            want[(c["when"], c["operand"])] += P
        assert ocomm.comm_elements(P, d, stage) == (want[("micro_step", "parameters")], want[("micro_step", "gradients")],
                                                    want[("optimizer_step", "parameters")], want[("optimizer_step", "gradients")]), stage
    # textbook cross-check of the stage 0 total: a ring all-reduce moves 2 (d-1)/d P elements per device, which the
    # paper's count (no (d-1)/d deduction) bounds from above and meets as d grows
    for dd in (2, 8, 1024):
        ring = 2 * (dd - 1) / dd * P
        paper = sum(ocomm.comm_elements(P, dd, 0))
        assert ring <= paper and paper / ring == pytest.approx(dd / (dd - 1))


def test_collectives_per_stage_follow_the_appendix():
    P, d = 1000, 4
    # stage 0: all-reduce = reduce-scatter + all-gather of the gradients, at the end of the step
    assert ocomm.comm_elements(P, d, 0) == (0, 0, 0, 2 * P)
    # stage 1: the same, then an all-gather of the updated parameters
    assert ocomm.comm_elements(P, d, 1) == (0, 0, P, 2 * P)
    # stage 2: reduce-scatter instead of all-reduce (every micro-step), all-gather of the parameters
    assert ocomm.comm_elements(P, d, 2) == (0, P, P, 0)
    # nothing to exchange alone
    for s in range(4):
        assert ocomm.comm_elements(P, 1, s) == (0, 0, 0, 0)
    with pytest.raises(ValueError):
        ocomm.comm_elements(P, d, 4)


def test_time_is_bytes_over_bandwidth_and_grows_with_the_stage_per_micro_step():
    P, d, bw = 124_439_808, 8, 7 * 153e9
    t = [ocomm.comm_model(P, d, s, 2, 4, bw) for s in range(4)]
    assert t[0]["t_micro"] == t[1]["t_micro"] == 0.0 < t[2]["t_micro"] < t[3]["t_micro"]
    assert t[2]["micro_bytes"] == 4 * P and t[3]["micro_bytes"] == 2 * 2 * P + 4 * P
    assert t[3]["t_micro"] == pytest.approx(8 * P / bw, rel=1e-15)
    assert t[1]["step_bytes"] == 2 * P + 2 * 4 * P


def test_host_library_matches_the_oracle_exactly():
    rng = np.random.default_rng(0)
    for _ in range(200):
        P = int(rng.integers(0, 10**10))
        world = int(rng.integers(1, 65))
        stage = int(rng.integers(0, 4))
        pbytes, gbytes = float(rng.choice([2, 4])), float(rng.choice([2, 4]))
        bw = float(rng.uniform(1e9, 2e12))
        got = pb.comm_model(P, world, stage, pbytes, gbytes, bw)
        ref = ocomm.comm_model(P, world, stage, pbytes, gbytes, bw)
        assert got == ref
    for bad in ((-1, 2, 1, 2, 4, 1e9), (10, 0, 1, 2, 4, 1e9), (10, 2, 4, 2, 4, 1e9), (10, 2, 1, 0, 4, 1e9), (10, 2, 1, 2, 4, 0.0)):
        with pytest.raises(pb.PoplarError):
            pb.comm_model(*bad)
