"""The paper's curve claim measured on this device (Appendix "Cubic Spline Interpolation": the curve through the
profiled points is almost the measured data), and Algorithm 2's stage 2/3 sweep with a modelled communication time."""
import numpy as np
import pytest
import torch

from oracle import allocate as oal
from oracle import comm as ocomm
from paper_2408_12596_amd import binding as pb
from paper_2408_12596_amd import synth
from gpu_util import DEV, scratch, to_dev, sync

pytestmark = pytest.mark.gpu
MODEL = dict(arch="gpt", L=2, H=768, nh=12, F=3072, S=1024, V=8192)   # two layers of the GPT-2-small shape
WORLD, STAGE, MAXB = 4, 2, 8


def measured_curve(reps=5):
    cfg = pb.make_cfg(**MODEL, dtype="bf16", world=WORLD, rank=0, zero_stage=STAGE)
    ctx = pb.Context(cfg)
    P = pb.model_param_count(cfg)
    spec = [(name, shape) for name, shape, _ in pb.model_spec(cfg)]
    flat = synth.init_params(spec, seed=0)
    off, ln, valid = pb.shard_range(P, WORLD, 0)
    tok, tgt = synth.tokens(MAXB, MODEL["S"], MODEL["V"], seed=0)
    keep = dict(
        params=to_dev(flat, "bf16"), master=to_dev(np.pad(flat, (0, WORLD * ln - P))[off:off + ln]),
        m=torch.zeros(ln, device=DEV), v=torch.zeros(ln, device=DEV), grads=torch.zeros(ln, device=DEV),
        tokens=to_dev(np.concatenate([tok, tgt[:, -1:]], axis=1).astype(np.int32)), loss=torch.zeros(1, device=DEV))
    wsb = pb.step_workspace_bytes(cfg, STAGE, MAXB)
    keep["ws"] = scratch(wsb)
    ctx.bind_state(keep["params"], keep["master"], keep["m"], keep["v"], keep["grads"], keep["tokens"], MAXB, keep["ws"], wsb,
                   keep["loss"], adam_t=1, lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8)
    dense = {}
    for b in range(1, MAXB + 1):
        ctx.profile_step(STAGE, b)   # warm-up at this shape
        dense[b] = float(np.median([ctx.profile_step(STAGE, b)["t_consumed"] for _ in range(reps)]))
    sync()
    return P, dense


def test_spline_through_the_visited_batches_predicts_the_others():
    P, dense = measured_curve()
    # time grows with the batch and the speed b / t rises towards a plateau (Section "Optimal Batch Size Searching")
    ts = [dense[b] for b in sorted(dense)]
    assert all(t > 0 for t in ts) and ts[-1] > ts[0]
    assert MAXB / dense[MAXB] > 2.0 * (1 / dense[1])
    visited = [1, 2, 4, 8]                       # what Algorithm 1's doubling sweep records
    speed = pb.speed_curve(visited, [dense[b] for b in visited], MAXB)
    for b in visited:
        assert speed[b] == pytest.approx(b / dense[b], rel=1e-12)
    err = [abs(speed[b] * dense[b] / b - 1.0) for b in dense if b not in visited]
    assert max(err) <= 0.10, err                 # measured on MI355X: 1-4 %

    # Algorithm 2, stages 2 and 3, on a four-device mix of this curve with the modelled communication time per
    # micro-step: same integers as the oracle, and more communication never makes the optimum shorter
    bs = sorted(dense)
    curves = [(bs, [dense[b] * k for b in bs], MAXB) for k in (1.0, 1.5, 2.0, 3.0)]
    last_T = 0.0
    for stage in (2, 3):
        cm = pb.comm_model(P, WORLD, stage, 2.0, 4.0, 7 * 153e9)
        assert cm == ocomm.comm_model(P, WORLD, stage, 2.0, 4.0, 7 * 153e9) and cm["t_micro"] > 0
        got = pb.allocate(stage, 96, curves, cm["t_micro"])
        ref = oal.allocate(stage, 96, curves, cm["t_micro"])
        for k in ("gmbs", "b", "lbs"):
            assert got[k] == ref[k], k
        assert got["gas"] == [ref["gas"]] * 4     # one accumulation count for the whole cluster at these stages
        assert got["T"] == pytest.approx(ref["wall"], rel=1e-12) and got["t"] == pytest.approx(ref["t"], rel=1e-12)
        assert sum(got["gmbs"]) == 96 and got["T"] >= last_T
        free = pb.allocate(stage, 96, curves, 0.0)
        assert got["T"] >= free["T"]
        last_T = got["T"]
