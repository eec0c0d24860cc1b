"""The backward pass that allocates nothing (poplar_layer_bwd_static) against poplar_layer_bwd: same inputs, same
outputs, two calls in a row on the library's own scratch, the second on a smaller batch."""
import numpy as np
import pytest
import torch

from oracle import transformer as otr
from paper_2408_12596_amd import binding as pb
from paper_2408_12596_amd import synth
from gpu_util import DEV, rel_l2, scratch, to_dev, to_np, sync

pytestmark = pytest.mark.gpu

CASES = [
    (dict(arch="gpt", L=1, H=256, nh=4, F=1024, S=128, V=1), "f32", (2, 1)),
    (dict(arch="llama", L=1, H=256, nh=2, F=344, S=130, V=1), "bf16", (3, 2)),
    (dict(arch="gpt", L=1, H=768, nh=12, F=3072, S=1024, V=1), "bf16", (1,)),     # the largest layer the scratch holds
    (dict(arch="gpt", L=1, H=128, nh=2, F=256, S=64, V=1), "bf16", (5, 1)),
]


def run_pair(ctx, cfg, case, dtype, B, seed):
    S, H = case["S"], case["H"]
    spec = [(f"l0.{n}", s) for n, s in otr.layer_spec(case["arch"], H, case["F"])]
    flat = synth.init_params(spec, seed=seed, jitter=True)
    d_params = to_dev(flat, dtype)
    d_x = to_dev(synth.activations((B, S, H), seed=seed + 1), dtype)
    d_dy = to_dev(synth.activations((B, S, H), seed=seed + 2), dtype)
    d_out = torch.empty_like(d_x)
    saved = scratch(pb.layer_saved_bytes(cfg, B))
    ctx.layer_fwd(B, d_x, d_params, d_out, saved)
    wsb = pb.layer_workspace_bytes(cfg, B)
    assert wsb <= pb.static_scratch_bytes()
    ws = scratch(wsb)
    dx_a, dx_b = torch.empty_like(d_x), torch.empty_like(d_x)
    g_a = torch.full((len(flat),), float("nan"), device=DEV)
    g_b = torch.full((len(flat),), float("nan"), device=DEV)
    ctx.layer_bwd(B, d_x, d_dy, d_params, saved, dx_a, g_a, 0, ws, wsb)
    sync()
    before = torch.cuda.memory_allocated(), torch.cuda.memory_reserved()
    ctx.layer_bwd_static(B, d_x, d_dy, d_params, saved, dx_b, g_b, 0)
    ctx.layer_bwd_static(B, d_x, d_dy, d_params, saved, dx_b, g_b, 1)       # accumulates: twice the gradient
    sync()
    assert before == (torch.cuda.memory_allocated(), torch.cuda.memory_reserved())
    tol = 2e-2 if dtype == "bf16" else 5e-5
    assert np.isfinite(to_np(g_b)).all()
    assert rel_l2(to_np(dx_b), to_np(dx_a)) <= min(tol, 1e-5)    # same kernels on the same data: far inside the bar
    assert rel_l2(to_np(g_b), 2.0 * to_np(g_a)) <= min(tol, 1e-5)


@pytest.mark.parametrize("case,dtype,batches", CASES, ids=lambda v: str(v) if not isinstance(v, dict) else f"{v['arch']}-H{v['H']}-S{v['S']}")
def test_static_backward_matches_the_workspace_one_on_calls_in_a_row(case, dtype, batches):
    cfg = pb.make_cfg(**case, dtype=dtype)
    ctx = pb.Context(cfg)
    for i, B in enumerate(batches):          # the later, smaller call finds the earlier one's leftovers in the scratch
        run_pair(ctx, cfg, case, dtype, B, seed=10 * i + 1)


def test_static_backward_refuses_what_does_not_fit():
    case = dict(arch="gpt", L=1, H=768, nh=12, F=3072, S=1024, V=1)
    cfg = pb.make_cfg(**case, dtype="bf16")
    ctx = pb.Context(cfg)
    assert pb.layer_workspace_bytes(cfg, 2) > pb.static_scratch_bytes() == 64 << 20
    t = torch.zeros(8, device=DEV)
    with pytest.raises(pb.PoplarError) as e:
        ctx.layer_bwd_static(2, t, t, t, t, t, t, 0)        # refused on its size before any pointer is used
    assert e.value.status == pb.ERR_INVALID and "static scratch" in str(e.value)
    with pytest.raises(pb.PoplarError):
        ctx.layer_bwd_static(1, None, t, t, t, t, t, 0)
