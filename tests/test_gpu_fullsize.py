"""GPU parity at the workloads' real shapes: one decoder layer forward +
backward of the ~1.3B GPT shape and of the Llama-7B shape (head dim 128,
seq 2048, SwiGLU, RoPE) against the fp64 oracle, and the heterogeneous
allocation scenario on the 1.3B model under an emulated 40 GB cap."""
import numpy as np
import pytest
import torch

from oracle import allocate as oal
from oracle import profiling as opf
from oracle import transformer as otr
from paper_2408_12596_amd import binding as pb
from paper_2408_12596_amd import synth
from gpu_util import DEV, assert_close_blockwise, quantize, rel_l2, scratch, to_dev, to_np, sync

pytestmark = pytest.mark.gpu

SHAPES = [
    dict(arch="gpt", L=1, H=2048, nh=16, F=8192, S=2048, V=1, B=1),
    dict(arch="llama", L=1, H=4096, nh=32, F=11008, S=2048, V=1, B=1),
    # three samples of the GPT-2-small shape: a token count that is not a multiple of the 256-row tile
    dict(arch="gpt", L=1, H=768, nh=12, F=3072, S=1024, V=1, B=3),
    # nine samples: the contraction over 9216 tokens is long enough for the weight-gradient group to be cut in two
    # along it (second half summed into buffers of its own and added afterwards)
    dict(arch="gpt", L=1, H=768, nh=12, F=3072, S=1024, V=1, B=9),
    # an odd local batch of the ~1.3B shape (the allocation stress runs 3, 5, 7 and 13; the larger ones follow below)
    dict(arch="gpt", L=1, H=2048, nh=16, F=8192, S=2048, V=1, B=3),
]


@pytest.mark.parametrize("case", SHAPES, ids=lambda c: f"{c['arch']}-H{c['H']}-S{c['S']}-B{c['B']}")
def test_layer_at_workload_shape(case):
    B, S, H, nh = case["B"], case["S"], case["H"], case["nh"]
    cfg = pb.make_cfg(**{k: case[k] for k in ("arch", "L", "H", "nh", "F", "S", "V")}, dtype="bf16")
    ctx = pb.Context(cfg)
    spec = [(f"l0.{n}", s) for n, s in otr.layer_spec(case["arch"], H, case["F"])]
    flat = synth.init_params(spec, seed=1, jitter=True)
    x = synth.activations((B, S, H), seed=1)
    dy = synth.activations((B, S, H), seed=2)
    d_params, d_x, d_dy = to_dev(flat, "bf16"), to_dev(x, "bf16"), to_dev(dy, "bf16")
    d_out, d_dx = torch.empty_like(d_x), torch.empty_like(d_x)
    saved = scratch(pb.layer_saved_bytes(cfg, B))
    wsb = pb.layer_workspace_bytes(cfg, B)
    ws = scratch(wsb)
    grads = torch.full((len(flat),), float("nan"), device=DEV)
    ctx.layer_fwd(B, d_x, d_params, d_out, saved)
    ctx.layer_bwd(B, d_x, d_dy, d_params, saved, d_dx, grads, 0, ws, wsb)
    sync()
    p = {k[3:]: v for k, v in otr.unpack(quantize(flat, "bf16"), spec).items()}
    ref_out, cache = otr.layer_fwd(case["arch"], p, quantize(x, "bf16"), nh)
    ref_dx, ref_g = otr.layer_bwd(case["arch"], p, quantize(dy, "bf16"), cache, nh)
    assert_close_blockwise(to_np(d_out).reshape(B * S, H), ref_out.reshape(B * S, H), 2e-2, "out")
    assert_close_blockwise(to_np(d_dx).reshape(B * S, H), ref_dx.reshape(B * S, H), 2e-2, "dx")
    got = to_np(grads)
    assert np.isfinite(got).all()
    table, _ = otr.offsets(spec)
    for name, (off, shape) in table.items():
        k = int(np.prod(shape))
        assert_close_blockwise(got[off:off + k].reshape(shape), np.asarray(ref_g[name[3:]]).reshape(shape), 2e-2, name)


@pytest.mark.parametrize("B", [5, 7, 13])
def test_1p3b_layer_at_the_odd_batches_of_the_allocation_stress(B):
    """One ~1.3B-shaped layer at local batch 5, 7 and 13, the launch configurations of the allocation stress.  The
    fp64 oracle costs ten seconds a sample, so only the first and the last sample carry an output gradient; samples
    are independent inside a layer and the backward pass is linear in dy, hence out and dx of those two samples and
    every weight gradient equal the oracle's on the two samples alone, and dx of the others is exactly zero.  (That
    the contraction over ALL tokens is complete is what test_gemm_full_size_every_tile shows at 26624 tokens.)"""
    case = dict(arch="gpt", L=1, H=2048, nh=16, F=8192, S=2048, V=1)
    S, H, nh = case["S"], case["H"], case["nh"]
    cfg = pb.make_cfg(**case, dtype="bf16")
    ctx = pb.Context(cfg)
    spec = [(f"l0.{n}", s) for n, s in otr.layer_spec("gpt", H, case["F"])]
    flat = synth.init_params(spec, seed=B, jitter=True)
    x = synth.activations((B, S, H), seed=10 + B)
    dy = synth.activations((B, S, H), seed=20 + B)
    live = [0, B - 1]
    dy[1:B - 1] = 0.0
    d_params, d_x, d_dy = to_dev(flat, "bf16"), to_dev(x, "bf16"), to_dev(dy, "bf16")
    d_out, d_dx = torch.empty_like(d_x), torch.empty_like(d_x)
    saved = scratch(pb.layer_saved_bytes(cfg, B))
    wsb = pb.layer_workspace_bytes(cfg, B)
    ws = scratch(wsb)
    grads = torch.full((len(flat),), float("nan"), device=DEV)
    ctx.layer_fwd(B, d_x, d_params, d_out, saved)
    ctx.layer_bwd(B, d_x, d_dy, d_params, saved, d_dx, grads, 0, ws, wsb)
    sync()
    out, dx, got = to_np(d_out), to_np(d_dx), to_np(grads)
    assert np.isfinite(out).all() and np.isfinite(got).all()
    assert np.all(dx[1:B - 1] == 0.0)
    p = {k[3:]: v for k, v in otr.unpack(quantize(flat, "bf16"), spec).items()}
    total = None
    for b in live:
        ref_out, cache = otr.layer_fwd("gpt", p, quantize(x[b:b + 1], "bf16"), nh)
        ref_dx, ref_g = otr.layer_bwd("gpt", p, quantize(dy[b:b + 1], "bf16"), cache, nh)
        assert_close_blockwise(out[b], ref_out[0], 2e-2, ("out", b))
        assert_close_blockwise(dx[b], ref_dx[0], 2e-2, ("dx", b))
        total = ref_g if total is None else {k: total[k] + ref_g[k] for k in total}
    table, _ = otr.offsets(spec)
    for name, (off, shape) in table.items():
        k = int(np.prod(shape))
        assert_close_blockwise(got[off:off + k].reshape(shape), np.asarray(total[name[3:]]).reshape(shape), 2e-2, name)


def test_heterogeneous_allocation_on_the_1p3b_model():
    """24-layer ~1.3B GPT, simulated world of 4, emulated 40 GiB device: largest batch per
    ZeRO stage by Algorithm 1, odd local batches (tail tiles), measured curves scaled to a
    1 : 1.5 : 2 : 3 device mix and split by Algorithm 2 for a global batch of 64."""
    model = dict(arch="gpt", L=24, H=2048, nh=16, F=8192, S=2048, V=50257)
    world, cap, max_b = 4, 40 * 2 ** 30, 16
    base = pb.make_cfg(**model, dtype="bf16", world=world, rank=0)
    P = pb.model_param_count(base)
    off, ln, valid = pb.shard_range(P, world, 0)
    g = torch.Generator(device=DEV).manual_seed(0)
    params = (torch.randn(P, device=DEV, generator=g) * 0.02).to(torch.bfloat16)
    own = params[off:off + ln].clone()
    master = params[off:off + ln].float()
    m, v = torch.zeros(ln, device=DEV), torch.zeros(ln, device=DEV)
    grads = torch.zeros(P, device=DEV)
    tok, tgt = synth.tokens(max_b, model["S"], model["V"], seed=0)
    tokens = to_dev(np.concatenate([tok, tgt[:, -1:]], axis=1).astype(np.int32))
    loss = torch.zeros(1, device=DEV)
    wsb = max(pb.step_workspace_bytes(base, s, max_b) for s in (1, 2, 3))
    ws = scratch(wsb)
    found = {}
    for stage in (1, 2, 3):
        cfg = pb.make_cfg(**model, dtype="bf16", world=world, rank=0, zero_stage=stage, cap_bytes=cap)
        ctx = pb.Context(cfg)
        ctx.bind_state(params, master, m, v, grads, tokens, max_b, ws, wsb, loss, own_shard=own, lr=1e-5)
        mbs, samples = ctx.search_mbs(stage)
        brute = max(b for b in range(0, max_b + 1) if pb.step_accounted_bytes(cfg, stage, b) <= cap)
        assert mbs == brute and mbs >= 1
        found[stage] = mbs
        assert all(np.isfinite(s["loss"]) and abs(s["loss"] - np.log(model["V"])) < 1.0 for s in samples)
        # an odd batch inside the range runs and is timed like any other
        odd = [b for b in (3, 5, 7, 13) if b <= mbs]
        extra = [ctx.profile_step(stage, b) for b in odd]
        pts = samples + extra
        bs = [s["batch"] for s in pts]
        ts = [s["t_consumed"] for s in pts]
        assert all(t > 0 for t in ts)
        curves = [(bs, [t * k for t in ts], mbs) for k in (1.0, 1 / 1.5, 1 / 2.0, 1 / 3.0)]
        got = pb.allocate(stage, 64, curves, 0.0)
        ref = oal.allocate(stage, 64, curves, 0.0)
        for key in ("gmbs", "b", "lbs"):
            assert got[key] == ref[key], (stage, key, got, ref)
        assert sum(got["gmbs"]) == 64
        assert all(bi <= mbs for bi in got["b"])
        # devices are listed slowest first: a faster device never gets fewer samples
        assert got["gmbs"] == sorted(got["gmbs"])
    # more sharding leaves more room for activations
    assert found[1] <= found[2] <= found[3]


def test_gpt2_small_step_at_the_benchmark_configuration():
    """The GPT-2-small configuration (12 layers, hidden 768, seq 1024, vocab 50257, bf16, ZeRO-1 on rank 0 of 8):
    two samples through the whole model against the fp64 oracle, tensor by tensor, and Adam on the shard; then the
    local batch of 16, the top of the sweep, against the oracle as well: the loss is a sum over samples, so the
    oracle's gradient for 16 samples is the sum of its gradients for eight pairs, each weighted 1 / (16 S), added up
    in float64 (the whole batch at once would hold every layer's attention matrices in float64: tens of GB)."""
    from oracle import optimizer as oopt
    from test_gpu_step import HP, Rank
    model = dict(arch="gpt", L=12, H=768, nh=12, F=3072, S=1024, V=50257)
    rk = Rank(model, "bf16", 1, 8, 0, max_batch=16)
    B = 2
    prof = rk.ctx.profile_step(1, B)
    sync()
    got = to_np(rk.grads)
    loss, grad, _ = otr.model_fwd_bwd(model, quantize(rk.flat, "bf16"), rk.tok[:B], rk.tgt[:B], 1.0 / (B * model["S"]))
    assert abs(prof["loss"] - loss) <= 5e-3 * abs(loss)
    assert abs(loss - np.log(model["V"])) < 0.5          # near-uniform predictions at initialisation
    table, _ = otr.offsets(rk.spec)
    for name, (off, shape) in table.items():
        k = int(np.prod(shape))
        assert rel_l2(got[off:off + k], grad[off:off + k]) <= 2e-2, name
    sl = slice(rk.off, rk.off + rk.valid)
    p0 = rk.flat[sl].astype(np.float64)
    z = np.zeros_like(p0)
    rp, rm, rv = oopt.adam_step(p0, z, z, got[sl], 1, **HP)
    assert rel_l2(to_np(rk.master)[:rk.valid], rp) <= 1e-6
    assert rel_l2(to_np(rk.m)[:rk.valid], rm) <= 1e-6
    assert rel_l2(to_np(rk.v)[:rk.valid], rv) <= 1e-6

    one = Rank(model, "bf16", 1, 8, 0, max_batch=16)
    p16 = one.ctx.profile_step(1, 16)
    sync()
    g16 = to_np(one.grads)
    assert np.isfinite(g16).all()
    fq = quantize(one.flat, "bf16")
    loss16, grad16 = 0.0, np.zeros(len(fq), np.float64)
    for b in range(0, 16, 2):
        l2, g2, _ = otr.model_fwd_bwd(model, fq, one.tok[b:b + 2], one.tgt[b:b + 2], 1.0 / (16 * model["S"]))
        loss16 += l2
        grad16 += g2
    assert abs(p16["loss"] - loss16) <= 5e-3 * abs(loss16)
    for name, (off, shape) in table.items():
        k = int(np.prod(shape))
        assert_close_blockwise(g16[off:off + k].reshape(shape), grad16[off:off + k].reshape(shape), 2e-2, name)
    sl = slice(one.off, one.off + one.valid)
    rp, rm, rv = oopt.adam_step(one.flat[sl].astype(np.float64), z, z, g16[sl], 1, **HP)
    assert rel_l2(to_np(one.master)[:one.valid], rp) <= 1e-6

    # the same batch as two accumulated micro-steps of 9 and 7 at ZeRO-2 (the weight gradients of the first are cut
    # in two along its 9216 tokens and land in the staging bucket; the second adds through the local reduce)
    acc = Rank(model, "bf16", 2, 8, 3, max_batch=16)       # rank 3 of 8 owns layers 1 to 3
    pacc = acc.ctx.accum_step(2, [9, 7], 16)
    sync()
    gacc = to_np(acc.grads)
    assert abs(pacc["loss"] - loss16) <= 5e-3 * abs(loss16)
    assert rel_l2(gacc[:acc.valid], grad16[acc.off:acc.off + acc.valid]) <= 2e-2
    seen = 0
    for name, (off, shape) in table.items():      # tensor by tensor, the rows that lie inside the shard
        cols = shape[-1] if len(shape) == 2 else 1
        lo, hi = max(off, acc.off), min(off + int(np.prod(shape)), acc.off + acc.valid)
        lo += (-(lo - off)) % cols
        hi -= (hi - off) % cols
        if hi > lo:
            seen += 1
            got_t, ref_t = gacc[lo - acc.off:hi - acc.off], grad16[lo:hi]
            assert_close_blockwise(got_t.reshape(-1, cols) if cols > 1 else got_t, ref_t.reshape(-1, cols) if cols > 1 else ref_t, 2e-2, name)
    assert seen >= 24                               # two whole layers at least


def test_layer_backward_accumulates_and_may_overwrite_dy():
    """GPT-2-small layer at nine samples (weight gradients cut in two along the 9216 tokens): a second backward pass
    with accumulate = 1 doubles every gradient, also when dx is written over dy."""
    case = dict(arch="gpt", L=1, H=768, nh=12, F=3072, S=1024, V=1)
    B, S, H, nh = 9, case["S"], case["H"], case["nh"]
    cfg = pb.make_cfg(**case, dtype="bf16")
    ctx = pb.Context(cfg)
    spec = [(f"l0.{n}", s) for n, s in otr.layer_spec("gpt", H, case["F"])]
    flat = synth.init_params(spec, seed=4, jitter=True)
    x = synth.activations((B, S, H), seed=5)
    dy = synth.activations((B, S, H), seed=6)
    d_params, d_x, d_dy = to_dev(flat, "bf16"), to_dev(x, "bf16"), to_dev(dy, "bf16")
    d_out, d_dx = torch.empty_like(d_x), torch.empty_like(d_x)
    saved = scratch(pb.layer_saved_bytes(cfg, B))
    wsb = pb.layer_workspace_bytes(cfg, B)
    ws = scratch(wsb)
    grads = torch.full((len(flat),), float("nan"), device=DEV)
    ctx.layer_fwd(B, d_x, d_params, d_out, saved)
    ctx.layer_bwd(B, d_x, d_dy, d_params, saved, d_dx, grads, 0, ws, wsb)
    inplace = d_dy.clone()
    ctx.layer_bwd(B, d_x, inplace, d_params, saved, inplace, grads, 1, ws, wsb)
    sync()
    p = {k[3:]: v for k, v in otr.unpack(quantize(flat, "bf16"), spec).items()}
    _, cache = otr.layer_fwd("gpt", p, quantize(x, "bf16"), nh)
    ref_dx, ref_g = otr.layer_bwd("gpt", p, quantize(dy, "bf16"), cache, nh)
    assert_close_blockwise(to_np(d_dx).reshape(B * S, H), ref_dx.reshape(B * S, H), 2e-2, "dx")
    assert_close_blockwise(to_np(inplace).reshape(B * S, H), ref_dx.reshape(B * S, H), 2e-2, "dx over dy")
    got = to_np(grads)
    table, _ = otr.offsets(spec)
    for name, (off, shape) in table.items():
        k = int(np.prod(shape))
        assert_close_blockwise(got[off:off + k].reshape(shape), 2.0 * np.asarray(ref_g[name[3:]]).reshape(shape), 2e-2, name)
