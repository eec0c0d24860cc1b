"""GPU parity: one rank's whole step at every ZeRO stage (profile_step), the
max-batch search under an emulated cap, and the allocator on measured curves."""
import numpy as np
import pytest
import torch

from oracle import allocate as oal
from oracle import optimizer as oopt
from oracle import profiling as opf
from oracle import transformer as otr
from paper_2408_12596_amd import binding as pb
from paper_2408_12596_amd import synth
from gpu_util import DEV, quantize, rel_l2, scratch, to_dev, to_np, sync, tdtype

pytestmark = pytest.mark.gpu
TOL = {"bf16": 2e-2, "f32": 5e-5}
# the C ABI takes float hyper-parameters: the oracle gets the same float values
HP = {k: float(np.float32(x)) for k, x in dict(lr=1e-3, b1=0.9, b2=0.999, eps=1e-8).items()}

MODELS = {
    "gpt": dict(arch="gpt", L=2, H=128, nh=2, F=256, S=64, V=211),
    "llama": dict(arch="llama", L=2, H=128, nh=2, F=200, S=64, V=157),
}


class Rank:
    """Device state of one simulated rank, built from the same flat fp32 vector the oracle sees."""

    def __init__(self, model, dtype, stage, world, rank, max_batch, cap_bytes=0, seed=0, deterministic=False):
        self.model, self.dtype, self.stage = model, dtype, stage
        self.cfg = pb.make_cfg(**model, dtype=dtype, world=world, rank=rank, zero_stage=stage, cap_bytes=cap_bytes,
                               deterministic=deterministic)
        self.ctx = pb.Context(self.cfg)
        self.spec = otr.model_spec(model)
        self.flat = synth.init_params(self.spec, seed=seed, jitter=True)
        self.P = len(self.flat)
        assert self.P == pb.model_param_count(self.cfg)
        if stage == 0:
            self.off, self.len, self.valid = 0, self.P, self.P
        else:
            self.off, self.len, self.valid = pb.shard_range(self.P, world, rank)
        padded = np.zeros(max(self.off + self.len, self.P), np.float32)
        padded[:self.P] = self.flat
        self.params = to_dev(self.flat, dtype)
        self.master = to_dev(padded[self.off:self.off + self.len])
        self.own = to_dev(padded[self.off:self.off + self.len], dtype) if stage == 3 else None
        if stage == 3:   # the rank's own range must come from its shard, not from the stand-in
            self.params[self.off:self.off + self.valid] = float("nan")
        self.m = torch.zeros(self.len, device=DEV)
        self.v = torch.zeros(self.len, device=DEV)
        self.grads = torch.full((self.P if stage < 2 else self.len,), float("nan"), device=DEV)
        tok, tgt = synth.tokens(max_batch, model["S"], model["V"], seed=seed)
        self.tok, self.tgt = tok, tgt
        both = np.concatenate([tok, tgt[:, -1:]], axis=1).astype(np.int32)
        self.tokens = to_dev(both)
        self.wsb = pb.step_workspace_bytes(self.cfg, stage, max_batch)
        self.ws = scratch(self.wsb)
        self.loss = torch.zeros(1, device=DEV)
        self.ctx.bind_state(self.params, self.master, self.m, self.v, self.grads, self.tokens, max_batch, self.ws, self.wsb,
                            self.loss, own_shard=self.own, adam_t=1, lr=HP["lr"], beta1=HP["b1"], beta2=HP["b2"], eps=HP["eps"])


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("stage", [0, 1, 2, 3])
@pytest.mark.parametrize("arch", ["gpt", "llama"])
def test_profile_step_matches_oracle(arch, stage, dtype):
    model, B, world, rank = MODELS[arch], 3, 4, 1
    rk = Rank(model, dtype, stage, world, rank, max_batch=4)
    prof = rk.ctx.profile_step(stage, B)
    sync()
    fq = quantize(rk.flat, dtype)
    loss, grad, _ = otr.model_fwd_bwd(model, fq, rk.tok[:B], rk.tgt[:B], 1.0 / (B * model["S"]))
    tol = TOL[dtype]
    assert abs(prof["loss"] - loss) <= (5e-3 if dtype == "bf16" else 1e-5) * abs(loss)
    got = to_np(rk.grads)
    sl = slice(rk.off, rk.off + rk.valid)
    if stage < 2:
        table, _ = otr.offsets(rk.spec)
        for name, (off, shape) in table.items():
            k = int(np.prod(shape))
            assert rel_l2(got[off:off + k], grad[off:off + k]) <= tol, name
        g_used = got[sl]
    else:
        assert rel_l2(got[:rk.valid], grad[sl]) <= tol
        assert np.all(got[rk.valid:] == 0)
        g_used = got[:rk.valid]
    # Adam on the shard: the oracle applied to the gradient the device produced (1e-6), and end to end
    p0 = rk.flat[sl].astype(np.float64)
    z = np.zeros_like(p0)
    rp, rm, rv = oopt.adam_step(p0, z, z, g_used, 1, **HP)
    assert rel_l2(to_np(rk.master)[:rk.valid], rp) <= 1e-6
    assert rel_l2(to_np(rk.m)[:rk.valid], rm) <= 1e-6
    assert rel_l2(to_np(rk.v)[:rk.valid], rv) <= 1e-6
    low = rk.own[:rk.valid] if stage == 3 else rk.params[sl]
    np.testing.assert_array_equal(low.to(torch.float32).cpu().numpy(),
                                  oopt.bf16_round(rk.master[:rk.valid].cpu().numpy()) if dtype == "bf16" else rk.master[:rk.valid].cpu().numpy())
    # what a profile sample means, per stage
    ref_t = opf.time_consumed(stage, prof["t_fwd"], prof["t_bwd"], prof["t_gather_fwd"], prof["t_gather_bwd"], prof["t_reduce_bwd"])
    assert abs(prof["t_consumed"] - ref_t) <= 1e-12
    assert prof["t_fwd"] > 0 and prof["t_bwd"] > 0 and prof["t_adam"] > 0
    assert (prof["t_reduce_bwd"] > 0) == (stage >= 2) and (prof["t_gather_fwd"] > 0) == (stage == 3)
    assert prof["accounted_bytes"] == pb.step_accounted_bytes(rk.cfg, stage, B)
    S, H, F, V, L = (model[k] for k in "SHFVL")
    mlp = 3 if arch == "llama" else 2
    assert prof["flops"] == B * (L * (6 * S * (4 * H * H + mlp * H * F) + 7 * S * S * H) + 6 * S * H * V)


def test_all_ranks_together_equal_the_unsharded_update():
    """ZeRO world of 4 simulated by shard offsets: the four shards' updates tile the full update."""
    model, B, world = MODELS["gpt"], 2, 4
    full = Rank(model, "f32", 0, 1, 0, max_batch=B)
    full.ctx.profile_step(0, B)
    sync()
    ref = to_np(full.master)
    for stage in (1, 2):
        parts = []
        for r in range(world):
            rk = Rank(model, "f32", stage, world, r, max_batch=B)
            rk.ctx.profile_step(stage, B)
            sync()
            parts.append(to_np(rk.master)[:rk.valid])
        got = np.concatenate(parts)
        # same kernels, same inputs: only the scatter-add order of the embedding gradient may differ
        assert rel_l2(got, ref) <= 1e-7


def test_profile_step_errors_leave_state_untouched():
    model = MODELS["gpt"]
    rk = Rank(model, "f32", 1, 4, 0, max_batch=2, cap_bytes=1)
    before = rk.master.clone()
    with pytest.raises(pb.OutOfMemory):
        rk.ctx.profile_step(1, 1)
    with pytest.raises(pb.PoplarError):
        rk.ctx.profile_step(1, 3)          # above the bound token buffer
    with pytest.raises(pb.PoplarError):
        rk.ctx.profile_step(3, 1)          # stage 3 needs own_shard
    with pytest.raises(pb.PoplarError):
        pb.Context(rk.cfg).profile_step(1, 1)   # nothing bound
    sync()
    assert torch.equal(before, rk.master)


@pytest.mark.parametrize("stage", [1, 2, 3])
def test_search_mbs_under_an_emulated_cap(stage):
    model, world = MODELS["gpt"], 4
    probe = pb.make_cfg(**model, dtype="bf16", world=world, zero_stage=stage)
    want = 11
    cap = pb.step_accounted_bytes(probe, stage, want) + 100    # room for 11 samples, not 12
    rk = Rank(model, "bf16", stage, world, 0, max_batch=16, cap_bytes=cap)
    mbs, samples = rk.ctx.search_mbs(stage)
    brute = max(b for b in range(0, 17) if pb.step_accounted_bytes(rk.cfg, stage, b) <= cap)
    assert mbs == brute == want
    # the oracle's search on the same memory model visits the same batches in the same order
    calls = []

    def step(b):
        calls.append(b)
        if pb.step_accounted_bytes(rk.cfg, stage, b) > cap:
            raise opf.OutOfMemory()
        return 1.0
    now = [pb.step_accounted_bytes(rk.cfg, stage, 0, True)]

    def forward(b):
        now[0] = pb.step_accounted_bytes(rk.cfg, stage, b, True)
    o_mbs, o_samples = opf.search_mbs(lambda: now[0], forward, step, cap)
    assert o_mbs == mbs
    assert [s["batch"] for s in samples] == [b for b, _ in o_samples]
    assert all(s["t_consumed"] > 0 for s in samples)
    # curves from the measured samples, scaled for a 4-device mix 1 : 1.5 : 2 : 3, go through Algorithm 2
    bs = [s["batch"] for s in samples]
    ts = [s["t_consumed"] for s in samples]
    curves = [(bs, [t * k for t in ts], mbs) for k in (1.0, 1 / 1.5, 1 / 2.0, 1 / 3.0)]
    got = pb.allocate(stage, 64, curves, 0.0)
    ref = oal.allocate(stage, 64, curves, 0.0)
    assert got["gmbs"] == ref["gmbs"] and got["b"] == ref["b"] and got["lbs"] == ref["lbs"]
    assert sum(got["gmbs"]) == 64


def test_search_mbs_returns_zero_when_nothing_fits():
    model = MODELS["gpt"]
    rk = Rank(model, "bf16", 1, 4, 0, max_batch=4, cap_bytes=1000)
    mbs, samples = rk.ctx.search_mbs(1)
    assert mbs == 0 and samples == []


# ---- gradient accumulation over uneven micro-batches (the gas / lbs outputs of Algorithm 2) ------------------------
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("stage", [0, 1, 2, 3])
@pytest.mark.parametrize("arch", ["gpt", "llama"])
def test_accum_step_equals_one_step_on_the_whole_run(arch, stage, dtype):
    """gas - 1 micro-steps at b and a last one at lbs give the gradient, loss and update of one big batch."""
    model, world, rank = MODELS[arch], 4, 2
    micro = [2, 2, 1]                     # b = 2, gas = 3, lbs = 1
    n = sum(micro)
    rk = Rank(model, dtype, stage, world, rank, max_batch=n)
    prof = rk.ctx.accum_step(stage, micro, n)
    sync()
    fq = quantize(rk.flat, dtype)
    loss, grad, _ = otr.model_fwd_bwd(model, fq, rk.tok[:n], rk.tgt[:n], 1.0 / (n * model["S"]))
    tol = TOL[dtype]
    assert prof["batch"] == n
    assert abs(prof["loss"] - loss) <= (5e-3 if dtype == "bf16" else 1e-5) * abs(loss)
    got = to_np(rk.grads)
    sl = slice(rk.off, rk.off + rk.valid)
    if stage < 2:
        table, _ = otr.offsets(rk.spec)
        for name, (off, shape) in table.items():
            k = int(np.prod(shape))
            assert rel_l2(got[off:off + k], grad[off:off + k]) <= tol, name
        g_used = got[sl]
    else:
        assert rel_l2(got[:rk.valid], grad[sl]) <= tol
        assert np.all(got[rk.valid:] == 0)
        g_used = got[:rk.valid]
    # one optimizer step, taken on the accumulated gradient
    p0 = rk.flat[sl].astype(np.float64)
    z = np.zeros_like(p0)
    rp, rm, rv = oopt.adam_step(p0, z, z, g_used, 1, **HP)
    assert rel_l2(to_np(rk.master)[:rk.valid], rp) <= 1e-6
    assert rel_l2(to_np(rk.m)[:rk.valid], rm) <= 1e-6
    assert rel_l2(to_np(rk.v)[:rk.valid], rv) <= 1e-6
    assert prof["t_adam"] > 0 and prof["t_fwd"] > 0 and prof["n_gemm"] == 0


def test_accum_step_of_one_micro_batch_is_profile_step():
    model = MODELS["gpt"]
    # the last rank's shard holds no part of wte, whose gradient collects float atomics in free order:
    # everything else is bit-equal
    a = Rank(model, "f32", 1, 4, 3, max_batch=3)
    b = Rank(model, "f32", 1, 4, 3, max_batch=3)
    V, H = model["V"], model["H"]
    assert a.off >= V * H
    a.ctx.profile_step(1, 3)
    b.ctx.accum_step(1, [3], 3)
    sync()
    assert torch.equal(a.master, b.master) and torch.equal(a.m, b.m) and torch.equal(a.v, b.v)
    assert torch.equal(a.grads[V * H:], b.grads[V * H:])
    assert rel_l2(to_np(a.grads[:V * H]), to_np(b.grads[:V * H])) <= 1e-6


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("arch", ["gpt", "llama"])
def test_deterministic_step_repeats_bit_for_bit(arch, dtype):
    """cfg.deterministic: the embedding-matrix gradient is summed in sequence order and no contraction is split over
    atomics, so the whole gradient, wte included, repeats bit for bit, equals the accumulation path's, and is still
    the oracle's gradient."""
    model, B = dict(MODELS[arch], V=37), 4        # a small vocabulary: every id occurs many times
    a = Rank(model, dtype, 0, 1, 0, max_batch=B, deterministic=True)
    b = Rank(model, dtype, 0, 1, 0, max_batch=B, deterministic=True)
    c = Rank(model, dtype, 0, 1, 0, max_batch=B, deterministic=True)
    pa = a.ctx.profile_step(0, B)
    pb_ = b.ctx.profile_step(0, B)
    c.ctx.accum_step(0, [B], B)
    sync()
    assert torch.equal(a.grads, b.grads) and torch.equal(a.grads, c.grads) and torch.equal(a.master, b.master)
    assert pa["loss"] == pb_["loss"]
    loss, grad, _ = otr.model_fwd_bwd(model, quantize(a.flat, dtype), a.tok[:B], a.tgt[:B], 1.0 / (B * model["S"]))
    table, _ = otr.offsets(a.spec)
    got = to_np(a.grads)
    for name, (off, shape) in table.items():
        k = int(np.prod(shape))
        assert rel_l2(got[off:off + k], grad[off:off + k]) <= TOL[dtype], name
    # ids outside the vocabulary embed as zero and get no gradient, in this path too
    d = Rank(model, dtype, 0, 1, 0, max_batch=B, deterministic=True)
    bad = d.tokens.clone()
    bad[0, 3], bad[1, 5] = -7, model["V"] + 2
    d.ctx.bind_state(d.params, d.master, d.m, d.v, d.grads, bad, B, d.ws, d.wsb, d.loss, adam_t=1)
    pd = d.ctx.profile_step(0, B)
    sync()
    assert np.isfinite(pd["loss"]) and torch.isfinite(d.grads).all()


def test_allocation_is_executable_on_two_unequal_devices():
    """Algorithm 2's output for a fast and a slow device, run as accumulation steps on each device's share of the
    global batch; the two gradients together are the gradient of the global batch."""
    model, gbs = MODELS["gpt"], 7
    bs = [1, 2, 3, 4]
    curves = [(bs, [0.010 * b + 0.004 for b in bs], 4), (bs, [0.021 * b + 0.006 for b in bs], 2)]
    plan = pb.allocate(1, gbs, curves, 0.0)
    ref = oal.allocate(1, gbs, curves, 0.0)
    assert plan["gmbs"] == ref["gmbs"] and plan["b"] == ref["b"] and plan["lbs"] == ref["lbs"]
    assert sum(plan["gmbs"]) == gbs and plan["gmbs"][0] > plan["gmbs"][1] > 0
    tok, tgt = synth.tokens(gbs, model["S"], model["V"], seed=3)
    flat = synth.init_params(otr.model_spec(model), seed=0, jitter=True)
    total = np.zeros(len(flat), np.float64)
    row = 0
    for dev in range(2):
        g, b = plan["gmbs"][dev], plan["b"][dev]
        gas = -(-g // b)
        micro = [b] * (gas - 1) + [g - (gas - 1) * b]
        assert micro[-1] == plan["lbs"][dev] and all(1 <= x <= curves[dev][2] for x in micro)
        rk = Rank(model, "f32", 0, 1, 0, max_batch=g)
        both = np.concatenate([tok[row:row + g], tgt[row:row + g, -1:]], axis=1).astype(np.int32)
        rk.tokens.copy_(torch.from_numpy(both))
        rk.ctx.accum_step(0, micro, gbs)
        sync()
        total += to_np(rk.grads).astype(np.float64)
        row += g
    _, grad, _ = otr.model_fwd_bwd(model, flat, tok, tgt, 1.0 / (gbs * model["S"]))
    assert rel_l2(total, grad) <= 5e-5


def test_accum_step_errors():
    model = MODELS["gpt"]
    rk = Rank(model, "f32", 1, 4, 0, max_batch=4)
    before = rk.master.clone()
    with pytest.raises(pb.PoplarError):
        rk.ctx.accum_step(1, [3, 2], 5)      # five rows, the token buffer holds four
    with pytest.raises(pb.PoplarError):
        rk.ctx.accum_step(1, [2, 0], 2)      # empty micro-batch
    with pytest.raises(pb.PoplarError):
        rk.ctx.accum_step(1, [], 1)
    with pytest.raises(pb.PoplarError):
        rk.ctx.accum_step(1, [2], 0)
    sync()
    assert torch.equal(before, rk.master)


# ---- a bidirectional model with a masked-language-model loss (the BERT-shaped workload) ----------------------------
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("stage", [1, 3])
def test_bidirectional_masked_lm_step_matches_oracle(stage, dtype):
    model, B, world, rank = MODELS["gpt"], 3, 4, 1
    rk = Rank(model, dtype, stage, world, rank, max_batch=B)
    cfg = pb.make_cfg(**model, dtype=dtype, world=world, rank=rank, zero_stage=stage, causal=False)
    ctx = pb.Context(cfg)
    rng = np.random.default_rng(5)
    tgt = np.where(rng.random((B, model["S"])) < 0.15, rk.tgt[:B], -1).astype(np.int32)
    n_scored = int((tgt >= 0).sum())
    assert 0 < n_scored < B * model["S"]
    d_tgt = to_dev(tgt)
    ctx.bind_state(rk.params, rk.master, rk.m, rk.v, rk.grads, rk.tokens, B, rk.ws, rk.wsb, rk.loss, own_shard=rk.own,
                   adam_t=1, lr=HP["lr"], beta1=HP["b1"], beta2=HP["b2"], eps=HP["eps"], targets=d_tgt)
    prof = ctx.profile_step(stage, B)
    sync()
    # profile_step weights every token by 1 / (B S), scored or not
    scale = 1.0 / (B * model["S"])
    loss, grad, _ = otr.model_fwd_bwd(model, quantize(rk.flat, dtype), rk.tok[:B], tgt, scale, causal=False)
    assert abs(prof["loss"] - loss) <= (5e-3 if dtype == "bf16" else 1e-5) * abs(loss)
    got = to_np(rk.grads)
    sl = slice(rk.off, rk.off + rk.valid)
    ref = grad if stage < 2 else grad[sl]
    got = got if stage < 2 else got[:rk.valid]
    assert rel_l2(got, ref) <= TOL[dtype]
    # without the mask the gradient is a different one
    _, grad_c, _ = otr.model_fwd_bwd(model, quantize(rk.flat, dtype), rk.tok[:B], tgt, scale, causal=True)
    assert rel_l2(grad_c if stage < 2 else grad_c[sl], ref) > 10 * TOL[dtype]
    assert prof["flops"] == B * (model["L"] * (6 * model["S"] * (4 * model["H"] ** 2 + 2 * model["H"] * model["F"])
                                               + 14 * model["S"] ** 2 * model["H"]) + 6 * model["S"] * model["H"] * model["V"])


# ---- memory knobs of the search: activation checkpointing, moving to the next ZeRO stage ---------------------------
def test_checkpointed_step_is_the_same_step_in_less_memory():
    model, B = MODELS["gpt"], 3
    a = Rank(model, "f32", 1, 4, 3, max_batch=B)
    b = Rank(model, "f32", 1, 4, 3, max_batch=B)
    cfg = pb.make_cfg(**model, dtype="f32", world=4, rank=3, zero_stage=1, checkpoint=True)
    ctx = pb.Context(cfg)
    wsb = pb.step_workspace_bytes(cfg, 1, B)
    assert wsb < b.wsb
    ctx.bind_state(b.params, b.master, b.m, b.v, b.grads, b.tokens, B, b.ws, wsb, b.loss, adam_t=1, lr=HP["lr"], beta1=HP["b1"],
                   beta2=HP["b2"], eps=HP["eps"])
    pa = a.ctx.profile_step(1, B)
    pc = ctx.profile_step(1, B)
    sync()
    V, H = model["V"], model["H"]
    assert a.off >= V * H          # this shard holds no part of wte, whose gradient collects atomics in free order
    assert pa["loss"] == pc["loss"]
    assert torch.equal(a.grads[V * H:], b.grads[V * H:]) and torch.equal(a.master, b.master)
    assert pc["accounted_bytes"] < pa["accounted_bytes"] and pc["flops"] == pa["flops"]


def test_checkpointing_raises_the_largest_batch_under_the_same_cap():
    model, world, stage = dict(MODELS["gpt"], L=6), 4, 1
    plain = pb.make_cfg(**model, dtype="bf16", world=world, zero_stage=stage)
    cap = pb.step_accounted_bytes(plain, stage, 4) + 100     # room for 4 samples with a stash per layer
    got = {}
    for ck in (False, True):
        cfg = pb.make_cfg(**model, dtype="bf16", world=world, zero_stage=stage, cap_bytes=cap, checkpoint=ck)
        rk = Rank(model, "bf16", stage, world, 0, max_batch=16)
        ctx = pb.Context(cfg)
        ctx.bind_state(rk.params, rk.master, rk.m, rk.v, rk.grads, rk.tokens, 16, rk.ws, rk.wsb, rk.loss, adam_t=1)
        mbs, samples = ctx.search_mbs(stage)
        assert mbs == max(b for b in range(0, 17) if pb.step_accounted_bytes(cfg, stage, b) <= cap)
        got[ck] = mbs
    assert got[False] == 4 and got[True] > 4


def test_search_moves_to_the_next_stage_when_nothing_fits():
    model, world = dict(MODELS["gpt"], L=8), 4      # deep enough for the model states to outweigh the staging bucket
    probe = pb.make_cfg(**model, dtype="bf16", world=world, zero_stage=1)
    need = [pb.step_accounted_bytes(probe, s, 1) for s in range(4)]
    assert need[0] > need[1] > need[2] > need[3]
    cap = need[2] + 10                                                        # stage 2 holds one sample, stage 1 none
    assert cap < need[1] and cap < pb.step_accounted_bytes(probe, 2, 2)
    rk = Rank(model, "bf16", 3, world, 0, max_batch=8, cap_bytes=cap)          # built for stage 3: has own_shard
    grads = torch.zeros(rk.P, device=DEV)                                      # a gradient buffer that serves every stage
    # stage 0 keeps the whole optimizer on the rank: master, m, v of P elements (rank 0's shard is their head)
    master, m, v = to_dev(rk.flat), torch.zeros(rk.P, device=DEV), torch.zeros(rk.P, device=DEV)
    rk.ctx.bind_state(rk.params, master, m, v, grads, rk.tokens, 8, rk.ws, rk.wsb, rk.loss, own_shard=rk.own, adam_t=1)
    stage, mbs, samples = rk.ctx.search_stage(0)

    def search(s):
        fits = max([b for b in range(0, 9) if pb.step_accounted_bytes(rk.cfg, s, b) <= cap], default=0)
        return fits, [None] * fits
    o_stage, o_mbs, _ = opf.search_stage(0, search)
    assert (stage, mbs) == (o_stage, o_mbs) == (2, 1)
    assert [s["batch"] for s in samples] == [1] and all(s["stage"] == 2 for s in samples)
    # nothing fits anywhere
    tiny = Rank(model, "bf16", 3, world, 0, max_batch=2, cap_bytes=1000)
    tiny.ctx.bind_state(tiny.params, tiny.master, tiny.m, tiny.v, grads, tiny.tokens, 2, tiny.ws, tiny.wsb, tiny.loss, own_shard=tiny.own, adam_t=1)
    assert tiny.ctx.search_stage(1) == (-1, 0, [])
    # a state sized for the shard cannot serve stage 0, where Adam runs over all P elements: refused before anything
    # is launched, also when stage 0 would fit the cap
    roomy = Rank(model, "bf16", 3, world, 0, max_batch=2)
    roomy.ctx.bind_state(roomy.params, roomy.master, roomy.m, roomy.v, grads, roomy.tokens, 2, roomy.ws, roomy.wsb, roomy.loss,
                         own_shard=roomy.own, adam_t=1)
    before = roomy.master.clone()
    for call in (lambda: roomy.ctx.search_stage(0), lambda: roomy.ctx.profile_step(0, 1), lambda: roomy.ctx.accum_step(0, [1], 1)):
        with pytest.raises(pb.PoplarError) as e:
            call()
        assert e.value.status == pb.ERR_INVALID and "optimizer elements" in str(e.value)
    sync()
    assert torch.equal(before, roomy.master)
    assert roomy.ctx.search_stage(1)[0] == 1          # from stage 1 on the same state serves


# ---- how many runs stand behind a profile sample ------------------------------------------------------------------
def test_sampling_runs_warmup_and_repeats_and_reports_the_median_run():
    model = MODELS["gpt"]
    # rank 3's shard holds no part of wte (float atomics in free order): everything else is bit-reproducible
    a = Rank(model, "f32", 1, 4, 3, max_batch=3)
    b = Rank(model, "f32", 1, 4, 3, max_batch=3)
    a.ctx.set_sampling(1, 3)
    pa = a.ctx.profile_step(1, 3)
    runs = [b.ctx.profile_step(1, 3) for _ in range(4)]
    sync()
    assert torch.equal(a.master, b.master) and torch.equal(a.m, b.m)       # four real steps each
    assert pa["loss"] in [r["loss"] for r in runs[1:]]                     # one of the three timed runs, reported whole
    assert pa["t_consumed"] > 0 and pa["batch"] == 3
    for bad in ((-1, 1), (0, 0), (65, 1), (0, 66)):
        with pytest.raises(pb.PoplarError):
            a.ctx.set_sampling(*bad)
    # the median of three is never the slowest run: a warmed-up sample does not carry first-launch costs
    # (on a step long enough to be bound by the GPU, not by the host's launch rate)
    c = Rank(dict(arch="gpt", L=2, H=768, nh=12, F=3072, S=1024, V=2000), "bf16", 1, 4, 0, max_batch=4)
    cold = c.ctx.profile_step(1, 4)["t_consumed"]
    c.ctx.set_sampling(1, 5)
    warm = [c.ctx.profile_step(1, 4)["t_consumed"] for _ in range(3)]
    assert max(warm) <= 1.5 * min(warm)                                      # stated spread of repeated samples
    assert min(warm) <= cold


def test_two_searches_give_the_same_allocation():
    # a step long enough to be bound by the GPU rather than by the host's launch rate: on the tiny parity model one
    # step is a quarter of a millisecond of launches, and two medians of five can differ by half of that
    model, world, stage = dict(arch="gpt", L=2, H=768, nh=12, F=3072, S=256, V=2000), 4, 1
    probe = pb.make_cfg(**model, dtype="bf16", world=world, zero_stage=stage)
    cap = pb.step_accounted_bytes(probe, stage, 12) + 100
    rk = Rank(model, "bf16", stage, world, 0, max_batch=16, cap_bytes=cap)
    rk.ctx.set_sampling(2, 5)
    found = [rk.ctx.search_mbs(stage) for _ in range(2)]
    assert found[0][0] == found[1][0] == 12
    assert [s["batch"] for s in found[0][1]] == [s["batch"] for s in found[1][1]]
    for s0, s1 in zip(found[0][1], found[1][1]):
        assert abs(s0["t_consumed"] - s1["t_consumed"]) <= 0.5 * min(s0["t_consumed"], s1["t_consumed"])
    plans = []
    for mbs, samples in found:
        bs, ts = [s["batch"] for s in samples], [s["t_consumed"] for s in samples]
        curves = [(bs, [t * k for t in ts], mbs) for k in (1.0, 1 / 1.5, 1 / 2.0, 1 / 3.0)]
        plans.append(pb.allocate(stage, 64, curves, 0.0))
    assert plans[0]["gmbs"] == plans[1]["gmbs"] and sum(plans[0]["gmbs"]) == 64


# ---- memory by measurement: the search against a real allocator with a byte budget --------------------------------
class BudgetAllocator:
    """torch's caching allocator behind a byte budget: alloc() hands out device memory while the bytes requested
    so far (on top of what was held when the budget began) stay inside it, else refuses."""

    def __init__(self, budget):
        self.base = torch.cuda.memory_allocated()
        self.budget, self.held, self.requested, self.log = budget, {}, 0, []

    def alloc(self, n):
        self.log.append(n)
        if self.base + self.requested + n > self.budget:
            return 0
        t = torch.full((n,), 255, dtype=torch.uint8, device=DEV)      # poisoned like every other scratch here
        self.held[t.data_ptr()] = (t, n)
        self.requested += n
        return t.data_ptr()

    def release(self, p):
        self.requested -= self.held.pop(p)[1]

    def bytes_now(self):
        return self.base + self.requested

    def bytes_total(self):
        return self.budget


@pytest.mark.parametrize("stage", [1, 3])
def test_search_mbs_against_a_measuring_allocator(stage):
    model, world, want = MODELS["gpt"], 4, 11
    rk = Rank(model, "bf16", stage, world, 0, max_batch=16)
    ws_bytes = lambda b: pb.step_workspace_bytes(rk.cfg, stage, b)
    al = BudgetAllocator(0)
    al.budget = al.base + ws_bytes(want) + 100                        # room for the workspace of 11 samples, not of 12
    rk.ctx.bind_state(rk.params, rk.master, rk.m, rk.v, rk.grads, rk.tokens, 16, None, 0, rk.loss, own_shard=rk.own, adam_t=1)
    rk.ctx.set_mem_hooks(al.alloc, al.release, al.bytes_now, al.bytes_total)
    mbs, samples = rk.ctx.search_mbs(stage)
    asked = list(al.log)
    assert mbs == want == max(b for b in range(1, 17) if al.base + ws_bytes(b) <= al.budget)
    assert not al.held and al.requested == 0                          # every workspace went back
    fwd1 = pb.step_forward_bytes(rk.cfg, stage, 1)
    assert al.log[0] == fwd1 and fwd1 < ws_bytes(1)
    # the oracle's Algorithm 1 on the same allocator model visits the same batches in the same order
    now = [al.base]

    def forward(b):
        now[0] = al.base + pb.step_forward_bytes(rk.cfg, stage, b)

    tried = []

    def step(b):
        tried.append(b)
        if al.base + ws_bytes(b) > al.budget:
            raise opf.OutOfMemory()
        return 1.0
    o_mbs, o_samples = opf.search_mbs(lambda: now[0], forward, step, al.budget)
    assert o_mbs == mbs and [s["batch"] for s in samples] == [b for b, _ in o_samples]
    assert asked[1:] == [ws_bytes(b) for b in tried] and tried == [1, 2, 4, 8, 16, 12, 10, 11]
    for s in samples:
        assert s["measured_bytes"] == al.base + ws_bytes(s["batch"]) and s["t_consumed"] > 0 and np.isfinite(s["loss"])
    # a refused allocation is POPLAR_ERR_OOM with the state as it was
    before = rk.master.clone()
    with pytest.raises(pb.OutOfMemory):
        rk.ctx.profile_step(stage, 12)
    sync()
    assert torch.equal(before, rk.master)
    # and the result of a step in an allocator-supplied workspace is the step's: same loss as with a bound workspace
    twin = Rank(model, "bf16", stage, world, 0, max_batch=16)
    rk2 = Rank(model, "bf16", stage, world, 0, max_batch=16)
    al2 = BudgetAllocator(1 << 60)
    rk2.ctx.set_mem_hooks(al2.alloc, al2.release, al2.bytes_now, al2.bytes_total)
    p_hook, p_bound = rk2.ctx.profile_step(stage, 3), twin.ctx.profile_step(stage, 3)
    sync()
    assert p_hook["loss"] == p_bound["loss"] and p_bound["measured_bytes"] == 0
    rk2.ctx.set_mem_hooks()
    assert rk2.ctx.profile_step(stage, 3)["measured_bytes"] == 0


@pytest.mark.parametrize("rank", [0, 3])
@pytest.mark.parametrize("stage", [1, 2, 3])
@pytest.mark.parametrize("arch", ["gpt", "llama"])
def test_profile_counts_the_elements_its_local_reduces_move(arch, stage, rank):
    """reduce_elems: nothing below stage 2; at stages 2 and 3 every gradient element of the rank's shard once, and the
    part of a tied embedding matrix that lies in the shard once more (its head term and its embedding term are
    reduced one after the other: Appendix "Details about ZeRO", gradients leave for their owner as they are formed)."""
    model, world, B = MODELS[arch], 4, 2
    rk = Rank(model, "bf16", stage, world, rank, max_batch=2)
    p = rk.ctx.profile_step(stage, B)
    sync()
    if stage < 2:
        assert p["reduce_elems"] == 0 and p["t_reduce_bwd"] == 0.0
        return
    lo, hi = rk.off, min(rk.off + rk.len, rk.P)
    tied = model["V"] * model["H"] if arch == "gpt" else 0      # the flat vector begins with the embedding matrix
    assert p["reduce_elems"] == (hi - lo) + max(0, min(hi, tied) - lo)
    assert p["t_reduce_bwd"] > 0.0


def test_kernel_timing_selects_and_counts_the_launches():
    """Per-launch timing inside a profiled step: what is selected is counted with its algorithmic flop, the rest is not,
    and the summed kernel time fits inside the step's forward + backward time."""
    model = dict(arch="gpt", L=2, H=128, nh=2, F=256, S=64, V=211)
    B = 3
    r = Rank(model, "bf16", 1, 2, 0, B)
    L, H, F, S, V = model["L"], model["H"], model["F"], model["S"], model["V"]
    T = B * S
    gemm_flop = 3 * (L * 2 * T * (4 * H * H + 2 * H * F) + 2 * T * H * V)
    attn_flop = L * B * 7 * S * S * H                     # causal: 2 S^2 H forward + 5 S^2 H backward per sample
    p = r.ctx.profile_step(1, B)
    assert p["n_gemm"] == 0 and p["n_attn"] == 0 and p["t_gemm"] == 0.0
    for sel in (1, 2, 3):
        r.ctx.set_kernel_timing(sel)
        p = r.ctx.profile_step(1, B)
        if sel & 1:
            # forward 4, backward 4 input gradients + the weight gradients as one grouped launch or four; head 3
            assert p["n_gemm"] in (L * 9 + 3, L * 12 + 3)
            assert p["n_gemm"] <= p["n_gemm_kernels"] <= 2 * p["n_gemm"]   # a span holds one kernel, or two when it is cut
            assert p["gemm_flops"] == pytest.approx(gemm_flop, rel=1e-12)
            assert 0.0 < p["t_gemm"] < p["t_fwd"] + p["t_bwd"]
        else:
            assert p["n_gemm"] == 0 and p["n_gemm_kernels"] == 0 and p["t_gemm"] == 0.0
        if sel & 2:
            assert p["n_attn"] == 2 * L
            assert p["attn_flops"] == pytest.approx(attn_flop, rel=1e-12)
            assert 0.0 < p["t_attn"] < p["t_fwd"] + p["t_bwd"]
        else:
            assert p["n_attn"] == 0 and p["t_attn"] == 0.0
    with pytest.raises(pb.PoplarError):
        r.ctx.set_kernel_timing(4)
    r.ctx.set_kernel_timing(0)
    p = r.ctx.profile_step(1, B)
    assert p["n_gemm"] == 0 and p["n_attn"] == 0
