"""GPU parity: one decoder layer forward + backward, embedding, head + loss,
against the fp64 oracle on the same seeded inputs."""
import numpy as np
import pytest
import torch

from oracle import transformer as otr
from paper_2408_12596_amd import binding as pb
from paper_2408_12596_amd import synth
from gpu_util import DEV, quantize, rel_l2, scratch, to_dev, to_np, sync, tdtype

pytestmark = pytest.mark.gpu

# relative-L2 bars: bf16 activations and gradients 2e-2; the fp32 path accumulates
# in float over K <= 1024 terms, so 2e-5 leaves a wide margin over sqrt(K) * 6e-8
TOL = {"bf16": 2e-2, "f32": 2e-5}

LAYER_CASES = [
    # the small parity configuration: pre-LN GPT layer, hidden 256, 4 heads, MLP 1024, seq 128, batch 2
    dict(arch="gpt", L=1, H=256, nh=4, F=1024, S=128, V=1, B=2),
    dict(arch="llama", L=1, H=128, nh=2, F=192, S=96, V=1, B=3),
    # ragged: tokens and widths that are not multiples of the GEMM tiles
    dict(arch="gpt", L=1, H=192, nh=3, F=328, S=77, V=1, B=3),
    dict(arch="llama", L=1, H=256, nh=2, F=1000, S=130, V=1, B=1),
    # wide rows (the norm backward takes a block per row above hidden 1024 in bf16, 512 in fp32), not a multiple of its 256 lanes
    dict(arch="gpt", L=1, H=1536, nh=12, F=512, S=40, V=1, B=2),
    dict(arch="llama", L=1, H=1152, nh=9, F=256, S=33, V=1, B=1),
]


def layer_inputs(case, dtype, seed=0):
    spec = [(f"l0.{n}", s) for n, s in otr.layer_spec(case["arch"], case["H"], case["F"])]
    flat = synth.init_params(spec, seed=seed, jitter=True)
    x = synth.activations((case["B"], case["S"], case["H"]), seed=seed)
    dy = synth.activations((case["B"], case["S"], case["H"]), seed=seed + 1)
    return spec, flat, x, dy


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("case", LAYER_CASES, ids=lambda c: f"{c['arch']}-H{c['H']}-S{c['S']}-B{c['B']}")
def test_layer_fwd_bwd_matches_oracle(case, dtype):
    if dtype == "bf16" and case["H"] // case["nh"] not in (64, 128):
        pytest.skip("bf16 attention supports head_dim 64 and 128")
    B, S, H, nh = case["B"], case["S"], case["H"], case["nh"]
    cfg = pb.make_cfg(**{k: case[k] for k in ("arch", "L", "H", "nh", "F", "S", "V")}, dtype=dtype)
    ctx = pb.Context(cfg)
    spec, flat, x, dy = layer_inputs(case, dtype)
    n = len(flat)
    assert n == pb.layer_param_count(cfg)
    d_params, d_x, d_dy = to_dev(flat, dtype), to_dev(x, dtype), to_dev(dy, dtype)
    d_out = torch.empty_like(d_x)
    d_dx = torch.empty_like(d_x)
    saved = scratch(pb.layer_saved_bytes(cfg, B))
    wsb = pb.layer_workspace_bytes(cfg, B)
    ws = scratch(wsb)
    grads = torch.full((n,), float("nan"), device=DEV)
    ctx.layer_fwd(B, d_x, d_params, d_out, saved)
    ctx.layer_bwd(B, d_x, d_dy, d_params, saved, d_dx, grads, 0, ws, wsb)
    sync()

    p = {k[3:]: v for k, v in otr.unpack(quantize(flat, dtype), spec).items()}
    ref_out, cache = otr.layer_fwd(case["arch"], p, quantize(x, dtype), nh)
    ref_dx, ref_g = otr.layer_bwd(case["arch"], p, quantize(dy, dtype), cache, nh)
    tol = TOL[dtype]
    assert rel_l2(to_np(d_out), ref_out) <= tol
    assert rel_l2(to_np(d_dx), ref_dx) <= tol
    table, _ = otr.offsets(spec)
    got = to_np(grads)
    assert np.isfinite(got).all()
    for name, (off, shape) in table.items():
        k = int(np.prod(shape))
        assert rel_l2(got[off:off + k], ref_g[name[3:]]) <= tol, name

    # accumulate = 1 adds the same gradient again
    ctx.layer_bwd(B, d_x, d_dy, d_params, saved, d_dx, grads, 1, ws, wsb)
    sync()
    assert rel_l2(to_np(grads), 2 * got) <= 1e-6

    # dx may share dy's buffer (the interface allows it): same results
    d_io = d_dy.clone()
    grads2 = torch.full((n,), float("nan"), device=DEV)
    ctx.layer_bwd(B, d_x, d_io, d_params, saved, d_io, grads2, 0, ws, wsb)
    sync()
    assert rel_l2(to_np(d_io), to_np(d_dx)) <= 1e-6
    assert rel_l2(to_np(grads2), got) <= 1e-5


def test_layer_bwd_rejects_small_workspace():
    case = LAYER_CASES[0]
    cfg = pb.make_cfg(**{k: case[k] for k in ("arch", "L", "H", "nh", "F", "S", "V")}, dtype="f32")
    ctx = pb.Context(cfg)
    t = torch.zeros(16, device=DEV)
    with pytest.raises(pb.OutOfMemory):
        ctx.layer_bwd(2, t, t, t, t, t, t, 0, t, 64)
    with pytest.raises(pb.PoplarError):
        ctx.layer_fwd(0, t, t, t, t)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("arch", ["gpt", "llama"])
def test_embedding_fwd_bwd(arch, dtype):
    B, S, H, V = 3, 40, 64, 97
    cfg = pb.make_cfg(arch=arch, L=1, H=H, nh=1, F=64, S=S, V=V, dtype=dtype)
    ctx = pb.Context(cfg)
    rng = np.random.default_rng(0)
    wte = (rng.standard_normal((V, H)) * 0.5).astype(np.float32)
    wpe = (rng.standard_normal((S, H)) * 0.5).astype(np.float32)
    tok, _ = synth.tokens(B, S, V, seed=0)
    tok[0, :5] = tok[1, 0]          # repeated ids exercise the scatter-add
    dx = synth.activations((B, S, H), seed=3)
    d_tok = to_dev(tok)
    d_x = torch.empty((B, S, H), dtype=tdtype(dtype), device=DEV)
    ctx.embed_fwd(B, d_tok, to_dev(wte, dtype), to_dev(wpe, dtype) if arch == "gpt" else None, d_x)
    dwte = torch.zeros((V, H), device=DEV)
    dwpe = torch.full((S, H), float("nan"), device=DEV) if arch == "gpt" else None
    ctx.embed_bwd(B, d_tok, to_dev(dx, dtype), dwte, dwpe, 0)
    sync()
    ref_x = otr.embed_fwd(arch, quantize(wte, dtype), quantize(wpe, dtype), tok)
    assert rel_l2(to_np(d_x), ref_x) <= (4e-3 if dtype == "bf16" else 1e-7)
    r_dwte, r_dwpe = otr.embed_bwd(arch, quantize(dx, dtype), tok, V, S)
    assert rel_l2(to_np(dwte), r_dwte) <= 1e-6
    if arch == "gpt":
        assert rel_l2(to_np(dwpe), r_dwpe) <= 1e-6

    # ids outside [0, V) embed as zero rows and receive no gradient
    bad = tok.copy()
    bad[0, 0], bad[1, 5] = V, -3
    d_bad = to_dev(bad)
    ctx.embed_fwd(B, d_bad, to_dev(wte, dtype), to_dev(wpe, dtype) if arch == "gpt" else None, d_x)
    dwte2 = torch.zeros((V, H), device=DEV)
    ctx.embed_bwd(B, d_bad, to_dev(dx, dtype), dwte2, dwpe, 0)
    sync()
    ok = tok.copy()
    ref_ok = otr.embed_fwd(arch, quantize(wte, dtype), quantize(wpe, dtype), ok)
    got_x = to_np(d_x)
    pos = quantize(wpe, dtype) if arch == "gpt" else np.zeros((S, H))
    for (b, s_) in ((0, 0), (1, 5)):
        np.testing.assert_allclose(got_x[b, s_], pos[s_], atol=1e-6)
        ref_ok[b, s_] = got_x[b, s_]
    assert rel_l2(got_x, ref_ok) <= (4e-3 if dtype == "bf16" else 1e-7)
    r2 = r_dwte.copy()
    for (b, s_) in ((0, 0), (1, 5)):
        r2[tok[b, s_]] -= quantize(dx, dtype)[b, s_]
    assert rel_l2(to_np(dwte2), r2) <= 1e-6


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("arch,V", [("gpt", 211), ("llama", 256), ("gpt", 1031), ("llama", 20011), ("gpt", 50257), ("llama", 70001)])
def test_head_loss_fwd_bwd(arch, V, dtype):
    check_head_loss(arch, V, dtype, 2, 48, 128)


# Row counts that make the row kernels (final norm forward / backward, loss) walk several rows per wave or block, with
# an odd count so that the last pair of rows is half empty; hidden 128 takes the wave-per-row norm kernels, 1152 the
# block-per-row backward; the vocabularies give the loss kernel 1, 2 and 3 vectors per thread.
@pytest.mark.parametrize("arch,V,H", [("gpt", 1031, 128), ("llama", 9001, 128), ("gpt", 20011, 1152)])
def test_head_loss_over_many_rows(arch, V, H):
    check_head_loss(arch, V, "bf16", 5, 379, H)


def check_head_loss(arch, V, dtype, B, S, H):
    cfg = pb.make_cfg(arch=arch, L=1, H=H, nh=H // 64, F=128, S=S, V=V, dtype=dtype)
    ctx = pb.Context(cfg)
    rng = np.random.default_rng(1)
    x = synth.activations((B, S, H), seed=5)
    gf = (1 + 0.1 * rng.standard_normal(H)).astype(np.float32)
    bf = (0.1 * rng.standard_normal(H)).astype(np.float32)
    wh = (rng.standard_normal((V, H)) * 0.1).astype(np.float32)
    _, tgt = synth.tokens(B, S, V, seed=2)
    scale = 1.0 / (B * S)
    loss = torch.zeros(1, device=DEV)
    d_dx = torch.empty((B, S, H), dtype=tdtype(dtype), device=DEV)
    d_gf, d_bf = torch.full((H,), float("nan"), device=DEV), torch.full((H,), float("nan"), device=DEV)
    d_wh = torch.full((V, H), float("nan"), device=DEV)
    wsb = pb.head_workspace_bytes(cfg, B)
    ws = scratch(wsb)
    ctx.head_loss_fwd_bwd(B, to_dev(x, dtype), to_dev(tgt.reshape(-1)), to_dev(gf, dtype), to_dev(bf, dtype) if arch == "gpt" else None,
                          to_dev(wh, dtype), scale, loss, d_dx, d_gf, d_bf if arch == "gpt" else None, d_wh, 0, ws, wsb)
    sync()
    xq, gq, bq, wq = quantize(x, dtype), quantize(gf, dtype), quantize(bf, dtype), quantize(wh, dtype)
    if arch == "gpt":
        hf, nc = otr.layernorm_fwd(xq, gq, bq)
    else:
        hf, nc = otr.rmsnorm_fwd(xq, gq)
    logits = hf.reshape(-1, H) @ wq.T
    r_loss, dlog = otr.xent_fwd_bwd(logits, tgt.reshape(-1), scale)
    r_dwh = dlog.T @ hf.reshape(-1, H)
    dhf = (dlog @ wq).reshape(hf.shape)
    tol = TOL[dtype]
    assert abs(loss.item() - r_loss) <= (5e-3 if dtype == "bf16" else 1e-5) * abs(r_loss)
    if arch == "gpt":
        r_dx, r_dg, r_db = otr.layernorm_bwd(dhf, gq, nc)
        assert rel_l2(to_np(d_bf), r_db) <= tol
    else:
        r_dx, r_dg = otr.rmsnorm_bwd(dhf, gq, nc)
    assert rel_l2(to_np(d_dx), r_dx) <= tol
    assert rel_l2(to_np(d_gf), r_dg) <= tol
    assert rel_l2(to_np(d_wh), r_dwh) <= tol


# ---- bidirectional attention and a masked-language-model loss (the BERT-shaped workload) ---------------------------
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("S", [128, 200])
def test_layer_without_causal_mask_matches_oracle(S, dtype):
    case = dict(arch="gpt", L=1, H=256, nh=4, F=512, S=S, V=64, B=2)
    B, H, nh = case["B"], case["H"], case["nh"]
    cfg = pb.make_cfg(**{k: case[k] for k in ("arch", "L", "H", "nh", "F", "S", "V")}, dtype=dtype, causal=False)
    ctx = pb.Context(cfg)
    spec, flat, x, dy = layer_inputs(case, dtype, seed=4)
    n = len(flat)
    d_params, d_x, d_dy = to_dev(flat, dtype), to_dev(x, dtype), to_dev(dy, dtype)
    d_out, d_dx = torch.empty_like(d_x), torch.empty_like(d_x)
    saved = scratch(pb.layer_saved_bytes(cfg, B))
    wsb = pb.layer_workspace_bytes(cfg, B)
    ws = scratch(wsb)
    grads = torch.full((n,), float("nan"), device=DEV)
    ctx.layer_fwd(B, d_x, d_params, d_out, saved)
    ctx.layer_bwd(B, d_x, d_dy, d_params, saved, d_dx, grads, 0, ws, wsb)
    sync()
    p = {k[3:]: v for k, v in otr.unpack(quantize(flat, dtype), spec).items()}
    ref_out, cache = otr.layer_fwd("gpt", p, quantize(x, dtype), nh, causal=False)
    ref_dx, ref_g = otr.layer_bwd("gpt", p, quantize(dy, dtype), cache, nh)
    tol = TOL[dtype]
    assert rel_l2(to_np(d_out), ref_out) <= tol
    assert rel_l2(to_np(d_dx), ref_dx) <= tol
    # the mask matters: the attention weights' gradient under the causal mask is far from this one (the layer
    # output itself is dominated by the residual stream and would not tell the two apart at the bf16 tolerance)
    _, cache_c = otr.layer_fwd("gpt", p, quantize(x, dtype), nh, causal=True)
    _, ref_g_c = otr.layer_bwd("gpt", p, quantize(dy, dtype), cache_c, nh)
    assert rel_l2(ref_g["Wqkv"], ref_g_c["Wqkv"]) > 10 * tol
    table, _ = otr.offsets(spec)
    got = to_np(grads)
    for name, (off, shape) in table.items():
        k = int(np.prod(shape))
        assert rel_l2(got[off:off + k], ref_g[name[3:]]) <= tol, name


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_head_loss_scores_only_positions_with_a_target(dtype):
    B, S, H, V = 2, 48, 128, 211
    cfg = pb.make_cfg(arch="gpt", L=1, H=H, nh=2, F=128, S=S, V=V, dtype=dtype, causal=False)
    ctx = pb.Context(cfg)
    rng = np.random.default_rng(3)
    x = synth.activations((B, S, H), seed=6)
    gf = (1 + 0.1 * rng.standard_normal(H)).astype(np.float32)
    bf = (0.1 * rng.standard_normal(H)).astype(np.float32)
    wh = (rng.standard_normal((V, H)) * 0.1).astype(np.float32)
    _, tgt = synth.tokens(B, S, V, seed=2)
    tgt = np.where(rng.random((B, S)) < 0.15, tgt, -1).astype(np.int32)     # 15 % of the positions are scored
    assert 0 < (tgt >= 0).sum() < B * S
    scale = 1.0 / (tgt >= 0).sum()
    loss = torch.zeros(1, device=DEV)
    d_dx = torch.empty((B, S, H), dtype=tdtype(dtype), device=DEV)
    d_gf, d_bf = torch.full((H,), float("nan"), device=DEV), torch.full((H,), float("nan"), device=DEV)
    d_wh = torch.full((V, H), float("nan"), device=DEV)
    wsb = pb.head_workspace_bytes(cfg, B)
    ws = scratch(wsb)
    # a class index of V or more counts as "no prediction" too (the kernel never reads outside the row)
    sent = tgt.reshape(-1).copy()
    unscored = np.flatnonzero(sent < 0)
    sent[unscored[::3]] = V
    sent[unscored[1::3]] = V + 100000
    ctx.head_loss_fwd_bwd(B, to_dev(x, dtype), to_dev(sent), to_dev(gf, dtype), to_dev(bf, dtype), to_dev(wh, dtype), scale,
                          loss, d_dx, d_gf, d_bf, d_wh, 0, ws, wsb)
    sync()
    xq, gq, bq, wq = quantize(x, dtype), quantize(gf, dtype), quantize(bf, dtype), quantize(wh, dtype)
    hf, nc = otr.layernorm_fwd(xq, gq, bq)
    logits = hf.reshape(-1, H) @ wq.T
    r_loss, dlog = otr.xent_fwd_bwd(logits, tgt.reshape(-1), scale)
    r_dwh = dlog.T @ hf.reshape(-1, H)
    r_dx, r_dg, r_db = otr.layernorm_bwd((dlog @ wq).reshape(hf.shape), gq, nc)
    tol = TOL[dtype]
    assert abs(loss.item() - r_loss) <= (5e-3 if dtype == "bf16" else 1e-5) * abs(r_loss)
    assert rel_l2(to_np(d_dx), r_dx) <= tol
    assert rel_l2(to_np(d_gf), r_dg) <= tol and rel_l2(to_np(d_bf), r_db) <= tol
    assert rel_l2(to_np(d_wh), r_dwh) <= tol
