"""Pins for oracle/transformer.py: finite differences, library routines,
special cases and invariants.  CPU only."""
import json
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import transformer as tr

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")

TINY = {
    "gpt": dict(arch="gpt", L=2, H=8, nh=2, F=16, S=4, V=11),
    "llama": dict(arch="llama", L=2, H=8, nh=2, F=12, S=4, V=11),
}


def rand_model(cfg, seed=0):
    rng = np.random.default_rng(seed)
    spec = tr.model_spec(cfg)
    _, P = tr.offsets(spec)
    flat = rng.standard_normal(P) * 0.3
    tok = rng.integers(0, cfg["V"], size=(2, cfg["S"]))
    tgt = rng.integers(0, cfg["V"], size=(2, cfg["S"]))
    return flat, tok, tgt


@pytest.mark.parametrize("arch", ["gpt", "llama"])
def test_backward_matches_central_differences(arch):
    cfg = TINY[arch]
    flat, tok, tgt = rand_model(cfg)
    scale = 1.0 / tok.size
    loss, grad, _ = tr.model_fwd_bwd(cfg, flat, tok, tgt, scale)
    rng = np.random.default_rng(1)
    # every tensor gets probed: 6 random entries each
    table, _ = tr.offsets(tr.model_spec(cfg))
    eps = 1e-6
    for name, (off, shape) in table.items():
        n = int(np.prod(shape))
        for j in rng.choice(n, size=min(6, n), replace=False):
            i = off + int(j)
            fp, fm = flat.copy(), flat.copy()
            fp[i] += eps
            fm[i] -= eps
            lp = tr.model_fwd_bwd(cfg, fp, tok, tgt, scale)[0]
            lm = tr.model_fwd_bwd(cfg, fm, tok, tgt, scale)[0]
            fd = (lp - lm) / (2 * eps)
            assert abs(fd - grad[i]) <= 1e-6 * max(1.0, abs(fd)) + 1e-8, (name, j, fd, grad[i])


@pytest.mark.parametrize("arch", ["gpt", "llama"])
def test_layer_input_gradient_by_central_differences(arch):
    cfg = TINY[arch]
    H, F_, nh, S = cfg["H"], cfg["F"], cfg["nh"], cfg["S"]
    rng = np.random.default_rng(2)
    p = {n: rng.standard_normal(s) * 0.4 for n, s in tr.layer_spec(arch, H, F_)}
    x = rng.standard_normal((2, S, H))
    w = rng.standard_normal((2, S, H))
    out, c = tr.layer_fwd(arch, p, x, nh)
    dx, _ = tr.layer_bwd(arch, p, w, c, nh)
    eps = 1e-6
    for _ in range(20):
        idx = tuple(rng.integers(0, d) for d in x.shape)
        xp, xm = x.copy(), x.copy()
        xp[idx] += eps
        xm[idx] -= eps
        fd = ((tr.layer_fwd(arch, p, xp, nh)[0] * w).sum() - (tr.layer_fwd(arch, p, xm, nh)[0] * w).sum()) / (2 * eps)
        assert abs(fd - dx[idx]) <= 1e-6 * max(1.0, abs(fd))


def _torch_model_loss(cfg, flat_t, tok, tgt, scale):
    """The same model from torch's library routines (third opinion)."""
    arch, L, H, nh, S, V = cfg["arch"], cfg["L"], cfg["H"], cfg["nh"], cfg["S"], cfg["V"]
    table, _ = tr.offsets(tr.model_spec(cfg))

    def get(name):
        off, shape = table[name]
        return flat_t[off:off + int(np.prod(shape))].reshape(shape)

    tok_t = torch.from_numpy(tok)
    x = get("wte")[tok_t]
    if arch == "gpt":
        x = x + get("wpe")[None, :S]
    d = H // nh
    B = tok.shape[0]
    for l in range(L):
        g = lambda n: get(f"l{l}.{n}")
        if arch == "gpt":
            a = F.layer_norm(x, (H,), g("g1"), g("b1"), 1e-5)
            qkv = F.linear(a, g("Wqkv"), g("bqkv"))
        else:
            a = x * torch.rsqrt((x * x).mean(-1, keepdim=True) + 1e-5) * g("g1")
            qkv = F.linear(a, g("Wqkv"))
        q, k, v = (t.reshape(B, S, nh, d).transpose(1, 2) for t in qkv.chunk(3, -1))
        if arch == "llama":
            inv = 10000.0 ** (-torch.arange(0, d, 2, dtype=torch.float64) / d)
            ang = torch.arange(S, dtype=torch.float64)[:, None] * inv[None]
            cos, sin = torch.cat([ang.cos(), ang.cos()], -1), torch.cat([ang.sin(), ang.sin()], -1)

            def rot(t):
                t1, t2 = t[..., :d // 2], t[..., d // 2:]
                return t * cos + torch.cat([-t2, t1], -1) * sin
            q, k = rot(q), rot(k)
        o = F.scaled_dot_product_attention(q, k, v, is_causal=True)
        o = o.transpose(1, 2).reshape(B, S, H)
        if arch == "gpt":
            x = x + F.linear(o, g("Wo"), g("bo"))
            m = F.layer_norm(x, (H,), g("g2"), g("b2"), 1e-5)
            x = x + F.linear(F.gelu(F.linear(m, g("W1"), g("bm1")), approximate="tanh"), g("W2"), g("bm2"))
        else:
            x = x + F.linear(o, g("Wo"))
            m = x * torch.rsqrt((x * x).mean(-1, keepdim=True) + 1e-5) * g("g2")
            x = x + F.linear(F.silu(F.linear(m, g("Wg"))) * F.linear(m, g("Wu")), g("Wd"))
    if arch == "gpt":
        hf = F.layer_norm(x, (H,), get("gf"), get("bf"), 1e-5)
        logits = F.linear(hf, get("wte"))
    else:
        hf = x * torch.rsqrt((x * x).mean(-1, keepdim=True) + 1e-5) * get("gf")
        logits = F.linear(hf, get("Whead"))
    return scale * F.cross_entropy(logits.reshape(-1, V), torch.from_numpy(tgt).reshape(-1), reduction="sum")


@pytest.mark.parametrize("arch", ["gpt", "llama"])
def test_against_torch_library_routines(arch):
    cfg = dict(TINY[arch], S=6, H=16, nh=4, F=24, L=3)
    flat, tok, tgt = rand_model(cfg, seed=3)
    scale = 0.37
    loss, grad, _ = tr.model_fwd_bwd(cfg, flat, tok, tgt, scale)
    ft = torch.tensor(flat, dtype=torch.float64, requires_grad=True)
    lt = _torch_model_loss(cfg, ft, tok, tgt, scale)
    lt.backward()
    assert abs(loss - lt.item()) < 1e-10 * max(1, abs(loss))
    np.testing.assert_allclose(grad, ft.grad.numpy(), rtol=1e-8, atol=1e-11)


def test_causal_first_row_and_single_token():
    rng = np.random.default_rng(4)
    q, k, v = (rng.standard_normal((1, 2, 5, 4)) for _ in range(3))
    o, p = tr.attention_fwd(q, k, v)
    np.testing.assert_allclose(o[:, :, 0], v[:, :, 0], rtol=1e-14)
    assert np.all(np.triu(p[0, 0], 1) == 0)
    np.testing.assert_allclose(p.sum(-1), 1.0, rtol=1e-14)
    o1, _ = tr.attention_fwd(q[:, :, :1], k[:, :, :1], v[:, :, :1])
    np.testing.assert_allclose(o1, v[:, :, :1], rtol=1e-14)


def test_attention_matches_scipy_softmax():
    from scipy.special import softmax
    rng = np.random.default_rng(5)
    q, k, v = (rng.standard_normal((1, 1, 6, 8)) for _ in range(3))
    o, _ = tr.attention_fwd(q, k, v, causal=False)
    ref = softmax(q[0, 0] @ k[0, 0].T / np.sqrt(8), axis=-1) @ v[0, 0]
    np.testing.assert_allclose(o[0, 0], ref, rtol=1e-12)


@pytest.mark.parametrize("arch", ["gpt", "llama"])
def test_zero_output_projections_give_identity(arch):
    cfg = TINY[arch]
    rng = np.random.default_rng(6)
    p = {n: rng.standard_normal(s) for n, s in tr.layer_spec(arch, cfg["H"], cfg["F"])}
    p["Wo"][:] = 0
    if arch == "gpt":
        p["W2"][:] = 0
        p["bo"][:] = 0
        p["bm2"][:] = 0
    else:
        p["Wd"][:] = 0
    x = rng.standard_normal((2, cfg["S"], cfg["H"]))
    out, c = tr.layer_fwd(arch, p, x, cfg["nh"])
    np.testing.assert_array_equal(out, x)
    # residual path: d(sum out)/dx = 1 when both branches are cut
    dx, _ = tr.layer_bwd(arch, p, np.ones_like(x), c, cfg["nh"])
    np.testing.assert_allclose(dx, 1.0, atol=1e-13)


def test_rope_properties():
    S, d = 9, 8
    cos, sin = tr.rope_tables(S, d)
    rng = np.random.default_rng(7)
    q = rng.standard_normal((1, 1, S, d))
    k = rng.standard_normal((1, 1, S, d))
    rq = tr.rope_apply(q, cos, sin)
    np.testing.assert_allclose(np.linalg.norm(rq, axis=-1), np.linalg.norm(q, axis=-1), rtol=1e-13)
    np.testing.assert_array_equal(rq[:, :, 0], q[:, :, 0])
    # relative-position property: same vectors at every position
    qq = np.broadcast_to(q[:, :, :1], q.shape)
    kk = np.broadcast_to(k[:, :, :1], k.shape)
    dots = tr.rope_apply(qq, cos, sin)[0, 0] @ tr.rope_apply(kk, cos, sin)[0, 0].T
    for off in range(-3, 4):
        diag = np.diagonal(dots, off)
        np.testing.assert_allclose(diag, diag[0], rtol=1e-12, atol=1e-12)
    # adjoint undoes the rotation
    np.testing.assert_allclose(tr.rope_apply(rq, cos, sin, -1.0), q, atol=1e-13)
    # first pair of position 1 rotates by exactly 1 radian (base**0)
    e = np.zeros((1, 1, 2, d))
    e[0, 0, 1, 0] = 1.0
    r = tr.rope_apply(e, *tr.rope_tables(2, d))
    np.testing.assert_allclose([r[0, 0, 1, 0], r[0, 0, 1, d // 2]], [np.cos(1.0), np.sin(1.0)], rtol=1e-14)


def test_cross_entropy_closed_forms():
    V, T = 13, 5
    loss, dl = tr.xent_fwd_bwd(np.full((T, V), 2.5), np.arange(T), 1.0 / T)
    assert abs(loss - np.log(V)) < 1e-13
    np.testing.assert_allclose(dl.sum(-1), 0.0, atol=1e-15)
    rng = np.random.default_rng(8)
    lg = rng.standard_normal((T, V)) * 3
    _, dl = tr.xent_fwd_bwd(lg, np.arange(T), 0.5)
    np.testing.assert_allclose(dl.sum(-1), 0.0, atol=1e-15)


def test_cross_entropy_skips_positions_without_a_target():
    """Negative targets: against torch's ignore_index (loss and its autograd gradient), and by restriction
    to the scored rows."""
    rng = np.random.default_rng(11)
    T, V = 9, 17
    lg = rng.standard_normal((T, V)) * 2
    tgt = rng.integers(0, V, T)
    tgt[[1, 4, 5]] = -1
    loss, dl = tr.xent_fwd_bwd(lg, tgt, 0.25)
    tl = torch.tensor(lg, requires_grad=True)
    tt = torch.tensor(np.where(tgt < 0, -100, tgt))
    ref = 0.25 * F.cross_entropy(tl, tt, ignore_index=-100, reduction="sum")
    ref.backward()
    assert abs(loss - ref.item()) < 1e-12
    np.testing.assert_allclose(dl, tl.grad.numpy(), atol=1e-14)
    assert np.all(dl[[1, 4, 5]] == 0)
    keep = tgt >= 0
    loss_k, dl_k = tr.xent_fwd_bwd(lg[keep], tgt[keep], 0.25)
    assert abs(loss - loss_k) < 1e-13
    np.testing.assert_array_equal(dl[keep], dl_k)
    # nothing scored: zero loss, zero gradient
    loss0, dl0 = tr.xent_fwd_bwd(lg, np.full(T, -1), 1.0)
    assert loss0 == 0 and not dl0.any()


def test_gelu_and_silu_values():
    # tanh-form GeLU at 1: 0.5*(1+tanh(sqrt(2/pi)*1.044715))
    assert abs(tr.gelu_fwd(np.array(1.0)) - 0.8411919906082768) < 1e-15
    assert tr.gelu_fwd(np.array(0.0)) == 0.0
    x = np.linspace(-4, 4, 33)
    np.testing.assert_allclose(tr.gelu_fwd(x), F.gelu(torch.tensor(x), approximate="tanh").numpy(), rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(tr.silu_fwd(x), F.silu(torch.tensor(x)).numpy(), rtol=1e-13, atol=1e-15)
    e = 1e-6
    np.testing.assert_allclose(tr.gelu_bwd(1.0, x), (tr.gelu_fwd(x + e) - tr.gelu_fwd(x - e)) / (2 * e), rtol=1e-7, atol=1e-9)
    np.testing.assert_allclose(tr.silu_bwd(1.0, x), (tr.silu_fwd(x + e) - tr.silu_fwd(x - e)) / (2 * e), rtol=1e-7, atol=1e-9)


def test_norms_against_definitions():
    rng = np.random.default_rng(9)
    x = rng.standard_normal((3, 16)) * 2 + 1
    g, b = rng.standard_normal(16), rng.standard_normal(16)
    y, _ = tr.layernorm_fwd(x, g, b)
    yn = (y - b) / g
    np.testing.assert_allclose(yn.mean(-1), 0, atol=1e-13)
    np.testing.assert_allclose((yn ** 2).mean(-1), x.var(-1) / (x.var(-1) + 1e-5), rtol=1e-12)
    y, _ = tr.rmsnorm_fwd(x, g)
    np.testing.assert_allclose(((y / g) ** 2).mean(-1), (x * x).mean(-1) / ((x * x).mean(-1) + 1e-5), rtol=1e-12)


def test_parameter_counts_match_fixture():
    """Model sizes of the four workload shapes (derived from the layer
    definitions; see the fixture's header)."""
    with open(os.path.join(GOLDEN, "param_counts.json")) as f:
        gold = json.load(f)
    for case in gold["cases"]:
        cfg = case["cfg"]
        _, per_layer = tr.offsets(tr.layer_spec(cfg["arch"], cfg["H"], cfg["F"]))
        assert per_layer == case["per_layer"]
        if "total" in case:
            _, P = tr.offsets(tr.model_spec(cfg))
            assert P == case["total"]
            assert P % case["world"] == 0 and P // case["world"] == case["shard"]
