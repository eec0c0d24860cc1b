"""Oracle: decoder-transformer forward and backward in fp64 NumPy.

TEST INFRASTRUCTURE ONLY - never imported by the product path.

The paper trains stock GPT-2 / Llama / BERT models through PyTorch and says
nothing about their internals (Section "Models and Baselines"); what one rank
computes in `model.step(batch)` (Algorithm 1) is therefore the textbook
definition of those models, written out here without blocking, fusion or
reordering.  Every backward function is the hand-derived adjoint of the
forward function directly above it.

Conventions (the paper is silent on all of them; the HIP path uses the same
ones so that flat indices agree):
  * every Linear weight is stored [out, in] row-major, y = x @ W.T + b;
  * fused QKV weight rows are all-q, then all-k, then all-v; head h owns rows
    h*d .. (h+1)*d of each third;
  * GPT layer block order: g1, b1, Wqkv, bqkv, Wo, bo, g2, b2, W1, bm1, W2, bm2
    model order: wte, wpe, layer 0..L-1, gf, bf;  LM head tied to wte;
  * Llama layer block order: g1, Wqkv, Wo, g2, Wg, Wu, Wd
    model order: wte, layer 0..L-1, gf, Whead (untied);
  * LayerNorm / RMSNorm eps 1e-5, biased variance;
  * GeLU is the tanh form used by GPT-2;
  * attention scores scaled by 1/sqrt(d), causal mask, no dropout;
  * RoPE pairs element i with i + d/2, angle pos * base**(-2i/d), pos from 0;
  * loss = loss_scale * sum over tokens of cross-entropy(logits_t, target_t).
"""
import numpy as np

EPS_NORM = 1e-5


# ----------------------------------------------------------------------------
# flat parameter layout
# ----------------------------------------------------------------------------
def layer_spec(arch, H, F):
    """Ordered (name, shape) list of one layer's tensors."""
    if arch == "gpt":
        return [("g1", (H,)), ("b1", (H,)), ("Wqkv", (3 * H, H)), ("bqkv", (3 * H,)),
                ("Wo", (H, H)), ("bo", (H,)), ("g2", (H,)), ("b2", (H,)),
                ("W1", (F, H)), ("bm1", (F,)), ("W2", (H, F)), ("bm2", (H,))]
    if arch == "llama":
        return [("g1", (H,)), ("Wqkv", (3 * H, H)), ("Wo", (H, H)), ("g2", (H,)),
                ("Wg", (F, H)), ("Wu", (F, H)), ("Wd", (H, F))]
    raise ValueError(arch)


def model_spec(cfg):
    """Ordered (name, shape) list of the whole model's tensors."""
    arch, L, H, F, S, V = cfg["arch"], cfg["L"], cfg["H"], cfg["F"], cfg["S"], cfg["V"]
    out = [("wte", (V, H))]
    if arch == "gpt":
        out.append(("wpe", (S, H)))
    for l in range(L):
        out += [(f"l{l}.{n}", s) for n, s in layer_spec(arch, H, F)]
    out.append(("gf", (H,)))
    if arch == "gpt":
        out.append(("bf", (H,)))
    else:
        out.append(("Whead", (V, H)))
    return out


def offsets(spec):
    """name -> (offset, shape) and the total element count."""
    table, off = {}, 0
    for name, shape in spec:
        table[name] = (off, shape)
        off += int(np.prod(shape))
    return table, off


def unpack(flat, spec, prefix=""):
    """Views into `flat` for every tensor whose name starts with prefix."""
    table, _ = offsets(spec)
    out = {}
    for name, (off, shape) in table.items():
        if name.startswith(prefix):
            out[name[len(prefix):]] = flat[off:off + int(np.prod(shape))].reshape(shape)
    return out


# ----------------------------------------------------------------------------
# elementary operations
# ----------------------------------------------------------------------------
def layernorm_fwd(x, g, b):
    mu = x.mean(-1, keepdims=True)
    var = ((x - mu) ** 2).mean(-1, keepdims=True)
    rstd = 1.0 / np.sqrt(var + EPS_NORM)
    xhat = (x - mu) * rstd
    return xhat * g + b, (xhat, rstd)


def layernorm_bwd(dy, g, cache):
    xhat, rstd = cache
    dxhat = dy * g
    dx = rstd * (dxhat - dxhat.mean(-1, keepdims=True)
                 - xhat * (dxhat * xhat).mean(-1, keepdims=True))
    red = tuple(range(dy.ndim - 1))
    return dx, (dy * xhat).sum(red), dy.sum(red)


def rmsnorm_fwd(x, g):
    rstd = 1.0 / np.sqrt((x * x).mean(-1, keepdims=True) + EPS_NORM)
    xhat = x * rstd
    return xhat * g, (xhat, rstd)


def rmsnorm_bwd(dy, g, cache):
    xhat, rstd = cache
    dxhat = dy * g
    dx = rstd * (dxhat - xhat * (dxhat * xhat).mean(-1, keepdims=True))
    red = tuple(range(dy.ndim - 1))
    return dx, (dy * xhat).sum(red)


_K0 = np.sqrt(2.0 / np.pi)
_K1 = 0.044715


def gelu_fwd(h):
    return 0.5 * h * (1.0 + np.tanh(_K0 * (h + _K1 * h ** 3)))


def gelu_bwd(dg, h):
    t = np.tanh(_K0 * (h + _K1 * h ** 3))
    dt = (1.0 - t * t) * _K0 * (1.0 + 3.0 * _K1 * h * h)
    return dg * (0.5 * (1.0 + t) + 0.5 * h * dt)


def silu_fwd(h):
    return h / (1.0 + np.exp(-h))


def silu_bwd(dy, h):
    s = 1.0 / (1.0 + np.exp(-h))
    return dy * (s + h * s * (1.0 - s))


def rope_tables(S, d, base=10000.0):
    i = np.arange(d // 2, dtype=np.float64)
    ang = np.arange(S, dtype=np.float64)[:, None] * base ** (-2.0 * i / d)[None, :]
    return np.cos(ang), np.sin(ang)


def rope_apply(x, cos, sin, sign=1.0):
    """x: [B, nh, S, d]; rotates pairs (i, i+d/2).  sign=-1 is the adjoint."""
    h = x.shape[-1] // 2
    x1, x2 = x[..., :h], x[..., h:]
    s = sign * sin
    return np.concatenate([x1 * cos - x2 * s, x2 * cos + x1 * s], axis=-1)


def split_heads(x, nh):
    """[B, S, H] -> [B, nh, S, d]"""
    B, S, H = x.shape
    return x.reshape(B, S, nh, H // nh).transpose(0, 2, 1, 3)


def merge_heads(x):
    """[B, nh, S, d] -> [B, S, H]"""
    B, nh, S, d = x.shape
    return x.transpose(0, 2, 1, 3).reshape(B, S, nh * d)


def attention_fwd(q, k, v, causal=True):
    """q, k, v: [B, nh, S, d].  Returns o and the probabilities."""
    B, nh, S, d = q.shape
    o = np.empty_like(q)
    p_all = np.empty((B, nh, S, S))
    for b in range(B):
        for h in range(nh):
            s = q[b, h] @ k[b, h].T / np.sqrt(d)
            if causal:
                s = np.where(np.tril(np.ones((S, S), bool)), s, -np.inf)
            s = s - s.max(-1, keepdims=True)
            e = np.exp(s)
            p = e / e.sum(-1, keepdims=True)
            p_all[b, h] = p
            o[b, h] = p @ v[b, h]
    return o, p_all


def attention_bwd(do, q, k, v, p_all):
    B, nh, S, d = q.shape
    dq, dk, dv = np.empty_like(q), np.empty_like(k), np.empty_like(v)
    for b in range(B):
        for h in range(nh):
            p = p_all[b, h]
            dv[b, h] = p.T @ do[b, h]
            dp = do[b, h] @ v[b, h].T
            ds = p * (dp - (dp * p).sum(-1, keepdims=True))
            dq[b, h] = ds @ k[b, h] / np.sqrt(d)
            dk[b, h] = ds.T @ q[b, h] / np.sqrt(d)
    return dq, dk, dv


# ----------------------------------------------------------------------------
# one decoder layer
# ----------------------------------------------------------------------------
def layer_fwd(arch, p, x, nh, causal=True):
    """x: [B, S, H]; p: dict of this layer's tensors.  Returns out, cache."""
    B, S, H = x.shape
    c = {"x": x}
    if arch == "gpt":
        a, c["n1"] = layernorm_fwd(x, p["g1"], p["b1"])
        qkv = a @ p["Wqkv"].T + p["bqkv"]
    else:
        a, c["n1"] = rmsnorm_fwd(x, p["g1"])
        qkv = a @ p["Wqkv"].T
    q, k, v = (split_heads(t, nh) for t in np.split(qkv, 3, axis=-1))
    if arch == "llama":
        cos, sin = rope_tables(S, H // nh)
        q, k = rope_apply(q, cos, sin), rope_apply(k, cos, sin)
    o, prob = attention_fwd(q, k, v, causal)
    om = merge_heads(o)
    x1 = x + om @ p["Wo"].T + (p["bo"] if arch == "gpt" else 0.0)
    c.update(a=a, q=q, k=k, v=v, prob=prob, om=om, x1=x1)
    if arch == "gpt":
        m, c["n2"] = layernorm_fwd(x1, p["g2"], p["b2"])
        h = m @ p["W1"].T + p["bm1"]
        g = gelu_fwd(h)
        out = x1 + g @ p["W2"].T + p["bm2"]
        c.update(m=m, h=h, g=g)
    else:
        m, c["n2"] = rmsnorm_fwd(x1, p["g2"])
        hg, hu = m @ p["Wg"].T, m @ p["Wu"].T
        g = silu_fwd(hg) * hu
        out = x1 + g @ p["Wd"].T
        c.update(m=m, hg=hg, hu=hu, g=g)
    return out, c


def _flat2(t):
    return t.reshape(-1, t.shape[-1])


def layer_bwd(arch, p, dout, c, nh):
    """Adjoint of layer_fwd.  Returns dx and a dict of parameter gradients."""
    B, S, H = dout.shape
    gr = {}
    # MLP branch
    if arch == "gpt":
        gr["bm2"] = _flat2(dout).sum(0)
        gr["W2"] = _flat2(dout).T @ _flat2(c["g"])
        dg = dout @ p["W2"]
        dh = gelu_bwd(dg, c["h"])
        gr["bm1"] = _flat2(dh).sum(0)
        gr["W1"] = _flat2(dh).T @ _flat2(c["m"])
        dm = dh @ p["W1"]
        dx1n, gr["g2"], gr["b2"] = layernorm_bwd(dm, p["g2"], c["n2"])
    else:
        gr["Wd"] = _flat2(dout).T @ _flat2(c["g"])
        dg = dout @ p["Wd"]
        dhg = silu_bwd(dg * c["hu"], c["hg"])
        dhu = dg * silu_fwd(c["hg"])
        gr["Wg"] = _flat2(dhg).T @ _flat2(c["m"])
        gr["Wu"] = _flat2(dhu).T @ _flat2(c["m"])
        dm = dhg @ p["Wg"] + dhu @ p["Wu"]
        dx1n, gr["g2"] = rmsnorm_bwd(dm, p["g2"], c["n2"])
    dx1 = dout + dx1n
    # attention branch
    if arch == "gpt":
        gr["bo"] = _flat2(dx1).sum(0)
    gr["Wo"] = _flat2(dx1).T @ _flat2(c["om"])
    do = split_heads(dx1 @ p["Wo"], nh)
    dq, dk, dv = attention_bwd(do, c["q"], c["k"], c["v"], c["prob"])
    if arch == "llama":
        cos, sin = rope_tables(S, H // nh)
        dq, dk = rope_apply(dq, cos, sin, -1.0), rope_apply(dk, cos, sin, -1.0)
    dqkv = np.concatenate([merge_heads(dq), merge_heads(dk), merge_heads(dv)], axis=-1)
    gr["Wqkv"] = _flat2(dqkv).T @ _flat2(c["a"])
    da = dqkv @ p["Wqkv"]
    if arch == "gpt":
        gr["bqkv"] = _flat2(dqkv).sum(0)
        dxn, gr["g1"], gr["b1"] = layernorm_bwd(da, p["g1"], c["n1"])
    else:
        dxn, gr["g1"] = rmsnorm_bwd(da, p["g1"], c["n1"])
    return dx1 + dxn, gr


# ----------------------------------------------------------------------------
# embedding, head and loss
# ----------------------------------------------------------------------------
def embed_fwd(arch, wte, wpe, tok):
    """tok: [B, S] ints -> [B, S, H]"""
    x = wte[tok]
    if arch == "gpt":
        x = x + wpe[np.arange(tok.shape[1])][None]
    return x


def embed_bwd(arch, dx, tok, V, S):
    dwte = np.zeros((V, dx.shape[-1]))
    np.add.at(dwte, tok.reshape(-1), _flat2(dx))
    dwpe = dx.sum(0) if arch == "gpt" else None
    return dwte, dwpe


def xent_fwd_bwd(logits, targets, loss_scale):
    """logits [T, V], targets [T].  loss = loss_scale * sum_t CE_t over the positions
    whose target is >= 0; a negative target marks a position that is not predicted
    (a masked-language-model batch scores only its masked positions): no loss, zero
    gradient."""
    targets = np.asarray(targets)
    z = logits - logits.max(-1, keepdims=True)
    lse = np.log(np.exp(z).sum(-1, keepdims=True))
    logp = z - lse
    T = logits.shape[0]
    use = targets >= 0
    rows = np.arange(T)[use]
    loss = -loss_scale * logp[rows, targets[use]].sum()
    dlogits = np.exp(logp)
    dlogits[rows, targets[use]] -= 1.0
    dlogits[~use] = 0.0
    return loss, dlogits * loss_scale


# ----------------------------------------------------------------------------
# whole model: one rank's forward + backward at local batch B
# ----------------------------------------------------------------------------
def model_fwd_bwd(cfg, flat, tok, targets, loss_scale, causal=True):
    """flat: fp64 parameter vector in model_spec order.
    tok, targets: [B, S] ints.  Returns loss, flat gradient, and the list of
    per-layer outputs (for intermediate parity checks)."""
    arch, L, nh, S, V = cfg["arch"], cfg["L"], cfg["nh"], cfg["S"], cfg["V"]
    spec = model_spec(cfg)
    P = unpack(flat, spec)
    grad = np.zeros_like(flat)
    G = unpack(grad, spec)
    x = embed_fwd(arch, P["wte"], P.get("wpe"), tok)
    caches, acts = [], [x]
    for l in range(L):
        lp = {n: P[f"l{l}.{n}"] for n, _ in layer_spec(arch, cfg["H"], cfg["F"])}
        x, c = layer_fwd(arch, lp, x, nh, causal)
        caches.append((lp, c))
        acts.append(x)
    if arch == "gpt":
        hf, nc = layernorm_fwd(x, P["gf"], P["bf"])
        Whead = P["wte"]
    else:
        hf, nc = rmsnorm_fwd(x, P["gf"])
        Whead = P["Whead"]
    logits = _flat2(hf) @ Whead.T
    loss, dlogits = xent_fwd_bwd(logits, targets.reshape(-1), loss_scale)
    dWhead = dlogits.T @ _flat2(hf)
    dhf = (dlogits @ Whead).reshape(hf.shape)
    if arch == "gpt":
        dx, G["gf"][:], G["bf"][:] = layernorm_bwd(dhf, P["gf"], nc)
        G["wte"][:] += dWhead
    else:
        dx, G["gf"][:] = rmsnorm_bwd(dhf, P["gf"], nc)
        G["Whead"][:] = dWhead
    for l in reversed(range(L)):
        lp, c = caches[l]
        dx, gr = layer_bwd(arch, lp, dx, c, nh)
        for n, gval in gr.items():
            G[f"l{l}.{n}"][:] = gval
    dwte, dwpe = embed_bwd(arch, dx, tok, V, S)
    G["wte"][:] += dwte
    if arch == "gpt":
        G["wpe"][:] = dwpe
    return loss, grad, acts
