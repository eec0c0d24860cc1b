"""Oracle: Adam on a ZeRO shard, shard index arithmetic, and the single-rank
share of the ZeRO-2 gradient reduction and ZeRO-3 parameter gather.

TEST INFRASTRUCTURE ONLY - never imported by the product path.

The paper (Appendix "Details about ZeRO") says that optimizer states (stage 1),
gradients (stage 2) and parameters (stage 3) are split across the GPUs and that
each rank updates only its own partition; it names no optimizer and no split
rule.  Readings used here: Adam with bias correction and eps outside the
square root, no weight decay; contiguous equal-length partitions of the flat
parameter vector, the last one zero-padded.
"""
import numpy as np


def shard_range(P, N, r):
    """Partition [0, P) into N contiguous shards of length ceil(P/N).
    Returns (offset, length, valid) for rank r; `valid` elements of the shard
    lie inside [0, P), the rest is padding."""
    length = -(-P // N)
    off = r * length
    valid = max(0, min(length, P - off))
    return off, length, valid


def adam_step(p, m, v, g, t, lr, b1, b2, eps):
    """One Adam update (t counts from 1).  Returns new (p, m, v); inputs are
    left untouched.  Works in the dtype of the inputs (fp64 for the oracle)."""
    m = b1 * m + (1.0 - b1) * g
    v = b2 * v + (1.0 - b2) * g * g
    mhat = m / (1.0 - b1 ** t)
    vhat = v / (1.0 - b2 ** t)
    p = p - lr * mhat / (np.sqrt(vhat) + eps)
    return p, m, v


def adam_shard(p_flat, m_flat, v_flat, g_flat, N, r, t, lr, b1, b2, eps):
    """Rank r's update: Adam on its slice of the flat vectors, nothing else
    touched.  Returns the new shard-sized (p, m, v), padded with zeros."""
    P = p_flat.shape[0]
    off, length, valid = shard_range(P, N, r)
    out = []
    sl = slice(off, off + valid)
    pn, mn, vn = adam_step(p_flat[sl], m_flat[sl], v_flat[sl], g_flat[sl], t, lr, b1, b2, eps)
    for a in (pn, mn, vn):
        buf = np.zeros(length, dtype=a.dtype)
        buf[:valid] = a
        out.append(buf)
    return tuple(out)


def bf16_round(x):
    """Round fp32 values to the nearest bfloat16 (ties to even) and return them
    as fp32.  Follows the IEEE definition on the bit pattern."""
    u = np.asarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    r = ((u + 0x7FFF + lsb) >> 16) << 16
    return r.astype(np.uint32).view(np.float32)


def zero2_reduce_local(gshard, g_full, N, r):
    """ZeRO-2, one rank's own contribution to the reduce-scatter: add the part
    of this rank's full gradient that falls in its partition into the shard
    buffer.  Returns the new shard buffer."""
    off, length, valid = shard_range(g_full.shape[0], N, r)
    out = gshard.copy()
    out[:valid] += g_full[off:off + valid]
    return out


def zero3_gather(shards, P, lo, hi):
    """ZeRO-3 all-gather of flat range [lo, hi): `shards` is the list of all N
    shard buffers (each ceil(P/N) long).  Result equals flat[lo:hi]."""
    N = len(shards)
    length = -(-P // N)
    idx = np.arange(lo, hi)
    out = np.empty(hi - lo, dtype=shards[0].dtype)
    for r in range(N):
        sel = (idx // length) == r
        out[sel] = shards[r][idx[sel] - r * length]
    return out
