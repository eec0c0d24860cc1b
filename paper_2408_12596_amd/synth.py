"""Seeded synthetic inputs shared by the tests, the smoke check and the benchmark.

Holds no arithmetic of the method: it only draws random numbers.  The recipe
follows the workloads the paper trains (Section "Models and Baselines": GPT /
Llama shaped decoders fed token ids; the dataset fixes nothing but the shapes):
weights N(0, 0.02), norm gains 1, biases 0, activations N(0, 1), token ids
uniform in [0, V).  The caller supplies the tensor list (name, shape) in flat
order, so this module knows no layout either.
"""
import numpy as np


def _is_gain(name):
    return name.split(".")[-1] in ("g1", "g2", "gf")


def init_params(spec, seed=0, jitter=False):
    """Flat fp32 parameter vector for `spec` = [(name, shape), ...].
    jitter=False: matrices N(0,0.02), gains 1, biases 0 (the benchmark recipe).
    jitter=True : gains 1+N(0,0.1), biases N(0,0.02), so that tests see every
    term of the forward pass."""
    rng = np.random.default_rng(seed)
    parts = []
    for name, shape in spec:
        n = int(np.prod(shape))
        if len(shape) == 2:
            a = rng.standard_normal(n, dtype=np.float32) * np.float32(0.02)
        elif _is_gain(name):
            a = np.ones(n, np.float32)
            if jitter:
                a += rng.standard_normal(n, dtype=np.float32) * np.float32(0.1)
        else:
            a = np.zeros(n, np.float32)
            if jitter:
                a += rng.standard_normal(n, dtype=np.float32) * np.float32(0.02)
        parts.append(a)
    return np.concatenate(parts)


def tokens(B, S, V, seed=0):
    """[B, S+1] uniform ids; inputs are [:, :S], next-token targets [:, 1:]."""
    rng = np.random.default_rng(seed + 1000003)
    t = rng.integers(0, V, size=(B, S + 1), dtype=np.int64)
    return t[:, :S].astype(np.int32), t[:, 1:].astype(np.int32)


def activations(shape, seed=0, scale=1.0):
    rng = np.random.default_rng(seed + 7919)
    return (rng.standard_normal(int(np.prod(shape)), dtype=np.float32) * np.float32(scale)).reshape(shape)


def adam_state(n, seed=0, warm=False):
    """(g, m, v) for an n-element shard.  warm=False: zero moments (first step);
    warm=True: m ~ N(0,1e-3), v ~ |N(0,1e-6)| as after some steps."""
    rng = np.random.default_rng(seed + 104729)
    g = rng.standard_normal(n, dtype=np.float32) * np.float32(1e-2)
    if warm:
        m = rng.standard_normal(n, dtype=np.float32) * np.float32(1e-3)
        v = np.abs(rng.standard_normal(n, dtype=np.float32)) * np.float32(1e-6)
    else:
        m = np.zeros(n, np.float32)
        v = np.zeros(n, np.float32)
    return g, m, v
