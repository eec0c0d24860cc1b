"""Pins for oracle/optimizer.py.  CPU only."""
import numpy as np
import pytest
import torch

from oracle import optimizer as opt

HP = dict(lr=1e-3, b1=0.9, b2=0.999, eps=1e-8)


def test_adam_first_step_closed_form():
    rng = np.random.default_rng(0)
    g = rng.standard_normal(1000) * 1e-2
    p = rng.standard_normal(1000)
    z = np.zeros(1000)
    pn, mn, vn = opt.adam_step(p, z, z, g, 1, **HP)
    # from zero state: mhat = g, vhat = g^2 -> dp = -lr g / (|g| + eps)
    np.testing.assert_allclose(pn - p, -HP["lr"] * g / (np.abs(g) + HP["eps"]), rtol=1e-9, atol=1e-18)
    np.testing.assert_allclose(mn, 0.1 * g, rtol=1e-12)
    np.testing.assert_allclose(vn, 0.001 * g * g, rtol=1e-9)
    # |dp| is lr up to eps/|g|
    big = np.abs(g) > 1e-4
    np.testing.assert_allclose(np.abs(pn - p)[big], HP["lr"], rtol=2e-4)


def test_adam_zero_gradient_zero_state_is_noop():
    p = np.linspace(-1, 1, 17)
    z = np.zeros(17)
    pn, mn, vn = opt.adam_step(p, z, z, z, 1, **HP)
    np.testing.assert_array_equal(pn, p)
    np.testing.assert_array_equal(mn, z)
    np.testing.assert_array_equal(vn, z)


def test_adam_matches_torch_optimizer_over_steps():
    rng = np.random.default_rng(1)
    p = rng.standard_normal(257)
    pt = torch.tensor(p, dtype=torch.float64, requires_grad=True)
    o = torch.optim.Adam([pt], lr=HP["lr"], betas=(HP["b1"], HP["b2"]), eps=HP["eps"])
    m = np.zeros_like(p)
    v = np.zeros_like(p)
    for t in range(1, 8):
        g = rng.standard_normal(257) * 10.0 ** rng.integers(-4, 1)
        pt.grad = torch.tensor(g)
        o.step()
        p, m, v = opt.adam_step(p, m, v, g, t, **HP)
        np.testing.assert_allclose(p, pt.detach().numpy(), rtol=1e-12, atol=1e-14)


@pytest.mark.parametrize("P,N", [(1000, 4), (1001, 4), (17, 3), (50, 7), (5, 8)])
def test_shards_partition_and_concat_equals_unsharded(P, N):
    rng = np.random.default_rng(2)
    p, g = rng.standard_normal(P), rng.standard_normal(P)
    m, v = rng.standard_normal(P) * 1e-3, np.abs(rng.standard_normal(P)) * 1e-6
    full = opt.adam_step(p, m, v, g, 3, **HP)
    covered = np.zeros(P, int)
    length = -(-P // N)
    for r in range(N):
        off, ln, valid = opt.shard_range(P, N, r)
        assert ln == length and off == r * length and 0 <= valid <= ln
        covered[off:off + valid] += 1
        sh = opt.adam_shard(p, m, v, g, N, r, 3, **HP)
        for a, b in zip(sh, full):
            assert a.shape == (length,)
            np.testing.assert_array_equal(a[:valid], b[off:off + valid])  # bit-equal
            np.testing.assert_array_equal(a[valid:], 0.0)
    np.testing.assert_array_equal(covered, 1)


def test_shard_range_of_workload_shapes():
    assert opt.shard_range(124439808, 8, 0) == (0, 15554976, 15554976)
    assert opt.shard_range(124439808, 8, 7) == (108884832, 15554976, 15554976)
    assert opt.shard_range(789760, 4, 0) == (0, 197440, 197440)
    assert opt.shard_range(10, 4, 3) == (9, 3, 1)
    assert opt.shard_range(9, 4, 3) == (9, 3, 0)


def test_bf16_round_matches_torch():
    rng = np.random.default_rng(3)
    x = np.concatenate([rng.standard_normal(4096).astype(np.float32) * 10.0 ** rng.integers(-6, 6, 4096).astype(np.float32),
                        np.array([1.0, 1.00390625, 1.01171875, -1.00390625, 0.0, 3.0e38], np.float32)])
    ref = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    np.testing.assert_array_equal(opt.bf16_round(x), ref)
    # ties to even: 1 + 2^-8 is halfway between 1 and 1 + 2^-7
    assert opt.bf16_round(np.float32(1.00390625)) == np.float32(1.0)
    assert opt.bf16_round(np.float32(1.01171875)) == np.float32(1.015625)


def test_zero2_local_reduce_and_accumulation():
    rng = np.random.default_rng(4)
    P, N = 103, 4
    g1, g2 = rng.standard_normal(P), rng.standard_normal(P)
    for r in range(N):
        off, ln, valid = opt.shard_range(P, N, r)
        sh = opt.zero2_reduce_local(np.zeros(ln), g1, N, r)
        np.testing.assert_array_equal(sh[:valid], g1[off:off + valid])
        np.testing.assert_array_equal(sh[valid:], 0.0)
        sh2 = opt.zero2_reduce_local(sh, g2, N, r)
        np.testing.assert_array_equal(sh2[:valid], (g1 + g2)[off:off + valid])


def test_zero3_gather_reassembles_flat_vector():
    rng = np.random.default_rng(5)
    P, N = 103, 4
    flat = rng.standard_normal(P)
    ln = -(-P // N)
    padded = np.concatenate([flat, np.zeros(N * ln - P)])
    shards = [padded[r * ln:(r + 1) * ln] for r in range(N)]
    for lo, hi in [(0, P), (10, 60), (25, 27), (77, 103)]:
        np.testing.assert_array_equal(opt.zero3_gather(shards, P, lo, hi), flat[lo:hi])
