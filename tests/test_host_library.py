"""Host-side logic of libpoplar against the oracle; no GPU needed.
Covers: exported symbols, flat layout, shard arithmetic, speed curves,
Algorithm 2 (bit-exact integers) and error reporting."""
import ctypes
import re
import os

import numpy as np
import pytest

from oracle import allocate as oal
from oracle import optimizer as oopt
from oracle import transformer as otr
from paper_2408_12596_amd import binding as pb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

CFGS = [
    dict(arch="gpt", L=1, H=256, nh=4, F=1024, S=128, V=1),
    dict(arch="gpt", L=12, H=768, nh=12, F=3072, S=1024, V=50257),
    dict(arch="gpt", L=24, H=2048, nh=16, F=8192, S=2048, V=50257),
    dict(arch="llama", L=32, H=4096, nh=32, F=11008, S=2048, V=32000),
    dict(arch="llama", L=2, H=64, nh=1, F=24, S=8, V=11),
]


def test_every_declared_symbol_is_exported():
    header = open(os.path.join(ROOT, "include", "poplar.h")).read()
    declared = set(re.findall(r"^(?:int|const char\*) (poplar_[a-z0-9_]+)\(", header, re.M))
    assert declared == set(pb.EXPORTS)
    lib = pb.lib()
    for name in declared:
        assert getattr(lib, name) is not None


@pytest.mark.parametrize("cfg", CFGS)
def test_layout_matches_oracle(cfg):
    c = pb.make_cfg(**cfg)
    table, P = otr.offsets(otr.model_spec(cfg))
    assert pb.model_param_count(c) == P
    assert pb.layer_param_count(c) == otr.offsets(otr.layer_spec(cfg["arch"], cfg["H"], cfg["F"]))[1]
    for name, shape, off in pb.model_spec(c):
        if name.endswith("Wgu"):   # the library treats gate|up as one [2F, H] matrix
            o_off, o_shape = table[name.replace("Wgu", "Wg")]
            assert off == o_off and shape == (2 * o_shape[0], o_shape[1])
            assert table[name.replace("Wgu", "Wu")][0] == off + o_shape[0] * o_shape[1]
        else:
            assert (off, tuple(shape)) == (table[name][0], tuple(table[name][1])), name


def test_shard_range_bit_exact():
    rng = np.random.default_rng(0)
    cases = [(124439808, 8), (1315723264, 4), (6738415616, 16), (789760, 4), (10, 4), (9, 4), (5, 8), (0, 3)]
    cases += [(int(rng.integers(0, 10**10)), int(rng.integers(1, 65))) for _ in range(200)]
    for P, N in cases:
        for r in {0, N - 1, N // 2}:
            assert pb.shard_range(P, N, r) == oopt.shard_range(P, N, r)
    with pytest.raises(pb.PoplarError):
        pb.shard_range(10, 4, 4)
    with pytest.raises(pb.PoplarError):
        pb.shard_range(10, 0, 0)


def random_curve(rng):
    mbs = int(rng.integers(1, 40))
    pts = sorted(set([1, mbs] + [int(b) for b in rng.integers(1, mbs + 1, int(rng.integers(0, 6)))]))
    if rng.random() < 0.3:
        pts = pts + [pts[-1]]          # a repeated sample
    sat, half = float(rng.uniform(1, 50)), float(rng.uniform(0.3, 8))
    times = [b / (sat * b / (b + half)) * float(rng.uniform(0.97, 1.03)) for b in pts]
    return (pts, times, mbs)


def test_speed_curve_matches_oracle():
    rng = np.random.default_rng(1)
    for _ in range(200):
        c = random_curve(rng)
        np.testing.assert_allclose(pb.speed_curve(*c), oal.speed_curve(*c), rtol=1e-11, atol=0)
    # a single sample is a constant curve; mbs above the sampled range clamps
    assert pb.speed_curve([4], [2.0], 6) == [0.0] + [2.0] * 6
    s = pb.speed_curve([1, 2, 4], [1.0, 1.5, 2.5], 8)
    assert s[5] == s[4] == s[8]


@pytest.mark.parametrize("stage", [0, 1, 2, 3])
def test_allocate_bit_exact_on_random_curves(stage):
    rng = np.random.default_rng(10 + stage)
    for _ in range(150):
        n = int(rng.integers(1, 7))
        curves = [random_curve(rng) for _ in range(n)]
        gbs = int(rng.integers(1, 400))
        tc = float(rng.choice([0.0, 0.01, 0.5, 20.0]))
        got = pb.allocate(stage, gbs, curves, tc)
        ref = oal.allocate(stage, gbs, curves, tc)
        for k in ("gmbs", "b", "gas", "lbs"):
            assert got[k] == (ref[k] if isinstance(ref[k], list) else [ref[k]] * n), (k, got, ref)
        assert sum(got["gmbs"]) == gbs
        T_ref = ref["T"] if stage < 2 else ref["wall"]
        assert abs(got["T"] - T_ref) <= 1e-10 * abs(T_ref)


def test_allocate_hand_case_and_ties():
    # speeds 1 : 1.5 : 2 : 3, gbs 64 -> 8, 13, 17, 26 (worked in tests/golden/alloc_hand_cases.json)
    pts = [1, 2, 4, 8, 16, 32, 64]
    curves = [(pts, [b / s for b in pts], 64) for s in (1.0, 1.5, 2.0, 3.0)]
    got = pb.allocate(1, 64, curves)
    assert got["gmbs"] == [8, 13, 17, 26]
    assert abs(got["T"] - 26 / 3) < 1e-12
    # equal devices: ties go to the lowest index, sum is exact
    got = pb.allocate(0, 10, [curves[0]] * 4)
    assert got["gmbs"] == [3, 3, 2, 2]
    # a device with mbs = 0 gets nothing
    got = pb.allocate(1, 9, [curves[0], ([], [], 0)])
    assert got["gmbs"] == [9, 0] and got["b"][1] == 0 and got["gas"][1] == 0


def test_allocate_rejects_bad_input():
    ok = ([1, 2], [1.0, 1.5], 2)
    for args in [(4, 8, [ok]), (1, 0, [ok]), (1, 8, [([1], [0.0], 1)]), (1, 8, [([0], [1.0], 1)]), (1, 8, [([], [], 0)])]:
        with pytest.raises(pb.PoplarError) as e:
            pb.allocate(*args)
        assert e.value.status == pb.ERR_INVALID and str(e.value)
    with pytest.raises(pb.PoplarError):
        pb.allocate(1, 8, [ok], peak_frac=0.0)


def test_config_validation_and_byte_queries():
    with pytest.raises(pb.PoplarError):
        pb.model_param_count(pb.make_cfg(H=100))              # not a multiple of 8
    with pytest.raises(pb.PoplarError):
        pb.model_param_count(pb.make_cfg(H=256, nh=3))
    with pytest.raises(pb.PoplarError):
        pb.model_param_count(pb.make_cfg(H=256, nh=2, dtype="bf16"))   # head_dim 128 ok
        pb.model_param_count(pb.make_cfg(H=256, nh=8, dtype="bf16"))   # head_dim 32 is not
    with pytest.raises(pb.PoplarError):
        pb.model_param_count(pb.make_cfg(world=4, rank=4))
    # accounted memory is affine in the batch at the workload shapes (memory linear in batch size)
    for cfg in CFGS[1:3]:
        for stage in range(4):
            c = pb.make_cfg(**cfg, world=4)
            a = [pb.step_accounted_bytes(c, stage, b) for b in (1, 2, 3, 7)]
            assert a[1] - a[0] == a[2] - a[1] == (a[3] - a[2]) // 4
            assert pb.step_accounted_bytes(c, stage, 1, forward_only=True) < a[0]
    # more sharding, less state
    c = pb.make_cfg(**CFGS[2], world=4)
    st = [pb.step_accounted_bytes(c, s, 0) for s in range(4)]
    assert st[0] > st[1] > st[2] > st[3]


def test_checkpointing_keeps_one_stash_instead_of_one_per_layer():
    base = dict(arch="gpt", L=6, H=128, nh=2, F=256, S=64, V=211, dtype="bf16", world=4, zero_stage=1)
    plain, ckpt = pb.make_cfg(**base), pb.make_cfg(**base, checkpoint=True)
    for stage in range(4):
        for B in (1, 3, 8):
            saved = pb.layer_saved_bytes(plain, B)
            assert pb.step_accounted_bytes(plain, stage, B) - pb.step_accounted_bytes(ckpt, stage, B) == 5 * saved
            assert pb.step_workspace_bytes(plain, stage, B) - pb.step_workspace_bytes(ckpt, stage, B) == 5 * saved
        assert pb.step_accounted_bytes(plain, stage, 0) == pb.step_accounted_bytes(ckpt, stage, 0)
    with pytest.raises(pb.PoplarError):
        bad = pb.make_cfg(**base)
        bad.checkpoint = 2
        pb.model_param_count(bad)
