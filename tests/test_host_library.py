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


# ---- the allocator against things the oracle does not supply ------------------------------------------------------
def test_dipping_and_negative_splines_from_fixture():
    """tests/golden/alloc_dip_cases.json: hand-worked curves whose spline dips in time or falls below zero in speed."""
    import json
    with open(os.path.join(ROOT, "tests", "golden", "alloc_dip_cases.json")) as f:
        gold = json.load(f)
    for case in gold["cases"]:
        curve = (case["batches"], case["times"], case["mbs"])
        sp = pb.speed_curve(*curve)
        assert sp[0] == 0.0
        np.testing.assert_allclose(sp[1:], case["speed"], rtol=1e-12)
        a = case["alloc"]
        got = pb.allocate(a["stage"], a["gbs"], [curve], a["time_communication"])
        assert got["b"] == a["b"] and got["gas"] == [a["gas"]] and got["lbs"] == a["lbs"] and got["gmbs"] == a["gmbs"]
        assert abs(got["t"] - a["t"]) < 1e-12 and abs(got["T"] - a["wall"]) < 1e-12 and got["T_steps"] == got["T"]
        # `find` through the library: with communication so costly that only the step count matters, a lone device
        # whose gbs equals its batch at time t runs that batch in one step
        for t, b in case["find"]:
            if b == 0:
                continue
            one = pb.allocate(2, b, [curve], 1e12)
            assert one["gas"] == [1] and one["b"][0] >= b


def _compositions(total, n):
    import itertools
    for c in itertools.combinations(range(total + n - 1), n - 1):
        yield [b - a - 1 for a, b in zip((-1,) + c, c + (total + n - 1,))]


def test_stage01_split_minimises_eq1_and_eq4_by_brute_force_on_the_library():
    """Every split of gbs over the devices, Eq. (1) and Eq. (4) evaluated here from the devices' peak speeds: the
    library's split attains both minima, and its remainder hand-out never leaves a device that could take a sample
    and still finish before the slowest one (the equal-step-time property, as far as integers allow)."""
    rng = np.random.default_rng(7)
    for _ in range(60):
        n = int(rng.integers(2, 5))
        gbs = int(rng.integers(1, 19))
        speeds = [float(rng.integers(1, 9)) / 2 for _ in range(n)]
        pts = [1, 2, 4, 8, 16, 32]
        got = pb.allocate(0, gbs, [(pts, [b / s for b in pts], 32) for s in speeds])
        g = got["gmbs"]
        assert sum(g) == gbs and min(g) >= 0
        best_T = best_U = np.inf
        for B in _compositions(gbs, n):
            t = [b / s for b, s in zip(B, speeds)]
            T = max(t)
            best_T = min(best_T, T)
            best_U = min(best_U, sum((T - ti) * pi for ti, pi in zip(t, speeds)))
        t = [gi / s for gi, s in zip(g, speeds)]
        T = max(t)
        assert abs(T - best_T) < 1e-12 and abs(got["T"] - best_T) < 1e-12
        assert abs(sum((T - ti) * pi for ti, pi in zip(t, speeds)) - best_U) < 1e-9
        last = int(np.argmax(t))          # no other device could take one more sample and finish before the slowest one
        assert all((g[j] + 1) / speeds[j] >= T - 1e-12 for j in range(n) if j != last)


def test_stage23_wall_time_is_the_brute_force_minimum_on_the_library():
    """All micro-batch vectors (b_1..b_n): wall = (max_i time_i(b_i) + t_comm) ceil(gbs / sum b), with time_i read
    from the library's own speed curve; the sweep over t with `find` must reach the exhaustive minimum."""
    import itertools
    rng = np.random.default_rng(8)
    for _ in range(40):
        n = int(rng.integers(2, 4))
        curves = []
        for _i in range(n):
            mbs = int(rng.integers(1, 7))
            bs = sorted(set([1, mbs] + [int(b) for b in rng.integers(1, mbs + 1, 2)]))
            sat, half = float(rng.uniform(1, 6)), float(rng.uniform(0.5, 4))
            noise = rng.uniform(0.8, 1.25, len(bs))                       # noisy enough for dips
            curves.append((bs, [b / (sat * b / (b + half)) * float(k) for b, k in zip(bs, noise)], mbs))
        gbs = int(rng.integers(1, 40))
        tc = float(rng.choice([0.0, 0.3, 5.0]))
        got = pb.allocate(3, gbs, curves, tc)
        tms = []
        for c in curves:
            sp = pb.speed_curve(*c)
            tms.append(np.concatenate([[0.0], np.maximum.accumulate([b / sp[b] for b in range(1, c[2] + 1)])]))
        best = np.inf
        for B in itertools.product(*[range(0, c[2] + 1) for c in curves]):
            if sum(B):
                best = min(best, (max(tms[i][b] for i, b in enumerate(B)) + tc) * -(-gbs // sum(B)))
        assert abs(got["T"] - best) <= 1e-12 * max(1.0, best)
        assert sum(got["gmbs"]) == gbs
        assert all(0 <= l <= b <= c[2] for l, b, c in zip(got["lbs"], got["b"], curves))
        assert all(tms[i][b] <= got["t"] * (1 + 1e-15) for i, b in enumerate(got["b"]))


def test_stage01_predicted_time_on_the_curve_itself():
    bs = list(range(1, 9))
    sp = [1.0, 2.0, 3.0, 3.9, 4.0, 4.0, 4.0, 4.0]
    fast = (bs, [b / s for b, s in zip(bs, sp)], 8)
    slow = (bs, [b / (s / 2) for b, s in zip(bs, sp)], 6)
    got = pb.allocate(1, 30, [fast, slow])
    ref = oal.allocate(1, 30, [fast, slow])
    assert got["gmbs"] == [20, 10] and got["b"] == [8, 6] and got["gas"] == [3, 2] and got["lbs"] == [4, 4]
    assert abs(got["T"] - 5.0) < 1e-12
    assert abs(got["T_steps"] - max(2 * 8 / 4.0 + 4 / 3.9, 6 / 2.0 + 4 / 1.95)) < 1e-12
    assert abs(got["T_steps"] - ref["T_steps"]) < 1e-12 and got["T_steps"] >= got["T"]


def test_state_sized_for_a_shard_cannot_run_stage_0():
    """Host-side check only (nothing is launched, so no GPU is needed): stage 0 runs the optimizer over all P
    elements; a state whose master / m / v hold one shard is refused."""
    cfg = pb.make_cfg(arch="gpt", L=2, H=128, nh=2, F=256, S=64, V=211, dtype="bf16", world=4, rank=0)
    P = pb.model_param_count(cfg)
    off, ln, valid = pb.shard_range(P, 4, 0)
    ctx = pb.Context(cfg)
    fake = 0x1000   # never dereferenced: every call below fails its argument checks first
    ctx.bind_state(fake, fake, fake, fake, fake, fake, 4, fake, 1 << 40, fake, master_len=ln, grads_len=P, own_len=0)
    for stage, word in ((0, "optimizer elements"), (3, "own_shard")):
        with pytest.raises(pb.PoplarError) as e:
            ctx.profile_step(stage, 1)
        assert e.value.status == pb.ERR_INVALID and word in str(e.value)
    ctx.bind_state(fake, fake, fake, fake, fake, fake, 4, fake, 1 << 40, fake, master_len=ln, grads_len=ln, own_len=0)
    with pytest.raises(pb.PoplarError) as e:
        ctx.profile_step(1, 1)                      # stage 1 keeps the whole gradient
    assert "gradient buffer" in str(e.value)
    with pytest.raises(pb.PoplarError):
        ctx.bind_state(fake, fake, fake, fake, fake, fake, 4, fake, 0, fake, master_len=0, grads_len=P, own_len=0)
    with pytest.raises(pb.PoplarError):
        ctx.bind_state(fake, fake, fake, fake, fake, fake, 4, fake, 0, fake, own_shard=fake, master_len=ln, grads_len=P, own_len=0)
    with pytest.raises(pb.PoplarError):
        ctx.set_sampling(0, 0)


def test_host_code_under_address_and_undefined_behaviour_sanitizers():
    """layout.cpp and analysis.cpp rebuilt for the host with ASan + UBSan (any finding aborts the driver) and fed the
    kinds of input the library gets, valid and invalid: the sanitized build must agree with the library to the last bit."""
    import subprocess
    from paper_2408_12596_amd import build as pbuild
    exe = pbuild.build_host_sanitized()
    rng = np.random.default_rng(99)
    lines, expect = [], []

    def curve_text(c):
        return f"{c[2]} {len(c[0])} " + " ".join(f"{b} {t!r}" for b, t in zip(c[0], c[1]))
    for P, N, r in [(10, 4, 3), (0, 3, 0), (124439808, 8, 7), (10, 4, 4)] + [(int(rng.integers(0, 10**12)), int(rng.integers(1, 65)), 0) for _ in range(30)]:
        lines.append(f"shard {P} {N} {r}")
        try:
            expect.append("0 " + " ".join(str(v) for v in pb.shard_range(P, N, r)))
        except pb.PoplarError as e:
            expect.append(f"{e.status} 0 0 0")
    for cfg in CFGS:
        c = pb.make_cfg(**cfg)
        lines.append(f"count {c.arch} {c.n_layer} {c.hidden} {c.n_head} {c.ffn} {c.seq} {c.vocab} {c.dtype}")
        expect.append(f"0 {pb.model_param_count(c)} {pb.layer_param_count(c)}")
        for layer, tid in ((0, pb.T_WQKV), (cfg["L"] - 1, pb.T_W2), (0, pb.T_GF), (cfg["L"], pb.T_G1), (0, pb.T_BQKV)):
            lines.append(f"offset {c.arch} {c.n_layer} {c.hidden} {c.n_head} {c.ffn} {c.seq} {c.vocab} {c.dtype} {layer} {tid}")
            try:
                expect.append("0 " + " ".join(str(v) for v in pb.param_offset(c, layer, tid)))
            except pb.PoplarError as e:
                expect.append(f"{e.status} 0 0 0")
    for _ in range(40):
        P, world, stage = int(rng.integers(0, 10**10)), int(rng.integers(1, 65)), int(rng.integers(0, 4))
        bw = float(rng.uniform(1e9, 2e12))
        lines.append(f"comm {P} {world} {stage} 2.0 4.0 {bw!r}")
        m = pb.comm_model(P, world, stage, 2.0, 4.0, bw)
        expect.append("0 " + " ".join(repr(float(m[k])) for k in ("micro_bytes", "step_bytes", "total_micro_elements", "t_micro", "t_step")))
    import json
    with open(os.path.join(ROOT, "tests", "golden", "alloc_dip_cases.json")) as f:
        dips = [(c["batches"], c["times"], c["mbs"]) for c in json.load(f)["cases"]]
    for c in dips + [random_curve(rng) for _ in range(60)] + [([4], [2.0], 6)]:
        lines.append("curve " + curve_text(c))
        expect.append("0 " + " ".join(repr(float(v)) for v in pb.speed_curve(*c)))
    for stage in range(4):
        for _ in range(40):
            n = int(rng.integers(1, 7))
            curves = [random_curve(rng) for _ in range(n)] if rng.random() < 0.9 else [dips[0], dips[1]]
            n = len(curves)
            gbs, tc = int(rng.integers(1, 400)), float(rng.choice([0.0, 0.01, 0.5, 20.0]))
            lines.append(f"alloc {stage} {gbs} {tc!r} 0.95 {n} " + " ".join(curve_text(c) for c in curves))
            a = pb.allocate(stage, gbs, curves, tc)
            expect.append("0 " + " ".join(f"{a['gmbs'][i]} {a['b'][i]} {a['gas'][i]} {a['lbs'][i]}" for i in range(n))
                          + f" {a['T']!r} {a['t']!r} {a['T_steps']!r}")
    lines.append("alloc 1 8 0.0 0.95 1 0 0")                 # no device can run a sample
    lines.append("alloc 7 8 0.0 0.95 1 2 2 1 1.0 2 1.5")     # no such stage
    lines.append("curve 3 2 1 0.0 2 1.0")                    # a zero time
    expect += [None, None, None]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=1", UBSAN_OPTIONS="halt_on_error=1")
    env.pop("LD_PRELOAD", None)   # the sanitizer runtime must come first in the process
    r = subprocess.run([exe], input="\n".join(lines) + "\n", capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0, r.stderr[-2000:]
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr
    got = r.stdout.strip().split("\n")
    assert len(got) == len(lines)
    for line, g, e in zip(lines, got, expect):
        if e is None:
            assert g.split()[0] == str(pb.ERR_INVALID), (line, g)
        else:
            gt, et = g.split(), e.split()
            assert gt[0] == et[0], (line, g, e)
            if et[0] == "0":
                assert [float(x) for x in gt] == [float(x) for x in et], (line, g, e)
