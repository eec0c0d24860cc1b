"""Benchmark: one rank's ZeRO-1 training step of the GPT-2-small-shaped workload
on one MI355X, through libpoplar's C ABI.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--batch B]
                    [--curve-report] [--layer-report] [--model-report] [--clock-report]

A step is poplar_profile_step(stage 1, B): embedding, 12 layers forward, head
and loss, backward, Adam on the rank's 1/8 shard, all on synthetic inputs that
already sit in HBM.  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

WORKLOAD = dict(arch="gpt", L=12, H=768, nh=12, F=3072, S=1024, V=50257)
WORLD, RANK, STAGE = 8, 0, 1
SWEEP = (1, 2, 4, 8, 16)
PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0
# Bytes that cross the L2 per GEMM launch at local batch 16, averaged over the 111 launches of a step: rocprofv3
# counters FETCH_SIZE x 2.0 (calibrated on kernels of known size) + WRITE_SIZE, summarised under profiles/.
# Valid for the GEMM kernel as profiled; set to None when that kernel changes until the counters are taken again.
GEMM_TRAFFIC_BYTES_PER_LAUNCH = 296.2e6
# Events ride on the GEMM launches of every GEMM_EVENTS_EVERY-th timed step (the first, the sixth, ...): an attached
# pair of events costs about 4.5 us per launch, 0.5 ms on a step's 111 launches, and the headline number should
# carry as little of the instrument as the measurement allows.
GEMM_EVENTS_EVERY = 5


def cpu_baseline(model, flat, tok, tgt):
    """The oracle as it stands, timed on this host: forward + backward of THREE samples
    through all layers and the head, then Adam on the 1/8 shard (10-20 s of CPU work)."""
    from oracle import optimizer as oopt
    from oracle import transformer as otr
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    f64 = flat.astype(np.float64)
    t0 = time.perf_counter()
    n = 3
    loss, grad, _ = otr.model_fwd_bwd(model, f64, tok[:n], tgt[:n], 1.0 / (n * model["S"]))
    off, ln, valid = oopt.shard_range(len(f64), WORLD, RANK)
    sl = slice(off, off + valid)
    z = np.zeros(valid)
    oopt.adam_step(f64[sl], z, z, grad[sl], 1, 1e-3, 0.9, 0.999, 1e-8)
    dt = time.perf_counter() - t0
    return {"value": n / dt, "unit": "samples/s", "cores": int(cores), "kind": "oracle",
            "sample": "3 samples (3072 tokens) through the full 12-layer model fwd+bwd + Adam on the 1/8 shard, fp64 NumPy",
            "seconds": dt, "loss": float(loss)}


def device_info(pb, torch):
    """What the device reports, and the bf16 matrix-core peak that follows from it (4096 flop per clock per CU)."""
    d = pb.device_info()
    ghz = d["clock_khz"] / 1e6
    return {"name": torch.cuda.get_device_properties(0).name, "compute_units": d["compute_units"], "clock_mhz": d["clock_khz"] / 1e3,
            "bf16_peak_tflops_from_device": d["compute_units"] * 4096 * ghz / 1e3,
            "bf16_peak_tflops_used": PEAK_BF16_TFLOPS, "hbm_gib": d["memory_bytes"] / 2**30}


def curve_report(pb, ctx, P, max_b, reps=5):
    """The paper's curve claim on this device (Appendix "Cubic Spline Interpolation": the curve through the
    profiled points is almost the measured one): a dense sweep of TimeConsumedDuringStep over every batch,
    the spline through the batches Algorithm 1 visits, its error at the batches it does not visit; then
    Algorithm 2 at stages 2 and 3 on a four-device mix built from the measured curve (times x 1, 1.5, 2, 3),
    with the communication time of the volume model over an xGMI mesh (7 links x 153 GB/s per device)."""
    dense = {}
    for b in range(1, max_b + 1):
        ctx.profile_step(STAGE, b)
        dense[b] = float(np.median([ctx.profile_step(STAGE, b)["t_consumed"] for _ in range(reps)]))
    visited = sorted({1 << k for k in range(max_b.bit_length()) if (1 << k) <= max_b} | {max_b})
    speed = pb.speed_curve(visited, [dense[b] for b in visited], max_b)
    rel = {b: speed[b] * dense[b] / b - 1.0 for b in dense if b not in visited}
    out = {"stage": STAGE, "batches": list(dense), "t_consumed_ms": [dense[b] * 1e3 for b in dense], "visited": visited,
           "spline_rel_err_at_unvisited": {str(b): e for b, e in rel.items()},
           "spline_max_abs_rel_err": max(abs(e) for e in rel.values()) if rel else 0.0,
           "spline_mean_abs_rel_err": float(np.mean([abs(e) for e in rel.values()])) if rel else 0.0}
    bs = list(dense)
    curves = [(bs, [dense[b] * k for b in bs], max_b) for k in (1.0, 1.5, 2.0, 3.0)]
    gbs, alloc = 256, {}
    for stage in (2, 3):
        cm = pb.comm_model(P, 4, stage, 2.0, 4.0, 7 * 153e9)
        with_comm = pb.allocate(stage, gbs, curves, cm["t_micro"])
        without = pb.allocate(stage, gbs, curves, 0.0)
        alloc[str(stage)] = {"t_comm_ms": cm["t_micro"] * 1e3, "micro_bytes": cm["micro_bytes"],
                             "b": with_comm["b"], "gas": with_comm["gas"], "T_ms": with_comm["T"] * 1e3,
                             "b_no_comm": without["b"], "gas_no_comm": without["gas"], "T_no_comm_ms": without["T"] * 1e3}
    out["allocate_gbs256_mix_1_1.5_2_3"] = alloc
    return out


def adam_large(pb, ctx, torch, elems=128 * 1024 * 1024, iters=5):
    """Adam on a shard far larger than the 256 MB Infinity Cache (30 bytes per element: 4 GB at the default size)."""
    dev = "cuda:0"
    p, m, v = (torch.zeros(elems, device=dev) for _ in range(3))
    g = torch.full((elems,), 1e-3, device=dev)
    low = torch.empty(elems, dtype=torch.bfloat16, device=dev)
    ctx.adam_shard(p, m, v, g, low, elems, 1, 1e-3, 0.9, 0.999, 1e-8)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for t in range(iters):
        ctx.adam_shard(p, m, v, g, low, elems, t + 2, 1e-3, 0.9, 0.999, 1e-8)
    e1.record()
    torch.cuda.synchronize()
    gbs = 30.0 * elems * iters / (e0.elapsed_time(e1) * 1e-3) / 1e9
    return {"achieved": gbs, "unit": "GB/s", "peak": PEAK_HBM_GBS, "frac": gbs / PEAK_HBM_GBS, "bytes_per_elem": 30, "elems": elems}


LAYER_SHAPES = {   # one decoder layer of the larger configurations, at the batches their parity tests use
    "gpt-1.3B (H 2048, 16 heads of 128, F 8192, S 2048)": (dict(arch="gpt", L=1, H=2048, nh=16, F=8192, S=2048, V=64), (1, 2, 4, 8)),
    "llama-7B (H 4096, 32 heads of 128, F 11008, S 2048)": (dict(arch="llama", L=1, H=4096, nh=32, F=11008, S=2048, V=64), (1, 2, 4)),
}


def layer_report(pb, torch, iters=5):
    """Forward and backward of ONE layer at the shapes of the larger configurations (their whole models need
    more than a bench run should take): milliseconds and algorithmic TFLOP/s, causal attention at half density."""
    dev, out = "cuda:0", {}
    for name, (case, batches) in LAYER_SHAPES.items():
        cfg = pb.make_cfg(**case, dtype="bf16")
        ctx = pb.Context(cfg, torch.cuda.current_stream().cuda_stream)
        n, H, S, F = pb.layer_param_count(cfg), case["H"], case["S"], case["F"]
        params = (torch.randn(n, device=dev) * 0.02).to(torch.bfloat16)
        grads = torch.zeros(n, device=dev)
        rows = []
        for B in batches:
            x = torch.randn(B * S, H, device=dev).to(torch.bfloat16)
            dy = torch.randn(B * S, H, device=dev).to(torch.bfloat16)
            y, dx = torch.empty_like(x), torch.empty_like(x)
            saved = torch.empty(pb.layer_saved_bytes(cfg, B) + 256, dtype=torch.uint8, device=dev)
            wsb = pb.layer_workspace_bytes(cfg, B)
            ws = torch.empty(wsb + 256, dtype=torch.uint8, device=dev)
            ctx.layer_fwd(B, x, params, y, saved)
            ctx.layer_bwd(B, x, dy, params, saved, dx, grads, 0, ws, wsb)
            torch.cuda.synchronize()
            e = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
            e[0].record()
            for _ in range(iters):
                ctx.layer_fwd(B, x, params, y, saved)
            e[1].record()
            for _ in range(iters):
                ctx.layer_bwd(B, x, dy, params, saved, dx, grads, 0, ws, wsb)
            e[2].record()
            torch.cuda.synchronize()
            tf, tb = e[0].elapsed_time(e[1]) / iters, e[1].elapsed_time(e[2]) / iters
            gemm = 2 * S * (4 * H * H + (3 if case["arch"] == "llama" else 2) * H * F)
            ff, fb = B * (gemm + 2 * S * S * H), B * (2 * gemm + 5 * S * S * H)
            rows.append({"batch": B, "fwd_ms": tf, "bwd_ms": tb, "fwd_tflops": ff / tf / 1e9, "bwd_tflops": fb / tb / 1e9,
                         "tflops": (ff + fb) / (tf + tb) / 1e9})
            del x, dy, y, dx, saved, ws
        out[name] = rows
    return out


def clock_report(pb, ctx, torch, shapes=((16384, 3072, 768), (8192, 2048, 8192)), iters=200):
    """The same GEMM launches on operands of zeros, ones and normal values: the matrix pipes draw power with the
    bits that toggle, the chip holds its power limit by lowering the shader clock, and so the rate a GEMM reaches
    depends on its data.  Reports the rate per kind of data and the shader clock rocm-smi shows during a long run."""
    import re
    import subprocess
    dev, rows = "cuda:0", []

    def operands(kind, M, N, K):
        if kind == "normal":
            return (torch.randn(M, K, device=dev) * 0.5).to(torch.bfloat16), (torch.randn(N, K, device=dev) * 0.5).to(torch.bfloat16)
        fill = torch.zeros if kind == "zeros" else torch.ones
        return fill(M, K, device=dev, dtype=torch.bfloat16), fill(N, K, device=dev, dtype=torch.bfloat16)

    def timed(A, B, C, M, N, K, n, sample):
        for _ in range(3):
            ctx.gemm(0, M, N, K, A, K, B, K, C, N, False, 0.0)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(n):
            ctx.gemm(0, M, N, K, A, K, B, K, C, N, False, 0.0)
        e1.record()
        mhz = None
        if sample:   # the launches are queued and still running: read the clock while they do
            time.sleep(0.05)
            try:
                txt = subprocess.run(["rocm-smi", "--showclocks"], capture_output=True, text=True, timeout=30).stdout
                m = re.search(r"sclk clock level.*?\((\d+)Mhz\)", txt)
                mhz = int(m.group(1)) if m else None
            except (OSError, subprocess.SubprocessError):
                mhz = None
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e-3 / n, mhz

    for (M, N, K) in shapes:
        C = torch.empty(M, N, device=dev, dtype=torch.bfloat16)
        for kind in ("zeros", "ones", "normal"):
            A, B = operands(kind, M, N, K)
            t, _ = timed(A, B, C, M, N, K, iters, False)
            seconds_each = max(t, 1e-6)
            _, mhz = timed(A, B, C, M, N, K, int(min(40000, max(iters, 2.0 / seconds_each))), True)
            rows.append({"M": M, "N": N, "K": K, "data": kind, "us": t * 1e6, "tflops": 2.0 * M * N * K / t / 1e12,
                         "frac_mfma_peak": 2.0 * M * N * K / t / 1e12 / PEAK_BF16_TFLOPS, "sclk_mhz_during_run": mhz})
            del A, B
    return rows


MODEL_CONFIGS = {   # the larger configurations: (model, world, ZeRO stage, local batches)
    # (after the sweep 1, 2, 4, 8: the odd batches of the allocation stress, whose token counts leave partial tiles)
    "gpt-1.3B, ZeRO-2 on a 1/4 shard": (dict(arch="gpt", L=24, H=2048, nh=16, F=8192, S=2048, V=50257), 4, 2, (1, 2, 4, 8, 3, 5, 7, 13)),
    "llama-7B, ZeRO-3 on a 1/16 shard": (dict(arch="llama", L=32, H=4096, nh=32, F=11008, S=2048, V=32000), 16, 3, (1, 2, 4)),
}


class DeviceRank:
    """One simulated rank whose state is drawn on the device (same recipe as synth.init_params: matrices N(0, 0.02),
    gains 1, biases 0; seed 0), for models too large to draw on the host in a bench run."""

    def __init__(self, pb, torch, model, world, stage, max_b, cap_bytes=0):
        dev = "cuda:0"
        self.cfg = pb.make_cfg(**model, dtype="bf16", world=world, rank=0, zero_stage=stage, cap_bytes=cap_bytes)
        self.P = pb.model_param_count(self.cfg)
        off, ln, valid = (0, self.P, self.P) if stage == 0 else pb.shard_range(self.P, world, 0)
        self.valid = valid
        g = torch.Generator(device=dev).manual_seed(0)
        flat = torch.zeros(max(self.P, off + ln), device=dev)
        for name, shape, o in pb.model_spec(self.cfg):
            n = int(np.prod(shape))
            if len(shape) == 2:
                flat[o:o + n].normal_(0.0, 0.02, generator=g)
            elif name.split(".")[-1] in ("g1", "g2", "gf"):
                flat[o:o + n] = 1.0
        params = flat[:self.P].to(torch.bfloat16)
        master = flat[off:off + ln].clone()
        own = master.to(torch.bfloat16) if stage == 3 else None
        del flat
        m, v = torch.zeros(ln, device=dev), torch.zeros(ln, device=dev)
        grads = torch.zeros(self.P if stage < 2 else ln, device=dev)
        tok = torch.randint(0, model["V"], (max_b, model["S"] + 1), generator=g, device=dev, dtype=torch.int32)
        self.wsb = pb.step_workspace_bytes(self.cfg, stage, max_b)
        ws = torch.empty(self.wsb + 256, dtype=torch.uint8, device=dev)
        loss = torch.zeros(1, device=dev)
        self.ctx = pb.Context(self.cfg, torch.cuda.current_stream().cuda_stream)
        self.ctx.bind_state(params, master, m, v, grads, tok, max_b, ws, self.wsb, loss, own_shard=own, adam_t=1, lr=1e-4)


def model_report(pb, torch):
    """Whole steps of the larger configurations (1.3 B parameters at ZeRO-2, the Llama-7B shape at ZeRO-3) over their
    local-batch sweeps, then the allocation stress on the 1.3 B model: odd local batches, Algorithm 1 under an
    emulated cap of 40 GiB at stages 1-3, and Algorithm 2 over four devices whose step times are the measured curve
    times 1, 1.5, 2 and 3, to a global batch of 64."""
    out = {}
    for name, (model, world, stage, batches) in MODEL_CONFIGS.items():
        r = DeviceRank(pb, torch, model, world, stage, max(batches))
        rows = []
        for B in batches:
            r.ctx.profile_step(stage, B)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            profs = [r.ctx.profile_step(stage, B) for _ in range(2)]
            torch.cuda.synchronize()
            dt = (time.perf_counter() - t0) / 2
            p = profs[-1]
            rows.append({"local_batch": B, "ms_per_step": dt * 1e3, "samples_per_s": B / dt, "tflops": p["flops"] / dt / 1e12,
                         "frac_mfma_peak": p["flops"] / dt / 1e12 / PEAK_BF16_TFLOPS, "t_consumed_ms": p["t_consumed"] * 1e3,
                         "t_adam_ms": p["t_adam"] * 1e3, "adam_gbs": 30.0 * r.valid / p["t_adam"] / 1e9,
                         "t_reduce_ms": p["t_reduce_bwd"] * 1e3, "t_gather_ms": (p["t_gather_fwd"] + p["t_gather_bwd"]) * 1e3,
                         "accounted_gib": p["accounted_bytes"] / 2**30, "loss": p["loss"]})
        out[name] = {"params": r.P, "shard_elems": r.valid, "sweep": rows}
        del r
        torch.cuda.empty_cache()
    model, world = MODEL_CONFIGS["gpt-1.3B, ZeRO-2 on a 1/4 shard"][0], 4
    cap = 40 * 2**30
    stress = {"cap_bytes": cap, "stages": {}}
    for stage in (1, 2, 3):
        r = DeviceRank(pb, torch, model, world, stage, 16, cap_bytes=cap)
        mbs, samples = r.ctx.search_mbs(stage)
        pts = {p["batch"]: p["t_consumed"] for p in samples}
        entry = {"mbs": mbs, "visited": sorted(pts), "t_consumed_ms": [pts[b] * 1e3 for b in sorted(pts)]}
        bs = sorted(pts)
        curves = [(bs, [pts[b] * k for b in bs], mbs) for k in (1.0, 1.5, 2.0, 3.0)]
        cm = pb.comm_model(r.P, 4, stage, 2.0, 4.0, 7 * 153e9) if stage >= 2 else {"t_micro": 0.0}
        al = pb.allocate(stage, 64, curves, cm["t_micro"])
        entry["allocate_gbs64"] = {"t_comm_ms": cm["t_micro"] * 1e3, "gmbs": al["gmbs"], "b": al["b"], "gas": al["gas"], "lbs": al["lbs"],
                                   "T_ms": al["T"] * 1e3}
        stress["stages"][str(stage)] = entry
        del r
        torch.cuda.empty_cache()
    out["allocation stress, gpt-1.3B, cap 40 GiB, devices 1 : 1.5 : 2 : 3, gbs 64"] = stress
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--batch", type=int, default=16, help="local batch of the headline number")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-sweep", action="store_true")
    ap.add_argument("--curve-report", action="store_true", help="add the dense-sweep / spline / Algorithm 2 report to the line")
    ap.add_argument("--layer-report", action="store_true", help="add one-layer timings at the larger configurations' shapes")
    ap.add_argument("--clock-report", action="store_true", help="add GEMM rates on zero, one and normal operands with the shader "
                    "clock during each run")
    ap.add_argument("--model-report", action="store_true", help="add whole-model steps of the 1.3B and Llama-7B-shaped configurations "
                    "and the allocation stress under an emulated 40 GiB cap (a few minutes, about 120 GB of HBM)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one rank on ONE GPU (the ZeRO world is simulated by shard offsets); --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2408_12596_amd import binding as pb
    from paper_2408_12596_amd import synth

    pb.lib()   # fails loudly if the HIP library has not been built
    dev = "cuda:0"
    model = WORKLOAD
    cfg = pb.make_cfg(**model, dtype="bf16", world=WORLD, rank=RANK, zero_stage=STAGE)
    P = pb.model_param_count(cfg)
    off, ln, valid = pb.shard_range(P, WORLD, RANK)
    spec = [(name, shape) for name, shape, _ in pb.model_spec(cfg)]   # the library's own flat layout
    assert sum(int(np.prod(s)) for _, s in spec) == P
    flat = synth.init_params(spec, seed=0)
    max_b = max(max(SWEEP), args.batch)
    tok, tgt = synth.tokens(max_b, model["S"], model["V"], seed=0)
    both = np.concatenate([tok, tgt[:, -1:]], axis=1).astype(np.int32)

    params = torch.from_numpy(flat).to(dev).to(torch.bfloat16)
    master = torch.from_numpy(flat[off:off + ln].copy()).to(dev)
    m = torch.zeros(ln, device=dev)
    v = torch.zeros(ln, device=dev)
    grads = torch.zeros(P, device=dev)
    tokens = torch.from_numpy(both).to(dev)
    wsb = pb.step_workspace_bytes(cfg, STAGE, max_b)
    ws = torch.empty(wsb + 256, dtype=torch.uint8, device=dev)
    loss = torch.zeros(1, device=dev)
    stream = torch.cuda.current_stream().cuda_stream
    ctx = pb.Context(cfg, stream)
    ctx.bind_state(params, master, m, v, grads, tokens, max_b, ws, wsb, loss, adam_t=1, lr=1e-4)

    def run(B, steps, warmup, timing, every=1):
        """`steps` timed steps after `warmup` untimed ones; the launches selected by `timing` carry events in every
        `every`-th timed step (the first, the (every+1)-th, ...)."""
        ctx.set_kernel_timing(0)
        for _ in range(warmup):
            ctx.profile_step(STAGE, B)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        profs = []
        for i in range(steps):
            ctx.set_kernel_timing(timing if i % every == 0 else 0)
            profs.append(ctx.profile_step(STAGE, B))
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / steps
        ctx.set_kernel_timing(0)
        return dt, profs

    B = args.batch
    # the timed steps carry events on the GEMM launches only (the roofline kernel); the attention kernels are timed in
    # three more steps afterwards, outside the headline number
    dt, profs = run(B, args.steps, args.warmup, 1, every=GEMM_EVENTS_EVERY)
    mean = lambda k: float(np.mean([p[k] for p in profs]))
    flops = profs[0]["flops"]
    evp = profs[::GEMM_EVENTS_EVERY]   # the timed steps whose GEMM launches carried events
    t_gemm, f_gemm, n_gemm = float(np.mean([p["t_gemm"] for p in evp])), evp[0]["gemm_flops"], evp[0]["n_gemm"]
    _, aprofs = run(B, 3, 0, 2)
    t_attn, f_attn = float(np.mean([p["t_attn"] for p in aprofs])), aprofs[0]["attn_flops"]
    gemm_tflops = f_gemm / t_gemm / 1e12 if t_gemm > 0 else 0.0
    adam_gbs = 30.0 * valid / mean("t_adam") / 1e9
    out = {
        "metric": "samples/sec", "value": B / dt, "unit": "samples/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": dt * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": "GPT-2-small-shaped decoder (12 layers, hidden 768, 12 heads, MLP 3072 GeLU, seq 1024, vocab 50257), "
                               "bf16 compute, fp32 master; ZeRO-1 step of rank 0 of a simulated world of 8: fwd + bwd + Adam on the 1/8 shard",
                   "local_batch": B, "zero_stage": STAGE, "world": WORLD, "params": P, "shard_elems": valid},
        "tflops": flops / dt / 1e12,
        "frac_mfma_peak_step": flops / dt / 1e12 / PEAK_BF16_TFLOPS,
        "samples_per_s_time_consumed": B / mean("t_consumed"),
        "step_breakdown_ms": dict({k: mean(k) * 1e3 for k in ("t_fwd", "t_bwd", "t_adam")}, t_gemm=t_gemm * 1e3, t_attn=t_attn * 1e3),
        "roofline": {"bound": "mfma", "kernel": "gemm_dtl_kernel (all GEMM launches of the step)", "achieved": gemm_tflops,
                     "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": gemm_tflops / PEAK_BF16_TFLOPS,
                     "traffic": GEMM_TRAFFIC_BYTES_PER_LAUNCH if B == 16 else None, "traffic_unit": "bytes per launch",
                     "launches_per_step": n_gemm, "avg_launch_ms": t_gemm / max(n_gemm, 1) * 1e3,
                     "timed_steps_with_events": len(evp),
                     "flop_per_launch": f_gemm / max(n_gemm, 1)},
        "attention": {"achieved": f_attn / t_attn / 1e12 if t_attn > 0 else 0.0, "unit": "TFLOP/s", "peak": PEAK_BF16_TFLOPS,
                      "frac": (f_attn / t_attn / 1e12 / PEAK_BF16_TFLOPS) if t_attn > 0 else 0.0},
        "adam": {"achieved": adam_gbs, "unit": "GB/s", "peak": PEAK_HBM_GBS, "frac": adam_gbs / PEAK_HBM_GBS,
                 "bytes_per_elem": 30, "elems": valid},
        "adam_4GB": adam_large(pb, ctx, torch),
        "loss": profs[-1]["loss"],
        "device": device_info(pb, torch),
    }
    if not args.no_sweep:
        sweep = []
        for b in SWEEP:
            d, pr = run(b, 3, 1, False)
            sweep.append({"local_batch": b, "samples_per_s": b / d, "ms_per_step": d * 1e3, "tflops": pr[0]["flops"] / d / 1e12,
                          "frac_mfma_peak": pr[0]["flops"] / d / 1e12 / PEAK_BF16_TFLOPS,
                          "t_consumed_ms": float(np.mean([p["t_consumed"] for p in pr])) * 1e3})
        out["sweep"] = sweep
    if args.curve_report:
        out["curve_report"] = curve_report(pb, ctx, P, max_b)
    if args.layer_report:
        out["layer_report"] = layer_report(pb, torch)
    if args.clock_report:
        out["clock_report"] = clock_report(pb, ctx, torch)
    if args.model_report:
        out["model_report"] = model_report(pb, torch)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(model, flat, tok, tgt)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
