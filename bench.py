"""Benchmark: one rank's ZeRO training step on one MI355X, through libpoplar's C ABI.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--batch B] [--headline-only]
                    [--workload llama7b|gpt1p3b|gpt2small] [--curve-report] [--layer-report] [--clock-report]

Headline: the Llama-7B-shaped configuration (32 layers, hidden 4096, SwiGLU 11008, seq 2048, vocab 32000) at
ZeRO-3 on a 1/16 shard, the largest configuration that fits one GPU.  A step is poplar_profile_step(3, B):
per-layer parameter gather, embedding, 32 layers forward, head and loss, backward with the local gradient reduce,
Adam on the shard, all on synthetic inputs that already sit in HBM.  The ~1.3B configuration (ZeRO-2, 1/4 shard,
with the odd batches and the 40 GiB allocation stress) and the GPT-2-small one (ZeRO-1, 1/8 shard) follow as
sub-records with their own sweeps and rooflines.  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

WORKLOAD = dict(arch="gpt", L=12, H=768, nh=12, F=3072, S=1024, V=50257)   # the GPT-2-small sub-record (and the curve report)
WORLD, RANK, STAGE = 8, 0, 1
SWEEP = (1, 2, 4, 8, 16)
HEADLINE = dict(arch="llama", L=32, H=4096, nh=32, F=11008, S=2048, V=32000)
HEADLINE_WORLD, HEADLINE_STAGE, HEADLINE_SWEEP = 16, 3, (1, 2, 4)
MID = dict(arch="gpt", L=24, H=2048, nh=16, F=8192, S=2048, V=50257)
MID_WORLD, MID_STAGE, MID_SWEEP, MID_ODD = 4, 2, (1, 2, 4, 8), (3, 5, 7, 13)
WORKLOADS = {   # name -> (model, simulated world, ZeRO stage, local-batch sweep, description)
    "llama7b": (HEADLINE, HEADLINE_WORLD, HEADLINE_STAGE, HEADLINE_SWEEP,
                "Llama-7B-shaped decoder (32 layers, hidden 4096, 32 heads of 128, SwiGLU MLP 11008, RMSNorm, RoPE, seq 2048, vocab 32000), "
                "bf16 compute, fp32 master; ZeRO-3 step of rank 0 of a simulated world of 16: per-layer parameter gather, fwd + bwd with the "
                "local gradient reduce, Adam on the 1/16 shard"),
    "gpt1p3b": (MID, MID_WORLD, MID_STAGE, MID_SWEEP,
                "~1.3B GPT decoder (24 layers, hidden 2048, 16 heads of 128, MLP 8192 GeLU, seq 2048, vocab 50257), bf16 compute, fp32 master; "
                "ZeRO-2 step of rank 0 of a simulated world of 4: fwd + bwd with the local gradient reduce, Adam on the 1/4 shard"),
    "gpt2small": (WORKLOAD, WORLD, STAGE, SWEEP,
                  "GPT-2-small-shaped decoder (12 layers, hidden 768, 12 heads of 64, MLP 3072 GeLU, seq 1024, vocab 50257), bf16 compute, "
                  "fp32 master; ZeRO-1 step of rank 0 of a simulated world of 8: fwd + bwd, Adam on the 1/8 shard"),
}
PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0
# Bytes that cross the L2 per GEMM launch of the headline step, averaged over its launches: rocprofv3 counters
# FETCH_SIZE and WRITE_SIZE, scaled by the factors a copy of known size gives, summarised under profiles/.
# Per kernel launch (355 per step: a weight-gradient group or a product whose partial last round is cut off is two).
# Valid for the GEMM kernel as profiled; set to None when that kernel changes until the counters are taken again.
GEMM_TRAFFIC_BYTES_PER_LAUNCH = 1606e6
# Events ride on the GEMM launches of every GEMM_EVENTS_EVERY-th timed step (the first, the sixth, ...): an attached
# pair of events costs about 4.5 us per launch, 0.5 ms on a step's 111 launches, and the headline number should
# carry as little of the instrument as the measurement allows.
GEMM_EVENTS_EVERY = 5


def cpu_baseline(model, n):
    """The oracle as it stands, timed on this host, on a bounded sample of the headline workload: forward +
    backward of the headline's local batch (4 samples) through ONE decoder layer of the model's shape (fp64 NumPy;
    10 TFLOP at the Llama-7B shape, 10-30 s).  The whole step is 32 such layers plus embedding, head and optimizer,
    which a CPU run of bounded length cannot hold: samples/s is the layer time taken 32 times, the rest left out,
    and says so."""
    from oracle import transformer as otr
    from paper_2408_12596_amd import synth
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    H, S, L = model["H"], model["S"], model["L"]
    spec = [(f"l0.{n}", s) for n, s in otr.layer_spec(model["arch"], H, model["F"])]
    flat = synth.init_params(spec, seed=0).astype(np.float64)
    p = {k[3:]: v for k, v in otr.unpack(flat, spec).items()}
    x = synth.activations((n, S, H), seed=1).astype(np.float64)
    dy = synth.activations((n, S, H), seed=2).astype(np.float64)
    t0 = time.perf_counter()
    out, cache = otr.layer_fwd(model["arch"], p, x, model["nh"])
    otr.layer_bwd(model["arch"], p, dy, cache, model["nh"])
    dt = time.perf_counter() - t0
    return {"value": n / (L * dt), "unit": "samples/s", "cores": int(cores), "kind": "oracle",
            "sample": f"{n} samples ({n * S} tokens) through one decoder layer of the headline shape, forward + backward, fp64 NumPy: "
                      f"{dt:.1f} s; value = {n} / ({L} layers x that), embedding, head, loss and optimizer left out",
            "seconds": dt}


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


class DeviceRank:
    """One simulated rank whose state is drawn on the device (same recipe as synth.init_params: matrices N(0, 0.02),
    gains 1, biases 0; seed 0), for models too large to draw on the host in a bench run."""

    def __init__(self, pb, torch, model, world, stage, max_b, cap_bytes=0):
        dev = "cuda:0"
        self.cfg = pb.make_cfg(**model, dtype="bf16", world=world, rank=0, zero_stage=stage, cap_bytes=cap_bytes)
        self.P = pb.model_param_count(self.cfg)
        off, ln, valid = (0, self.P, self.P) if stage == 0 else pb.shard_range(self.P, world, 0)
        self.valid = valid
        self.emb = next(o for name, shape, o in pb.model_spec(self.cfg) if name.startswith("l0."))   # elements before layer 0
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
        self.ctx.bind_state(params, master, m, v, grads, tok, max_b, ws, self.wsb, loss, own_shard=own, adam_t=1, lr=1e-6)   # the steps repeat one batch: a rate that leaves the loss near ln V


def rank_hbm_figures(P_model, emb, shard_valid, stage, p, tied):
    """Bandwidth of the streaming kernels a whole step times on its own: Adam (30 B per element: g, p, m, v read,
    p, m, v and the bf16 copy written), the ZeRO-3 parameter gathers (read 2 B, write 2 B per element; the forward
    pass gathers every unit, the backward pass all but the embedding), the local gradient reduce (12 B per owned
    element: the unit's gradient and the shard read, the shard written; a tied embedding matrix passes twice)."""
    out = {"adam": {"achieved": 30.0 * shard_valid / p["t_adam"] / 1e9, "unit": "GB/s", "peak": PEAK_HBM_GBS, "bytes_per_elem": 30,
                    "elems": shard_valid, "ms": p["t_adam"] * 1e3}}
    if stage >= 3:
        t = p["t_gather_fwd"] + p["t_gather_bwd"]
        gathered = 2 * P_model + (emb if tied else -emb)   # a tied head gathers the embedding matrix again in both passes
        out["gather"] = {"achieved": 4.0 * gathered / t / 1e9, "unit": "GB/s", "peak": PEAK_HBM_GBS, "bytes_per_elem": 4, "elems": gathered, "ms": t * 1e3}
    if stage >= 2:
        red = p["reduce_elems"]   # what the step's reduce launches moved: more than the shard where a tied embedding matrix lies in it
        out["local_reduce"] = {"achieved": 12.0 * red / p["t_reduce_bwd"] / 1e9, "unit": "GB/s", "peak": PEAK_HBM_GBS,
                               "bytes_per_elem": 12, "elems": red, "ms": p["t_reduce_bwd"] * 1e3}
    for v in out.values():
        v["frac"] = v["achieved"] / v["peak"]
    return out


def timed_steps(ctx, torch, stage, B, steps, warmup, timing=0, every=1):
    """`steps` timed steps after `warmup` untimed ones, bracketed by synchronisations; the launches selected by
    `timing` carry events in every `every`-th timed step (the first, the (every+1)-th, ...)."""
    ctx.set_kernel_timing(0)
    for _ in range(warmup):
        ctx.profile_step(stage, B)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    profs = []
    for i in range(steps):
        ctx.set_kernel_timing(timing if i % every == 0 else 0)
        profs.append(ctx.profile_step(stage, B))
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / steps
    ctx.set_kernel_timing(0)
    return dt, profs


def kernel_rooflines(ctx, torch, stage, B):
    """GEMM and attention launches of two steps with events on the launches themselves."""
    _, g = timed_steps(ctx, torch, stage, B, 2, 0, 1)
    _, a = timed_steps(ctx, torch, stage, B, 2, 0, 2)
    tg, ta = float(np.mean([p["t_gemm"] for p in g])), float(np.mean([p["t_attn"] for p in a]))
    out = {"gemm": {"achieved": g[0]["gemm_flops"] / tg / 1e12, "launches_per_step": g[0]["n_gemm_kernels"], "ms_per_step": tg * 1e3},
           "attention": {"achieved": a[0]["attn_flops"] / ta / 1e12, "launches_per_step": a[0]["n_attn"], "ms_per_step": ta * 1e3}}
    for v in out.values():
        v.update(unit="TFLOP/s", peak=PEAK_BF16_TFLOPS, frac=v["achieved"] / PEAK_BF16_TFLOPS)
    return out


def sweep_rows(r, torch, stage, batches, steps=3, warmup=1):
    rows = []
    for b in batches:
        d, pr = timed_steps(r.ctx, torch, stage, b, steps, warmup)
        rows.append({"local_batch": b, "samples_per_s": b / d, "ms_per_step": d * 1e3, "tflops": pr[0]["flops"] / d / 1e12,
                     "frac_mfma_peak": pr[0]["flops"] / d / 1e12 / PEAK_BF16_TFLOPS,
                     "t_consumed_ms": float(np.mean([p["t_consumed"] for p in pr])) * 1e3,
                     "accounted_gib": pr[0]["accounted_bytes"] / 2**30})
    return rows


def sub_record(pb, torch, name, model, world, stage, batches, extra_batches=()):
    """One configuration as a sub-record: its local-batch sweep, and at the top of the sweep the GEMM / attention
    rooflines and the bandwidth of the optimizer and of the collectives' local share."""
    r = DeviceRank(pb, torch, model, world, stage, max(batches + tuple(extra_batches)))
    top = max(batches)
    rec = {"workload": name, "zero_stage": stage, "world": world, "params": r.P, "shard_elems": r.valid,
           "sweep": sweep_rows(r, torch, stage, batches)}
    if extra_batches:
        rec["odd_batches"] = sweep_rows(r, torch, stage, extra_batches)
    _, pr = timed_steps(r.ctx, torch, stage, top, 2, 0)
    rec["at_local_batch"] = top
    rec["roofline"] = kernel_rooflines(r.ctx, torch, stage, top)
    rec["hbm_kernels"] = rank_hbm_figures(r.P, r.emb, r.valid, stage, pr[-1], model["arch"] == "gpt")
    del r
    torch.cuda.empty_cache()
    return rec


def allocation_stress(pb, torch, model, world, cap, gbs=64):
    """Algorithm 1 under an emulated cap at stages 1-3 (each sample the median of three warmed-up runs), then
    Algorithm 2 for four devices whose step times are the measured curve times 1, 1.5, 2 and 3."""
    stress = {"cap_bytes": cap, "gbs": gbs, "device_mix_time_factors": [1.0, 1.5, 2.0, 3.0], "stages": {}}
    for stage in (1, 2, 3):
        r = DeviceRank(pb, torch, model, world, stage, 16, cap_bytes=cap)
        r.ctx.set_sampling(1, 3)
        mbs, samples = r.ctx.search_mbs(stage)
        pts = {p["batch"]: p["t_consumed"] for p in samples}
        bs = sorted(pts)
        entry = {"mbs": mbs, "visited": [p["batch"] for p in samples], "t_consumed_ms": [pts[b] * 1e3 for b in bs]}
        curves = [(bs, [pts[b] * k for b in bs], mbs) for k in (1.0, 1.5, 2.0, 3.0)]
        cm = pb.comm_model(r.P, world, stage, 2.0, 4.0, 7 * 153e9) if stage >= 2 else {"t_micro": 0.0}
        al = pb.allocate(stage, gbs, curves, cm["t_micro"])
        entry["allocate"] = {"t_comm_ms": cm["t_micro"] * 1e3, "gmbs": al["gmbs"], "b": al["b"], "gas": al["gas"], "lbs": al["lbs"],
                             "T_ms": al["T"] * 1e3, "T_steps_ms": al["T_steps"] * 1e3}
        stress["stages"][str(stage)] = entry
        del r
        torch.cuda.empty_cache()
    return stress


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--batch", type=int, default=0, help="local batch of the headline number (default: the top of the workload's sweep)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--headline-only", action="store_true", help="the headline configuration's timed steps and rooflines only "
                    "(no sweeps, no sub-records, no CPU leg): the short run the rocprofv3 summaries under profiles/ are taken from")
    ap.add_argument("--workload", choices=sorted(WORKLOADS), default="llama7b", help="which configuration takes the headline's place "
                    "(default: the Llama-7B shape; the others exist so that the profiler can be pointed at them with --headline-only)")
    ap.add_argument("--curve-report", action="store_true", help="add the dense-sweep / spline / Algorithm 2 report (GPT-2-small) to the line")
    ap.add_argument("--layer-report", action="store_true", help="add one-layer timings at the larger configurations' shapes")
    ap.add_argument("--clock-report", action="store_true", help="add GEMM rates on zero, one and normal operands with the shader "
                    "clock during each run")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one rank on ONE GPU (the ZeRO world is simulated by shard offsets); --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2408_12596_amd import binding as pb

    pb.lib()   # fails loudly if the HIP library has not been built
    model, world, stage, sweep, label = WORKLOADS[args.workload]
    B = args.batch if args.batch else max(sweep)
    r = DeviceRank(pb, torch, model, world, stage, max(max(sweep), B))
    ctx = r.ctx
    # the timed steps carry events on the GEMM launches of every fifth step (the roofline kernel, measured live in the
    # timed region on the launch stream); the attention kernels are timed in further steps afterwards
    dt, profs = timed_steps(ctx, torch, stage, B, args.steps, args.warmup, 1, every=GEMM_EVENTS_EVERY)
    mean = lambda k: float(np.mean([p[k] for p in profs]))
    flops = profs[0]["flops"]
    evp = profs[::GEMM_EVENTS_EVERY]
    t_gemm, f_gemm, n_gemm = float(np.mean([p["t_gemm"] for p in evp])), evp[0]["gemm_flops"], evp[0]["n_gemm_kernels"]
    gemm_tflops = f_gemm / t_gemm / 1e12 if t_gemm > 0 else 0.0
    _, aprofs = timed_steps(ctx, torch, stage, B, 2, 0, 2)
    t_attn, f_attn = float(np.mean([p["t_attn"] for p in aprofs])), aprofs[0]["attn_flops"]
    out = {
        "metric": "samples/sec", "value": B / dt, "unit": "samples/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": dt * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": label, "local_batch": B, "zero_stage": stage, "world": world, "params": r.P, "shard_elems": r.valid},
        "tflops": flops / dt / 1e12,
        "frac_mfma_peak_step": flops / dt / 1e12 / PEAK_BF16_TFLOPS,
        "samples_per_s_time_consumed": B / mean("t_consumed"),
        "step_breakdown_ms": dict({k: mean(k) * 1e3 for k in ("t_fwd", "t_bwd", "t_adam", "t_gather_fwd", "t_gather_bwd", "t_reduce_bwd")},
                                  t_gemm=t_gemm * 1e3, t_attn=t_attn * 1e3),
        "roofline": {"bound": "mfma", "kernel": "gemm_dtl_kernel (all GEMM launches of the step)", "achieved": gemm_tflops,
                     "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": gemm_tflops / PEAK_BF16_TFLOPS,
                     "traffic": GEMM_TRAFFIC_BYTES_PER_LAUNCH if (args.workload == "llama7b" and B == max(HEADLINE_SWEEP)) else None,
                     "traffic_unit": "bytes between the L2 caches and memory per GEMM kernel launch",
                     "launches_per_step": n_gemm, "timed_spans_per_step": evp[0]["n_gemm"], "avg_launch_ms": t_gemm / max(n_gemm, 1) * 1e3,
                     "timed_steps_with_events": len(evp), "flop_per_launch": f_gemm / max(n_gemm, 1)},
        "attention": {"achieved": f_attn / t_attn / 1e12 if t_attn > 0 else 0.0, "unit": "TFLOP/s", "peak": PEAK_BF16_TFLOPS,
                      "frac": (f_attn / t_attn / 1e12 / PEAK_BF16_TFLOPS) if t_attn > 0 else 0.0, "head_dim": model["H"] // model["nh"],
                      "ms_per_step": t_attn * 1e3},
        "hbm_kernels": rank_hbm_figures(r.P, r.emb, r.valid, stage, dict({k: mean(k) for k in ("t_adam", "t_gather_fwd", "t_gather_bwd", "t_reduce_bwd")}, reduce_elems=profs[-1]["reduce_elems"]), model["arch"] == "gpt"),
        "loss": profs[-1]["loss"],
        "device": device_info(pb, torch),
    }
    if not args.headline_only:
        out["sweep"] = sweep_rows(r, torch, stage, sweep)
    del r, ctx
    torch.cuda.empty_cache()
    if not args.headline_only and args.workload == "llama7b":
        mid = sub_record(pb, torch, WORKLOADS["gpt1p3b"][4], MID, MID_WORLD, MID_STAGE, MID_SWEEP, MID_ODD)
        mid["allocation_stress"] = allocation_stress(pb, torch, MID, MID_WORLD, 40 * 2**30)
        small = sub_record(pb, torch, WORKLOADS["gpt2small"][4], WORKLOAD, WORLD, STAGE, SWEEP)
        out["sub_records"] = {"gpt_1p3b_zero2": mid, "gpt2_small_zero1": small}
    if args.curve_report or args.clock_report:
        rs = DeviceRank(pb, torch, WORKLOAD, WORLD, STAGE, max(SWEEP))
        if args.curve_report:
            out["curve_report"] = curve_report(pb, rs.ctx, rs.P, max(SWEEP))
        if args.clock_report:
            out["clock_report"] = clock_report(pb, rs.ctx, torch)
        del rs
    if args.layer_report:
        out["layer_report"] = layer_report(pb, torch)
    if not args.no_cpu_baseline and not args.headline_only:
        out["cpu_baseline"] = cpu_baseline(model, max(sweep))
    print(json.dumps(out))


if __name__ == "__main__":
    main()
