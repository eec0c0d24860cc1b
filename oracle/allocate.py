"""Oracle: performance curves and Algorithm 2 ("Optimal Batch Size Searching").

TEST INFRASTRUCTURE ONLY - never imported by the product path.

Follows Section "Problem Formulation" (Eq. 1-4), Section "Optimal Batch Size
Searching" and Algorithm 2, in the paper's notation: gbs, mbs_i, speed_i,
time_optimal, gmbs_i, gas, lbs_i, time_communication.

Readings where the paper is silent or the listing is garbled:
  * p_i holds step times; it is first turned into speed points b / time(b),
    samples at the same batch are averaged, and a natural cubic spline through
    them is read at every integer batch in [1, mbs_i] (clamped to the end
    knots outside the sampled range, floored at 1e-9 of the largest knot);
  * speed_i = max of that curve; time_optimal = gbs / sum(speed_i);
    gmbs_i = floor(time_optimal * speed_i);
  * the listing's delta_i / u_i lines cancel to a constant; following the text
    (Eq. 2 and 3 are used to hand the remaining samples to the devices with the
    lower workload) each remaining sample goes to the device that would finish
    earliest after taking it, argmin (gmbs_i + 1) / speed_i, lowest index on
    ties.  With constant speeds sum_i (T - t_i) speed_i = T sum(speed) - gbs, so
    minimising Eq. 4 is minimising T, which this greedy does;
  * mbs_i bounds the micro-batch, not gmbs_i (gradient accumulation covers the
    rest); the micro-batch is the largest batch of the peak range
    {b : speed_i(b) >= peak_frac * max}, peak_frac = 0.95 by default;
    gas_i = ceil(gmbs_i / b_i), lbs_i = gmbs_i - (gas_i - 1) b_i;
  * stage 2/3: candidate t are all distinct values of time_i(b); find(g_i, t)
    is the largest b <= mbs_i with time_i(b) <= t, where time_i is the running
    maximum of b / speed_i(b) (a spline through noisy samples may dip; with the
    running maximum "can finish b samples within t" is monotone in b);
    gas = ceil(gbs / sum_i b_i); wall = (t + time_communication) * gas; the
    first strict minimum wins; the last accumulation step carries
    gbs - (gas - 1) sum_i b_i samples, handed out one at a time to the device
    whose time after taking it is smallest (never above b_i);
  * stage 0/1 reports two predictions: T, Eq. 1 with t_i = gmbs_i / speed_i
    (what the split was made for), and T_steps, Eq. 1 with t_i summed over the
    accumulation steps the device will really run on its own curve,
    (gas_i - 1) time_i(b_i) + time_i(lbs_i) with time_i(b) = b / speed_i(b).
"""
import math
import numpy as np
from .spline import natural_spline_coeffs, natural_spline_eval

SPEED_FLOOR = 1e-9


def speed_curve(batches, times, mbs):
    """Speeds at b = 0..mbs (index 0 unused, set to 0)."""
    pts = {}
    for b, t in zip(batches, times):
        pts.setdefault(int(b), []).append(float(b) / float(t))
    xs = sorted(pts)
    ys = [sum(pts[b]) / len(pts[b]) for b in xs]
    out = np.zeros(mbs + 1)
    q = np.clip(np.arange(1, mbs + 1, dtype=np.float64), xs[0], xs[-1])
    if len(xs) == 1:
        out[1:] = ys[0]
    else:
        out[1:] = natural_spline_eval(xs, natural_spline_coeffs(xs, ys), q)
    out[1:] = np.maximum(out[1:], SPEED_FLOOR * max(ys))
    return out


def time_curve(speed):
    """Monotone step time at b = 0..mbs from a speed curve: running maximum of
    b / speed(b)."""
    t = np.zeros_like(speed)
    for b in range(1, len(speed)):
        t[b] = max(t[b - 1], b / speed[b])
    return t


def find(tm, t):
    """Largest batch whose step time does not exceed t (0 if none): the `find`
    of Algorithm 2, written as its definition over the whole curve."""
    fits = [b for b in range(1, len(tm)) if tm[b] <= t]
    return max(fits) if fits else 0


def iteration_time(t):
    """Eq. 1."""
    return max(t)


def under_utilization(t, p):
    """Eq. 2-4: sum_i (T - t_i) p_i."""
    T = iteration_time(t)
    return sum((T - ti) * pi for ti, pi in zip(t, p))


def allocate_stage01(gbs, curves, peak_frac=0.95):
    """curves: list of (batches, times, mbs).  Returns dict with gmbs, b, gas,
    lbs (lists of ints) and T (predicted iteration time, Eq. 1)."""
    n = len(curves)
    sp = [speed_curve(*c) for c in curves]
    mbs = [c[2] for c in curves]
    speed = [float(sp[i][1:].max()) if mbs[i] >= 1 else 0.0 for i in range(n)]
    speed_cluster = 0.0
    for s in speed:
        speed_cluster += s
    if speed_cluster <= 0.0:
        raise ValueError("no device can run a single sample")
    time_optimal = gbs / speed_cluster
    gmbs = [int(math.floor(time_optimal * s)) for s in speed]
    remain = gbs - sum(gmbs)
    while remain > 0:
        best, best_t = -1, math.inf
        for i in range(n):
            if speed[i] > 0.0:
                t = (gmbs[i] + 1) / speed[i]
                if t < best_t:
                    best, best_t = i, t
        gmbs[best] += 1
        remain -= 1
    b, gas, lbs = [], [], []
    for i in range(n):
        if gmbs[i] == 0:
            b.append(0), gas.append(0), lbs.append(0)
            continue
        peak = [k for k in range(1, mbs[i] + 1) if sp[i][k] >= peak_frac * speed[i]]
        bi = min(gmbs[i], max(peak))
        gi = -(-gmbs[i] // bi)
        b.append(bi), gas.append(gi), lbs.append(gmbs[i] - (gi - 1) * bi)
    T = max(gmbs[i] / speed[i] for i in range(n) if speed[i] > 0.0)
    T_steps = max((gas[i] - 1) * (b[i] / sp[i][b[i]]) + lbs[i] / sp[i][lbs[i]] for i in range(n) if gmbs[i] > 0)
    return dict(gmbs=gmbs, b=b, gas=gas, lbs=lbs, T=T, T_steps=T_steps)


def allocate_stage23(gbs, curves, time_communication):
    """Returns dict with b (micro-batch per device), gas, lbs, gmbs, t, wall."""
    n = len(curves)
    tm = [time_curve(speed_curve(*c)) if c[2] >= 1 else np.zeros(1) for c in curves]
    cand = sorted({float(tm[i][k]) for i in range(n) for k in range(1, len(tm[i]))})
    best = None
    for t in cand:
        bs = [find(tm[i], t) for i in range(n)]
        mb = sum(bs)
        if mb == 0:
            continue
        gas = -(-gbs // mb)
        wall = (t + time_communication) * gas
        if best is None or wall < best["wall"]:
            best = dict(b=bs, gas=gas, t=t, wall=wall)
    if best is None:
        raise ValueError("no device can run a single sample")
    b, gas = best["b"], best["gas"]
    R = gbs - (gas - 1) * sum(b)
    lbs = [0] * n
    for _ in range(R):
        pick, pick_t = -1, math.inf
        for i in range(n):
            if lbs[i] < b[i] and tm[i][lbs[i] + 1] < pick_t:
                pick, pick_t = i, tm[i][lbs[i] + 1]
        lbs[pick] += 1
    best["lbs"] = lbs
    best["gmbs"] = [(gas - 1) * b[i] + lbs[i] for i in range(n)]
    return best


def allocate(stage, gbs, curves, time_communication=0.0, peak_frac=0.95):
    if stage in (0, 1):
        return allocate_stage01(gbs, curves, peak_frac)
    if stage in (2, 3):
        return allocate_stage23(gbs, curves, time_communication)
    raise ValueError(stage)
