"""Oracle: what one profile sample means and the max-batch-size search.

TEST INFRASTRUCTURE ONLY - never imported by the product path.

Section "Time Consumed Estimation" defines TimeConsumedDuringStep per ZeRO
stage; Algorithm 1 ("Heterogeneity Aware of each GPU") and Section
"Heterogeneity Aware" define the search for the largest batch that does not
run out of memory.

Readings where the printed algorithm cannot be followed literally:
  * the binary search as printed updates low and high to mid under
    `while low <= high` and never ends; here `lo` is the largest batch known
    to fit, `hi` the largest batch not known to fail, the midpoint is rounded
    up, and the loop ends when they meet;
  * after an out-of-memory error at batch 2^k in the doubling sweep the
    search interval is [2^(k-1), 2^k - 1];
  * the doubling sweep visits the powers of two not above the estimate, and
    the estimate itself stays as the upper bound;
  * a result of 0 means that batch 1 does not fit and the caller moves to the
    next ZeRO stage.
"""


class OutOfMemory(Exception):
    pass


def time_consumed(stage, t_fwd, t_bwd, t_gather_fwd=0.0, t_gather_bwd=0.0, t_reduce_bwd=0.0):
    """TimeConsumedDuringStep.
    stage 0, 1: forward + backward run time.
    stage 2   : forward + (backward minus the collective time inside it).
    stage 3   : total minus all-gather in forward, all-gather in backward and
                reduce-scatter in backward.
    t_fwd / t_bwd include the collective (here: stand-in) time."""
    if stage in (0, 1):
        return t_fwd + t_bwd
    if stage == 2:
        return t_fwd + (t_bwd - t_reduce_bwd)
    if stage == 3:
        return (t_fwd + t_bwd) - t_gather_fwd - t_gather_bwd - t_reduce_bwd
    raise ValueError(stage)


def search_mbs(bytes_now, forward, step, total_memory):
    """Algorithm 1 for one device.
    bytes_now()  -> bytes currently allocated
    forward(b)   -> runs a forward pass at batch b (may leave memory allocated)
    step(b)      -> runs one training step, returns its time or raises
                    OutOfMemory
    Returns (mbs, samples) with samples = [(batch, time), ...] in call order."""
    bf = bytes_now()
    forward(1)
    af = bytes_now()
    if af <= bf:
        raise ValueError("forward pass allocated nothing")
    est = int((total_memory - bf) // (af - bf))
    samples = []
    lo, hi = 0, est
    b = 1
    while b <= est:
        try:
            t = step(b)
        except OutOfMemory:
            hi = b - 1
            break
        samples.append((b, t))
        lo = b
        b *= 2
    while lo < hi:
        mid = (lo + hi + 1) // 2
        try:
            t = step(mid)
        except OutOfMemory:
            hi = mid - 1
            continue
        samples.append((mid, t))
        lo = mid
    return lo, samples


def search_stage(first_stage, search):
    """Section "Heterogeneity Aware": a stage at which not even one sample fits
    (mbs = 0) is given up for the next one.  search(stage) -> (mbs, samples).
    Returns (stage, mbs, samples) of the first stage >= first_stage with
    mbs > 0, or (-1, 0, []) when none has."""
    for stage in range(first_stage, 4):
        mbs, samples = search(stage)
        if mbs > 0:
            return stage, mbs, samples
    return -1, 0, []
