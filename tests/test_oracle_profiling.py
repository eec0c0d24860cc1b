"""Pins for oracle/profiling.py.  CPU only."""
import numpy as np
import pytest

from oracle import profiling as pf


def test_time_consumed_per_stage():
    # Section "Time Consumed Estimation": stage 0/1 fwd+bwd; stage 2 subtracts
    # the collective inside backward; stage 3 subtracts three collectives.
    assert pf.time_consumed(0, 3.0, 5.0, 0.25, 0.5, 1.0) == 8.0
    assert pf.time_consumed(1, 3.0, 5.0, 0.25, 0.5, 1.0) == 8.0
    assert pf.time_consumed(2, 3.0, 5.0, 0.25, 0.5, 1.0) == 7.0
    assert pf.time_consumed(3, 3.0, 5.0, 0.25, 0.5, 1.0) == 6.25
    with pytest.raises(ValueError):
        pf.time_consumed(4, 1, 1)


class FakeDevice:
    """Affine memory model: state + b * (fwd part [+ extra held only by step])."""

    def __init__(self, total, state, fwd_per_sample, step_extra_per_sample, step_const=0):
        self.total, self.state = total, state
        self.fwd, self.extra, self.const = fwd_per_sample, step_extra_per_sample, step_const
        self.now = state
        self.calls = []

    def bytes_now(self):
        return self.now

    def forward(self, b):
        self.now = self.state + b * self.fwd

    def step(self, b):
        self.calls.append(b)
        need = self.state + b * (self.fwd + self.extra) + self.const
        if need > self.total:
            raise pf.OutOfMemory()
        return 1.0 + 0.5 * b

    def brute(self):
        b = 0
        while self.state + (b + 1) * (self.fwd + self.extra) + self.const <= self.total:
            b += 1
        return b


def test_search_equals_brute_force_on_random_affine_models():
    rng = np.random.default_rng(0)
    for _ in range(300):
        total = int(rng.integers(1000, 200000))
        dev = FakeDevice(total, int(rng.integers(0, total // 2)), int(rng.integers(1, 3000)),
                         int(rng.integers(0, 2000)), int(rng.integers(0, 500)))
        mbs, samples = pf.search_mbs(dev.bytes_now, dev.forward, dev.step, dev.total)
        assert mbs == dev.brute()
        ok = [b for b, _ in samples]
        assert all(b <= mbs for b in ok)
        if mbs >= 1:
            assert 1 in ok and mbs in ok          # both ends of the curve are sampled
            assert len(dev.calls) <= 2 * int(np.log2(max(mbs, 1))) + 4
        assert len(set(dev.calls)) == len(dev.calls)  # no batch size tried twice


def test_search_exact_when_forward_estimate_is_tight():
    dev = FakeDevice(total=1000, state=100, fwd_per_sample=90, step_extra_per_sample=0)
    mbs, samples = pf.search_mbs(dev.bytes_now, dev.forward, dev.step, dev.total)
    assert mbs == 10
    assert dev.calls == [1, 2, 4, 8, 9, 10]
    assert samples[-1] == (10, 6.0)


def test_search_returns_zero_when_one_sample_does_not_fit():
    dev = FakeDevice(total=1000, state=900, fwd_per_sample=50, step_extra_per_sample=100)
    mbs, samples = pf.search_mbs(dev.bytes_now, dev.forward, dev.step, dev.total)
    assert mbs == 0 and samples == []


def test_stage_escalation_stops_at_the_first_stage_that_fits():
    # Section "Heterogeneity Aware": mbs = 0 at a stage sends the search to the next one
    table = {0: (0, []), 1: (0, []), 2: (5, [(1, .1), (2, .2), (4, .4), (5, .5)]), 3: (9, [(1, .1)])}
    seen = []

    def search(stage):
        seen.append(stage)
        return table[stage]
    assert pf.search_stage(0, search) == (2, 5, table[2][1]) and seen == [0, 1, 2]
    seen.clear()
    assert pf.search_stage(3, search) == (3, 9, table[3][1]) and seen == [3]
    assert pf.search_stage(0, lambda s: (0, [])) == (-1, 0, [])
