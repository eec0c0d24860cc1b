"""The parity helpers themselves (CPU): the blockwise bound must catch what the whole-tensor bound lets through."""
import numpy as np

from gpu_util import blockwise_rel_l2, rel_l2


def test_blockwise_bound_catches_a_dropped_tile_and_a_lost_tail():
    rng = np.random.default_rng(0)
    ref = rng.standard_normal((16384, 768))
    noisy = ref * (1 + 2e-3 * rng.standard_normal(ref.shape))          # bf16-sized rounding everywhere
    assert rel_l2(noisy, ref) < 3e-3 and blockwise_rel_l2(noisy, ref) < 4e-3
    dropped = noisy.copy()
    dropped[640:704, 128:192] = 0.0                                      # one 64 x 64 tile never written
    assert rel_l2(dropped, ref) < 2e-2                                    # the whole-tensor bar does not see it
    assert blockwise_rel_l2(dropped, ref) > 0.9
    tail = noisy.copy()
    tail[-8:, :] = 0.0                                                    # the last eight rows lost
    assert rel_l2(tail, ref) < 2.5e-2 and blockwise_rel_l2(tail, ref) > 0.3


def test_blockwise_bound_on_ragged_shapes_and_vectors():
    rng = np.random.default_rng(1)
    ref = rng.standard_normal((130, 70))
    got = ref.copy()
    got[128:, 64:] += 1.0                                                 # only the 2 x 6 corner tile is wrong
    assert blockwise_rel_l2(got, ref) > 0.5 and rel_l2(got, ref) < 0.05
    v = rng.standard_normal(1000)
    w = v.copy()
    w[960:] = 0.0                                                         # the trailing partial run of 40
    assert blockwise_rel_l2(w, v) > 0.9
    assert blockwise_rel_l2(v, v) == 0.0
    # a tile of near-zeros is measured against the tensor's scale, not against itself
    z = ref.copy()
    z[:64, :64] *= 1e-9
    assert blockwise_rel_l2(z * (1 + 1e-3), z) < 2e-3
    assert blockwise_rel_l2(np.zeros((4, 4)), np.zeros((4, 4))) == 0.0
