"""The bound the GPU parity tests put on O: max-abs 1e-2 as stated, loosened only where half a bf16
ulp of the reference value is larger, which starts at |O| = 4."""

import numpy as np

from tests import gpu_util as G


def test_o_bound_is_the_stated_one_below_four():
    x = np.array([0.0, 1e-30, 0.3, 1.0, 2.0, 2.56, 3.0, 3.999, -3.999])
    assert np.all(G.o_bound(x) == 1e-2)


def test_o_bound_is_half_a_bf16_ulp_from_four_on():
    # bf16 keeps 8 significant bits: the spacing on [4, 8) is 2^-5, on [8, 16) 2^-4
    assert G.o_bound(np.array([4.0]))[0] == 2.0 ** -6
    assert G.o_bound(np.array([-7.99]))[0] == 2.0 ** -6
    assert G.o_bound(np.array([8.0]))[0] == 2.0 ** -5
    # and it is what rounding to bf16 can cost, no more: nearest-even rounding of values in [4, 8)
    rng = np.random.default_rng(0)
    v = rng.uniform(4.0, 8.0, 1000).astype(np.float32)
    bits = v.view(np.uint32)
    rounded = (((bits + 0x7FFF + ((bits >> 16) & 1)) >> 16) << 16).astype(np.uint32).view(np.float32)
    err = np.abs(rounded.astype(np.float64) - v.astype(np.float64))
    assert err.max() <= 2.0 ** -6 and err.max() > 2.0 ** -7


def test_o_excess_sign():
    want = np.array([1.0, 5.0])
    assert G.o_excess(want + np.array([0.009, 0.015]), want) < 0
    assert G.o_excess(want + np.array([0.011, 0.0]), want) > 0
    assert G.o_excess(want + np.array([0.0, 0.016]), want) > 0
