"""The comparison helpers of the GPU parity tests, checked on the CPU: the parameter regions tile the flat
vector, a planted error in a small region is caught, and the threaded oracle update equals the plain one."""
import copy

import numpy as np
import pytest

from paper_2104_06272_amd import workloads as W
import parity as PT


@pytest.mark.parametrize("name", W.ORDER)
def test_regions_tile_the_parameter_vector(orc, name):
    cfg = W.get(name, B=16, T=2)
    o = orc.Oracle(cfg, seed=0)
    regions, P = PT.param_regions(cfg)
    assert P == o.P
    cover = np.zeros(P, np.int32)
    for _, sl in regions:
        cover[sl] += 1
    assert np.all(cover == 1)
    names = [n for n, _ in regions]
    assert ("W1[agent]" in names) == (cfg["env"]["kind"] == "maze")
    # biases are zero at initialisation, weights are not: the regions sit where the oracle puts them
    for n, sl in regions:
        assert np.all(o.theta[sl] == 0) == n.startswith("b"), n


def test_small_region_error_is_caught():
    cfg = W.get("catch_4096")
    regions, P = PT.param_regions(cfg)
    rng = np.random.default_rng(0)
    ref = rng.standard_normal(P)
    got = ref * (1 + 1e-6 * rng.standard_normal(P))
    PT.assert_regions_close("x", got, ref, regions, 1e-4)
    bad = got.copy()
    bad[-4:] *= 1.5                                   # the head bias: 4 of 79 876 entries
    assert PT.rel(bad, ref) < 1e-2                    # invisible in one global norm at the bf16 tolerance
    with pytest.raises(AssertionError, match="bh"):
        PT.assert_regions_close("x", bad, ref, regions, 2e-2)
    one = got.copy()
    one[regions[0][1].start + 7] += 0.5               # a single entry of the first weight matrix
    with pytest.raises(AssertionError, match="W1"):
        PT.assert_regions_close("x", one, ref, regions, 2e-2)


@pytest.mark.parametrize("kind", ["catch", "maze_bf16"])
def test_threaded_oracle_update_equals_plain(orc, kind):
    if kind == "catch":
        cfg = W.get("catch_small", B=32, T=7)
    else:
        cfg = W.get("maze_16384", B=16, T=12)
        cfg["net"]["hidden"] = [32, 16]
        cfg["env"] = dict(cfg["env"], rows=4, cols=4, max_steps=5)
    a = orc.Oracle(cfg, seed=4); b = orc.Oracle(copy.deepcopy(cfg), seed=4)
    for o in (a, b):
        o.rollout()
    a.learn()
    PT.oracle_learn_parallel(b, workers=3)
    assert np.allclose(a.ret, b.ret, rtol=0, atol=0) and np.allclose(a.adv, b.adv, rtol=0, atol=0)
    assert np.allclose(a.loss, b.loss, rtol=1e-12)
    assert PT.rel(b.grad, a.grad) < 1e-6
    assert PT.rel(b.theta, a.theta) < 1e-6 and a.adam_t == b.adam_t == 1
    assert np.allclose(a.m, b.m, rtol=1e-5, atol=1e-12)
