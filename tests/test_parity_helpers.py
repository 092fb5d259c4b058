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


def _stored_forward(o):
    """the oracle's own acting forward pass at every (t, b) of its stored unroll, as the arrays a GPU trajectory holds"""
    T, B = o.T, o.B
    hid = list(o.cfg["net"]["hidden"])
    acts = [np.zeros((T, B, h), np.float32) for h in hid]
    head = np.zeros((T, B, o.NH), np.float32)
    for t in range(T):
        for b in range(B):
            hd, a = PT.oracle_forward_at(o, t, b)
            head[t, b] = hd
            off = 0
            for l, h in enumerate(hid):
                acts[l][t, b] = a[off:off + h]; off += h
    return acts, head


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_numpy_maze_backward_equals_the_oracle(orc, dtype):
    """np_maze_backward_from_stored (the stand-in for the oracle at sizes it cannot reach) against the oracle's own
    loss and gradient on a small maze, to rounding in both precisions -- and, in bf16, clearly worse with the weights
    left unrounded, so the rounding point is seen."""
    cfg = W.get("maze_16384", B=24, T=6)
    cfg["net"]["hidden"] = [48, 40, 32]
    cfg["net"]["dtype"] = dtype
    cfg["env"] = dict(cfg["env"], rows=6, cols=6, max_steps=9)
    o = orc.Oracle(cfg, seed=5)
    rng = np.random.default_rng(1)
    o.theta[:] += (0.05 * rng.standard_normal(o.P)).astype(np.float32)       # biases away from zero
    o.rollout()
    theta0 = o.theta.copy()
    acts, head = _stored_forward(o)
    cells = 36
    walls = np.unpackbits(o.walls.view(np.uint8), axis=1, bitorder="little")[:, :cells].astype(bool)
    o.learn()
    regions, P = PT.param_regions(cfg)
    loss, g = PT.np_maze_backward_from_stored(cfg, theta0, walls, o.tr_state_i[:-1, :, 0], acts, head, o.tr_action,
                                              o.adv, o.ret, t_chunk=4)
    tol = 2e-6                # the oracle's gradient is stored in binary32; in this case no activation rounds differently
    assert np.abs(loss - o.loss).max() <= tol * np.abs(o.loss).max()
    worst = PT.assert_regions_close("gradient", g, o.grad, regions, tol)
    if dtype == "bf16":
        cfg32 = copy.deepcopy(cfg); cfg32["net"]["dtype"] = "fp32"
        _, g_unrounded = PT.np_maze_backward_from_stored(cfg32, theta0, walls, o.tr_state_i[:-1, :, 0], acts, head,
                                                         o.tr_action, o.adv, o.ret, t_chunk=4)
        assert PT.rel(g_unrounded, o.grad) > 3 * max(PT.rel(g, o.grad), 1e-4)


def test_numpy_maze_layer_forward_equals_the_oracle(orc):
    """np_maze_forward_layers_from_stored against the oracle's own bf16 acting forward pass on a small maze: fed with
    the oracle's stored activations, every layer's reference reproduces the next stored activation and the heads."""
    cfg = W.get("maze_16384", B=24, T=6)
    cfg["net"]["hidden"] = [48, 40, 32]
    cfg["env"] = dict(cfg["env"], rows=6, cols=6, max_steps=9)
    o = orc.Oracle(cfg, seed=8)
    rng = np.random.default_rng(2)
    o.theta[:] += (0.05 * rng.standard_normal(o.P)).astype(np.float32)
    o.rollout()
    acts, head = _stored_forward(o)
    walls = np.unpackbits(o.walls.view(np.uint8), axis=1, bitorder="little")[:, :36].astype(bool)
    seen = 0
    for t0, t1, refs, heads in PT.np_maze_forward_layers_from_stored(cfg, o.theta, walls, o.tr_state_i[:-1, :, 0], acts, t_chunk=4):
        for l, r in enumerate(refs):
            assert PT.assert_bf16_layers_close(f"layer {l + 1}", acts[l][t0:t1], r) <= 0.002
        assert np.abs(heads - head[t0:t1]).max() <= 1e-5 * np.abs(head).max()
        seen += t1 - t0
    assert seen == o.T
    # a planted mistake is seen: one weight of the second layer changed by a bfloat16 step
    th = o.theta.copy()
    regions, _ = PT.param_regions(cfg)
    w2 = dict(regions)["W2"]
    th[w2.start + 5] *= 1.02
    with pytest.raises(AssertionError):
        for t0, t1, refs, heads in PT.np_maze_forward_layers_from_stored(cfg, th, walls, o.tr_state_i[:-1, :, 0], acts, t_chunk=4):
            for l, r in enumerate(refs):
                PT.assert_bf16_layers_close(f"layer {l + 1}", acts[l][t0:t1], r)
