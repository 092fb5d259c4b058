"""Pins of the CPU oracle against things other than itself: published
known answers, closed forms, invariants, brute force, library routines.
None of these tests needs a GPU."""
import math
import os
from fractions import Fraction

import numpy as np
import pytest

from paper_2104_06272_amd import workloads as W

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def tiny(kind, hidden=(4, 4), B=4, T=5, **kw):
    if kind == "catch":
        env = dict(kind="catch", rows=kw.get("rows", 4), cols=kw.get("cols", 3), max_steps=0)
        cfg = W.get("catch_small")
    elif kind == "pendulum":
        env = dict(kind="pendulum", rows=0, cols=0, max_steps=kw.get("max_steps", 200))
        cfg = W.get("pendulum_8192")
    else:
        env = dict(kind="maze", rows=kw.get("rows", 16), cols=kw.get("cols", 16),
                   max_steps=kw.get("max_steps", 256), p_wall=kw.get("p_wall", 0.2))
        cfg = W.get("maze_16384")
    cfg["env"] = env
    cfg["net"]["hidden"] = list(hidden)
    cfg["net"]["dtype"] = kw.get("dtype", "fp32")
    if "lam" in kw:
        cfg["net"]["lambda"] = kw["lam"]
    cfg["B"], cfg["T"] = B, T
    return cfg


# --------------------------------------------------------------------------- RNG
def test_philox_known_answers(orc):
    rows = [l.split() for l in open(os.path.join(GOLD, "philox4x32_10_kat.txt")) if not l.startswith("#")]
    assert len(rows) == 3
    for r in rows:
        v = [int(x, 16) for x in r]
        assert list(orc.philox(v[0:4], v[4:6])) == v[6:10]


def test_uniform_and_bounded_statistics(orc):
    L = orc.lib()
    words = np.concatenate([orc.draw(7, i, 0, 0) for i in range(5000)])
    u = np.array([L.orc_u01(int(w)) for w in words])
    assert u.min() >= 0.0 and u.max() < 1.0
    assert abs(u.mean() - 0.5) < 4 * math.sqrt(1 / 12 / u.size)
    assert abs(u.var() - 1 / 12) < 0.003
    assert L.orc_u01(0xFFFFFFFF) == 1.0 - 2.0 ** -24 and L.orc_u01(0) == 0.0
    assert L.orc_u01_plus(0xFFFFFFFF) == 1.0 and L.orc_u01_plus(0) == 2.0 ** -24
    k = np.array([L.orc_bounded(int(w), 5) for w in words])
    assert k.min() == 0 and k.max() == 4
    cnt = np.bincount(k, minlength=5)
    chi2 = ((cnt - k.size / 5) ** 2 / (k.size / 5)).sum()
    assert chi2 < 18.5          # chi-square, 4 dof, p = 0.001
    assert L.orc_bounded(0xFFFFFFFF, 5) == 4 and L.orc_bounded(0, 5) == 0


def test_counter_draws_are_independent_of_batch(orc):
    # same (seed, env, t) gives the same draw whatever else exists
    a = orc.Oracle(tiny("catch", B=3), seed=11)
    b = orc.Oracle(tiny("catch", B=9), seed=11)
    assert np.array_equal(a.state_i, b.state_i[:3])


# ----------------------------------------------------------------------- detmath
def _rel(a, b):
    return np.abs(a.astype(np.float64) - b) / np.maximum(np.abs(b), 1e-300)


def test_det_exp(orc):
    x = np.linspace(-86.9, 87.9, 200001).astype(np.float32)
    y = orc.f32fun("orc_exp")(x)
    assert _rel(y, np.exp(x.astype(np.float64))).max() < 3e-7
    f = orc.lib().orc_exp
    assert f(0.0) == 1.0
    assert f(-200.0) == f(-87.0) and f(-87.0) > 0.0
    # monotone on a fine grid near zero (softmax ordering)
    z = orc.f32fun("orc_exp")(np.linspace(-1, 0, 5001).astype(np.float32))
    assert np.all(np.diff(z.astype(np.float64)) >= 0)


def test_det_log(orc):
    x = np.concatenate([np.linspace(2.0 ** -24, 1.0, 100001), np.logspace(-30, 30, 20001)]).astype(np.float32)
    y = orc.f32fun("orc_log")(x).astype(np.float64)
    ref = np.log(x.astype(np.float64))
    err = np.abs(y - ref)
    assert np.all(err <= 3e-7 * np.abs(ref) + 1e-7)
    assert orc.lib().orc_log(1.0) == 0.0


def test_det_sin_cos(orc):
    pi_f = float(np.float32(math.pi))
    x = np.linspace(-pi_f, pi_f, 200001).astype(np.float32)
    s = orc.f32fun("orc_sin")(x).astype(np.float64)
    c = orc.f32fun("orc_cos")(x).astype(np.float64)
    xd = x.astype(np.float64)
    assert np.abs(s - np.sin(xd)).max() < 2e-7
    assert np.abs(c - np.cos(xd)).max() < 2e-7
    big = np.abs(np.sin(xd)) > 1e-2
    assert _rel(s[big], np.sin(xd)[big]).max() < 4e-7
    L = orc.lib()
    assert L.orc_sin(0.0) == 0.0 and L.orc_cos(0.0) == 1.0
    xs = x[::97]
    assert np.array_equal(orc.f32fun("orc_sin")(-xs), -orc.f32fun("orc_sin")(xs))
    assert np.array_equal(orc.f32fun("orc_cos")(-xs), orc.f32fun("orc_cos")(xs))


def test_det_cos2pi(orc):
    u = (np.arange(0, 1 << 24, 257, dtype=np.int64) * 2.0 ** -24).astype(np.float32)
    y = orc.f32fun("orc_cos2pi")(u).astype(np.float64)
    assert np.abs(y - np.cos(2 * np.pi * u.astype(np.float64))).max() < 3e-7
    L = orc.lib()
    assert L.orc_cos2pi(0.0) == 1.0 and L.orc_cos2pi(0.5) == -1.0
    assert L.orc_cos2pi(0.25) == 0.0 and L.orc_cos2pi(0.75) == 0.0


def test_det_tanh(orc):
    x = np.concatenate([np.linspace(-12, 12, 100001), np.linspace(-0.3, 0.3, 50001),
                        np.logspace(-20, -1, 2001)]).astype(np.float32)
    y = orc.f32fun("orc_tanh")(x)
    ref = np.tanh(x.astype(np.float64))
    nz = x != 0
    assert _rel(y[nz], ref[nz]).max() < 4e-7
    assert np.abs(y.astype(np.float64)).max() <= 1.0
    assert orc.lib().orc_tanh(0.0) == 0.0
    assert np.array_equal(orc.f32fun("orc_tanh")(-x), -y)


def test_bf16_round(orc):
    import torch
    x = np.random.default_rng(0).standard_normal(20000).astype(np.float32) * 37
    x = np.concatenate([x, np.array([1.0, 1.00390625, 1.005859375, 1.001953125, 0.0], np.float32)])
    mine = orc.f32fun("orc_bf16_round")(x)
    ref = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()   # library rounding
    assert np.array_equal(mine, ref)


# -------------------------------------------------------------------------- Catch
def test_catch_episodes_and_returns(orc):
    cfg = W.get("catch_small", B=200, T=45)
    o = orc.Oracle(cfg, seed=3)
    o.rollout()
    done, rew = o.tr_done, o.tr_reward
    # every episode lasts rows-1 = 9 steps: dones exactly at t = 8, 17, 26, ...
    t_idx = np.arange(45)[:, None]
    assert np.array_equal(done.astype(bool), np.broadcast_to(t_idx % 9 == 8, done.shape))
    # reward is +-1 exactly when done and exactly 0 otherwise
    assert np.all(np.isin(rew[done == 1], (-1.0, 1.0)))
    assert np.all(rew[done == 0] == 0.0)
    ep_ret = rew.reshape(5, 9, -1).sum(1)
    assert np.all(np.isin(ep_ret, (-1.0, 1.0)))
    # observed states: ball row = t mod 9 (never the bottom row), ball column fixed within an episode
    by = o.tr_state_i[:45, :, 1]
    assert np.array_equal(by, np.broadcast_to(t_idx % 9, by.shape))
    bx = o.tr_state_i[:45, :, 0].reshape(5, 9, -1)
    assert np.all(bx == bx[:, :1])
    # paddle moves by a-1 with clamping; it restarts in the middle column
    px = o.tr_state_i[:, :, 2]
    a = o.tr_action
    for t in range(45):
        want = np.clip(px[t] + a[t] - 1, 0, 4)
        if t % 9 == 8:
            want = np.full_like(want, 2)
        assert np.array_equal(px[t + 1], want)
    # reward sign: caught iff the paddle ends under the ball
    for t in range(8, 45, 9):
        final_px = np.clip(px[t] + a[t] - 1, 0, 4)
        assert np.array_equal(rew[t] > 0, final_px == o.tr_state_i[t, :, 0])


def test_catch_observation(orc):
    o = orc.Oracle(W.get("catch_small", B=50, T=20), seed=5)
    o.rollout()
    for b in range(50):
        x = o.observe(b).reshape(10, 5)
        bx, by, px, _ = o.state_i[b]
        want = np.zeros((10, 5), np.float32)
        want[by, bx] = 1
        want[9, px] = 1
        assert np.array_equal(x, want) and x.sum() == 2


def test_catch_scripted_policies(orc):
    # always "stay": caught iff the ball column is the middle one; ball column uniform
    B = 4000
    o = orc.Oracle(W.get("catch_small", B=B, T=9), seed=8)
    bx0 = o.state_i[:, 0].copy()
    rets = np.zeros(B)
    for b in range(B):
        for t in range(9):
            r, d = o.env_step(b, action=1, t=t)
            rets[b] += r
            assert d == (t == 8)
    assert np.array_equal(rets > 0, bx0 == 2)
    cnt = np.bincount(bx0, minlength=5)
    assert ((cnt - B / 5) ** 2 / (B / 5)).sum() < 18.5
    # zero weights -> uniform policy: P(catch) = 1/5 exactly in law, mean return -> -0.6,
    # and the paddle's final column follows the 9-step clamped random walk from column 2
    cfg = W.get("catch_small", B=B, T=9)
    o = orc.Oracle(cfg, seed=9)
    o.theta[:] = 0
    o.rollout()
    rets = o.tr_reward.sum(0)
    se = math.sqrt(0.2 * 0.8 * 4 / B)
    assert abs(rets.mean() + 0.6) < 4 * se
    law = [Fraction(0)] * 5
    law[2] = Fraction(1)
    for _ in range(9):
        nxt = [Fraction(0)] * 5
        for c, p in enumerate(law):
            for mv in (-1, 0, 1):
                nxt[min(4, max(0, c + mv))] += p / 3
        law = nxt
    assert law[0] == Fraction(1304, 6561) and law[1] == Fraction(3946, 19683) and law[2] == Fraction(3967, 19683)
    final_px = np.clip(o.tr_state_i[8, :, 2] + o.tr_action[8] - 1, 0, 4)
    cnt = np.bincount(final_px, minlength=5)
    exp = np.array([float(p) for p in law]) * B
    assert ((cnt - exp) ** 2 / exp).sum() < 18.5


# ----------------------------------------------------------------------- Pendulum
def _pend_ref(th, thd, a):
    """closed-form semi-implicit Euler update in float64 with libm"""
    u = min(2.0, max(-2.0, 2.0 * a))
    r = -(th * th + 0.1 * thd * thd + 0.001 * u * u)
    nthd = thd + (15.0 * math.sin(th) + 3.0 * u) * 0.05
    nthd = min(8.0, max(-8.0, nthd))
    nth = th + nthd * 0.05
    nth = (nth + math.pi) % (2 * math.pi) - math.pi
    return nth, nthd, r


def test_pendulum_step_vs_closed_form(orc):
    o = orc.Oracle(tiny("pendulum", B=1, T=4), seed=1)
    rng = np.random.default_rng(4)
    for _ in range(3000):
        th = np.float32(rng.uniform(-math.pi, math.pi))
        thd = np.float32(rng.uniform(-8, 8))
        a = np.float32(rng.uniform(-1, 1))
        o.state_f[0] = (th, thd)
        o.state_i[0, 0] = 0
        r, d = o.env_step(0, action_f=float(a))
        nth, nthd, rr = _pend_ref(float(th), float(thd), float(a))
        dth = (float(o.state_f[0, 0]) - nth + math.pi) % (2 * math.pi) - math.pi
        assert abs(dth) < 1e-5 and abs(float(o.state_f[0, 1]) - nthd) < 1e-5 and abs(r - rr) < 1e-5
        assert d == 0
        assert -float(np.float32(math.pi)) <= o.state_f[0, 0] < float(np.float32(math.pi))
        assert abs(o.state_f[0, 1]) <= 8.0
        assert r <= 0 and r >= -(math.pi ** 2 + 6.4 + 0.004) - 1e-4


def test_pendulum_fixed_point_and_episode_length(orc):
    o = orc.Oracle(tiny("pendulum", B=2, T=4, max_steps=200), seed=2)
    o.state_f[0] = (0.0, 0.0)
    for t in range(199):
        r, d = o.env_step(0, action_f=0.0, t=t)
        assert r == 0.0 and d == 0 and tuple(o.state_f[0]) == (0.0, 0.0)
    r, d = o.env_step(0, action_f=0.0, t=199)
    assert d == 1 and o.state_i[0, 0] == 0            # 200th step ends the episode and resets
    th, thd = o.state_f[0]
    assert -math.pi - 1e-6 <= th <= math.pi + 1e-6 and -1 <= thd < 1


def test_pendulum_angle_wrap_boundary(orc):
    """The stored angle lies in [-pi_f, pi_f) with pi_f the binary32 pi (R-10): walking the starting angle one
    binary32 step at a time takes the angle before wrapping through every value around pi_f, pi_f itself included,
    and the half-open interval must hold at each (pi_f wraps, the value just below it does not)."""
    o = orc.Oracle(tiny("pendulum", B=1, T=2, max_steps=200), seed=1)
    pi_f = np.float32(math.pi)

    def after_step(bits):
        o.state_i[0, 0] = 0
        o.state_f[0] = (np.uint32(bits).view(np.float32), 1.0)
        o.env_step(0, action_f=0.0, t=0)
        return o.state_f[0, 0]

    lo, hi = int(np.float32(3.0).view(np.uint32)), int(np.float32(3.14).view(np.uint32))   # stays / wraps
    assert after_step(lo) > 0 > after_step(hi)
    while hi - lo > 1:                                       # the first starting angle whose step wraps
        mid = (lo + hi) // 2
        lo, hi = (mid, hi) if after_step(mid) > 0 else (lo, mid)
    out = [after_step(hi + k) for k in range(-400, 400)]
    out = np.array(out, np.float32)
    assert (out >= -pi_f).all() and (out < pi_f).all()
    assert (out > 3.14).any() and (out < -3.14).any()       # both sides of the wrap were visited
    up = out[out > 0]
    assert up.max() == np.nextafter(pi_f, np.float32(0))     # the last value that stays is the one just below pi_f


def test_pendulum_init_distribution_and_obs(orc):
    B = 4000
    o = orc.Oracle(tiny("pendulum", B=B, T=2), seed=6)
    th, thd = o.state_f[:, 0].astype(np.float64), o.state_f[:, 1].astype(np.float64)
    assert th.min() >= -math.pi - 1e-6 and th.max() <= math.pi + 1e-6
    assert abs(th.mean()) < 4 * (2 * math.pi / math.sqrt(12)) / math.sqrt(B)
    assert abs(th.var() - (2 * math.pi) ** 2 / 12) < 0.25
    assert thd.min() >= -1 and thd.max() < 1 and abs(thd.mean()) < 4 * (2 / math.sqrt(12)) / math.sqrt(B)
    # the whole of U(-1, 1) and of U(-pi, pi): variance of the uniform law and both ends reached
    assert abs(thd.var() - 4 / 12) < 0.03 and thd.min() < -0.99 and thd.max() > 0.99
    assert th.min() < -0.99 * math.pi and th.max() > 0.99 * math.pi
    for b in range(0, B, 131):
        x = o.observe(b).astype(np.float64)
        assert abs(x[0] - math.cos(th[b])) < 3e-7 and abs(x[1] - math.sin(th[b])) < 3e-7 and x[2] == thd[b]


def test_pendulum_energy_drift_without_torque(orc):
    # with u = 0 and no clipping, E = thd^2/2 + 15 cos(th) is conserved by the flow; the
    # symplectic Euler map keeps it within O(dt) of its initial value
    o = orc.Oracle(tiny("pendulum", B=1, T=2, max_steps=100000), seed=1)
    o.state_f[0] = (2.0, 0.5)
    e0 = 0.5 * 0.5 ** 2 / 2 * 2 + 15 * math.cos(2.0)
    worst = 0.0
    for t in range(2000):
        o.env_step(0, action_f=0.0, t=t)
        th, thd = (float(v) for v in o.state_f[0])
        worst = max(worst, abs(0.5 * thd * thd + 15 * math.cos(th) - e0))
    assert worst < 0.05 * 15 * 3          # O(dt) band, dt = 0.05


# --------------------------------------------------------------------------- Maze
def _flood(walls, n=16):
    free = ~walls
    seen = np.zeros_like(free)
    seen[0, 0] = True
    while True:
        grow = seen.copy()
        grow[1:] |= seen[:-1]; grow[:-1] |= seen[1:]; grow[:, 1:] |= seen[:, :-1]; grow[:, :-1] |= seen[:, 1:]
        grow &= free
        if np.array_equal(grow, seen):
            return seen
        seen = grow


def _walls(o, b, n=16):
    bits = np.unpackbits(o.walls[b].view(np.uint8), bitorder="little")[: n * n]
    return bits.reshape(n, n).astype(bool)


def test_maze_generation(orc):
    B = 300
    o = orc.Oracle(tiny("maze", hidden=(8,), B=B, T=2), seed=4)
    dens = []
    for b in range(B):
        w = _walls(o, b)
        assert not w[0, 0] and not w[15, 15]
        assert _flood(w)[15, 15]                     # independent flood fill reaches the goal
        dens.append(w.mean())
    # accepted mazes are a connected subset, so density sits at or a little below 0.2*254/256
    assert 0.15 < np.mean(dens) < 0.2 * 254 / 256 + 0.005
    # unconditioned wall law: threshold floor(0.2 * 2^32) on raw words
    words = np.concatenate([orc.draw(4, b, (blk << 32) | 0, 4) for b in range(40) for blk in range(64)])
    p = (words < 0x33333333).mean()
    assert abs(p - 0.2) < 4 * math.sqrt(0.16 / words.size)
    # a rejected first attempt really is disconnected: rebuild attempt 0 by hand and compare
    rejected = 0
    for b in range(B):
        w0 = np.array([orc.draw(4, b, (blk << 32) | 0, 4) for blk in range(64)]).reshape(-1) < 0x33333333
        w0 = w0.reshape(16, 16).copy(); w0[0, 0] = False; w0[15, 15] = False
        if _flood(w0)[15, 15]:
            assert np.array_equal(w0, _walls(o, b))
        else:
            rejected += 1
            assert not np.array_equal(w0, _walls(o, b))
    assert 0 < rejected < B // 2


def _bfs_path(w):
    from collections import deque
    n = w.shape[0]
    prev = {(0, 0): None}
    q = deque([(0, 0)])
    moves = [(-1, 0, 0), (0, 1, 1), (1, 0, 2), (0, -1, 3)]
    while q:
        r, c = q.popleft()
        if (r, c) == (n - 1, n - 1):
            break
        for dr, dc, a in moves:
            rr, cc = r + dr, c + dc
            if 0 <= rr < n and 0 <= cc < n and not w[rr, cc] and (rr, cc) not in prev:
                prev[(rr, cc)] = ((r, c), a)
                q.append((rr, cc))
    acts, cur = [], (n - 1, n - 1)
    while prev[cur] is not None:
        cur, a = prev[cur]
        acts.append(a)
    return acts[::-1]


def test_maze_shortest_path_return_and_walls(orc):
    o = orc.Oracle(tiny("maze", hidden=(8,), B=20, T=2), seed=12)
    for b in range(20):
        w = _walls(o, b)
        acts = _bfs_path(w)
        d = len(acts)
        total = np.float32(0)
        for i, a in enumerate(acts):
            r, done = o.env_step(b, action=a, t=i)
            total = np.float32(total + np.float32(r))
            assert done == (i == d - 1)
            if not done:
                cell = o.state_i[b, 0]
                assert not w[cell // 16, cell % 16]
        assert abs(float(total) - (1 - 0.01 * (d - 1))) < 1e-5
        assert tuple(o.state_i[b, :2]) == (0, 0)
        # bumping into the border or a wall leaves the agent in place; the step cap ends the episode
        for i in range(256):
            r, done = o.env_step(b, action=0 if i % 2 == 0 else 3, t=i)
            assert o.state_i[b, 0] == 0
            assert abs(r + 0.01) < 1e-9 and done == (i == 255)
        x = o.observe(b).reshape(3, 16, 16)
        assert np.array_equal(x[0].astype(bool), w) and x[1].sum() == 1 and x[1, 0, 0] == 1
        assert x[2].sum() == 1 and x[2, 15, 15] == 1


# ------------------------------------------------------------------------ Network
def _unpack(o, theta=None):
    th = o.theta if theta is None else theta
    dims = [o.D] + list(o.cfg["net"]["hidden"])
    Ws, bs, off = [], [], 0
    for l in range(len(dims) - 1):
        Ws.append(th[off:off + dims[l] * dims[l + 1]].reshape(dims[l], dims[l + 1])); off += dims[l] * dims[l + 1]
        bs.append(th[off:off + dims[l + 1]]); off += dims[l + 1]
    Wh = th[off:off + dims[-1] * o.NH].reshape(dims[-1], o.NH); off += dims[-1] * o.NH
    bh = th[off:off + o.NH]; off += o.NH
    assert off == th.size
    return Ws, bs, Wh, bh


def test_glorot_init(orc):
    o = orc.Oracle(W.get("catch_4096", B=2, T=2), seed=0)
    assert o.P == 79876
    Ws, bs, Wh, bh = _unpack(o)
    for Wm in Ws:
        a = math.sqrt(6.0 / sum(Wm.shape))
        assert np.abs(Wm).max() <= a * (1 + 1e-6)
        assert abs(Wm.astype(np.float64).var() / (a * a / 3) - 1) < 0.05
        assert abs(Wm.mean()) < 4 * a / math.sqrt(3 * Wm.size)
    for b in bs + [bh]:
        assert np.all(b == 0)
    for cols, fo in ((slice(0, 3), 3), (slice(3, 4), 1)):
        a = math.sqrt(6.0 / (256 + fo))
        blk = Wh[:, cols]
        assert np.abs(blk).max() <= a * (1 + 1e-6) and np.abs(blk).max() > 0.9 * a
    # different seeds and different layers give different numbers
    o2 = orc.Oracle(W.get("catch_4096", B=2, T=2), seed=1)
    assert not np.array_equal(o.theta, o2.theta)
    assert o.P == sum(x.size for x in Ws + bs) + Wh.size + bh.size


@pytest.mark.parametrize("name", ["catch_small", "pendulum_8192"])
def test_forward_vs_float64(orc, name):
    o = orc.Oracle(W.get(name, B=6, T=3), seed=2)
    rng = np.random.default_rng(1)
    o.theta[:] += rng.standard_normal(o.P).astype(np.float32) * 0.05     # non-zero biases too
    Ws, bs, Wh, bh = _unpack(o)
    for b in range(6):
        x = o.observe(b)
        head, acts = o.forward(x, want_acts=True)
        hcur = x.astype(np.float64)
        ref_acts = []
        for Wm, bv in zip(Ws, bs):
            hcur = np.maximum(hcur @ Wm.astype(np.float64) + bv, 0)
            ref_acts.append(hcur)
        ref = hcur @ Wh.astype(np.float64) + bh
        assert np.allclose(head, ref, rtol=1e-5, atol=1e-6)
        assert np.allclose(acts, np.concatenate(ref_acts), rtol=1e-5, atol=1e-6)


def test_forward_zero_weights_gives_biases(orc):
    o = orc.Oracle(W.get("catch_small", B=2, T=2), seed=2)
    o.theta[:] = 0
    o.theta[-4:] = (0.25, -1.5, 3.0, 0.125)
    assert np.array_equal(o.forward(o.observe(0)), np.array([0.25, -1.5, 3.0, 0.125], np.float32))


def test_forward_bf16_rounding_points(orc):
    import torch
    o = orc.Oracle(tiny("maze", hidden=(32, 16), B=3, T=2, dtype="bf16"), seed=5)
    bf = lambda a: torch.from_numpy(np.ascontiguousarray(a, np.float32)).to(torch.bfloat16).to(torch.float32).numpy()
    Ws, bs, Wh, bh = _unpack(o)
    for b in range(3):
        x = o.observe(b)
        head, acts = o.forward(x, want_acts=True)
        hcur = bf(x).astype(np.float64)
        ref_acts = []
        for Wm, bv in zip(Ws, bs):
            z = hcur @ bf(Wm).astype(np.float64) + bv
            hcur = bf(np.maximum(z, 0).astype(np.float32)).astype(np.float64)
            ref_acts.append(hcur)
        ref = hcur @ bf(Wh).astype(np.float64) + bh
        # hidden activations may differ by one bf16 step where fp32 and fp64 sums straddle a tie
        assert np.allclose(acts, np.concatenate(ref_acts), rtol=2 ** -7, atol=1e-6)
        assert np.mean(acts == np.concatenate(ref_acts)) > 0.95
        assert np.allclose(head, ref, rtol=2e-2, atol=2e-3)
        assert np.array_equal(acts, bf(acts))          # stored activations are bf16 values


# ----------------------------------------------------------------------- Sampling
def test_categorical_sampler(orc):
    L = orc.lib()
    us = (np.arange(0, 1 << 24, 4099) * 2.0 ** -24).astype(np.float32)
    # equal logits: action = floor(3u) up to the rounding of the running sums
    a = np.array([orc.sample_categorical([0.7, 0.7, 0.7], u) for u in us])
    assert np.mean(a == np.floor(3 * us.astype(np.float64))) > 0.9995
    assert np.all(np.diff(a) >= 0) and set(a) == {0, 1, 2}
    # ties: "the first index whose running sum EXCEEDS u * total" -- with equal logits the running sums are exactly
    # 1, 2, ..., so u = k / A sits on a boundary and belongs to the upper action
    assert [orc.sample_categorical([0.0, 0.0], u) for u in (0.0, 0.25, 0.5, 0.75)] == [0, 0, 1, 1]
    assert [orc.sample_categorical([1.5] * 4, u) for u in (0.0, 0.25, 0.5, 0.75, 1 - 2.0 ** -24)] == [0, 1, 2, 3, 3]
    # a dominant logit wins wherever it sits (the others have mass e^-40, below the grid's smallest u > 0)
    for i in range(3):
        lg = [0.0, 0.0, 0.0]; lg[i] = 40.0
        assert all(orc.sample_categorical(lg, u) == i for u in us[1::50])
    # frequencies follow softmax
    lg = np.array([0.3, -1.2, 0.9, 0.1], np.float32)
    p = np.exp(lg.astype(np.float64)); p /= p.sum()
    words = np.concatenate([orc.draw(3, i, 5, 0) for i in range(6000)])
    acts = np.array([orc.sample_categorical(lg, L.orc_u01(int(w))) for w in words])
    cnt = np.bincount(acts, minlength=4)
    assert ((cnt - p * acts.size) ** 2 / (p * acts.size)).sum() < 16.3     # 3 dof, p = 0.001
    # monotone in u: inverse-CDF property
    a = np.array([orc.sample_categorical(lg, u) for u in us])
    assert np.all(np.diff(a) >= 0)
    cdf = np.cumsum(p)
    assert np.mean(a == np.searchsorted(cdf, us.astype(np.float64), side="right").clip(0, 3)) > 0.9995


def test_gaussian_sampler(orc):
    n = 20000
    ws = np.array([orc.draw(5, i, 0, 0) for i in range(n)])
    out = np.array([orc.sample_gaussian(0.3, -0.5, w[0], w[1]) for w in ws], np.float64)
    eps, z, act = out[:, 0], out[:, 1], out[:, 2]
    assert abs(eps.mean()) < 4 / math.sqrt(n) and abs(eps.var() - 1) < 0.05
    kurt = ((eps - eps.mean()) ** 4).mean() / eps.var() ** 2
    assert abs(kurt - 3) < 0.25
    sigma = math.exp(-0.5)
    assert np.allclose(z, 0.3 + sigma * eps, rtol=1e-6, atol=1e-6)
    assert np.allclose(act, np.tanh(z), rtol=1e-6, atol=1e-7)
    # Box-Muller against the textbook formula in float64
    L = orc.lib()
    u0 = np.array([L.orc_u01_plus(int(w[0])) for w in ws[:2000]], np.float64)
    u1 = np.array([L.orc_u01(int(w[1])) for w in ws[:2000]], np.float64)
    assert np.allclose(eps[:2000], np.sqrt(-2 * np.log(u0)) * np.cos(2 * np.pi * u1), rtol=2e-5, atol=2e-6)
    # clamp of log_sigma
    e1, z1, _ = orc.sample_gaussian(0.0, 7.0, ws[0][0], ws[0][1])
    assert abs(z1 - math.exp(2.0) * e1) < 1e-5 * abs(z1) + 1e-6
    e2, z2, _ = orc.sample_gaussian(0.0, -9.0, ws[0][0], ws[0][1])
    assert abs(z2 - math.exp(-5.0) * e2) < 1e-5 * abs(z2) + 1e-9


# ------------------------------------------------------------------------ Returns
def _brute_lambda_returns(rew, done, val, gamma, lam):
    """Mixture definition: G^lam_t = (1-lam) sum_{n<N} lam^(n-1) G^(n)_t + lam^(N-1) G^(N)_t, where
    G^(n)_t is the n-step return with explicit discount products, and N is the number of steps up
    to the end of the unroll or of the episode, whichever comes first."""
    T, B = rew.shape
    G = np.zeros((T, B))
    for b in range(B):
        for t in range(T):
            N = T - t
            for n in range(1, T - t + 1):
                if done[t + n - 1, b]:
                    N = n
                    break
            nstep = []
            for n in range(1, N + 1):
                g, disc = 0.0, 1.0
                for i in range(n):
                    g += disc * float(rew[t + i, b])
                    disc *= 0.0 if done[t + i, b] else gamma
                g += disc * float(val[t + n, b])
                nstep.append(g)
            G[t, b] = (1 - lam) * sum(lam ** (n - 1) * nstep[n - 1] for n in range(1, N)) + lam ** (N - 1) * nstep[N - 1]
    return G


@pytest.mark.parametrize("lam", [1.0, 0.95, 0.0, 0.5])
def test_returns_vs_bruteforce_and_gae(orc, lam):
    rng = np.random.default_rng(10)
    T, B, gamma = 13, 7, 0.99
    rew = rng.standard_normal((T, B)).astype(np.float32)
    done = (rng.random((T, B)) < 0.2).astype(np.uint8)
    val = rng.standard_normal((T + 1, B)).astype(np.float32)
    ret, adv = orc.returns(rew, done, val, gamma, lam)
    assert np.allclose(ret, _brute_lambda_returns(rew, done, val, gamma, lam), rtol=1e-12, atol=1e-12)
    # GAE form
    A = np.zeros((T + 1, B))
    for t in range(T - 1, -1, -1):
        disc = np.where(done[t] == 1, 0.0, gamma)
        delta = rew[t] + disc * val[t + 1] - val[t]
        A[t] = delta + disc * lam * A[t + 1]
    assert np.allclose(adv, A[:T], rtol=1e-12, atol=1e-12)
    assert np.allclose(adv, ret - val[:T], rtol=0, atol=1e-14)
    if lam == 0.0:
        assert np.allclose(ret, rew + np.where(done == 1, 0, gamma) * val[1:], atol=1e-14)


def test_returns_closed_forms(orc):
    for line in open(os.path.join(GOLD, "returns_closed_form.txt")):
        if line.startswith("#"):
            continue
        T, gamma, lam, r, v, what, value = line.split()
        T = int(T); gamma, lam, r, v, value = map(float, (gamma, lam, r, v, value))
        rew = np.full((T, 2), r, np.float32); done = np.zeros((T, 2), np.uint8)
        val = np.full((T + 1, 2), v, np.float32)
        ret, adv = orc.returns(rew, done, val, gamma, lam)
        got = ret[0, 0] if what == "G0" else adv[0, 0]
        assert abs(got - value) < 5e-9
        n = np.arange(T, 0, -1)
        if lam == 1.0:
            assert np.allclose(ret[:, 0], r * (1 - gamma ** n) / (1 - gamma) + gamma ** n * v, rtol=1e-12)
        assert np.allclose(adv[:, 0], (r + gamma * v - v) * (1 - (gamma * lam) ** n) / (1 - gamma * lam), rtol=1e-10)
    # an episode end at every step: G_t = r_{t+1}
    rew = np.arange(12, dtype=np.float32).reshape(6, 2)
    ret, _ = orc.returns(rew, np.ones((6, 2), np.uint8), np.full((7, 2), 9.0, np.float32), 0.99, 0.95)
    assert np.array_equal(ret, rew.astype(np.float64))


# ------------------------------------------------------------- Objective, gradient
def _np_surrogate(o, theta, obs, kind):
    """Independent float64 statement of the objective for fixed samples (a, z), A and G."""
    Ws, bs, Wh, bh = _unpack(o, theta.astype(np.float64))
    h = obs
    for Wm, bv in zip(Ws, bs):
        h = np.maximum(h @ Wm + bv, 0)
    head = h @ Wh + bh
    A, G = o.adv.reshape(-1), o.ret.reshape(-1)
    beta, cv = o.cfg["net"]["entropy_coef"], o.cfg["net"]["value_coef"]
    V = head[:, -1]
    if kind == "categorical":
        lg = head[:, :-1]
        lp = lg - lg.max(1, keepdims=True)
        lp = lp - np.log(np.exp(lp).sum(1, keepdims=True))
        H = -(np.exp(lp) * lp).sum(1)
        lpa = lp[np.arange(lp.shape[0]), o.tr_action.reshape(-1)]
    else:
        mu, ls = head[:, 0], np.clip(head[:, 1], -5, 2)
        z = o.tr_z.reshape(-1).astype(np.float64)
        lpa = -0.5 * ((z - mu) / np.exp(ls)) ** 2 - ls - 0.5 * math.log(2 * math.pi)
        H = ls + 0.5 * math.log(2 * math.pi * math.e)
    per = -A * lpa + cv * (G - V) ** 2 - beta * H
    return per.mean(), (-A * lpa).mean(), (cv * (G - V) ** 2).mean(), (-beta * H).mean()


@pytest.mark.parametrize("kind", ["catch", "pendulum", "maze"])
def test_gradient_vs_finite_differences(orc, kind):
    cfg = tiny(kind, hidden=(5, 4), B=3, T=5, rows=4, cols=4 if kind == "maze" else 3, max_steps=3, p_wall=0.1)
    o = orc.Oracle(cfg, seed=13)
    rng = np.random.default_rng(3)
    o.theta[:] += rng.standard_normal(o.P).astype(np.float32) * 0.3
    o.rollout()
    ret, adv = orc.returns(o.tr_reward, o.tr_done, o.tr_value, cfg["net"]["gamma"], cfg["net"]["lambda"])
    o.ret[:] = ret; o.adv[:] = adv + rng.standard_normal(adv.shape)     # any constants will do
    o.loss_and_grad()
    # observations rebuilt from the stored states by the test itself
    T, B = o.T, o.B
    obs = np.zeros((T * B, o.D))
    for t in range(T):
        for b in range(B):
            si, sf = o.tr_state_i[t, b], o.tr_state_f[t, b]
            if kind == "catch":
                x = np.zeros((4, 3)); x[si[1], si[0]] = 1; x[3, si[2]] = 1
            elif kind == "pendulum":
                x = np.array([math.cos(sf[0]), math.sin(sf[0]), sf[1]])
            else:
                n = 16
                wb = np.unpackbits(o.walls[b].view(np.uint8), bitorder="little")[:n].astype(float)
                ag = np.zeros(n); ag[si[0]] = 1
                gl = np.zeros(n); gl[n - 1] = 1
                x = np.concatenate([wb, ag, gl])
            obs[t * B + b] = np.ravel(x)
    pol = "categorical" if kind != "pendulum" else "gauss"
    th0 = o.theta.astype(np.float64)
    l0 = _np_surrogate(o, th0, obs, pol)
    assert np.allclose(o.loss, l0, rtol=1e-6, atol=1e-7)
    h = 1e-5
    fd = np.zeros(o.P)
    for i in range(o.P):
        tp, tm = th0.copy(), th0.copy()
        tp[i] += h; tm[i] -= h
        fd[i] = (_np_surrogate(o, tp, obs, pol)[0] - _np_surrogate(o, tm, obs, pol)[0]) / (2 * h)
    g = o.grad.astype(np.float64)
    assert np.linalg.norm(g) > 1e-3
    assert np.linalg.norm(g - fd) / np.linalg.norm(fd) < 1e-5
    assert np.abs(g - fd).max() < 1e-5 * np.abs(fd).max() + 1e-7


@pytest.mark.parametrize("shift", [4.0, -8.0])
def test_gaussian_gradient_outside_the_log_sigma_clamp(orc, shift):
    """R-19: log_sigma is clamped to [-5, 2], and a clamped log_sigma passes no gradient.  With the head's bias pushed
    far outside the clamp every sample is clamped: the objective (float64, written out by the test) then does not
    depend on that head at all, and central differences of it say so for every parameter."""
    cfg = tiny("pendulum", hidden=(5, 4), B=3, T=5, max_steps=3)
    o = orc.Oracle(cfg, seed=17)
    rng = np.random.default_rng(5)
    o.theta[:] += rng.standard_normal(o.P).astype(np.float32) * 0.2
    o.theta[-2] = shift                                   # bias of log_sigma (heads: mu, log_sigma, value)
    o.rollout()
    assert (o.tr_head[:-1, :, 1] > 2.5).all() if shift > 0 else (o.tr_head[:-1, :, 1] < -5.5).all()
    ret, adv = orc.returns(o.tr_reward, o.tr_done, o.tr_value, cfg["net"]["gamma"], cfg["net"]["lambda"])
    o.ret[:] = ret; o.adv[:] = adv + rng.standard_normal(adv.shape)
    o.loss_and_grad()
    T, B = o.T, o.B
    obs = np.array([[math.cos(o.tr_state_f[t, b, 0]), math.sin(o.tr_state_f[t, b, 0]), o.tr_state_f[t, b, 1]]
                    for t in range(T) for b in range(B)], np.float64)
    th0 = o.theta.astype(np.float64)
    assert np.allclose(o.loss, _np_surrogate(o, th0, obs, "gauss"), rtol=1e-6, atol=1e-7)
    h = 1e-5
    fd = np.zeros(o.P)
    for i in range(o.P):
        tp, tm = th0.copy(), th0.copy()
        tp[i] += h; tm[i] -= h
        fd[i] = (_np_surrogate(o, tp, obs, "gauss")[0] - _np_surrogate(o, tm, obs, "gauss")[0]) / (2 * h)
    g = o.grad.astype(np.float64)
    Wh = slice(o.P - 3 - 4 * 3, o.P - 3)
    assert np.abs(g[Wh].reshape(4, 3)[:, 1]).max() == 0.0 and g[-2] == 0.0      # the clamped head's column and bias
    assert np.abs(fd[Wh].reshape(4, 3)[:, 1]).max() < 1e-9 and abs(fd[-2]) < 1e-9
    assert np.linalg.norm(g) > 1e-3 and np.linalg.norm(g - fd) / np.linalg.norm(fd) < 1e-5


def test_head_gradient_identities(orc):
    cfg = tiny("catch", hidden=(4,), B=4, T=3)
    o = orc.Oracle(cfg, seed=3)
    # all-zero parameters: uniform policy, H = log 3, entropy gradient 0
    o.theta[:] = 0
    o.rollout()
    o.ret[:] = 0; o.adv[:] = 0
    o.loss_and_grad()
    assert abs(o.loss[3] + float(np.float32(0.01)) * math.log(3)) < 1e-12 and abs(math.log(3) - 1.0986123) < 1e-7
    assert np.abs(o.grad).max() < 1e-15             # A = 0, G = V = 0, uniform policy
    # bias gradient of the logits sums to zero for any A (softmax shift invariance)
    rng = np.random.default_rng(0)
    o.theta[:] = rng.standard_normal(o.P).astype(np.float32) * 0.5
    o.rollout()
    o.adv[:] = rng.standard_normal(o.adv.shape); o.ret[:] = rng.standard_normal(o.ret.shape)
    o.loss_and_grad()
    assert abs(o.grad[-4:-1].astype(np.float64).sum()) < 1e-7
    # mean over copies: duplicating every sample leaves loss and gradient unchanged
    g1, l1 = o.grad.copy(), o.loss.copy()
    cfg2 = tiny("catch", hidden=(4,), B=8, T=3)
    o2 = orc.Oracle(cfg2, seed=3)
    o2.theta[:] = o.theta
    for arr in ("tr_state_i", "tr_state_f", "tr_action", "tr_reward", "tr_done", "tr_value"):
        getattr(o2, arr)[:] = np.concatenate([getattr(o, arr)] * 2, axis=1)
    o2.adv[:] = np.concatenate([o.adv] * 2, axis=1); o2.ret[:] = np.concatenate([o.ret] * 2, axis=1)
    o2.loss_and_grad()
    assert np.allclose(o2.grad, g1, rtol=1e-6, atol=1e-9) and np.allclose(o2.loss, l1, rtol=1e-12)


# --------------------------------------------------------------------------- Adam
def test_adam_closed_forms(orc):
    g = np.array([0.5, -2.0, 0.0, 1e-3, -7e-6], np.float32)
    th = np.ones(5, np.float32); m = np.zeros(5); v = np.zeros(5)
    orc.adam(th, g, m, v, 1, 3e-4, 0.9, 0.999, 1e-8)
    want = 1 - 3e-4 * g.astype(np.float64) / (np.abs(g) + 1e-8)
    assert np.allclose(th, want, rtol=0, atol=1e-7) and th[2] == 1.0
    # constant gradient for t steps: theta_t = theta_0 - t lr g/(|g|+eps)
    th = np.zeros(5, np.float32); m = np.zeros(5); v = np.zeros(5)
    for t in range(1, 51):
        orc.adam(th, g, m, v, t, 3e-4, 0.9, 0.999, 1e-8)
    assert np.allclose(th, -50 * 3e-4 * g.astype(np.float64) / (np.abs(g) + 1e-8), rtol=1e-5, atol=1e-7)


def test_adam_vs_library(orc):
    import torch
    rng = np.random.default_rng(2)
    n = 300
    p = torch.nn.Parameter(torch.from_numpy(rng.standard_normal(n)).double())
    opt = torch.optim.Adam([p], lr=3e-4, betas=(0.9, 0.999), eps=1e-8)
    th = p.detach().numpy().astype(np.float32).copy(); m = np.zeros(n); v = np.zeros(n)
    p.data = torch.from_numpy(th.astype(np.float64))
    for t in range(1, 21):
        g = (rng.standard_normal(n) * 10 ** rng.uniform(-4, 1)).astype(np.float32)
        p.grad = torch.from_numpy(g.astype(np.float64))
        opt.step()
        orc.adam(th, g, m, v, t, 3e-4, 0.9, 0.999, 1e-8)
    assert np.abs(th - p.detach().numpy()).max() < 1e-6


# --------------------------------------------------------------- whole-agent checks
def test_unroll_continues_across_calls(orc):
    # two unrolls of 10 equal one of 20 when parameters do not change (state stays resident)
    a = orc.Oracle(W.get("catch_small", B=16, T=10), seed=21)
    b = orc.Oracle(W.get("catch_small", B=16, T=20), seed=21)
    a.rollout(); first = (a.tr_action.copy(), a.tr_reward.copy())
    a.rollout()
    b.rollout()
    assert np.array_equal(np.concatenate([first[0], a.tr_action]), b.tr_action)
    assert np.array_equal(np.concatenate([first[1], a.tr_reward]), b.tr_reward)
    assert a.global_step == b.global_step == 20


def test_n_updates_per_unroll(orc):
    """N updates on one unroll (the paper's remark on splitting the learner batch): with N = 1 it is the plain
    update; with N = 2 the two chunk gradients (at the acting-time parameters) average to the full-batch gradient,
    the reported loss is the full-batch loss, and the parameters are what two Adam steps in chunk order give."""
    cfg = W.get("catch_small", B=32, T=8)
    a = orc.Oracle(cfg, seed=5); b = orc.Oracle(cfg, seed=5)
    a.rollout(); b.rollout()
    a.learn(); b.learn_n(1)
    assert np.array_equal(a.theta, b.theta) and np.array_equal(a.m, b.m) and np.array_equal(a.v, b.v)
    # N = 2 from non-zero moments
    a.rollout(); b.rollout()
    assert np.array_equal(a.tr_action, b.tr_action)
    theta0 = b.theta.copy().astype(np.float64); m0 = b.m.copy(); v0 = b.v.copy(); t0 = b.adam_t
    # full-batch gradient and loss at theta0 (learn computes the returns first; loss_and_grad needs them)
    ret, adv = orc.returns(a.tr_reward, a.tr_done, a.tr_value, cfg["net"]["gamma"], cfg["net"]["lambda"])
    a.ret[:] = ret; a.adv[:] = adv
    a.loss_and_grad()
    g_full = a.grad.copy().astype(np.float64); loss_full = a.loss.copy()
    b.learn_n(2)
    g2 = b.grad.copy().astype(np.float64)
    g1 = 2.0 * g_full - g2
    assert np.abs(b.loss - loss_full).max() <= 1e-7 * max(1.0, np.abs(loss_full).max())
    lr, b1, b2, eps = cfg["net"]["lr"], cfg["net"]["beta1"], cfg["net"]["beta2"], cfg["net"]["eps"]
    th, m, v = theta0.copy(), m0.copy(), v0.copy()
    for k, g in enumerate((g1, g2)):
        t = t0 + k + 1
        m = b1 * m + (1 - b1) * g; v = b2 * v + (1 - b2) * g * g
        th = th - lr * (m / (1 - b1 ** t)) / (np.sqrt(v / (1 - b2 ** t)) + eps)
    assert b.adam_t == t0 + 2
    # g1 is known only through float32 gradients: a few 1e-7 relative on the step, far below one step (3e-4)
    assert np.abs(b.theta - th).max() <= 2e-6, np.abs(b.theta - th).max()
    assert np.abs(b.m - m).max() <= 1e-6 * max(1.0, np.abs(m).max()) and np.abs(b.v - v).max() <= 1e-6 * max(1e-3, np.abs(v).max())
    with pytest.raises(RuntimeError):
        b.rollout(); b.learn_n(3)               # 8 steps do not split into 3 chunks


@pytest.mark.parametrize("kind", ["catch", "pendulum"])
def test_n_updates_sequential_is_two_hand_applied_steps(orc, kind):
    """The sequential reading of several updates per unroll: chunk 1's gradient is the gradient of chunk 1's mean loss
    at the parameters AFTER the first update, with returns, advantages, actions and pre-squash samples of the stored
    unroll.  Rebuilt here from single calls: range gradient, Adam in numpy, parameters written back, range gradient."""
    cfg = tiny(kind, hidden=(6, 5), B=4, T=8, max_steps=5)
    cfg["net"]["lr"] = 1e-2                                   # one step moves the parameters visibly
    a = orc.Oracle(cfg, seed=9); b = orc.Oracle(cfg, seed=9)
    rng = np.random.default_rng(4)
    noise = rng.standard_normal(a.P).astype(np.float32) * 0.2
    a.theta[:] += noise; b.theta[:] += noise
    a.rollout(); b.rollout()
    f32 = lambda x: float(np.float32(x))
    net = cfg["net"]
    ret, adv = orc.returns(a.tr_reward, a.tr_done, a.tr_value, f32(net["gamma"]), f32(net["lambda"]))
    a.ret[:] = ret; a.adv[:] = adv
    n = a.T * a.B
    th = a.theta.astype(np.float64).copy(); m = np.zeros(a.P); v = np.zeros(a.P)
    lr, b1, b2, eps = (f32(net[k]) for k in ("lr", "beta1", "beta2", "eps"))
    grads = []
    for k in range(2):
        a.loss_and_grad(k * n // 2, (k + 1) * n // 2)         # at a.theta as it is now
        g = a.grad.astype(np.float64).copy(); grads.append(g)
        t = k + 1
        m = b1 * m + (1 - b1) * g; v = b2 * v + (1 - b2) * g * g
        th = th - lr * (m / (1 - b1 ** t)) / (np.sqrt(v / (1 - b2 ** t)) + eps)
        a.theta[:] = th.astype(np.float32); th = a.theta.astype(np.float64)      # parameters are binary32 between steps
    b.learn_n(2, sequential=True)
    assert b.adam_t == 2
    assert np.abs(b.theta.astype(np.float64) - th).max() <= 1e-6
    assert np.array_equal(b.grad, grads[1].astype(np.float32))
    # and it is not the acting-time reading: the second chunk's gradient moved with the parameters
    c = orc.Oracle(cfg, seed=9); c.theta[:] += noise; c.rollout(); c.learn_n(2)
    assert np.linalg.norm(c.grad.astype(np.float64) - grads[1]) > 1e-4 * np.linalg.norm(grads[1])
    assert np.abs(c.theta - b.theta).max() > 1e-5


# --------------------------------------------------------------------------- off-policy update, decoupled step
def test_maze_random_walk_against_the_rule(orc):
    """R-14 / R-15 written out by the test on its own copy of the wall bits: a move into a wall or off the grid
    leaves the agent where it is, any other move takes it there; the agent is never on a wall."""
    o = orc.Oracle(tiny("maze", hidden=(8,), B=6, T=2, max_steps=10 ** 6), seed=21)
    rng = np.random.default_rng(9)
    step = {0: (-1, 0), 1: (0, 1), 2: (1, 0), 3: (0, -1)}
    blocked = moved = 0
    for b in range(6):
        w = _walls(o, b)
        r_, c_ = 0, 0
        for i in range(600):
            a = int(rng.integers(4))
            nr, nc = r_ + step[a][0], c_ + step[a][1]
            ok = 0 <= nr < 16 and 0 <= nc < 16 and not w[nr, nc]
            blocked += (0 <= nr < 16 and 0 <= nc < 16 and bool(w[nr, nc])); moved += ok
            if ok:
                r_, c_ = nr, nc
            r, done = o.env_step(b, action=a, t=i)
            if (r_, c_) == (15, 15):
                assert done == 1 and r == 1.0 and o.state_i[b, 0] == 0
                r_, c_ = 0, 0
            else:
                assert done == 0 and o.state_i[b, 0] == r_ * 16 + c_ and not w[r_, c_]
    assert blocked > 100 and moved > 1000                  # walls were hit, and not every move was blocked


@pytest.mark.parametrize("kind", ["catch", "pendulum"])
def test_unroll_draws_follow_the_counter_layout(orc, kind):
    """R-1 / R-21 / R-22: the action of env b at global step g comes from words 0 (and 1) of the draw
    (index b, t = g, domain 0), the state after an episode end from the draw (b, g, domain 1); the test makes the
    draws itself through the Philox routine pinned above and replays sampling and reset from the stored head outputs."""
    cfg = tiny(kind, hidden=(6, 6), B=5, T=9, max_steps=4)
    seed = 77
    o = orc.Oracle(cfg, seed=seed)
    L = orc.lib()
    o.rollout()                                            # second unroll below: global step numbers 9..17
    g0 = o.global_step
    o.rollout()
    ends = 0
    for t in range(o.T):
        for b in range(o.B):
            wa, wr = orc.draw(seed, b, g0 + t, 0), orc.draw(seed, b, g0 + t, 1)
            head = o.tr_head[t, b]
            if kind == "catch":
                assert o.tr_action[t, b] == orc.sample_categorical(head[:3], L.orc_u01(int(wa[0])))
                if o.tr_done[t, b]:
                    ends += 1
                    assert tuple(o.tr_state_i[t + 1, b, :3]) == (int(L.orc_bounded(int(wr[0]), 3)), 0, 1)
            else:
                e, z, a = orc.sample_gaussian(head[0], head[1], wa[0], wa[1])
                assert (o.tr_eps[t, b], o.tr_z[t, b], o.tr_action_f[t, b]) == (e, z, a)
                if o.tr_done[t, b]:
                    ends += 1
                    th = np.float32(-math.pi) + np.float32(2 * math.pi) * np.float32(L.orc_u01(int(wr[0])))
                    thd = -1.0 + 2.0 * L.orc_u01(int(wr[1]))
                    assert abs(float(o.tr_state_f[t + 1, b, 0]) - float(th)) < 1e-6 and o.tr_state_f[t + 1, b, 1] == np.float32(thd)
    assert ends >= o.B


def _np_log_prob(head, kind, act, z):
    """log-probability of the stored action under head outputs [..., NH] (binary64, written out here)."""
    head = np.asarray(head, np.float64)
    if kind == "pendulum":
        mu, ls = head[..., 0], np.clip(head[..., 1], -5.0, 2.0)
        return -0.5 * ((z - mu) / np.exp(ls)) ** 2 - ls - 0.5 * math.log(2 * math.pi)
    lg = head[..., :-1]
    lse = np.log(np.exp(lg - lg.max(-1, keepdims=True)).sum(-1)) + lg.max(-1)
    return np.take_along_axis(lg, act[..., None], -1)[..., 0] - lse


@pytest.mark.parametrize("kind", ["catch", "pendulum", "pendulum-clamped"])
def test_vtrace_targets_vs_definition(orc, kind):
    """The backward recursion against V-trace written as its defining sum (Espeholt et al. 2018, eq. 1):
    v_s = V(x_s) + sum_{t>=s} (prod_{i=s}^{t-1} disc_i c_i) delta_t, delta_t = rho_t (r_t + disc_t V(x_{t+1}) - V(x_t)),
    with truncation levels below and above the ratios that occur, plus the advantage rho_s (r_s + disc_s v_{s+1} - V(x_s))."""
    clamped = kind == "pendulum-clamped"          # log_sigma above its clamp (R-19) in most samples, inside in a few
    kind = kind.split("-")[0]
    cfg = tiny(kind, hidden=(8, 8), B=6, T=12, lam=0.9, max_steps=7)
    o = orc.Oracle(cfg, seed=3)
    if clamped:
        o.theta[-2] = 3.0
    for _ in range(2):
        o.rollout()
    rng = np.random.default_rng(0)
    o.theta[:] = o.theta + rng.normal(0, 0.08, o.P).astype(np.float32)      # the learner has moved on
    if clamped:
        assert (o.tr_head[..., 1] > 2.1).mean() > 0.5 and (o.tr_head[..., 1] < 1.9).any()
    rho_bar, c_bar = 1.05, 0.9
    o.vtrace_targets(rho_bar, c_bar)
    T, B = o.T, o.B
    gamma, lam = float(np.float32(cfg["net"]["gamma"])), float(np.float32(cfg["net"]["lambda"]))   # stored as binary32
    # the learner's heads are the network's: float32 canonical forward of the same states, a few samples
    for (t, b) in [(0, 0), (5, 3), (T, B - 1)]:
        si, sf = o.tr_state_i[t, b].copy(), o.tr_state_f[t, b].copy()
        keep_i, keep_f = o.state_i[b].copy(), o.state_f[b].copy()
        o.state_i[b] = si; o.state_f[b] = sf
        h32 = o.forward(o.observe(b))
        o.state_i[b] = keep_i; o.state_f[b] = keep_f
        assert np.abs(o.cur_head[t, b] - h32).max() <= 1e-5 * max(1.0, np.abs(h32).max())
    V = o.cur_head[..., -1]
    w = np.exp(_np_log_prob(o.cur_head[:T], kind, o.tr_action, o.tr_z) - _np_log_prob(o.tr_head[:T], kind, o.tr_action, o.tr_z))
    if not clamped:
        assert (w > rho_bar).any() and (w < c_bar).any() and ((w > c_bar) & (w < rho_bar)).any()   # every branch of both min()
    else:
        assert (o.cur_head[..., 1] > 2.1).mean() > 0.5 and np.abs(w - 1).max() > 1e-3
    rho = np.minimum(rho_bar, w); c = lam * np.minimum(c_bar, w)
    assert np.allclose(o.rho, rho, rtol=1e-12, atol=0)
    disc = gamma * (1.0 - o.tr_done.astype(np.float64))
    assert o.tr_done.sum() > 0
    delta = rho * (o.tr_reward + disc * V[1:] - V[:-1])
    vs = np.zeros((T + 1, B)); vs[T] = V[T]
    for s_ in range(T):
        acc = np.zeros(B); coef = np.ones(B)
        for t in range(s_, T):
            acc += coef * delta[t]
            coef = coef * disc[t] * c[t]
        vs[s_] = V[s_] + acc
    adv = rho * (o.tr_reward + disc * vs[1:] - V[:-1])
    assert np.abs(o.ret - vs[:T]).max() <= 1e-12 * max(1.0, np.abs(vs).max())
    assert np.abs(o.adv - adv).max() <= 1e-12 * max(1.0, np.abs(adv).max())


@pytest.mark.parametrize("kind", ["catch", "pendulum"])
def test_vtrace_on_policy_is_the_a2c_update(orc, kind):
    """With the acting-time parameters (ratios 1 up to the float32/binary64 forward difference) and lambda = 1,
    the off-policy update is the on-policy one: same targets, same gradient, same step."""
    cfg = tiny(kind, hidden=(8, 8), B=8, T=10, lam=1.0, max_steps=6)
    a = orc.Oracle(cfg, seed=9); b = orc.Oracle(cfg, seed=9)
    for _ in range(2):
        a.rollout(); a.learn(); b.rollout(); b.learn_vtrace(1.0, 1.0)
        assert np.abs(a.ret - b.ret).max() <= 1e-5 * max(1.0, np.abs(a.ret).max())
        assert np.abs(a.adv - b.adv).max() <= 1e-5 * max(1.0, np.abs(a.adv).max())
        assert np.abs(a.grad - b.grad).max() <= 1e-5 * max(1e-3, np.abs(a.grad).max())
        assert np.abs(a.loss - b.loss).max() <= 1e-5 * max(1.0, np.abs(a.loss).max())
        # Adam normalises the step: near-zero gradient entries may move by a fraction of lr either way
        assert np.abs(a.theta - b.theta).max() <= 0.02 * cfg["net"]["lr"]
        b.theta[:] = a.theta; b.m[:] = a.m; b.v[:] = a.v
    assert a.adam_t == b.adam_t == 2


def test_decoupled_step_semantics(orc):
    """The first decoupled step only collects; from then on the learner is one unroll behind the actor, and the
    actor's parameters are those from before the update that runs beside it."""
    cfg = tiny("catch", hidden=(8, 8), B=8, T=6, lam=1.0)
    a = orc.Oracle(cfg, seed=4); ref = orc.Oracle(cfg, seed=4)
    theta0 = a.theta.copy()
    a.step_decoupled()
    ref.rollout()
    assert np.array_equal(a.theta, theta0) and a.adam_t == 0
    assert np.array_equal(a.tr_action, ref.tr_action) and np.array_equal(a.tr_head, ref.tr_head)
    # second step: update on unroll 0 (on-policy at theta0), unroll 1 acted with theta0
    a.step_decoupled()
    ref.learn_vtrace()
    theta1 = a.theta.copy()
    assert a.adam_t == 1 and np.array_equal(a.theta, ref.theta)
    ref_theta1 = ref.theta.copy()
    ref.theta[:] = theta0
    ref.rollout()
    assert np.array_equal(a.tr_action, ref.tr_action) and np.array_equal(a.tr_head, ref.tr_head)
    assert a.global_step == 2 * cfg["T"]
    # third step: off-policy update (behaviour theta0, learner theta1), unroll 2 acted with theta1
    ref.theta[:] = ref_theta1
    a.step_decoupled()
    ref.learn_vtrace()
    assert a.adam_t == 2 and np.array_equal(a.theta, ref.theta)
    assert (a.rho < 1.0 - 1e-4).any()                       # the update really was off-policy
    theta2 = ref.theta.copy()
    ref.theta[:] = theta1
    ref.rollout()
    assert np.array_equal(a.tr_head, ref.tr_head) and np.array_equal(a.tr_state_i, ref.tr_state_i)
    ref.theta[:] = theta2
    ref.forward(ref.observe(0))
    assert not np.array_equal(theta1, theta2)


# --------------------------------------------------------------------------- pathwise gradient through the env
def _simulate_path_loss(o, theta, max_steps):
    """-mean reward of the unroll as a function of the parameters, written out in float64: same noise, same start
    states, same reset states after an episode end; the pendulum's step and the tanh-Gaussian policy in plain
    formulas."""
    Ws, bs, Wh, bh = _unpack(o, theta)
    T, B = o.T, o.B
    dt, c_thd, c_u = float(np.float32(0.05)), float(np.float32(0.1)), float(np.float32(0.001))
    th = o.tr_state_f[0, :, 0].astype(np.float64); thd = o.tr_state_f[0, :, 1].astype(np.float64)
    total = 0.0
    for t in range(T):
        x = np.stack([np.cos(th), np.sin(th), thd], 1)
        for Wm, bv in zip(Ws, bs):
            x = np.maximum(x @ Wm + bv, 0)
        head = x @ Wh + bh
        u = 2 * np.tanh(head[:, 0] + np.exp(np.clip(head[:, 1], -5, 2)) * o.tr_eps[t])
        total += -(th ** 2 + c_thd * thd ** 2 + c_u * u ** 2).sum()
        nthd = np.clip(thd + dt * (15 * np.sin(th) + 3 * u), -8, 8)
        nth = th + dt * nthd
        nth = np.where(nth >= math.pi, nth - 2 * math.pi, np.where(nth < -math.pi, nth + 2 * math.pi, nth))
        done = o.tr_done[t].astype(bool)
        th = np.where(done, o.tr_state_f[t + 1, :, 0], nth); thd = np.where(done, o.tr_state_f[t + 1, :, 1], nthd)
    return -total / (T * B)


def test_pathwise_gradient_vs_finite_differences(orc):
    """Reverse accumulation through policy and dynamics against central differences of the re-simulated unroll
    (episode ends inside the unroll cut the adjoint; one env runs into the velocity clip)."""
    cfg = tiny("pendulum", hidden=(6, 5), B=5, T=9, max_steps=4)
    o = orc.Oracle(cfg, seed=21)
    rng = np.random.default_rng(5)
    o.theta[:] += rng.standard_normal(o.P).astype(np.float32) * 0.4
    o.state_f[0] = (2.0, 7.9)                       # fast enough to hit the clip at +-8 within the unroll
    o.rollout()
    assert o.tr_done.sum() >= 2 and (np.abs(o.tr_state_f[..., 1]) == 8.0).any()
    th0 = o.theta.astype(np.float64)
    # the re-simulation follows the stored unroll (binary32 states) to rounding
    assert abs(_simulate_path_loss(o, th0, 4) + o.tr_reward.astype(np.float64).mean()) < 1e-5
    g, ph = o.pathwise_grad()
    h = 1e-6
    fd = np.zeros(o.P)
    for i in range(o.P):
        tp, tm = th0.copy(), th0.copy()
        tp[i] += h; tm[i] -= h
        fd[i] = (_simulate_path_loss(o, tp, 4) - _simulate_path_loss(o, tm, 4)) / (2 * h)
    assert np.linalg.norm(fd) > 1e-3
    # the adjoint is linearised at the stored binary32 states, the differences re-simulate in float64
    assert np.linalg.norm(g - fd) / np.linalg.norm(fd) < 2e-5, np.linalg.norm(g - fd) / np.linalg.norm(fd)
    # a one-step unroll has no dynamics in it: d(-r)/du = 0.002 u through u = 2 tanh(z)
    cfg1 = tiny("pendulum", hidden=(6, 5), B=4, T=1)
    o1 = orc.Oracle(cfg1, seed=2)
    o1.rollout()
    _, ph1 = o1.pathwise_grad()
    a = o1.tr_action_f[0].astype(np.float64)
    sigma = np.exp(np.clip(o1.tr_head[0, :, 1].astype(np.float64), -5, 2))
    gz = (2 * float(np.float32(0.001)) * 2 * a) * 2 * (1 - a * a) / 4
    assert np.allclose(ph1[0, :, 0], gz, rtol=1e-5, atol=1e-12)
    assert np.allclose(ph1[0, :, 1], gz * sigma * o1.tr_eps[0], rtol=1e-5, atol=1e-12)


def test_pathwise_update_composition(orc):
    """learn_pathwise = value and entropy terms of the usual objective (no score-function term) plus the pathwise
    gradient, one Adam step; the reported policy loss is minus the mean reward.  Board envs are refused."""
    cfg = tiny("pendulum", hidden=(6, 5), B=6, T=8, max_steps=5)
    a = orc.Oracle(cfg, seed=8); b = orc.Oracle(cfg, seed=8)
    a.rollout(); b.rollout()
    ret, adv = orc.returns(b.tr_reward, b.tr_done, b.tr_value, float(np.float32(cfg["net"]["gamma"])),
                           float(np.float32(cfg["net"]["lambda"])))
    b.ret[:] = ret; b.adv[:] = 0.0
    b.loss_and_grad()
    gp, _ = b.pathwise_grad()
    g = b.grad.astype(np.float64) + gp
    a.learn_pathwise()
    assert np.abs(a.grad - g).max() <= 1e-6 * max(1.0, np.abs(g).max())
    assert abs(a.loss[1] + a.tr_reward.astype(np.float64).mean()) < 1e-12
    assert abs(a.loss[2] - b.loss[2]) < 1e-12 and abs(a.loss[3] - b.loss[3]) < 1e-12
    th = b.theta.astype(np.float64); m = np.zeros(b.P); v = np.zeros(b.P)
    lr, b1, b2, eps = (cfg["net"][k] for k in ("lr", "beta1", "beta2", "eps"))
    gf = a.grad.astype(np.float64)
    m = (1 - b1) * gf; v = (1 - b2) * gf * gf
    th = th - lr * (m / (1 - b1)) / (np.sqrt(v / (1 - b2)) + eps)
    assert np.abs(a.theta - th).max() <= 2e-7 and a.adam_t == 1
    c = orc.Oracle(tiny("catch"), seed=0)
    c.rollout()
    with pytest.raises(RuntimeError):
        c.learn_pathwise()


def test_catch_learning_sanity(orc):
    # not a parity criterion: the mean episode return should rise from about -0.6
    cfg = W.get("catch_small", B=64, T=20)
    cfg["net"]["lr"] = 3e-3
    o = orc.Oracle(cfg, seed=0)
    first = last = 0.0
    for i in range(150):
        o.rollout()
        r = o.tr_reward.sum() / max(1, o.tr_done.sum())
        if i < 10: first += r / 10
        if i >= 140: last += r / 10
        o.learn()
    assert last > first + 0.3


# ------------------------------------------- bf16 nets: the learn-time forward pass and its gradient
def _bf(a):
    """binary32 -> bfloat16 -> binary64 through the library's cast (round to nearest even)"""
    import torch
    a32 = np.ascontiguousarray(np.asarray(a, np.float64).astype(np.float32))
    return torch.from_numpy(a32).to(torch.bfloat16).to(torch.float32).numpy().astype(np.float64)


def _obs_rows(o, kind, rows=4, cols=3, t_max=None):
    """observations rebuilt by the test from the stored states, [(t_max)*B][D] in binary64"""
    T1, B = (o.T + 1 if t_max is None else t_max), o.B
    obs = np.zeros((T1 * B, o.D))
    for t in range(T1):
        for b in range(B):
            si, sf = o.tr_state_i[t, b], o.tr_state_f[t, b]
            if kind == "catch":
                x = np.zeros((rows, cols)); x[si[1], si[0]] = 1; x[rows - 1, si[2]] = 1
            elif kind == "pendulum":
                x = np.array([math.cos(sf[0]), math.sin(sf[0]), sf[1]])
            else:
                n = rows * cols
                wb = np.unpackbits(o.walls[b].view(np.uint8), bitorder="little")[:n].astype(float)
                ag = np.zeros(n); ag[si[0]] = 1
                gl = np.zeros(n); gl[n - 1] = 1
                x = np.concatenate([wb, ag, gl])
            obs[t * B + b] = np.ravel(x)
    return obs


def _np_forward_bf16(o, theta, obs):
    """The bf16 forward pass with explicit casts at every rounding point: layer inputs (the observation
    included) and weight matrices rounded to bfloat16, sums in binary64, bias and ReLU, the result rounded to
    binary32 and then to bfloat16; the head outputs are left unrounded."""
    Ws, bs, Wh, bh = _unpack(o, np.asarray(theta, np.float64))
    h = _bf(obs)
    acts = []
    for Wm, bv in zip(Ws, bs):
        h = _bf(np.maximum(h @ _bf(Wm) + bv, 0))
        acts.append(h)
    return h @ _bf(Wh) + bh, acts


@pytest.mark.parametrize("kind", ["pendulum", "maze", "catch"])
def test_bf16_learn_forward_rounding_points(orc, kind):
    """The binary64 forward pass the bf16 update differentiates (weights, observation and hidden activations
    rounded to bfloat16, heads not) against (a) a numpy forward with the library's bfloat16 casts written out
    here and (b) the acting-time binary32 forward, which has its own pin."""
    cfg = tiny(kind, hidden=(16, 8), B=5, T=6, rows=4, cols=4 if kind == "maze" else 3, max_steps=4, p_wall=0.1, dtype="bf16")
    o = orc.Oracle(cfg, seed=21)
    rng = np.random.default_rng(8)
    o.theta[:] += rng.standard_normal(o.P).astype(np.float32) * 0.2      # biases off zero and off the bf16 grid
    assert not np.array_equal(_bf(o.theta), o.theta.astype(np.float64))
    o.rollout()
    o.vtrace_targets()                                                    # fills cur_head at the current parameters
    obs = _obs_rows(o, kind, rows=4, cols=4 if kind == "maze" else 3)
    if kind == "pendulum":
        assert not np.array_equal(_bf(obs), obs)                          # the observation itself needs rounding
    ref, _ = _np_forward_bf16(o, o.theta, obs)
    got = o.cur_head.reshape(-1, o.NH)
    # same rounding points, binary64 sums: equal up to the order of the sums, except where that order decides a
    # bfloat16 tie in a hidden activation (rare)
    close = np.isclose(got, ref, rtol=1e-9, atol=1e-12).all(1)
    assert close.mean() > 0.9 and np.allclose(got, ref, rtol=0, atol=2e-2 * np.abs(ref).max())
    # the acting-time forward differs only by binary32 accumulation
    act_head = o.tr_head.reshape(-1, o.NH).astype(np.float64)
    assert np.isclose(got, act_head, rtol=1e-4, atol=1e-5).all(1).mean() > 0.9
    assert np.allclose(got, act_head, rtol=0, atol=2e-2 * np.abs(ref).max())
    # and a forward without the rounding points is measurably different (the pin would see a dropped cast)
    Ws, bs, Wh, bh = _unpack(o, o.theta.astype(np.float64))
    for drop in ("weights", "heads", "obs", "acts"):
        h = obs if drop == "obs" else _bf(obs)
        for Wm, bv in zip(Ws, bs):
            z = np.maximum(h @ (Wm if drop == "weights" else _bf(Wm)) + bv, 0)
            h = z if drop == "acts" else _bf(z)
        alt = h @ (Wh if drop == "heads" else _bf(Wh)) + bh
        if drop == "obs" and kind != "pendulum":
            continue                                                      # 0/1 boards are bfloat16 values already
        assert np.isclose(got, alt, rtol=1e-9, atol=1e-12).all(1).mean() < 0.5, drop


def _np_surrogate_frozen(o, wvars, obs_q, deltas, kind):
    """The objective of a bf16 net as a smooth binary64 function of the *rounded* weights: every rounding of a
    hidden activation is replaced by the additive offset it had at the point of expansion."""
    Ws, bs, Wh, bh = _unpack(o, wvars)
    h = obs_q
    for Wm, bv, d in zip(Ws, bs, deltas):
        h = np.maximum(h @ Wm + bv, 0) + d
    head = h @ Wh + bh
    A, G = o.adv.reshape(-1), o.ret.reshape(-1)
    beta, cv = o.cfg["net"]["entropy_coef"], o.cfg["net"]["value_coef"]
    V = head[:, -1]
    if kind == "categorical":
        lg = head[:, :-1]
        lp = lg - lg.max(1, keepdims=True)
        lp = lp - np.log(np.exp(lp).sum(1, keepdims=True))
        H = -(np.exp(lp) * lp).sum(1)
        lpa = lp[np.arange(lp.shape[0]), o.tr_action.reshape(-1)]
    else:
        mu, ls = head[:, 0], np.clip(head[:, 1], -5, 2)
        z = o.tr_z.reshape(-1).astype(np.float64)
        lpa = -0.5 * ((z - mu) / np.exp(ls)) ** 2 - ls - 0.5 * math.log(2 * math.pi)
        H = ls + 0.5 * math.log(2 * math.pi * math.e)
    return (-A * lpa + cv * (G - V) ** 2 - beta * H).mean()


@pytest.mark.parametrize("kind", ["pendulum", "maze"])
def test_bf16_gradient_vs_finite_differences(orc, kind):
    """Gradient of a bf16 net (taken with respect to the rounded weights the forward pass uses and applied to the
    binary32 master weights) against central differences of a binary64 objective written here, with the rounded
    weights as the variables and every activation rounding frozen as an offset."""
    cfg = tiny(kind, hidden=(6, 5), B=3, T=5, rows=4, cols=4, max_steps=3, p_wall=0.1, dtype="bf16")
    o = orc.Oracle(cfg, seed=17)
    rng = np.random.default_rng(5)
    o.theta[:] += rng.standard_normal(o.P).astype(np.float32) * 0.3
    o.rollout()
    ret, adv = orc.returns(o.tr_reward, o.tr_done, o.tr_value, cfg["net"]["gamma"], cfg["net"]["lambda"])
    o.ret[:] = ret; o.adv[:] = adv + rng.standard_normal(adv.shape)
    o.loss_and_grad()
    obs_q = _bf(_obs_rows(o, kind, rows=4, cols=4, t_max=o.T))
    # point of expansion: weight matrices rounded, biases as they are
    Ws, bs, Wh, bh = _unpack(o, o.theta.astype(np.float64))
    w0 = np.concatenate([np.concatenate([_bf(Wm).ravel(), bv]) for Wm, bv in zip(Ws, bs)] + [_bf(Wh).ravel(), bh])
    assert w0.size == o.P and not np.array_equal(w0, o.theta.astype(np.float64))
    Wq, bq, _, _ = _unpack(o, w0)
    deltas, h = [], obs_q
    for Wm, bv in zip(Wq, bq):
        z = np.maximum(h @ Wm + bv, 0)
        h = _bf(z)
        deltas.append(h - z)
    assert max(np.abs(d).max() for d in deltas) > 0                       # some activation really was rounded
    pol = "categorical" if kind != "pendulum" else "gauss"
    assert abs(_np_surrogate_frozen(o, w0, obs_q, deltas, pol) - o.loss[0]) < 1e-9 * max(1.0, abs(o.loss[0]))
    hstep = 1e-5
    fd = np.zeros(o.P)
    for i in range(o.P):
        tp, tm = w0.copy(), w0.copy()
        tp[i] += hstep; tm[i] -= hstep
        fd[i] = (_np_surrogate_frozen(o, tp, obs_q, deltas, pol) - _np_surrogate_frozen(o, tm, obs_q, deltas, pol)) / (2 * hstep)
    g = o.grad.astype(np.float64)
    assert np.linalg.norm(g) > 1e-3
    assert np.linalg.norm(g - fd) / np.linalg.norm(fd) < 1e-5
    assert np.abs(g - fd).max() < 1e-5 * np.abs(fd).max() + 1e-7
    # the same differences taken at the unrounded weights, or without the frozen offsets, do not reproduce it
    th = o.theta.astype(np.float64)
    zero = [np.zeros_like(d) for d in deltas]
    alt = np.zeros(o.P)
    for i in range(o.P):
        tp, tm = th.copy(), th.copy()
        tp[i] += hstep; tm[i] -= hstep
        alt[i] = (_np_surrogate_frozen(o, tp, obs_q, zero, pol) - _np_surrogate_frozen(o, tm, obs_q, zero, pol)) / (2 * hstep)
    assert np.linalg.norm(g - alt) / np.linalg.norm(alt) > 1e-4


def test_relu_side_is_taken_from_the_binary32_forward(orc):
    """A pre-activation within rounding of zero: the update differentiates the pass that acted, which ran in
    binary32, so its ReLU side is the binary32 one even where the binary64 sum lands on the other side.  Two
    hand-built units on the pendulum observation (1, 0, theta_dot) at theta = 0:
      unit 0: 1 - 2^-26 - (1 - 2^-26): binary32 rounds the first sum to 1 and ends at +2^-26 (on), binary64 at 0
      unit 1: 1 + 2^-25 - 1:           binary32 rounds the first sum to 1 and ends at 0 (off),     binary64 at +2^-25
    """
    cfg = tiny("pendulum", hidden=(2,), B=2, T=1)
    o = orc.Oracle(cfg, seed=1)
    rng = np.random.default_rng(2)
    o.theta[:] = rng.standard_normal(o.P).astype(np.float32) * 0.3
    Ws, bs, Wh, bh = _unpack(o)                      # views into o.theta
    Ws[0][:, 0] = (-2.0 ** -26, 0.0, -8193.0 / 8192.0); bs[0][0] = 1.0
    Ws[0][:, 1] = (2.0 ** -25, 0.0, -1.0); bs[0][1] = 1.0
    # unit 0 is probed at theta_dot = 8191/8192 (env 0), unit 1 at theta_dot = 1 (env 1)
    o.state_f[:] = [[0.0, 8191.0 / 8192.0], [0.0, 1.0]]
    o.state_i[:] = 0
    x0, x1 = o.observe(0), o.observe(1)
    assert np.array_equal(x0, np.array([1.0, 0.0, 8191.0 / 8192.0], np.float32)) and np.array_equal(x1, np.array([1.0, 0.0, 1.0], np.float32))
    _, a0 = o.forward(x0, want_acts=True); _, a1 = o.forward(x1, want_acts=True)
    assert a0[0] == np.float32(2.0 ** -26) and a1[1] == 0.0                     # binary32 sides: on, off
    z64 = lambda x, j: float(bs[0][j]) + sum(float(x[k]) * float(Ws[0][k, j]) for k in range(3))
    assert z64(x0, 0) == 0.0 and z64(x1, 1) == 2.0 ** -25                       # binary64 sides: off, on
    o.rollout()
    o.ret[:] = rng.standard_normal(o.ret.shape); o.adv[:] = rng.standard_normal(o.adv.shape)
    # per-sample head gradients from single-sample calls: dhead = gradient of the head bias
    regions, _ = __import__("parity").param_regions(cfg)
    R = dict(regions)
    grads = []
    for b in range(2):
        o.loss_and_grad(b, b + 1)
        grads.append(o.grad.astype(np.float64).copy())
    for b, unit, expect_on in ((0, 0, True), (1, 1, False)):
        g = grads[b]
        dhead = g[R["bh"]]
        assert np.abs(dhead).max() > 1e-3
        want = float(Wh[unit].astype(np.float64) @ dhead) if expect_on else 0.0
        got = g[R["b1"]][unit]
        assert abs(got - want) <= 1e-6 * max(abs(want), 1e-3), (b, unit, got, want)
        assert (got != 0.0) == expect_on
