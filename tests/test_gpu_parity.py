"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on
the same seeded workloads.  Env transitions, RNG draws, actions, rewards and
(on the canonical acting path) head outputs must match bit for bit; returns,
loss, gradients, parameters and Adam moments within 1e-4 (fp32) / 2e-2 (bf16),
per tensor in the l2 norm (spec tolerances)."""
import copy
import sys

import numpy as np
import pytest

from paper_2104_06272_amd import workloads as W
import parity as PT

pytestmark = pytest.mark.gpu

TOL_F32 = 1e-4
TOL_BF16 = 2e-2


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def gpu():
    from paper_2104_06272_amd import binding
    binding.load()
    return binding


def variant(name, hidden=None, B=None, T=None, **env_over):
    cfg = W.get(name, B=B, T=T)
    if hidden is not None:
        cfg["net"]["hidden"] = list(hidden)
    dtype = env_over.pop("dtype", None)
    if dtype:
        cfg["net"]["dtype"] = dtype
    cfg["env"] = dict(cfg["env"], **env_over)
    return cfg


LOCKSTEP_CASES = {
    # name: (cfg, seed, updates, tolerance)
    "catch_small": (variant("catch_small"), 0, 4, TOL_F32),
    "catch_256x256_B256": (variant("catch_4096", B=256), 1, 2, TOL_F32),
    "catch_ragged_B80_T7": (variant("catch_small", B=80, T=7), 2, 3, TOL_F32),
    "catch_tiny_net_B512": (variant("catch_262144", B=512), 0, 3, TOL_F32),
    "pendulum_B128": (variant("pendulum_8192", B=128), 0, 2, TOL_F32),
    "pendulum_short_episodes": (variant("pendulum_8192", hidden=[64, 64], B=64, T=32, max_steps=25), 2, 3, TOL_F32),
    "maze_fp32_small": (variant("maze_16384", hidden=[64, 64], B=64, T=32, dtype="fp32", max_steps=20), 1, 3, TOL_F32),
    "maze_bf16_canonical": (variant("maze_16384", hidden=[64, 64, 32], B=64, T=16, max_steps=40), 3, 2, TOL_BF16),
    "maze_fp32_8x8": (variant("maze_16384", hidden=[32], B=32, T=24, dtype="fp32", rows=8, cols=8, max_steps=30), 0, 2, TOL_F32),
    # 512 -> 256: the weights-resident dX kernel with two column blocks, tiled dW; three 256-wide layers: resident both ways
    "catch_512x256": (variant("catch_4096", hidden=[512, 256], B=64, T=10), 3, 2, TOL_F32),
    "catch_256x256x256": (variant("catch_4096", hidden=[256, 256, 256], B=96, T=9), 4, 2, TOL_F32),
    # 512-wide last layer: two column blocks in the head pass; 512-wide first layer of the pendulum kernel
    "catch_256x512": (variant("catch_4096", hidden=[256, 512], B=64, T=10), 5, 2, TOL_F32),
    "pendulum_512x256": (variant("pendulum_8192", hidden=[512, 256], B=64, T=12, max_steps=9), 6, 2, TOL_F32),
    # pendulum first layer summed inside the dX product of a middle layer, two 32-sample stages per workgroup;
    # and a sample count (272 tiles of 32) that 256 dX workgroups do not cut evenly, which keeps the separate kernel
    "pendulum_256x256x256_B512": (variant("pendulum_8192", hidden=[256, 256, 256], B=512, T=32), 11, 1, TOL_F32),
    "pendulum_256x256_B272": (variant("pendulum_8192", B=272, T=32), 12, 1, TOL_F32),
    # 143 = 11 x 13 stages of 32 samples: no chunk count near the number of compute units divides them, so the
    # 256 -> 256 layer's dW product stays with the tiled kernel while its dX product is the resident one
    "catch_256x256_B208_T22": (variant("catch_4096", B=208, T=22), 13, 1, TOL_F32),
    # degenerate shapes: a one-step unroll (the return is reward + bootstrap only), a single tile of envs,
    # an episode end at every step (max_steps = 1: every transition is terminal, nothing bootstraps)
    "catch_T1": (variant("catch_small", B=64, T=1), 7, 3, TOL_F32),
    "pendulum_T1_B16": (variant("pendulum_8192", hidden=[64, 64], B=16, T=1), 8, 2, TOL_F32),
    "pendulum_every_step_terminal": (variant("pendulum_8192", hidden=[64, 64], B=32, T=6, max_steps=1), 9, 2, TOL_F32),
    "maze_fp32_one_step_episodes": (variant("maze_16384", hidden=[64, 64], B=32, T=5, dtype="fp32", max_steps=1), 10, 2, TOL_F32),
}


@pytest.mark.parametrize("case", list(LOCKSTEP_CASES))
def test_lockstep(gpu, orc, case):
    """Parameter-synchronised lockstep: before every update the oracle takes the GPU's parameters;
    both roll out (bitwise equal), both learn (tolerance)."""
    cfg, seed, updates, tol = LOCKSTEP_CASES[case]
    kind = cfg["env"]["kind"]
    say(f"[lockstep] {case} seed={seed} B={cfg['B']} T={cfg['T']} hidden={cfg['net']['hidden']}")
    g = gpu.Anakin(cfg, seed=seed)
    o = orc.Oracle(cfg, seed=seed)
    PT.assert_same_init(g, o, kind)
    for u in range(updates):
        PT.sync_oracle_from_gpu(g, o)
        g.rollout(); o.rollout()
        tr = PT.assert_rollout_equal(g, o, kind)
        PT.assert_final_state_equal(g, o, kind)
        # hidden activations kept for the update equal the oracle's forward on the same states
        for (t, b) in ((0, 0), (g.T - 1, g.B - 1), (g.T // 2, g.B // 3)):
            head, acts = PT.oracle_forward_at(o, t, b)
            if tr["act"]:                 # one-layer nets keep no activations: the update rebuilds the layer
                got = np.concatenate([a[t, b] for a in tr["act"]])
                assert np.array_equal(got, acts), "stored activations differ"
        g.learn(); o.learn()
        e_g, e_p = PT.assert_learn_close(g, o, tol)
        say(f"  update {u}: grad rel {e_g:.2e}, param rel {e_p:.2e}, loss {o.loss[0]:+.5f}")
    g.close()


@pytest.mark.parametrize("hidden,B", [([64, 64], 64), ([256, 256], 128)])
@pytest.mark.parametrize("shift", [3.5, -7.5, 1.97])
def test_pendulum_log_sigma_at_and_outside_its_clamp(gpu, orc, hidden, B, shift):
    """log_sigma is clamped to [-5, 2] in the sampler, and a clamped log_sigma passes no gradient (neither from the
    score function nor from the entropy bonus).  With the head's bias pushed above or below the clamp every sample
    is clamped; with the bias just under the upper end some are and some are not.  Unrolls bit-exact, updates within
    tolerance, on the vector-ALU head pass (64-wide net) and on the head pass folded into the resident products
    (256-wide net)."""
    cfg = variant("pendulum_8192", hidden=hidden, B=B, T=16, max_steps=11)
    say(f"[log_sigma clamp] hidden={hidden} B={B} bias={shift}")
    g = gpu.Anakin(cfg, seed=31); o = orc.Oracle(cfg, seed=31)
    theta = g.get_params()
    theta[-2] = shift                              # heads: mu, log_sigma, value; their biases are the last three entries
    g.set_params(theta)
    for u in range(2):
        PT.sync_oracle_from_gpu(g, o)
        g.rollout(); o.rollout()
        tr = PT.assert_rollout_equal(g, o, "pendulum")
        ls = tr["head"][:-1, :, 1]
        if shift > 2.5:
            assert (ls > 2.0).all()
        elif shift < -5.5:
            assert (ls < -5.0).all()
        else:
            assert (ls > 2.0).any() and (ls < 2.0).any()
        g.learn(); o.learn()
        e_g, e_p = PT.assert_learn_close(g, o, TOL_F32)
        if abs(shift) > 2.5:
            nh, hl = 3, hidden[-1]
            wh = g.get_grads()[-(nh + hl * nh):-nh].reshape(hl, nh)
            assert np.abs(wh[:, 1]).max() == 0.0 and g.get_grads()[-2] == 0.0, "a clamped log_sigma passed a gradient"
        say(f"  update {u}: grad rel {e_g:.2e}, param rel {e_p:.2e}")
    g.close()


def test_pendulum_states_on_the_wrap_boundary(gpu, orc):
    """The stored angle lies in [-pi_f, pi_f): the env step wraps an angle of exactly pi_f (binary32 pi) and leaves
    the value just below it alone.  8192 envs start one binary32 step apart around the angle from which a step
    with velocity 1 and (nearly) no torque lands on pi_f; the policy's noise (sigma = e^-5) spreads the landing points
    over a few hundred steps, so several envs land exactly on pi_f, several just below and just above.  One step,
    every env bit-exact against the oracle."""
    cfg = variant("pendulum_8192", hidden=[64, 64], B=8192, T=1)
    say("[wrap boundary] pendulum B=8192 T=1")
    g = gpu.Anakin(cfg, seed=5); o = orc.Oracle(cfg, seed=5)
    theta = np.zeros(g.P, np.float32)
    theta[-2] = -7.5                                  # log_sigma below its clamp: sigma = e^-5; mu = 0, value = 0
    g.set_params(theta); o.theta[:] = theta
    pi_f = np.float32(np.pi)
    # the starting angle whose torque-free step lands nearest pi_f, found with the oracle's own env step (pinned on the CPU)
    lo, hi = int(np.float32(3.0).view(np.uint32)), int(np.float32(3.14).view(np.uint32))

    def lands_past(bits):
        o.state_i[0, 0] = 0; o.state_f[0] = (np.uint32(bits).view(np.float32), 1.0)
        o.env_step(0, action_f=0.0, t=0)
        return o.state_f[0, 0] < 0
    while hi - lo > 1:
        mid = (lo + hi) // 2
        lo, hi = (lo, mid) if lands_past(mid) else (mid, hi)
    si = np.zeros((g.B, 4), np.int32)
    sf = np.empty((g.B, 2), np.float32)
    sf[:, 0] = (np.uint32(hi) + (np.arange(g.B, dtype=np.int64) % 1024 - 512).astype(np.int64)).astype(np.uint32).view(np.float32)
    sf[:, 1] = 1.0
    g.set_env_state(si, sf); o.state_i[:] = si; o.state_f[:] = sf
    g.rollout(); o.rollout()
    PT.assert_rollout_equal(g, o, "pendulum")
    PT.assert_final_state_equal(g, o, "pendulum")
    th = o.state_f[:, 0]
    wrapped_pi = np.float32(np.float32(pi_f - np.float32(2) * pi_f) - np.float32(float.fromhex("-0x1.777a5cp-23")))
    assert (th >= -pi_f).all() and (th < pi_f).all()
    assert (th == np.nextafter(pi_f, np.float32(0))).sum() >= 1, "no env landed just below pi_f"
    assert (th == wrapped_pi).sum() >= 1, "no env landed exactly on pi_f"
    say(f"  {int((th == wrapped_pi).sum())} envs landed on pi_f, {int((th == np.nextafter(pi_f, np.float32(0))).sum())} just below")
    g.close()


def test_pendulum_velocity_clip_and_large_costs(gpu, orc):
    """Envs started at the edge of the state space: angular velocities at and next to the clip (+-8) with angles that
    push them further out, so the clip is active in most steps and the reward takes its largest magnitudes; two
    updates in lockstep."""
    cfg = variant("pendulum_8192", hidden=[64, 64], B=256, T=8)
    say("[velocity clip] pendulum B=256 T=8")
    g = gpu.Anakin(cfg, seed=9); o = orc.Oracle(cfg, seed=9)
    rng = np.random.default_rng(2)
    si = np.zeros((g.B, 4), np.int32)
    sf = np.empty((g.B, 2), np.float32)
    sign = np.where(np.arange(g.B) % 2 == 0, 1.0, -1.0).astype(np.float32)
    sf[:, 0] = sign * rng.uniform(0.2, 2.9, g.B).astype(np.float32)            # sin(theta) has the sign of the velocity
    sf[:, 1] = sign * rng.choice(np.float32([8.0, 7.999999, 7.9, 7.5]), g.B)
    g.set_env_state(si, sf); o.state_i[:] = si; o.state_f[:] = sf
    clipped = 0
    for u in range(2):
        PT.sync_oracle_from_gpu(g, o)
        g.rollout(); o.rollout()
        PT.assert_rollout_equal(g, o, "pendulum")
        PT.assert_final_state_equal(g, o, "pendulum")
        clipped += int((np.abs(o.tr_state_f[1:, :, 1]) == 8.0).sum())
        assert o.tr_reward.min() < -10.0
        g.learn(); o.learn()
        e_g, e_p = PT.assert_learn_close(g, o, TOL_F32)
        say(f"  update {u}: grad rel {e_g:.2e}, param rel {e_p:.2e}")
    assert clipped > g.B                                  # the clip was active in many steps
    g.close()


@pytest.mark.parametrize("dtype,hidden", [("fp32", [64, 64]), ("bf16", [64, 64, 32])])
def test_maze_goal_and_step_cap_inside_the_unroll(gpu, orc, dtype, hidden):
    """Envs placed next to the goal with 250 of their 256 steps used: within one unroll many reach the goal (+1,
    episode end, back to the start) and the rest run into the step cap; both kinds of episode end, the restart
    from the start cell and the step counter next to its limit, bit-exact, then the update."""
    cfg = variant("maze_16384", hidden=hidden, B=128, T=12, dtype=dtype)
    say(f"[maze goal and cap] {dtype} hidden={hidden}")
    g = gpu.Anakin(cfg, seed=4); o = orc.Oracle(cfg, seed=4)
    PT.assert_same_init(g, o, "maze")
    _place_next_to_goal(g, o)           # a free neighbour of the goal (it is reachable, so one of its two neighbours is free)
    PT.sync_oracle_from_gpu(g, o)
    g.rollout(); o.rollout()
    PT.assert_rollout_equal(g, o, "maze")
    PT.assert_final_state_equal(g, o, "maze")
    goals = int((o.tr_reward == 1.0).sum()); caps = int(o.tr_done.sum()) - goals
    assert goals >= 10 and caps >= 10, (goals, caps)
    g.learn(); o.learn()
    e_g, e_p = PT.assert_learn_close(g, o, TOL_F32 if dtype == "fp32" else TOL_BF16)
    say(f"  {goals} goals, {caps} step caps; grad rel {e_g:.2e}, param rel {e_p:.2e}")
    g.close()


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_seeded_shape_sweep(gpu, orc, seed):
    """A seeded sample of the shapes the library accepts -- one to four hidden layers of 32..1024 units in any order,
    batch sizes that are not powers of two, one-step unrolls, boards of other sizes -- each two updates in lockstep
    with the oracle.  Shapes without an acting tile (a 32-wide layer with B not a multiple of 32, a 1024-wide last
    layer) are refused at create with ANAKIN_E_BAD_CONFIG and counted; nothing else may be refused."""
    rng = np.random.default_rng(seed)
    base = {"catch": "catch_small", "pendulum": "pendulum_8192", "maze": "maze_16384"}
    ran = refused = 0
    for c in range(16):
        kind = ["catch", "pendulum", "maze"][c % 3]
        L = int(rng.integers(1, 5))
        widths = [int(rng.choice([32, 64, 128, 256, 512] if L > 2 else [32, 64, 128, 256, 512, 1024])) for _ in range(L)]
        B = int(rng.choice([16, 48, 112, 272]))
        T = int(rng.choice([1, 3, 6, 11]))
        over = {}
        if kind == "maze":
            r, co = [(4, 4), (8, 8), (16, 16), (5, 7)][int(rng.integers(4))]
            over = dict(rows=r, cols=co, max_steps=int(rng.integers(2, 12)))
        elif kind == "pendulum":
            over = dict(max_steps=int(rng.integers(2, 12)))
        else:
            r, co = [(10, 5), (4, 3), (6, 9)][int(rng.integers(3))]
            over = dict(rows=r, cols=co)
        cfg = variant(base[kind], hidden=widths, B=B, T=T, dtype="fp32", **over)
        s = int(rng.integers(1000))
        say(f"[shape sweep {seed}.{c}] {kind} {over} hidden={widths} B={B} T={T} seed={s}")
        try:
            g = gpu.Anakin(cfg, seed=s)
        except gpu.AnakinError as e:
            assert e.code == gpu.E_BAD_CONFIG and "no rollout tile" in str(e), str(e)
            assert (32 in widths and (B % 32 or 1024 in widths)) or widths[-1] == 1024, "refused without a reason this test knows"
            refused += 1
            continue
        o = orc.Oracle(cfg, seed=s)
        PT.assert_same_init(g, o, kind)
        for u in range(2):
            PT.sync_oracle_from_gpu(g, o)
            g.rollout(); o.rollout()
            PT.assert_rollout_equal(g, o, kind)
            PT.assert_final_state_equal(g, o, kind)
            g.learn(); o.learn()
            PT.assert_learn_close(g, o, TOL_F32)
        g.close()
        ran += 1
    say(f"  {ran} shapes in lockstep, {refused} refused at create")
    assert ran >= 8


def test_catch_small_100_updates_lockstep(gpu, orc):
    """The small Catch workload for its full 100 updates, parameter-synchronised."""
    cfg = W.get("catch_small")
    g = gpu.Anakin(cfg, seed=0); o = orc.Oracle(cfg, seed=0)
    worst = 0.0
    for u in range(cfg["updates"]):
        PT.sync_oracle_from_gpu(g, o)
        g.rollout(); o.rollout()
        PT.assert_rollout_equal(g, o, "catch")
        g.learn(); o.learn()
        e_g, e_p = PT.assert_learn_close(g, o, TOL_F32)
        worst = max(worst, e_g, e_p)
    say(f"[catch_small x100] worst rel error {worst:.2e}")
    g.close()


def test_catch_small_free_running(gpu, orc):
    """No re-synchronisation: trajectories stay bitwise equal until rounding in the parameters
    flips a sample; parameters must agree within tolerance for as long as they do."""
    cfg = W.get("catch_small")
    g = gpu.Anakin(cfg, seed=3); o = orc.Oracle(cfg, seed=3)
    diverged = None
    for u in range(cfg["updates"]):
        g.rollout(); o.rollout()
        tr = g.trajectory()
        if not (np.array_equal(tr["action"].astype(np.int32), o.tr_action) and np.array_equal(tr["reward"], o.tr_reward)):
            diverged = u
            break
        g.learn(); o.learn()
        assert PT.rel(g.get_params(), o.theta) <= TOL_F32
    say(f"[free running] first trajectory divergence: {diverged}")
    assert diverged is None or diverged >= 5
    g.close()


FULL_SIZE = {
    "catch_4096": 0, "pendulum_8192": 1, "catch_262144": 2,
    # the same launch shape (32 envs per workgroup) with episodes that end, twice per env, inside the two unrolls
    "pendulum_8192_short_episodes": 3,
}


@pytest.mark.parametrize("name", list(FULL_SIZE))
def test_full_size_rollout_sampled_envs(gpu, orc, name):
    """The full-size workloads in the launch shape the benchmark times: two unrolls with an update in
    between; the oracle replays a seeded sample of envs one by one (valid because every draw is keyed by
    (env, step) and envs are independent given the parameters)."""
    cfg = W.get(name.replace("_short_episodes", ""))
    if name.endswith("_short_episodes"):
        cfg["env"] = dict(cfg["env"], max_steps=25)
    seed = FULL_SIZE[name]
    kind = cfg["env"]["kind"]
    B = cfg["B"]
    rng = np.random.default_rng(seed)
    sel = np.unique(np.concatenate([[0, 1, 15, 16, 63, 64, 255, 256, B - 1, B - 16, B // 2],
                                    rng.integers(0, B, 13)])).astype(np.int32)
    say(f"[full size] {name} seed={seed} envs={sel.tolist()}")
    g = gpu.Anakin(cfg, seed=seed); o = orc.Oracle(cfg, seed=seed)
    PT.assert_same_init(g, o, kind)
    for u in range(2):
        PT.sync_oracle_from_gpu(g, o)
        g.rollout(); o.rollout(sel=sel)
        PT.assert_rollout_equal(g, o, kind, sel=sel)
        PT.assert_final_state_equal(g, o, kind, sel=sel)
        g.learn()
        m = g.metrics()
        assert m["nonfinite"] == 0
        say(f"  unroll {u}: loss {m['loss']:+.5f} reward_sum {m['reward_sum']:.1f} episodes {m['episodes']}")
        # properties that hold at any size
        tr = g.trajectory()
        if kind == "catch":
            assert np.all(np.isin(tr["reward"][tr["done"] == 1], (-1.0, 1.0))) and np.all(tr["reward"][tr["done"] == 0] == 0)
            by = (tr["state_s0"] >> 8) & 0xFF
            assert np.array_equal(tr["done"] == 1, by[:-1] == 8)
        else:
            assert np.all(np.abs(tr["state_f1"]) <= 8.0) and np.all(np.abs(tr["state_f0"]) <= np.float32(np.pi))
            assert np.all(tr["reward"] <= 0)
        ret_o, adv_o = orc.returns(tr["reward"], tr["done"], tr["value"], cfg["net"]["gamma"], cfg["net"]["lambda"])
        assert np.abs(tr["ret"] - ret_o).max() <= 1e-5 * max(1.0, np.abs(ret_o).max())
        assert np.abs(tr["adv"] - adv_o).max() <= 1e-5 * max(1.0, np.abs(ret_o).max())
    g.close()


@pytest.mark.parametrize("name,kw,forced", [
    ("catch_262144", dict(B=1 << 20), False),          # four times the tiny-net workload: a million envs
    ("catch_4096", dict(B=65536), False),              # sixteen times the headline batch
    ("maze_16384", dict(B=32768), True),               # twice the maze batch (bf16 matrix-core path)
])
def test_batches_larger_than_the_benchmark(gpu, orc, name, kw, forced):
    """Beyond the benchmark's sizes: two whole steps, a seeded sample of envs replayed by the oracle (bit-exact; the
    bf16 matrix-core path logit-forced), returns and advantages of every sample against the oracle's routine, and a
    finite update."""
    cfg = W.get(name, **kw)
    kind, B = cfg["env"]["kind"], cfg["B"]
    say(f"[large batch] {name} B={B} T={cfg['T']} workspace {gpu.workspace_bytes(cfg) / 2 ** 30:.1f} GiB")
    g = gpu.Anakin(cfg, seed=1); o = orc.Oracle(cfg, seed=1)
    rng = np.random.default_rng(1)
    sel = np.unique(np.concatenate([[0, 63, 64, B - 1, B - 64, B // 2], rng.integers(0, B, 10)])).astype(np.int32)
    for u in range(2):
        PT.sync_oracle_from_gpu(g, o)
        g.rollout()
        tr = g.trajectory()
        o.rollout(forced_head=tr["head"] if forced else None, sel=sel)
        PT.assert_rollout_equal(g, o, kind, sel=sel, forced=forced)
        PT.assert_final_state_equal(g, o, kind, sel=sel)
        g.learn()
        m = g.metrics()
        assert m["nonfinite"] == 0 and m["episodes"] == int(tr["done"].sum())
        tr2 = g.trajectory()
        ret_o, adv_o = orc.returns(tr["reward"], tr["done"], tr["value"], cfg["net"]["gamma"], cfg["net"]["lambda"])
        assert np.abs(tr2["ret"] - ret_o).max() <= 1e-5 * max(1.0, np.abs(ret_o).max())
        assert np.abs(tr2["adv"] - adv_o).max() <= 1e-5 * max(1.0, np.abs(ret_o).max())
        del tr, tr2
    g.close()


def test_full_size_headline_update(gpu, orc):
    """The headline workload (Catch, B=4096, T=20, MLP 50-256-256) at full size, one whole step in lockstep:
    every env of the unroll bit-exact, then loss, gradient, parameters and Adam moments of the update in the
    launch shape the benchmark times (one persistent workgroup per compute unit in the backward GEMMs).
    The oracle needs about ten seconds for this step."""
    cfg = W.get("catch_4096")
    say("[full size] catch_4096 whole step, all envs")
    g = gpu.Anakin(cfg, seed=7); o = orc.Oracle(cfg, seed=7)
    PT.assert_same_init(g, o, "catch")
    g.step()                                    # one free step first, so the compared update starts from non-initial parameters
    PT.sync_oracle_from_gpu(g, o)
    si, sf = g.get_env_state()
    o.state_i[:] = si
    o.global_step = g.global_step
    g.rollout(); o.rollout()
    PT.assert_rollout_equal(g, o, "catch")
    PT.assert_final_state_equal(g, o, "catch")
    g.learn(); o.learn()
    e_g, e_p = PT.assert_learn_close(g, o, TOL_F32)
    say(f"  gradient rel err {e_g:.2e}, parameter rel err {e_p:.2e}")
    g.close()


@pytest.mark.parametrize("name", ["catch_262144", "pendulum_8192"])
def test_full_size_whole_step(gpu, orc, name):
    """Two more workloads at their full size, one whole step in lockstep, in the launch shape the benchmark times:
    every env of the unroll bit-exact, then the update (the lane-per-env acting kernel and the one-layer update for
    the tiny net; the 32-env resident acting kernel, the pendulum's first-layer kernel and the head-folded products
    for the pendulum).  The oracle needs ten to thirty seconds for each."""
    cfg = W.get(name)
    kind = cfg["env"]["kind"]
    say(f"[full size] {name} whole step, all envs")
    g = gpu.Anakin(cfg, seed=11); o = orc.Oracle(cfg, seed=11)
    g.step()
    PT.sync_oracle_from_gpu(g, o)
    si, sf = g.get_env_state()
    o.state_i[:] = si; o.state_f[:] = sf
    o.global_step = g.global_step
    g.rollout()
    say("  unroll on the oracle ...")
    o.rollout()
    PT.assert_rollout_equal(g, o, kind)
    PT.assert_final_state_equal(g, o, kind)
    say("  update on the oracle ...")
    g.learn(); o.learn()
    e_g, e_p = PT.assert_learn_close(g, o, TOL_F32)
    say(f"  gradient rel err {e_g:.2e}, parameter rel err {e_p:.2e}")
    g.close()


# --------------------------------------------------------------------------- bf16 on the matrix cores
BF16_CASES = {
    "maze_bf16_128": (variant("maze_16384", hidden=[128, 128, 128], B=64, T=16, max_steps=40), 3, 2),
    "maze_bf16_256_512": (variant("maze_16384", hidden=[256, 512], B=128, T=8, rows=8, cols=8, max_steps=20), 1, 2),
    # 16x16 maze with 256-wide layers: 256 x 256 GEMM tiles and the first layer reduced plane by plane
    "maze_bf16_16x16_256": (variant("maze_16384", hidden=[256, 256], B=128, T=9, max_steps=20), 4, 2),
    # the benchmark's layer widths at a size the oracle can follow: every 512-wide update kernel
    "maze_bf16_16x16_512": (variant("maze_16384", B=64, T=8, max_steps=20), 5, 1),
    # three layers: all 256 wide (both dX products weights-resident, dZ in the packed layout only) and 128-256-256
    # (the 128 -> 256 layer's dX product is the tiled one, which reads rows: the layer above then runs tiled too)
    "maze_bf16_8x8_256x3": (variant("maze_16384", hidden=[256, 256, 256], B=64, T=8, rows=8, cols=8, max_steps=20), 6, 2),
    "maze_bf16_8x8_128_256_256": (variant("maze_16384", hidden=[128, 256, 256], B=64, T=8, rows=8, cols=8, max_steps=20), 7, 2),
    "catch_bf16_128": (variant("catch_4096", hidden=[128, 128], B=64, T=12, dtype="bf16"), 0, 2),
    "pendulum_bf16_128": (variant("pendulum_8192", hidden=[128, 128], B=64, T=10, dtype="bf16", max_steps=7), 2, 2),
}


def _forced_lockstep(gpu, orc, cfg, seed, updates, sel=None, learn=True, prepare=None):
    """Logit-forced protocol for the bf16 matrix-core acting path: the accumulation order inside the bf16
    MFMA is the hardware's, so (1) the GPU's head outputs are checked against the oracle's own sequential
    forward within the bf16 tolerance, (2) the oracle samples from the GPU's head outputs with its own
    sampler and RNG and steps its own envs -- actions, rewards, dones and states must then match bit for
    bit, (3) both learn on the identical unroll and gradients / parameters agree within 2e-2."""
    kind = cfg["env"]["kind"]
    g = gpu.Anakin(cfg, seed=seed); o = orc.Oracle(cfg, seed=seed)
    PT.assert_same_init(g, o, kind)
    if prepare is not None:
        prepare(g, o)                            # e.g. places the envs of both sides in chosen states
    for u in range(updates):
        PT.sync_oracle_from_gpu(g, o)
        g.rollout()
        tr = g.trajectory()
        o.rollout(forced_head=tr["head"], sel=sel)
        PT.assert_rollout_equal(g, o, kind, sel=sel, forced=True)
        PT.assert_final_state_equal(g, o, kind, sel=sel)
        # (1) head outputs and stored activations against the oracle's own forward on the same states, at every
        # step of every compared env
        worst = PT.assert_heads_close(g, o, tr, TOL_BF16, sel=sel)
        if learn:
            g.learn(); o.learn()
            e_g, e_p = PT.assert_learn_close(g, o, TOL_BF16)
            say(f"  update {u}: head err {worst:.2e}, grad rel {e_g:.2e}, param rel {e_p:.2e}")
        else:
            g.learn()
            assert g.metrics()["nonfinite"] == 0
            say(f"  unroll {u}: head err {worst:.2e}")
    g.close()


@pytest.mark.parametrize("case", list(BF16_CASES))
def test_bf16_matrix_core_path(gpu, orc, case):
    cfg, seed, updates = BF16_CASES[case]
    say(f"[bf16] {case} seed={seed} B={cfg['B']} T={cfg['T']} hidden={cfg['net']['hidden']}")
    _forced_lockstep(gpu, orc, cfg, seed, updates)


def _place_next_to_goal(g, o):
    """every env on a free neighbour of the goal with 250 - (b % 3) of its 256 steps used (16 x 16 maze)"""
    walls = np.unpackbits(o.walls.view(np.uint8), axis=1, bitorder="little").reshape(g.B, 16, 16).astype(bool)
    si = np.zeros((g.B, 4), np.int32)
    _, sf = g.get_env_state()
    for b in range(g.B):
        si[b, 0] = 15 * 16 + 14 if not walls[b, 15, 14] else 14 * 16 + 15
        assert not walls[b, si[b, 0] // 16, si[b, 0] % 16]
        si[b, 1] = 250 - (b % 3)
    g.set_env_state(si, sf); o.state_i[:] = si


def test_bf16_matrix_core_goal_and_step_cap(gpu, orc):
    """The matrix-core acting kernel keeps the maze state in registers and packs it on its own: goal arrivals, the
    step cap next to its limit and the restart from the start cell inside one unroll, logit-forced, then the update."""
    cfg = variant("maze_16384", hidden=[128, 128, 128], B=128, T=12)
    say("[bf16 goal and cap] hidden=[128, 128, 128] B=128 T=12")
    seen = {}

    def prepare(g, o):
        assert g.plan()["bf16_matrix_path"] == 1
        _place_next_to_goal(g, o)
        seen["o"] = o
    _forced_lockstep(gpu, orc, cfg, 4, 1, prepare=prepare)
    o = seen["o"]
    goals = int((o.tr_reward == 1.0).sum()); caps = int(o.tr_done.sum()) - goals
    say(f"  {goals} goals, {caps} step caps")
    assert goals >= 10 and caps >= 10, (goals, caps)


def test_seeded_shape_sweep_bf16_and_boards(gpu, orc):
    """More shapes off the benchmark's grid: Catch boards of other sizes (up to 32 x 32: the first-layer matrix no
    longer fits LDS and the acting kernel that keeps it there has to step aside), and a seeded sample of bf16 nets
    of one to three layers on all three envs -- on the matrix-core path where the plan takes it (logit-forced
    protocol), on the canonical path elsewhere (bit-exact unrolls)."""
    for (r, c, hid, B, T) in [(20, 20, [256, 256], 64, 4), (32, 32, [64, 64], 32, 3), (30, 7, [128, 128], 64, 5), (25, 25, [64], 64, 4)]:
        cfg = variant("catch_small", hidden=hid, B=B, T=T, rows=r, cols=c)
        say(f"[board] catch {r}x{c} hidden={hid} B={B} T={T}")
        g = gpu.Anakin(cfg, seed=3); o = orc.Oracle(cfg, seed=3)
        PT.assert_same_init(g, o, "catch")
        for u in range(2):
            PT.sync_oracle_from_gpu(g, o)
            g.rollout(); o.rollout()
            PT.assert_rollout_equal(g, o, "catch")
            g.learn(); o.learn()
            PT.assert_learn_close(g, o, TOL_F32)
        g.close()
    rng = np.random.default_rng(5)
    base = {"catch": "catch_small", "pendulum": "pendulum_8192", "maze": "maze_16384"}
    on_matrix_cores = 0
    for i in range(12):
        kind = ["maze", "catch", "pendulum"][i % 3]
        widths = [int(rng.choice([64, 128, 256, 512])) for _ in range(int(rng.integers(1, 4)))]
        B, T = int(rng.choice([64, 128, 192])), int(rng.choice([2, 5, 8]))
        over = dict(max_steps=int(rng.integers(2, 9))) if kind != "catch" else {}
        if kind == "maze":
            r, co = [(8, 8), (16, 16), (4, 4)][int(rng.integers(3))]
            over.update(rows=r, cols=co)
        cfg = variant(base[kind], hidden=widths, B=B, T=T, dtype="bf16", **over)
        s = int(rng.integers(100))
        g = gpu.Anakin(cfg, seed=s)
        matrix = g.plan()["bf16_matrix_path"]
        g.close()
        say(f"[bf16 shape {i}] {kind} {over} hidden={widths} B={B} T={T} seed={s} matrix cores: {matrix}")
        if matrix:
            on_matrix_cores += 1
            _forced_lockstep(gpu, orc, cfg, s, 2)
        else:
            g = gpu.Anakin(cfg, seed=s); o = orc.Oracle(cfg, seed=s)
            for u in range(2):
                PT.sync_oracle_from_gpu(g, o)
                g.rollout(); o.rollout()
                PT.assert_rollout_equal(g, o, kind)
                g.learn(); o.learn()
                PT.assert_learn_close(g, o, TOL_BF16)
            g.close()
    assert 3 <= on_matrix_cores <= 10


def _steady_state_update(gpu, orc, cfg, check_plan, n_head_envs):
    """One whole update of a bf16 maze net at a size where the update kernels run their steady-state loops:
    logit-forced lockstep over all envs, head outputs checked on a sample of envs at every time step, the oracle's
    update spread over threads by sample range.  check_plan(plan, B, T) asserts on the launch plan."""
    B, T = cfg["B"], cfg["T"]
    g = gpu.Anakin(cfg, seed=9); o = orc.Oracle(cfg, seed=9)
    plan = g.plan()
    say(f"  plan {plan}")
    assert plan["bf16_matrix_path"] == 1
    check_plan(plan, B, T)
    PT.assert_same_init(g, o, "maze")
    g.step()                                     # the compared update starts from non-initial parameters and moments
    PT.sync_oracle_from_gpu(g, o)
    si, sf = g.get_env_state()
    o.state_i[:] = si
    o.global_step = g.global_step
    g.rollout()
    tr = g.trajectory()
    o.rollout(forced_head=tr["head"])
    PT.assert_rollout_equal(g, o, "maze", forced=True)
    PT.assert_final_state_equal(g, o, "maze")
    rng = np.random.default_rng(9)
    sel = np.unique(np.concatenate([[0, 63, 64, B - 1], rng.integers(0, B, n_head_envs)])).astype(np.int32)
    worst = PT.assert_heads_close(g, o, tr, TOL_BF16, sel=sel)
    say(f"  head err {worst:.2e} over {sel.size} envs x {g.T + 1} steps; update on the oracle ...")
    g.learn()
    PT.oracle_learn_parallel(o, workers=16)
    e_g, e_p = PT.assert_learn_close(g, o, TOL_BF16)
    say(f"  gradient rel err {e_g:.2e}, parameter rel err {e_p:.2e}")
    g.close()


@pytest.mark.parametrize("B,T", [(1024, 32), (8192, 2)])
def test_bf16_benchmark_widths_steady_state(gpu, orc, B, T):
    """The maze workload's own layer widths (768-512-512-512, bf16) with enough samples that every update kernel
    runs its steady-state loop, not just its prologue.  B = 1024, T = 32: the weights-resident dX kernel walks
    >= 4 stages of 32 samples per workgroup (its ring holds rows two stages and the mask one stage ahead), the
    256 x 256-tile dW kernels (the top one forms dZ_L itself) >= 8 LDS stages of 64 samples per chunk on the hidden
    layers (double-buffered, next step prefetched) and >= 4 on the agent plane.  B = 8192, T = 2: the wall-plane
    product, whose rows are the 2 B time-summed ones, reaches >= 4 stages per chunk in several chunks."""
    cfg = variant("maze_16384", B=B, T=T)
    say(f"[bf16 steady state] B={cfg['B']} T={cfg['T']} hidden={cfg['net']['hidden']}")

    def check_plan(plan, B, T):
        M = B * T
        if T == 32:
            assert all(plan["dx_rows"][l] >= 4 * 32 for l in (1, 2)), "dX kernel: fewer than 4 stages per workgroup"
            assert all(M // plan["splits"][l] >= 8 * 64 for l in (1, 2)), "dW kernel: fewer than 8 LDS stages per chunk"
            assert M // plan["splits"][0] >= 4 * 64, "agent-plane product: fewer than 4 LDS stages per chunk"
            assert plan["splits"][3] == plan["splits"][2] and plan["head_fan"] == 1, "top layer: the head pass is not folded in"
        else:
            assert plan["splits_walls"] > 1 and 2 * B // plan["splits_walls"] >= 4 * 64, "wall-plane product: fewer than 4 LDS stages per chunk"

    _steady_state_update(gpu, orc, cfg, check_plan, 12 if T == 32 else 60)


def test_bf16_agent_plane_sums_over_time_in_the_product(gpu, orc):
    """The benchmark's batch size with a narrower net (768-256-256, so the oracle can follow all 131072 samples):
    B = 16384 divides into blocks of 128 environments per chunk of the agent-plane product, which then walks them as
    two passes of 64 environments over the T = 8 time steps and writes the time sum of dZ1 itself (no separate
    pass); the wall-plane product reads that sum.  Also the 256-wide form of the fused top layer (one row of tiles
    carries both the head matrix's gradient and the column sums)."""
    cfg = variant("maze_16384", hidden=[256, 256], B=16384, T=8)
    say(f"[bf16 agent plane by environment blocks] B={cfg['B']} T={cfg['T']} hidden={cfg['net']['hidden']}")

    def check_plan(plan, B, T):
        s0 = plan["splits"][0]
        assert B % (64 * s0) == 0 and B // s0 >= 128, "agent-plane chunks are not blocks of >= 128 environments"
        assert plan["splits"][2] == plan["splits"][1] and plan["head_fan"] == 1, "top layer: the head pass is not folded in"

    _steady_state_update(gpu, orc, cfg, check_plan, 40)


def test_bf16_reference_mode_is_exact(gpu, orc):
    """The same bf16 net on the sequential fp32-chain reference path matches the oracle bit for bit."""
    cfg, seed, _ = BF16_CASES["maze_bf16_128"]
    g = gpu.Anakin(cfg, seed=seed); o = orc.Oracle(cfg, seed=seed)
    g.set_mode(gpu.MODE_CANONICAL_ACTING | gpu.MODE_VALU_GEMM)
    with pytest.raises(gpu.AnakinError):
        g.set_mode(gpu.MODE_VALU_GEMM)
    g.set_mode(gpu.MODE_CANONICAL_ACTING | gpu.MODE_VALU_GEMM)
    PT.sync_oracle_from_gpu(g, o)
    g.rollout(); o.rollout()
    PT.assert_rollout_equal(g, o, "maze")
    g.learn(); o.learn()
    PT.assert_learn_close(g, o, TOL_BF16)
    g.close()


def test_full_size_maze_bf16_sampled_envs(gpu, orc):
    """The maze workload at full size (B=16384, 768-512-512-512 bf16) in the benchmark's launch shape:
    logit-forced replay of a seeded sample of envs, plus properties that hold at any size."""
    cfg = W.get("maze_16384")
    B = cfg["B"]
    rng = np.random.default_rng(4)
    sel = np.unique(np.concatenate([[0, 1, 63, 64, B - 1, B - 64, B // 2], rng.integers(0, B, 9)])).astype(np.int32)
    say(f"[full size] maze_16384 envs={sel.tolist()}")
    _forced_lockstep(gpu, orc, cfg, 0, 2, sel=sel, learn=False)


def test_full_size_maze_bf16_every_sample(gpu, orc):
    """The forward pass and the update of the maze workload at its full size (B=16384, T=32, 768-512-512-512 bf16: 524288 samples), in
    the launch shape the benchmark times.  The oracle would need an hour for it, so the reference is the same
    objective and backward rule written as binary64 matrix products over the forward pass the GPU stored
    (parity.np_maze_backward_from_stored, itself checked against the oracle on small cases by the CPU suite; the
    stored forward pass is compared first, layer by layer at every sample, with binary64 products from each layer's
    stored input; test_full_size_maze_bf16_sampled_envs replays whole envs on the oracle): returns and advantages by
    the oracle's routine, loss terms, every region of the gradient, then the Adam step replayed in binary64 from
    the GPU's own gradient."""
    from oracle import oracle as O
    cfg = W.get("maze_16384")
    net = cfg["net"]
    f32 = lambda x: float(np.float32(x))
    say("[full size] maze_16384 update against the binary64 backward pass over the stored forward pass")
    g = gpu.Anakin(cfg, seed=2)
    g.step()                                     # the compared update starts from non-initial parameters and moments
    g.rollout()
    theta0 = g.get_params()
    m0, v0, step0 = g.get_opt_state()
    tr = g.trajectory()
    walls = np.unpackbits(g.get_walls().view(np.uint8), axis=1, bitorder="little").astype(bool)
    pos = (tr["state_s0"][:-1] & 0xFFFF).astype(np.int64)
    # the acting kernel's forward pass at EVERY one of the 524288 stored samples, layer by layer from the stored
    # input of each layer (parity.np_maze_forward_layers_from_stored, checked against the oracle by the CPU suite)
    say("  trajectory on the host; every layer of every stored sample against binary64 products ...")
    share = [0.0] * len(tr["act"])
    head_err = 0.0
    hscale = float(np.abs(tr["head"]).max())
    for t0, t1, refs, heads in PT.np_maze_forward_layers_from_stored(cfg, theta0, walls, pos, tr["act"]):
        for l, r in enumerate(refs):
            share[l] = max(share[l], PT.assert_bf16_layers_close(f"layer {l + 1}, steps {t0}..{t1 - 1}", tr["act"][l][t0:t1], r))
        head_err = max(head_err, float(np.abs(heads - tr["head"][t0:t1]).max()) / hscale)
    assert head_err <= 1e-4, f"head outputs differ by {head_err:.3e} of their scale"
    say(f"  layers differ in at most {max(share):.4%} of their entries (one bfloat16 step), heads by {head_err:.2e}; update on the GPU ...")
    g.learn()
    assert g.metrics()["nonfinite"] == 0
    ret, adv = O.returns(tr["reward"], tr["done"], tr["value"], f32(net["gamma"]), f32(net["lambda"]))
    tr2 = g.trajectory()
    scale = max(1.0, float(np.abs(ret).max()))
    assert np.abs(tr2["ret"] - ret).max() <= 1e-5 * scale and np.abs(tr2["adv"] - adv).max() <= 1e-5 * scale
    say("  binary64 backward pass on the host ...")
    loss, ref = PT.np_maze_backward_from_stored(cfg, theta0, walls, pos, tr["act"], tr["head"][:-1], tr["action"], adv, ret)
    m = g.metrics()
    for k, i in (("loss", 0), ("policy_loss", 1), ("value_loss", 2), ("entropy_loss", 3)):
        assert abs(m[k] - loss[i]) <= 1e-4 * max(abs(loss[i]), 1e-3 * np.abs(loss).max()) + 1e-7, (k, m[k], loss[i])
    regions, P = PT.param_regions(cfg)
    g_gpu = g.get_grads()
    e_g = PT.rel(g_gpu, ref)
    say(f"  gradient rel err {e_g:.2e}")
    # both sides start from the same stored forward pass here, so what is left is the order of the sums and the
    # bfloat16 rounding of dZ_l between the layers' products: a twentieth of the bf16 tolerance holds per region
    worst = PT.assert_regions_close("gradient", g_gpu, ref, regions, TOL_BF16 / 20)
    # Adam on its own: binary64 Adam (the oracle's routine) on the GPU's gradient from the state before the update
    th_x, m_x, v_x = theta0.copy(), m0.astype(np.float64), v0.astype(np.float64)
    O.adam(th_x, g_gpu, m_x, v_x, step0 + 1, f32(net["lr"]), f32(net["beta1"]), f32(net["beta2"]), f32(net["eps"]))
    gm, gv, gt = g.get_opt_state()
    assert gt == step0 + 1
    th_gpu = g.get_params()
    assert np.abs(th_gpu.astype(np.float64) - th_x).max() <= 2.0 ** -22 * np.abs(th_x).max() + 1e-4 * net["lr"]
    assert np.abs(gm - m_x).max() <= 1e-6 * np.abs(m_x).max() and np.abs(gv - v_x).max() <= 1e-6 * np.abs(v_x).max()
    say(f"  worst region {worst:.2e}; Adam step matches binary64 Adam on the same gradient")
    g.close()


def _fast_lr(cfg, lr=1e-2):
    cfg = copy.deepcopy(cfg)
    cfg["net"]["lr"] = lr          # one update moves the policy enough for importance ratios on both sides of 1
    return cfg


N_UPDATE_CASES = {
    # name: (cfg, seed, N, tolerance)
    "catch_256x256_N2": (variant("catch_4096", B=128, T=8), 0, 2, TOL_F32),
    "catch_tiny_net_N4": (variant("catch_262144", B=512, T=16), 1, 4, TOL_F32),
    "pendulum_N2": (variant("pendulum_8192", B=128, T=8), 2, 2, TOL_F32),
    "maze_fp32_N2": (variant("maze_16384", hidden=[64, 64], B=64, T=16, dtype="fp32", max_steps=20), 3, 2, TOL_F32),
}


@pytest.mark.parametrize("case", list(N_UPDATE_CASES))
def test_n_updates_per_unroll(gpu, orc, case):
    """N Adam updates on one unroll, one per consecutive time chunk, gradients at the acting-time parameters
    (paper section 4): parameters, moments, loss and the last chunk's gradient against the oracle's learn_n."""
    cfg, seed, N, tol = N_UPDATE_CASES[case]
    say(f"[n updates] {case} seed={seed} N={N} B={cfg['B']} T={cfg['T']}")
    g = gpu.Anakin(cfg, seed=seed); o = orc.Oracle(cfg, seed=seed)
    g.set_updates_per_unroll(N)
    kind = cfg["env"]["kind"]
    for u in range(2):
        PT.sync_oracle_from_gpu(g, o)
        g.rollout(); o.rollout()
        PT.assert_rollout_equal(g, o, kind)
        g.learn(); o.learn_n(N)
        e_g, e_p = PT.assert_learn_close(g, o, tol, n_updates=N)
        say(f"  unroll {u}: gradient rel err {e_g:.2e}, parameter rel err {e_p:.2e}")
    with pytest.raises(gpu.AnakinError):
        g.set_updates_per_unroll(3 if cfg["T"] % 3 else 5)
    g.set_updates_per_unroll(1)                   # and back to one update per unroll
    PT.sync_oracle_from_gpu(g, o)
    g.rollout(); o.rollout(); g.learn(); o.learn()
    PT.assert_learn_close(g, o, tol)
    g.close()


@pytest.mark.parametrize("case", list(N_UPDATE_CASES))
def test_n_updates_sequential(gpu, orc, case):
    """The sequential reading: chunk k's gradient at the parameters after k updates (the forward pass over the
    stored states is repeated on the GPU before every further chunk), against the oracle's learn_n(sequential)."""
    cfg, seed, N, tol = N_UPDATE_CASES[case]
    cfg = _fast_lr(cfg, 3e-3)                     # the parameters move enough between chunks to tell the two readings apart
    say(f"[n updates, sequential] {case} seed={seed} N={N} B={cfg['B']} T={cfg['T']}")
    g = gpu.Anakin(cfg, seed=seed); o = orc.Oracle(cfg, seed=seed); o2 = orc.Oracle(cfg, seed=seed)
    g.set_updates_per_unroll(N, sequential=True)
    kind = cfg["env"]["kind"]
    for u in range(2):
        PT.sync_oracle_from_gpu(g, o)
        g.rollout(); o.rollout()
        PT.assert_rollout_equal(g, o, kind)
        g.learn(); o.learn_n(N, sequential=True)
        e_g, e_p = PT.assert_learn_close(g, o, tol, n_updates=N)
        say(f"  unroll {u}: gradient rel err {e_g:.2e}, parameter rel err {e_p:.2e}")
    # the acting-time reading gives a measurably different last gradient on the same unroll
    PT.sync_oracle_from_gpu(g, o); PT.sync_oracle_from_gpu(g, o2)
    o2.state_i[:] = o.state_i; o2.state_f[:] = o.state_f; o2.global_step = o.global_step
    g.rollout(); o.rollout(); o2.rollout()
    g.learn(); o.learn_n(N, sequential=True); o2.learn_n(N)
    assert PT.rel(g.get_grads(), o.grad) <= tol
    assert PT.rel(o2.grad, o.grad) > 10 * tol
    g.set_updates_per_unroll(1, sequential=False)
    g.close()


def test_n_updates_sequential_bf16(gpu, orc):
    """the same on the bf16 matrix-core path (logit-forced unroll), 256-wide maze net, N = 3"""
    cfg = _fast_lr(variant("maze_16384", hidden=[256, 256], B=128, T=9, max_steps=20), 3e-3)
    g = gpu.Anakin(cfg, seed=6); o = orc.Oracle(cfg, seed=6)
    g.set_updates_per_unroll(3, sequential=True)
    PT.sync_oracle_from_gpu(g, o)
    g.rollout()
    tr = g.trajectory()
    o.rollout(forced_head=tr["head"])
    g.learn(); o.learn_n(3, sequential=True)
    # The learner's forward pass at the moved parameters is the GPU's bf16 matrix-core one on one side and the
    # oracle's sequential one on the other (the forced protocol only pins the acting pass), and a chunk is 384
    # samples: single entries of the wall-plane rows, sums over the ~25 envs with a wall there, differ by up to a few
    # per cent of the largest entry while every region's norm stays within the tolerance.
    PT.assert_learn_close(g, o, TOL_BF16, n_updates=3, elem_factor=3.0)
    g.close()


def test_n_updates_per_unroll_bf16(gpu, orc):
    """the same on the bf16 matrix-core path (logit-forced unroll), 256-wide maze net, N = 3"""
    cfg = variant("maze_16384", hidden=[256, 256], B=128, T=9, max_steps=20)
    g = gpu.Anakin(cfg, seed=6); o = orc.Oracle(cfg, seed=6)
    g.set_updates_per_unroll(3)
    PT.sync_oracle_from_gpu(g, o)
    g.rollout()
    tr = g.trajectory()
    o.rollout(forced_head=tr["head"])
    g.learn(); o.learn_n(3)
    PT.assert_learn_close(g, o, TOL_BF16, n_updates=3)
    g.close()


DECOUPLED_CASES = {
    # name: (cfg, seed, steps) -- every fp32 acting kernel in its replay form, both policies, the one-layer update
    "catch_small": (_fast_lr(variant("catch_small")), 0, 4),
    "catch_256x256_B256": (_fast_lr(variant("catch_4096", B=256)), 1, 3),
    "catch_tiny_net_B512": (_fast_lr(variant("catch_262144", B=512)), 0, 3),
    "pendulum_B128": (_fast_lr(variant("pendulum_8192", B=128), 3e-3), 0, 3),
    "pendulum_short_episodes": (_fast_lr(variant("pendulum_8192", hidden=[64, 64], B=64, T=32, max_steps=25), 3e-3), 2, 3),
    "maze_fp32_small": (_fast_lr(variant("maze_16384", hidden=[64, 64], B=64, T=32, dtype="fp32", max_steps=20)), 1, 3),
    "catch_512x256": (_fast_lr(variant("catch_4096", hidden=[512, 256], B=64, T=10)), 3, 3),
    "catch_ragged_B80_T7": (_fast_lr(variant("catch_small", B=80, T=7)), 2, 3),
}


@pytest.mark.parametrize("case", list(DECOUPLED_CASES))
def test_decoupled_lockstep(gpu, orc, case):
    """Decoupled steps, parameter-synchronised: the actor's unroll (with the parameters from before the update
    that runs beside it) is bitwise the oracle's; the learner's off-policy update on the previous unroll --
    V-trace targets, loss, gradient, parameters, moments -- within tolerance."""
    cfg, seed, steps = DECOUPLED_CASES[case]
    kind = cfg["env"]["kind"]
    say(f"[decoupled] {case} seed={seed} B={cfg['B']} T={cfg['T']} hidden={cfg['net']['hidden']}")
    g = gpu.Anakin(cfg, seed=seed)
    o = orc.Oracle(cfg, seed=seed)
    if case == "catch_small":
        # the actor on a stream of the caller's instead of one the library creates
        import torch
        with pytest.raises(gpu.AnakinError):
            g.set_actor_stream(g.stream)            # must differ from the handle's own stream
        g.set_actor_stream(torch.cuda.Stream())
    off_policy = 0
    for k in range(steps):
        PT.sync_oracle_from_gpu(g, o)
        before = g.get_params().copy()
        learned_on = (o.tr_reward.copy(), o.tr_done.copy())
        g.step_decoupled(); o.step_decoupled()
        tr = PT.assert_rollout_equal(g, o, kind)
        PT.assert_final_state_equal(g, o, kind)
        if k == 0:
            assert np.array_equal(g.get_params(), before) and g.get_opt_state()[2] == 0      # the first step only collects
            continue
        e_g, e_p = PT.assert_learn_close(g, o, TOL_F32, tr_after=tr, learned_on=learned_on)
        off_policy += int((o.rho < 1.0 - 1e-3).sum())
        say(f"  step {k}: grad rel {e_g:.2e}, param rel {e_p:.2e}, loss {o.loss[0]:+.5f}, min rho {o.rho.min():.4f}")
    assert off_policy > 0, "no update was off-policy"
    # an on-policy update cannot use this unroll (older parameters, no activations kept)
    with pytest.raises(gpu.AnakinError):
        g.learn()
    # a plain step afterwards starts a fresh on-policy unroll
    PT.sync_oracle_from_gpu(g, o)
    g.step(); o.step()
    PT.assert_learn_close(g, o, TOL_F32)
    g.close()


DECOUPLED_BF16_CASES = {
    "maze_bf16_16x16_256": (_fast_lr(variant("maze_16384", hidden=[256, 256], B=128, T=9, max_steps=20), 3e-3), 4, 3),
    "maze_bf16_16x16_512": (_fast_lr(variant("maze_16384", B=64, T=8, max_steps=20), 3e-3), 5, 3),
    "pendulum_bf16_128": (_fast_lr(variant("pendulum_8192", hidden=[128, 128], B=64, T=10, dtype="bf16", max_steps=7), 3e-3), 2, 3),
    "catch_bf16_128": (_fast_lr(variant("catch_4096", hidden=[128, 128], B=64, T=12, dtype="bf16"), 3e-3), 0, 3),
}


@pytest.mark.parametrize("case", list(DECOUPLED_BF16_CASES))
def test_decoupled_bf16_forced_lockstep(gpu, orc, case):
    """Decoupled steps of a bf16 net on the matrix-core path, logit-forced: the oracle's actor samples from the GPU
    actor's head outputs (which must be its own forward within the bf16 tolerance) and must then reproduce the
    unroll bit for bit; the learner's off-policy update on the previous unroll agrees within 2e-2."""
    cfg, seed, steps = DECOUPLED_BF16_CASES[case]
    kind = cfg["env"]["kind"]
    say(f"[decoupled bf16] {case} seed={seed} B={cfg['B']} T={cfg['T']} hidden={cfg['net']['hidden']}")
    g = gpu.Anakin(cfg, seed=seed)
    o = orc.Oracle(cfg, seed=seed)
    for k in range(steps):
        PT.sync_oracle_from_gpu(g, o)
        behaviour = o.theta.copy()
        learned_on = (o.tr_reward.copy(), o.tr_done.copy())
        g.step_decoupled()
        tr = g.trajectory()
        o.step_decoupled(forced_head=tr["head"])
        PT.assert_rollout_equal(g, o, kind, forced=True)
        PT.assert_final_state_equal(g, o, kind)
        # the actor's head outputs are the forward pass of the parameters from before this step's update
        learner = o.theta.copy()
        o.theta[:] = behaviour
        scale = max(1e-3, float(np.abs(tr["head"]).max()))
        for (t, b) in [(0, 0), (g.T // 2, g.B // 2), (g.T, g.B - 1)]:
            save = (o.state_i[b].copy(), o.state_f[b].copy())
            o.state_i[b] = o.tr_state_i[t, b]; o.state_f[b] = o.tr_state_f[t, b]
            head = o.forward(o.observe(b))
            o.state_i[b], o.state_f[b] = save
            assert np.abs(head - tr["head"][t, b]).max() <= TOL_BF16 * scale, "actor head outputs differ"
        o.theta[:] = learner
        if k == 0:
            assert g.get_opt_state()[2] == 0
            continue
        # the V-trace targets come from the learner's own forward pass: bf16 tolerance for them too
        e_g, e_p = PT.assert_learn_close(g, o, TOL_BF16, tr_after=tr, learned_on=learned_on, target_tol=TOL_BF16)
        say(f"  step {k}: grad rel {e_g:.2e}, param rel {e_p:.2e}, min rho {o.rho.min():.4f}")
    g.close()


def _path_only(cfg):
    cfg = copy.deepcopy(cfg)
    cfg["net"]["value_coef"] = 0.0; cfg["net"]["entropy_coef"] = 0.0     # nothing but the pathwise term in the gradient
    return cfg


PATHWISE_CASES = {
    "pendulum_64_path_term_only": (_path_only(variant("pendulum_8192", hidden=[64, 64], B=32, T=20, max_steps=13)), 7, 2),
    # name: (cfg, seed, updates) -- the three widths of the sweep kernel, episode ends inside the unroll
    "pendulum_256_B128": (variant("pendulum_8192", B=128), 0, 2),
    "pendulum_64_short_episodes": (variant("pendulum_8192", hidden=[64, 64], B=64, T=32, max_steps=25), 2, 3),
    "pendulum_128_B48": (variant("pendulum_8192", hidden=[128, 128], B=48, T=12, max_steps=7), 4, 2),
    # enough envs for the 32-env form of the sweep (32x32x2 matrix instruction)
    "pendulum_128_B8192": (_path_only(variant("pendulum_8192", hidden=[128, 128], B=8192, T=6, max_steps=4)), 5, 1),
}


@pytest.mark.parametrize("case", list(PATHWISE_CASES))
def test_pathwise_lockstep(gpu, orc, case):
    """Policy gradient through the pendulum's dynamics: per-sample head gradients of the reverse sweep and the whole
    update against the oracle's binary64 reverse accumulation, parameter-synchronised."""
    cfg, seed, updates = PATHWISE_CASES[case]
    say(f"[pathwise] {case} seed={seed} B={cfg['B']} T={cfg['T']} hidden={cfg['net']['hidden']}")
    g = gpu.Anakin(cfg, seed=seed)
    o = orc.Oracle(cfg, seed=seed)
    g.set_policy_gradient(gpu.PG_PATHWISE)
    for u in range(updates):
        PT.sync_oracle_from_gpu(g, o)
        g.rollout(); o.rollout()
        PT.assert_rollout_equal(g, o, "pendulum")
        _, ph = o.pathwise_grad()
        rew, done = o.tr_reward.copy(), o.tr_done.copy()
        adv_zero = np.zeros_like(o.adv)
        g.learn(); o.learn_pathwise()
        tr = g.trajectory()
        tr["adv"] = adv_zero                 # the score-function advantage is not used on either side
        e_g, e_p = PT.assert_learn_close(g, o, TOL_F32, tr_after=tr, learned_on=(rew, done))
        say(f"  update {u}: grad rel {e_g:.2e}, param rel {e_p:.2e}, -mean reward {o.loss[1]:+.4f}, |path dhead| {np.abs(ph).max():.3e}")
    if cfg["env"]["max_steps"] < cfg["T"]:
        assert o.tr_done.sum() > 0                   # the adjoint was cut inside the unroll
    g.set_policy_gradient(gpu.PG_SCORE_FUNCTION)
    PT.sync_oracle_from_gpu(g, o)
    g.step(); o.step()
    PT.assert_learn_close(g, o, TOL_F32)
    g.close()


def test_pathwise_rejections(gpu):
    c = gpu.Anakin(variant("catch_small"), seed=0)
    with pytest.raises(gpu.AnakinError):
        c.set_policy_gradient(gpu.PG_PATHWISE)
    c.close()
    p = gpu.Anakin(variant("pendulum_8192", hidden=[64, 64], B=32, T=8), seed=0)
    p.set_policy_gradient(gpu.PG_PATHWISE)
    with pytest.raises(gpu.AnakinError):
        p.step_decoupled()
    with pytest.raises(gpu.AnakinError):        # chunks would cut the adjoint
        p.set_updates_per_unroll(2)
        p.rollout()
        p.learn()
    p.close()


def test_seeded_sweep_of_the_widened_calls(gpu, orc):
    """The calls beyond the fused step on a seeded sample of shapes (fp32, one to three layers of 64..512 units, batch
    sizes that are not powers of two, short unrolls): several updates per unroll in both readings, decoupled steps,
    the pathwise gradient (on the shapes it takes), and the static-scratch update against the workspace one."""
    rng = np.random.default_rng(0)
    base = {"catch": "catch_small", "pendulum": "pendulum_8192", "maze": "maze_16384"}

    def shape(kind):
        widths = [int(rng.choice([64, 128, 256, 512])) for _ in range(int(rng.integers(1, 4)))]
        B = int(rng.choice([16, 48, 112, 256]))
        over = {}
        if kind == "maze":
            r, co = [(4, 4), (8, 8), (16, 16)][int(rng.integers(3))]
            over = dict(rows=r, cols=co, max_steps=int(rng.integers(2, 12)))
        elif kind == "pendulum":
            over = dict(max_steps=int(rng.integers(2, 12)))
        return widths, B, over

    for i in range(6):
        kind = ["catch", "pendulum", "maze"][i % 3]
        widths, B, over = shape(kind)
        N = int(rng.choice([2, 3, 4])); T = N * int(rng.integers(1, 4))
        seq = bool(i % 2)
        cfg = _fast_lr(variant(base[kind], hidden=widths, B=B, T=T, dtype="fp32", **over), 3e-3)
        s = int(rng.integers(1000))
        say(f"[sweep: n updates {i}] {kind} {over} hidden={widths} B={B} T={T} N={N} sequential={seq} seed={s}")
        g = gpu.Anakin(cfg, seed=s); o = orc.Oracle(cfg, seed=s)
        g.step()                  # Adam's first steps from zero moments are +-lr whatever the gradient's size: with only
        g.step()                  # the last chunk's gradient visible, compare from moments that have settled
        o.global_step = g.global_step
        si, sf = g.get_env_state(); o.state_i[:] = si; o.state_f[:] = sf
        g.set_updates_per_unroll(N, sequential=seq)
        PT.sync_oracle_from_gpu(g, o)
        g.rollout(); o.rollout()
        PT.assert_rollout_equal(g, o, kind)
        g.learn(); o.learn_n(N, sequential=seq)
        PT.assert_learn_close(g, o, TOL_F32, n_updates=N)
        g.close()
    for i in range(6):
        kind = ["catch", "pendulum", "maze"][i % 3]
        widths, B, over = shape(kind)
        T = int(rng.choice([2, 5, 9]))
        cfg = _fast_lr(variant(base[kind], hidden=widths, B=B, T=T, dtype="fp32", **over), 3e-3)
        s = int(rng.integers(1000))
        say(f"[sweep: decoupled {i}] {kind} {over} hidden={widths} B={B} T={T} seed={s}")
        g = gpu.Anakin(cfg, seed=s); o = orc.Oracle(cfg, seed=s)
        for k in range(3):
            PT.sync_oracle_from_gpu(g, o)
            learned_on = (o.tr_reward.copy(), o.tr_done.copy())
            g.step_decoupled(); o.step_decoupled()
            tr = PT.assert_rollout_equal(g, o, kind)
            PT.assert_final_state_equal(g, o, kind)
            if k:
                PT.assert_learn_close(g, o, TOL_F32, tr_after=tr, learned_on=learned_on)
        g.close()
    for i in range(4):
        w = int(rng.choice([64, 128, 256]))
        B, T = int(rng.choice([16, 48, 112, 256])), int(rng.choice([2, 5, 9]))
        cfg = variant("pendulum_8192", hidden=[w, w], B=B, T=T, max_steps=int(rng.integers(2, 12)))
        s = int(rng.integers(1000))
        say(f"[sweep: pathwise {i}] hidden={[w, w]} B={B} T={T} max_steps={cfg['env']['max_steps']} seed={s}")
        g = gpu.Anakin(cfg, seed=s); o = orc.Oracle(cfg, seed=s)
        g.set_policy_gradient(gpu.PG_PATHWISE)
        for u in range(2):
            PT.sync_oracle_from_gpu(g, o)
            g.rollout(); o.rollout()
            PT.assert_rollout_equal(g, o, "pendulum")
            rew, done = o.tr_reward.copy(), o.tr_done.copy()
            g.learn(); o.learn_pathwise()
            tr = g.trajectory(); tr["adv"] = np.zeros_like(o.adv)
            PT.assert_learn_close(g, o, TOL_F32, tr_after=tr, learned_on=(rew, done))
        g.close()
    for i in range(6):
        kind = ["catch", "pendulum", "maze"][i % 3]
        widths, B, over = shape(kind)
        T = int(rng.choice([2, 5, 9]))
        dt = "bf16" if i % 2 else "fp32"
        cfg = variant(base[kind], hidden=widths, B=max(B, 64) if dt == "bf16" else B, T=T, dtype=dt, **over)
        s = int(rng.integers(1000))
        say(f"[sweep: static scratch {i}] {kind} {over} hidden={widths} B={cfg['B']} T={T} {dt} seed={s}")
        a = gpu.Anakin(cfg, seed=s); b = gpu.Anakin(cfg, seed=s)
        for _ in range(2):
            a.rollout(); a.learn(); b.rollout(); b.learn_static()
            assert np.array_equal(a.get_grads(), b.get_grads()) and np.array_equal(a.get_params(), b.get_params())
        a.close(); b.close()


def test_determinism_and_resume(gpu):
    """Same seed twice gives the same bytes; a byte copy of the workspace plus the two host counters
    resumes bit-exactly (explicit, device-resident state; counter-based RNG)."""
    import torch
    cfg = variant("catch_4096", B=256)
    a = gpu.Anakin(cfg, seed=5); b = gpu.Anakin(cfg, seed=5)
    for _ in range(3):
        a.step(); b.step()
    a.synchronize(); b.synchronize()
    assert np.array_equal(a.get_params(), b.get_params()), "two runs with the same seed differ"
    assert all(np.array_equal(x, y) for x, y in zip(a.get_opt_state()[:2], b.get_opt_state()[:2]))
    ta, tb = a.trajectory(), b.trajectory()
    for k in ("state_s0", "action", "reward", "done", "value", "head", "adv", "ret"):
        assert np.array_equal(ta[k], tb[k]), k
    assert all(np.array_equal(x, y) for x, y in zip(ta["act"], tb["act"]))
    snap = a.ws.clone(); gstep = a.global_step; m, v, t = a.get_opt_state()
    for _ in range(2):
        a.step()
    a.synchronize()
    c = gpu.Anakin(cfg, seed=5)
    c.ws.copy_(snap); c.global_step = gstep; c.set_opt_state(m, v, t)
    for _ in range(2):
        c.step()
    c.synchronize()
    assert np.array_equal(a.get_params(), c.get_params())
    assert np.array_equal(a.trajectory()["action"], c.trajectory()["action"])
    for x in (a, b, c):
        x.close()


def test_error_paths(gpu):
    cfg = variant("catch_small", B=64)
    g = gpu.Anakin(cfg, seed=0)
    m0 = g.metrics()                                # before the first update: zeros, not whatever the workspace held
    assert m0["nonfinite"] == 0 and m0["loss"] == 0.0 and m0["reward_sum"] == 0.0 and m0["episodes"] == 0
    with pytest.raises(gpu.AnakinError) as e:
        g.learn()
    assert e.value.code == gpu.E_STATE
    g.rollout(); g.learn()
    with pytest.raises(gpu.AnakinError):
        g.learn()
    with pytest.raises(gpu.AnakinError):
        g.set_params(np.zeros(3, np.float32))
    bad = np.zeros((64, 4), np.int32); bad[:, 1] = 200
    with pytest.raises(gpu.AnakinError):
        g.set_env_state(bad, np.zeros((64, 2), np.float32))
    # non-finite parameters are reported, not hidden
    th = g.get_params(); th[:] = np.nan
    g.set_params(th); g.rollout(); g.learn()
    assert g.metrics()["nonfinite"] == 1
    g.close()


def test_catch_learning_sanity(gpu):
    """Not a parity criterion: the mean episode return rises from about -0.6."""
    cfg = variant("catch_small")
    cfg["net"]["lr"] = 3e-3
    g = gpu.Anakin(cfg, seed=0)
    first = last = 0.0
    for i in range(150):
        g.step()
        m = g.metrics()
        r = m["reward_sum"] / max(1, m["episodes"])
        if i < 10: first += r / 10
        if i >= 140: last += r / 10
    say(f"[learning] mean return {first:+.2f} -> {last:+.2f}")
    assert last > first + 0.3
    g.close()
