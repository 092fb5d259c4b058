"""Helpers shared by the GPU parity tests: compare one GPU agent with one oracle
agent built from the same workload dict and seed."""
import numpy as np

from paper_2104_06272_amd import binding


def rel(a, b):
    a = np.asarray(a, np.float64).ravel(); b = np.asarray(b, np.float64).ravel()
    return np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-30)


def gpu_state_rows(kind, tr):
    """trajectory state snapshots of the GPU as the oracle's (int rows, float rows)."""
    si = binding.unpack_state_word(kind, tr["state_s0"])
    sf = np.stack([tr["state_f0"], tr["state_f1"]], axis=-1)
    return si, sf


def sync_oracle_from_gpu(g, o):
    """parameter-synchronised comparison: the oracle takes the GPU's parameters and optimiser state"""
    o.theta[:] = g.get_params()
    m, v, t = g.get_opt_state()
    o.m[:] = m; o.v[:] = v; o.adam_t = t


def assert_same_init(g, o, kind):
    assert np.array_equal(g.get_params(), o.theta), "initial parameters differ"
    si, sf = g.get_env_state()
    assert np.array_equal(si, o.state_i), "initial env states differ"
    if kind == "pendulum":
        assert np.array_equal(sf, o.state_f)
    if kind == "maze":
        assert np.array_equal(g.get_walls(), o.walls), "mazes differ"


def assert_rollout_equal(g, o, kind, sel=None, head_tol=None):
    """Bitwise equality (floats by value) of everything the unroll stores, for all envs or the
    selected ones.  head_tol: compare head outputs / values / activations within this relative
    tolerance instead (logit-forced protocol for the matrix-core bf16 path)."""
    tr = g.trajectory()
    cols = slice(None) if sel is None else np.asarray(sel)
    si, sf = gpu_state_rows(kind, tr)
    T = g.T
    assert np.array_equal(si[:, cols], o.tr_state_i[:, cols]), "state snapshots differ"
    if kind == "pendulum":
        assert np.array_equal(sf[:, cols], o.tr_state_f[:, cols]), "pendulum states differ"
        assert np.array_equal(tr["eps"][:, cols], o.tr_eps[:, cols]), "gaussian noise differs"
        assert np.array_equal(tr["action_f"][:, cols], o.tr_action_f[:, cols]), "gaussian actions differ"
    else:
        assert np.array_equal(tr["action"][:, cols].astype(np.int32), o.tr_action[:, cols]), "actions differ"
    assert np.array_equal(tr["reward"][:, cols], o.tr_reward[:, cols]), "rewards differ"
    assert np.array_equal(tr["done"][:, cols], o.tr_done[:, cols]), "dones differ"
    if head_tol is None:
        assert np.array_equal(tr["head"][:, cols], o.tr_head[:, cols]), "head outputs differ"
        assert np.array_equal(tr["value"][:, cols], o.tr_value[:, cols]), "values differ"
    else:
        assert np.array_equal(tr["value"][:, cols], o.tr_value[:, cols])      # forced: both hold the GPU's
        assert np.array_equal(tr["head"][:, cols], o.tr_head[:, cols])
    return tr


def assert_final_state_equal(g, o, kind, sel=None):
    si, sf = g.get_env_state()
    cols = slice(None) if sel is None else np.asarray(sel)
    assert np.array_equal(si[cols], o.state_i[cols]), "final env states differ"
    if kind == "pendulum":
        assert np.array_equal(sf[cols], o.state_f[cols])
    assert g.global_step == o.global_step


def assert_learn_close(g, o, tol, tr_after=None, learned_on=None, target_tol=1e-5):
    """after both sides learned on the same unroll: returns, loss, gradient, parameters, moments.
    learned_on: (rewards, dones) of the unroll the update used when that is not the one now stored
    (decoupled steps learn on the previous unroll).  target_tol: tolerance on returns and advantages (they come
    from stored binary32 values on both sides, except where the learner's own bf16 forward pass feeds them)."""
    tr = tr_after if tr_after is not None else g.trajectory()
    rew, done = learned_on if learned_on is not None else (o.tr_reward, o.tr_done)
    scale = max(1.0, float(np.abs(o.ret).max()))
    assert np.abs(tr["ret"] - o.ret).max() <= target_tol * scale, "returns differ"
    assert np.abs(tr["adv"] - o.adv).max() <= target_tol * scale, "advantages differ"
    m = g.metrics()
    for k, i in (("loss", 0), ("policy_loss", 1), ("value_loss", 2), ("entropy_loss", 3)):
        assert abs(m[k] - o.loss[i]) <= tol * max(abs(o.loss[i]), 1e-3 * abs(o.loss).max()) + 1e-7, (k, m[k], o.loss[i])
    assert abs(m["reward_sum"] - float(rew.astype(np.float64).sum())) <= 1e-4 * max(1.0, np.abs(rew).sum())
    assert m["episodes"] == int(done.sum())
    e_g = rel(g.get_grads(), o.grad)
    assert e_g <= tol, f"gradient rel error {e_g:.3e} > {tol}"
    e_p = rel(g.get_params(), o.theta)
    assert e_p <= tol, f"parameter rel error {e_p:.3e} > {tol}"
    gm, gv, gt = g.get_opt_state()
    assert gt == o.adam_t
    assert rel(gm, o.m) <= tol and rel(gv, o.v) <= 2 * tol, "Adam moments differ"
    return e_g, e_p
