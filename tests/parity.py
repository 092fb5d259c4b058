"""Helpers shared by the GPU parity tests: compare one GPU agent with one oracle
agent built from the same workload dict and seed."""
import threading

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
    """parameter-synchronised comparison: the oracle takes the GPU's parameters and optimiser state.
    The values are also kept on the oracle object, so that the check after the update can replay the
    optimiser step from them."""
    o.theta[:] = g.get_params()
    m, v, t = g.get_opt_state()
    o.m[:] = m; o.v[:] = v; o.adam_t = t
    o.before_update = (o.theta.copy(), o.m.copy(), o.v.copy(), t)


def assert_same_init(g, o, kind):
    assert np.array_equal(g.get_params(), o.theta), "initial parameters differ"
    si, sf = g.get_env_state()
    assert np.array_equal(si, o.state_i), "initial env states differ"
    if kind == "pendulum":
        assert np.array_equal(sf, o.state_f)
    if kind == "maze":
        assert np.array_equal(g.get_walls(), o.walls), "mazes differ"


def assert_rollout_equal(g, o, kind, sel=None, forced=False):
    """Bitwise equality (floats by value) of everything the unroll stores, for all envs or the
    selected ones.  forced: the oracle sampled from the GPU's head outputs (logit-forced protocol
    for the matrix-core bf16 path), so heads and values are not compared here -- assert_heads_close
    compares them with the oracle's own forward pass."""
    tr = g.trajectory()
    cols = slice(None) if sel is None else np.asarray(sel)
    si, sf = gpu_state_rows(kind, tr)
    assert np.array_equal(si[:, cols], o.tr_state_i[:, cols]), "state snapshots differ"
    if kind == "pendulum":
        assert np.array_equal(sf[:, cols], o.tr_state_f[:, cols]), "pendulum states differ"
        assert np.array_equal(tr["eps"][:, cols], o.tr_eps[:, cols]), "gaussian noise differs"
        assert np.array_equal(tr["action_f"][:, cols], o.tr_action_f[:, cols]), "gaussian actions differ"
    else:
        assert np.array_equal(tr["action"][:, cols].astype(np.int32), o.tr_action[:, cols]), "actions differ"
    assert np.array_equal(tr["reward"][:, cols], o.tr_reward[:, cols]), "rewards differ"
    assert np.array_equal(tr["done"][:, cols], o.tr_done[:, cols]), "dones differ"
    if not forced:
        assert np.array_equal(tr["head"][:, cols], o.tr_head[:, cols]), "head outputs differ"
        assert np.array_equal(tr["value"][:, cols], o.tr_value[:, cols]), "values differ"
    else:
        # the value row the update reads is the value head's output
        assert np.array_equal(tr["value"][:, cols], tr["head"][:, cols, -1]), "stored values are not the value head"
    return tr


def assert_final_state_equal(g, o, kind, sel=None):
    si, sf = g.get_env_state()
    cols = slice(None) if sel is None else np.asarray(sel)
    assert np.array_equal(si[cols], o.state_i[cols]), "final env states differ"
    if kind == "pendulum":
        assert np.array_equal(sf[cols], o.state_f[cols])
    assert g.global_step == o.global_step


def oracle_forward_at(o, t, b, want_acts=True):
    """the oracle's own acting forward pass on the state env b was in at step t of the stored unroll"""
    keep = (o.state_i[b].copy(), o.state_f[b].copy())
    o.state_i[b] = o.tr_state_i[t, b]; o.state_f[b] = o.tr_state_f[t, b]
    x = o.observe(b)
    o.state_i[b], o.state_f[b] = keep
    return o.forward(x, want_acts=want_acts)


def assert_heads_close(g, o, tr, tol, sel=None, act_tol=2.0 ** -6):
    """Logit-forced protocol, step (1): the GPU's head outputs at EVERY (t, b) of the selected envs (all envs when
    sel is None) against the oracle's own sequential forward pass on the same state, within tol of the head
    outputs' scale; the stored hidden activations within act_tol of theirs (one bfloat16 step is 2^-8 of the
    element; a different accumulation order moves a few elements by one step, deeper layers by a little more)."""
    cols = range(g.B) if sel is None else [int(b) for b in sel]
    scale = max(1e-3, float(np.abs(tr["head"]).max()))
    worst = 0.0
    for b in cols:
        for t in range(g.T + 1):
            head, acts = oracle_forward_at(o, t, b)
            worst = max(worst, float(np.abs(head - tr["head"][t, b]).max()) / scale)
            if t < g.T and tr["act"]:
                got = np.concatenate([a[t, b] for a in tr["act"]])
                assert np.abs(got - acts).max() <= act_tol * max(1.0, float(np.abs(acts).max())), f"activations differ at t={t} b={b}"
    assert worst <= tol, f"head outputs differ by {worst:.3e} of their scale"
    return worst


def param_regions(cfg):
    """[(name, slice)] over the flat parameter vector: every weight matrix and every bias vector on its own;
    the maze's first-layer matrix as its wall / agent / goal row blocks (they are reduced by different kernels)."""
    e, hid = cfg["env"], list(cfg["net"]["hidden"])
    kind = e["kind"]
    cells = e.get("rows", 0) * e.get("cols", 0)
    D = {"catch": cells, "pendulum": 3, "maze": 3 * cells}[kind]
    NH = 3 if kind == "pendulum" else ({"catch": 3, "maze": 4}[kind] + 1)
    dims = [D] + hid
    out, off = [], 0
    for l in range(len(hid)):
        K, N = dims[l], dims[l + 1]
        if l == 0 and kind == "maze":
            for i, plane in enumerate(("walls", "agent", "goal")):
                out.append((f"W1[{plane}]", slice(off + i * cells * N, off + (i + 1) * cells * N)))
        else:
            out.append((f"W{l + 1}", slice(off, off + K * N)))
        off += K * N
        out.append((f"b{l + 1}", slice(off, off + N))); off += N
    out.append(("Wh", slice(off, off + dims[-1] * NH))); off += dims[-1] * NH
    out.append(("bh", slice(off, off + NH))); off += NH
    return out, off


def assert_regions_close(name, got, ref, regions, tol, skip=None, elem_factor=1.0):
    """per parameter region: relative l2 error <= tol and max |difference| <= elem_factor * tol * max |reference|.
    skip: boolean mask of elements left out (see assert_learn_close).  Returns the worst relative l2 error."""
    got = np.asarray(got, np.float64); ref = np.asarray(ref, np.float64)
    worst = 0.0
    for rname, sl in regions:
        a, b = got[sl], ref[sl]
        if skip is not None:
            keep = ~skip[sl]
            a, b = a[keep], b[keep]
        if b.size == 0:
            continue
        top = np.abs(b).max()
        if top == 0.0:
            assert np.abs(a).max() <= 1e-12, f"{name} {rname}: reference is zero, got {np.abs(a).max():.3e}"
            continue
        e2 = np.linalg.norm(a - b) / np.linalg.norm(b)
        emax = np.abs(a - b).max() / top
        assert e2 <= tol, f"{name} {rname}: relative l2 error {e2:.3e} > {tol}"
        assert emax <= elem_factor * tol, f"{name} {rname}: max element error {emax:.3e} of the region's largest entry > {elem_factor * tol}"
        worst = max(worst, e2)
    return worst


def assert_learn_close(g, o, tol, tr_after=None, learned_on=None, target_tol=1e-5, n_updates=1, elem_factor=1.0):
    """after both sides learned on the same unroll: returns, loss, then per parameter region (param_regions)
    the gradient, the parameters and the Adam moments, each as a relative l2 norm and as the largest element
    error relative to the region's largest entry.
    learned_on: (rewards, dones) of the unroll the update used when that is not the one now stored
    (decoupled steps learn on the previous unroll).  target_tol: tolerance on returns and advantages (they come
    from stored binary32 values on both sides, except where the learner's own bf16 forward pass feeds them).
    n_updates: Adam steps this update applied (with several, only the last gradient is visible, so the
    optimiser step is not replayed).  elem_factor: widens the element-wise bounds only (a case whose per-sample
    terms cancel almost completely has binary32 summation noise above tol of the largest entry)."""
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
    regions, P = param_regions(g.cfg)
    assert P == g.P
    g_gpu, g_ref = g.get_grads(), o.grad
    e_g = rel(g_gpu, g_ref)
    assert e_g <= tol, f"gradient rel error {e_g:.3e} > {tol}"
    assert_regions_close("gradient", g_gpu, g_ref, regions, tol, elem_factor=elem_factor)
    th_gpu = g.get_params()
    gm, gv, gt = g.get_opt_state()
    assert gt == o.adam_t
    net = g.cfg["net"]
    pre = getattr(o, "before_update", None)
    if pre is not None and n_updates == 1 and pre[3] + 1 == gt:
        # the optimiser step on its own, element by element: Adam in binary64 (the oracle's routine) on the GPU's
        # own gradient, from the parameters and moments both sides started the update with
        th0, m0, v0, t0 = pre
        th_x, m_x, v_x = th0.copy(), m0.copy(), v0.copy()
        from oracle import oracle as O
        f32 = lambda x: float(np.float32(x))
        O.adam(th_x, g_gpu, m_x, v_x, gt, f32(net["lr"]), f32(net["beta1"]), f32(net["beta2"]), f32(net["eps"]))
        assert np.abs(th_gpu.astype(np.float64) - th_x).max() <= 2.0 ** -22 * np.abs(th_x).max() + 1e-4 * net["lr"], "Adam step differs from binary64 Adam on the same gradient"
        assert np.abs(gm - m_x).max() <= 1e-6 * max(np.abs(m_x).max(), 1e-30), "first moment differs"
        assert np.abs(gv - v_x).max() <= 1e-6 * max(np.abs(v_x).max(), 1e-30), "second moment differs"
    # parameters against the oracle's.  An Adam step is lr * m_hat / (sqrt(v_hat) + eps), whose sensitivity to a
    # gradient entry is inversely proportional to that entry: where the GPU's gradient entry is within the region's
    # tolerance (checked above) but not within tol of the entry itself, the step is not determined to tol (its sign
    # may differ: 2 lr).  Those entries are covered by the gradient check and by the replayed optimiser step; the
    # element-wise parameter comparison leaves them out.
    fragile = np.abs(g_gpu.astype(np.float64) - g_ref) > tol * np.abs(g_ref)
    assert fragile.mean() <= 0.25, f"{fragile.mean():.2%} of the gradient entries are off by more than tol of themselves"
    e_p = rel(th_gpu, o.theta)
    assert e_p <= tol, f"parameter rel error {e_p:.3e} > {tol}"
    # with several Adam steps only the last gradient is visible, so the entries whose step the earlier chunks left
    # undetermined cannot be told apart: parameters are then compared by region norms only
    pf = elem_factor if n_updates == 1 else float("inf")
    assert_regions_close("parameters", th_gpu, o.theta, regions, tol, skip=fragile, elem_factor=pf)
    assert rel(gm, o.m) <= tol and rel(gv, o.v) <= 2 * tol, "Adam moments differ"
    assert_regions_close("first moment", gm, o.m, regions, tol, elem_factor=elem_factor)
    assert_regions_close("second moment", gv, o.v, regions, 2 * tol, elem_factor=elem_factor)
    return e_g, e_p


def oracle_learn_parallel(o, workers=16):
    """What o.learn() computes, with the per-sample work (binary64 forward and backward pass of every sample, the
    part that takes minutes for wide nets) spread over `workers` oracle instances on disjoint, contiguous sample
    ranges, one thread each: returns over the whole unroll, every instance's mean loss and gradient over its own
    range, their sample-weighted sum (binary64), one Adam step.  Each range's gradient passes through binary32 once
    before the sum, which the update tolerances cover by orders of magnitude."""
    from oracle import oracle as O
    net = o.cfg["net"]
    f32 = lambda x: float(np.float32(x))                     # the hyper-parameters are binary32 in the config structs
    ret, adv = O.returns(o.tr_reward, o.tr_done, o.tr_value, f32(net["gamma"]), f32(net["lambda"]))
    o.ret[:] = ret; o.adv[:] = adv
    n = o.T * o.B
    workers = max(1, min(workers, n // 64))
    edges = [n * i // workers for i in range(workers + 1)]
    parts = []
    for i in range(workers):
        c = O.Oracle(o.cfg, B=o.B, T=o.T, seed=0)
        c.theta[:] = o.theta
        c.walls[:] = o.walls
        for arr in ("tr_state_i", "tr_state_f", "tr_action", "tr_z", "tr_eps", "tr_reward", "tr_done", "tr_value", "ret", "adv"):
            getattr(c, arr)[:] = getattr(o, arr)
        parts.append(c)
    threads = [threading.Thread(target=c.loss_and_grad, args=(edges[i], edges[i + 1])) for i, c in enumerate(parts)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    grad = np.zeros(o.P); loss = np.zeros(4)
    for i, c in enumerate(parts):
        w = (edges[i + 1] - edges[i]) / n
        grad += w * c.grad.astype(np.float64); loss += w * c.loss
    o.grad[:] = grad.astype(np.float32); o.loss[:] = loss
    o.adam_t = o.adam_t + 1
    O.adam(o.theta, o.grad, o.m, o.v, o.adam_t, f32(net["lr"]), f32(net["beta1"]), f32(net["beta2"]), f32(net["eps"]))


def bf16_round_np(x):
    """binary32 -> nearest bfloat16 (ties to even), as binary32; finite inputs"""
    u = np.ascontiguousarray(x, np.float32).view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32)


def np_maze_backward_from_stored(cfg, theta, walls, pos, acts, head, action, adv, ret, t_chunk=2):
    """The A2C objective's value and its gradient for a maze net, in binary64 with BLAS products, from a STORED
    forward pass: hidden activations acts[l] [T][B][H_l], head outputs head [T][B][NH], actions, agent cells pos
    [T][B] and wall bits walls [B][cells]; adv and ret [T][B] are constants.  Same objective and same backward rule
    as the oracle's (mean over the T*B samples of -A log pi(a|s) + c_v (G - V)^2 - beta H; ReLU sides from the sign
    of the stored activation; weights as the forward pass saw them, i.e. rounded to bfloat16 when dtype is bf16),
    only arranged as matrix products over blocks of t_chunk time steps so that half a million samples take seconds.
    It is checked against the oracle itself on small cases by the CPU suite, and stands in for it where the oracle
    would need an hour.  Returns (loss[4], grad[P]) in binary64."""
    net = cfg["net"]
    hid = list(net["hidden"])
    L = len(hid)
    T, B = action.shape
    cells = walls.shape[1]
    D = 3 * cells
    dims = [D] + hid
    A = head.shape[2] - 1
    NH = A + 1
    beta, cv = float(np.float32(net["entropy_coef"])), float(np.float32(net["value_coef"]))
    th = np.asarray(theta, np.float32)
    bf = net.get("dtype", "fp32") == "bf16"
    Ws, bs, off = [], [], 0
    w_off, b_off = [], []
    for l in range(L):
        K, N = dims[l], dims[l + 1]
        Wm = th[off:off + K * N]
        Ws.append((bf16_round_np(Wm) if bf else Wm).astype(np.float64).reshape(K, N)); w_off.append(off); off += K * N
        bs.append(th[off:off + N].astype(np.float64)); b_off.append(off); off += N
    wh_off = off
    Whm = th[off:off + hid[-1] * NH]
    Wh = (bf16_round_np(Whm) if bf else Whm).astype(np.float64).reshape(hid[-1], NH); off += hid[-1] * NH
    bh_off = off; off += NH
    P = off
    g = np.zeros(P)
    n_all = T * B
    wallsf = walls.astype(np.float64)                        # [B][cells]
    S = np.zeros((B, hid[0]))                                # sum over time of dZ_1, per env
    gW = [np.zeros((dims[l], dims[l + 1])) for l in range(L)]
    gb = [np.zeros(dims[l + 1]) for l in range(L)]
    gWh = np.zeros((hid[-1], NH)); gbh = np.zeros(NH)
    Lp = Lv = Le = 0.0
    for t0 in range(0, T, t_chunk):
        t1 = min(T, t0 + t_chunk)
        n = (t1 - t0) * B
        hd = head[t0:t1].reshape(n, NH).astype(np.float64)
        a = action[t0:t1].reshape(n).astype(np.int64)
        A_ = adv[t0:t1].reshape(n).astype(np.float64); G_ = ret[t0:t1].reshape(n).astype(np.float64)
        lg = hd[:, :A]
        lp = lg - lg.max(1, keepdims=True)
        lp = lp - np.log(np.exp(lp).sum(1, keepdims=True))
        p = np.exp(lp)
        H = -(p * lp).sum(1)
        V = hd[:, A]
        Lp += float((-A_ * lp[np.arange(n), a]).sum()); Lv += float((cv * (G_ - V) ** 2).sum()); Le += float((-beta * H).sum())
        onehot = np.zeros((n, A)); onehot[np.arange(n), a] = 1.0
        dhead = np.empty((n, NH))
        dhead[:, :A] = (-A_[:, None] * (onehot - p) + beta * p * (lp + H[:, None])) / n_all
        dhead[:, A] = -2.0 * cv * (G_ - V) / n_all
        hs = [acts[l][t0:t1].reshape(n, hid[l]).astype(np.float64) for l in range(L)]
        gWh += hs[-1].T @ dhead; gbh += dhead.sum(0)
        dz = (hs[-1] > 0) * (dhead @ Wh.T)
        for l in range(L - 1, 0, -1):
            gW[l] += hs[l - 1].T @ dz; gb[l] += dz.sum(0)
            dz = (hs[l - 1] > 0) * (dz @ Ws[l].T)
        gb[0] += dz.sum(0)
        S += dz.reshape(t1 - t0, B, hid[0]).sum(0)
        oh = np.zeros((cells, n)); oh[pos[t0:t1].reshape(n), np.arange(n)] = 1.0
        gW[0][cells:2 * cells] += oh @ dz
    gW[0][:cells] = wallsf.T @ S
    gW[0][2 * cells + cells - 1] = gb[0]                     # the goal plane has its one at the last cell, always
    for l in range(L):
        g[w_off[l]:w_off[l] + gW[l].size] = gW[l].ravel()
        g[b_off[l]:b_off[l] + gb[l].size] = gb[l]
    g[wh_off:wh_off + gWh.size] = gWh.ravel()
    g[bh_off:bh_off + NH] = gbh
    loss = np.array([Lp + Lv + Le, Lp, Lv, Le]) / n_all
    return loss, g


def np_maze_forward_layers_from_stored(cfg, theta, walls, pos, acts, t_chunk=2):
    """Every layer of a bf16 maze net's acting forward pass on its own, in binary64 with BLAS products, each from
    the STORED input of that layer: hidden layer 1 from the observation (wall bits of the env, agent cell pos[t][b],
    goal at the last cell), hidden layer l from the stored acts[l-2], the heads from the stored last activations --
    with the rounding points of the bf16 forward pass (weights and layer outputs rounded to bfloat16, biases and
    heads binary32/64).  Yields (t0, t1, [reference of acts[0], ..., acts[L-1]], reference heads) per block of
    time steps.  Because every layer starts from what the GPU stored, a difference is that layer's own."""
    net = cfg["net"]
    assert net.get("dtype") == "bf16"
    hid = list(net["hidden"])
    L = len(hid)
    T, B = pos.shape
    cells = walls.shape[1]
    dims = [3 * cells] + hid
    th = np.asarray(theta, np.float32)
    Ws, bs, off = [], [], 0
    for l in range(L):
        K, N = dims[l], dims[l + 1]
        Ws.append(bf16_round_np(th[off:off + K * N]).astype(np.float64).reshape(K, N)); off += K * N
        bs.append(th[off:off + N].astype(np.float64)); off += N
    NH = (th.size - off) // (hid[-1] + 1)
    Wh = bf16_round_np(th[off:off + hid[-1] * NH]).astype(np.float64).reshape(hid[-1], NH); off += hid[-1] * NH
    bh = th[off:off + NH].astype(np.float64)
    # the part of layer 1 that does not change within an unroll: bias + wall rows + goal row, per env
    prefix = bs[0] + walls.astype(np.float64) @ Ws[0][:cells] + Ws[0][2 * cells + cells - 1]
    for t0 in range(0, T, t_chunk):
        t1 = min(T, t0 + t_chunk)
        n = (t1 - t0) * B
        y = np.tile(prefix, (t1 - t0, 1)) + Ws[0][cells + pos[t0:t1].reshape(n)]
        refs = [bf16_round_np(np.maximum(y, 0).astype(np.float32))]
        for l in range(1, L):
            x = acts[l - 1][t0:t1].reshape(n, hid[l - 1]).astype(np.float64)
            refs.append(bf16_round_np(np.maximum(x @ Ws[l] + bs[l], 0).astype(np.float32)))
        heads = acts[L - 1][t0:t1].reshape(n, hid[-1]).astype(np.float64) @ Wh + bh
        yield t0, t1, [r.reshape(t1 - t0, B, -1) for r in refs], heads.reshape(t1 - t0, B, NH)


def assert_bf16_layers_close(name, got, ref):
    """stored bfloat16 activations against their reference: equal, or one bfloat16 step apart where the two
    accumulation orders round the sum to different neighbours (a small share of the entries; a sum within rounding
    of zero may sit on either side of the ReLU).  Returns the share of entries that differ."""
    got = np.asarray(got, np.float32); ref = np.asarray(ref, np.float32)
    d = np.abs(got - ref)
    step = 2.0 ** -7 * np.maximum(np.abs(ref), np.abs(got))          # one step of an 8-bit significand, at most
    bad = d > step + 1e-6
    assert not bad.any(), f"{name}: {int(bad.sum())} entries differ by more than one bfloat16 step (worst {d.max():.3e})"
    share = float((d > 0).mean())
    assert share <= 0.02, f"{name}: {share:.2%} of the entries differ"
    return share
