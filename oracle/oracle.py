"""ctypes binding of the CPU oracle (TEST INFRASTRUCTURE, not product code).

Only tests, the smoke check and the benchmark's CPU-baseline leg may import
this module.  It never imports the GPU package, and the GPU package never
imports it.
"""
import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "anakin_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

CFLAGS = ["-O2", "-std=c99", "-ffp-contract=off", "-mfma", "-Wall", "-shared", "-fPIC"]


def build(force=False):
    """Compile the oracle with gcc (no fast-math, no contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", *CFLAGS, "-o", _LIB, _SRC, "-lm"])
    return _LIB


class EnvCfg(C.Structure):
    _fields_ = [("kind", C.c_int32), ("rows", C.c_int32), ("cols", C.c_int32),
                ("max_steps", C.c_int32), ("p_wall", C.c_float)]


class NetCfg(C.Structure):
    _fields_ = [("n_hidden", C.c_int32), ("hidden", C.c_int32 * 4), ("policy", C.c_int32),
                ("dtype", C.c_int32), ("gamma", C.c_float), ("lambda_", C.c_float),
                ("entropy_coef", C.c_float), ("value_coef", C.c_float), ("lr", C.c_float),
                ("beta1", C.c_float), ("beta2", C.c_float), ("eps", C.c_float)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(_LIB)
        f32p, u32p, i32p, u8p, f64p = (C.POINTER(t) for t in
                                       (C.c_float, C.c_uint32, C.c_int32, C.c_uint8, C.c_double))
        L.orc_philox4x32_10.argtypes = [u32p, u32p, u32p]
        L.orc_philox4x32_10.restype = None
        for name in ("orc_exp", "orc_log", "orc_sin", "orc_cos", "orc_cos2pi", "orc_tanh", "orc_bf16_round"):
            getattr(L, name).argtypes = [C.c_float]
            getattr(L, name).restype = C.c_float
        L.orc_u01.argtypes = [C.c_uint32]; L.orc_u01.restype = C.c_float
        L.orc_u01_plus.argtypes = [C.c_uint32]; L.orc_u01_plus.restype = C.c_float
        L.orc_bounded.argtypes = [C.c_uint32, C.c_uint32]; L.orc_bounded.restype = C.c_uint32
        L.orc_sample_categorical.argtypes = [f32p, C.c_int, C.c_float]
        L.orc_sample_categorical.restype = C.c_int
        L.orc_sample_gaussian.argtypes = [C.c_float, C.c_float, C.c_uint32, C.c_uint32, f32p, f32p, f32p]
        L.orc_sample_gaussian.restype = None
        L.orc_create.argtypes = [C.POINTER(EnvCfg), C.POINTER(NetCfg), C.c_int, C.c_int, C.c_uint64]
        L.orc_create.restype = C.c_void_p
        L.orc_destroy.argtypes = [C.c_void_p]; L.orc_destroy.restype = None
        for name, rt in (("orc_param_count", C.c_int64), ("orc_obs_dim", C.c_int), ("orc_num_heads", C.c_int),
                         ("orc_act_width", C.c_int64), ("orc_global_step", C.c_uint64), ("orc_get_adam_t", C.c_int)):
            getattr(L, name).argtypes = [C.c_void_p]; getattr(L, name).restype = rt
        L.orc_set_global_step.argtypes = [C.c_void_p, C.c_uint64]; L.orc_set_global_step.restype = None
        L.orc_set_adam_t.argtypes = [C.c_void_p, C.c_int]; L.orc_set_adam_t.restype = None
        for name, rt in (("orc_theta", f32p), ("orc_grad", f32p), ("orc_adam_m", f64p), ("orc_adam_v", f64p),
                         ("orc_state_i", i32p), ("orc_state_f", f32p), ("orc_walls", u32p),
                         ("orc_traj_state_i", i32p), ("orc_traj_state_f", f32p), ("orc_traj_action", i32p),
                         ("orc_traj_action_f", f32p), ("orc_traj_eps", f32p), ("orc_traj_z", f32p),
                         ("orc_traj_reward", f32p), ("orc_traj_done", u8p), ("orc_traj_value", f32p),
                         ("orc_traj_head", f32p), ("orc_adv", f64p), ("orc_ret", f64p), ("orc_loss", f64p),
                         ("orc_cur_head", f64p), ("orc_rho", f64p)):
            getattr(L, name).argtypes = [C.c_void_p]; getattr(L, name).restype = rt
        L.orc_observe.argtypes = [C.c_void_p, C.c_int, f32p]; L.orc_observe.restype = None
        L.orc_forward.argtypes = [C.c_void_p, f32p, f32p, f32p]; L.orc_forward.restype = None
        L.orc_env_step.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_float, C.c_uint64, f32p, i32p]
        L.orc_env_step.restype = None
        L.orc_rollout.argtypes = [C.c_void_p, f32p]; L.orc_rollout.restype = None
        L.orc_rollout_sel.argtypes = [C.c_void_p, f32p, i32p, C.c_int]; L.orc_rollout_sel.restype = None
        L.orc_returns.argtypes = [C.c_int, C.c_int, f32p, u8p, f32p, C.c_double, C.c_double, f64p, f64p]
        L.orc_returns.restype = None
        L.orc_loss_and_grad.argtypes = [C.c_void_p]; L.orc_loss_and_grad.restype = None
        L.orc_loss_and_grad_range.argtypes = [C.c_void_p, C.c_int64, C.c_int64]; L.orc_loss_and_grad_range.restype = C.c_int
        L.orc_surrogate_loss.argtypes = [C.c_void_p]; L.orc_surrogate_loss.restype = C.c_double
        L.orc_adam.argtypes = [C.c_int64, f32p, f32p, f64p, f64p, C.c_int, C.c_double, C.c_double,
                               C.c_double, C.c_double]
        L.orc_adam.restype = None
        L.orc_learn.argtypes = [C.c_void_p]; L.orc_learn.restype = C.c_int
        L.orc_learn_n.argtypes = [C.c_void_p, C.c_int]; L.orc_learn_n.restype = C.c_int
        L.orc_learn_n_sequential.argtypes = [C.c_void_p, C.c_int]; L.orc_learn_n_sequential.restype = C.c_int
        L.orc_step.argtypes = [C.c_void_p]; L.orc_step.restype = None
        L.orc_vtrace_targets.argtypes = [C.c_void_p, C.c_double, C.c_double]; L.orc_vtrace_targets.restype = None
        L.orc_learn_vtrace.argtypes = [C.c_void_p, C.c_double, C.c_double]; L.orc_learn_vtrace.restype = C.c_int
        L.orc_step_decoupled.argtypes = [C.c_void_p]; L.orc_step_decoupled.restype = None
        L.orc_step_decoupled_forced.argtypes = [C.c_void_p, f32p]; L.orc_step_decoupled_forced.restype = None
        L.orc_pathwise_grad.argtypes = [C.c_void_p, f64p, f64p]; L.orc_pathwise_grad.restype = None
        L.orc_learn_pathwise.argtypes = [C.c_void_p]; L.orc_learn_pathwise.restype = C.c_int
        _lib = L
    return _lib


def _ptr(a, ct):
    return a.ctypes.data_as(C.POINTER(ct))


def _view(p, shape, dtype):
    n = int(np.prod(shape))
    if n == 0:
        return np.zeros(shape, dtype)
    return np.ctypeslib.as_array(p, shape=(n,)).view(dtype).reshape(shape)


ENV_KINDS = {"catch": 0, "pendulum": 1, "maze": 2}
POLICIES = {"categorical": 0, "tanh_gaussian": 1}
DTYPES = {"fp32": 0, "bf16": 1}


def make_cfgs(cfg):
    """cfg: a plain dict as in the workload table (env / net sub-dicts)."""
    e, n = cfg["env"], cfg["net"]
    env = EnvCfg(ENV_KINDS[e["kind"]], e.get("rows", 0), e.get("cols", 0), e.get("max_steps", 0),
                 float(e.get("p_wall", 0.0)))
    hid = list(n["hidden"]) + [0] * (4 - len(n["hidden"]))
    net = NetCfg(len(n["hidden"]), (C.c_int32 * 4)(*hid), POLICIES[n["policy"]], DTYPES[n.get("dtype", "fp32")],
                 n["gamma"], n["lambda"], n["entropy_coef"], n["value_coef"], n["lr"], n["beta1"], n["beta2"],
                 n["eps"])
    return env, net


def philox(ctr, key):
    c = np.asarray(ctr, np.uint32).copy(); k = np.asarray(key, np.uint32).copy()
    out = np.zeros(4, np.uint32)
    lib().orc_philox4x32_10(_ptr(c, C.c_uint32), _ptr(k, C.c_uint32), _ptr(out, C.c_uint32))
    return out


def draw(seed, index, t, domain):
    return philox([index, t & 0xFFFFFFFF, t >> 32, domain], [seed & 0xFFFFFFFF, seed >> 32])


def f32fun(name):
    f = getattr(lib(), name)
    return lambda xs: np.array([f(float(x)) for x in np.asarray(xs, np.float32).ravel()], np.float32)


def returns(rew, done, val, gamma, lam):
    T, B = rew.shape
    rew = np.ascontiguousarray(rew, np.float32); done = np.ascontiguousarray(done, np.uint8)
    val = np.ascontiguousarray(val, np.float32)
    ret = np.zeros((T, B)); adv = np.zeros((T, B))
    lib().orc_returns(T, B, _ptr(rew, C.c_float), _ptr(done, C.c_uint8), _ptr(val, C.c_float),
                      gamma, lam, _ptr(ret, C.c_double), _ptr(adv, C.c_double))
    return ret, adv


def adam(theta, grad, m, v, t, lr, b1, b2, eps):
    """In-place on theta (f32), m, v (f64)."""
    lib().orc_adam(theta.size, _ptr(theta, C.c_float), _ptr(np.ascontiguousarray(grad, np.float32), C.c_float),
                   _ptr(m, C.c_double), _ptr(v, C.c_double), t, lr, b1, b2, eps)


def sample_categorical(logits, u):
    lg = np.ascontiguousarray(logits, np.float32)
    return lib().orc_sample_categorical(_ptr(lg, C.c_float), lg.size, float(np.float32(u)))


def sample_gaussian(mu, log_sigma, w0, w1):
    e, z, a = C.c_float(), C.c_float(), C.c_float()
    lib().orc_sample_gaussian(float(mu), float(log_sigma), int(w0), int(w1), C.byref(e), C.byref(z), C.byref(a))
    return e.value, z.value, a.value


class Oracle:
    """One oracle agent: B envs, a network, an optimiser state."""

    def __init__(self, cfg, B=None, T=None, seed=0):
        self.L = lib()
        self.cfg = cfg
        self.B = int(B if B is not None else cfg["B"])
        self.T = int(T if T is not None else cfg["T"])
        env, net = make_cfgs(cfg)
        self.h = self.L.orc_create(C.byref(env), C.byref(net), self.B, self.T, seed)
        if not self.h:
            raise ValueError("oracle rejected the configuration")
        self.P = self.L.orc_param_count(self.h)
        self.D = self.L.orc_obs_dim(self.h)
        self.NH = self.L.orc_num_heads(self.h)
        self.AW = self.L.orc_act_width(self.h)
        B, T, NH, P = self.B, self.T, self.NH, self.P
        g = lambda name, shape, dt: _view(getattr(self.L, name)(self.h), shape, dt)
        self.theta = g("orc_theta", (P,), np.float32)
        self.grad = g("orc_grad", (P,), np.float32)
        self.m = g("orc_adam_m", (P,), np.float64)
        self.v = g("orc_adam_v", (P,), np.float64)
        self.state_i = g("orc_state_i", (B, 4), np.int32)
        self.state_f = g("orc_state_f", (B, 2), np.float32)
        self.walls = g("orc_walls", (B, 8), np.uint32)
        self.tr_state_i = g("orc_traj_state_i", (T + 1, B, 4), np.int32)
        self.tr_state_f = g("orc_traj_state_f", (T + 1, B, 2), np.float32)
        self.tr_action = g("orc_traj_action", (T, B), np.int32)
        self.tr_action_f = g("orc_traj_action_f", (T, B), np.float32)
        self.tr_eps = g("orc_traj_eps", (T, B), np.float32)
        self.tr_z = g("orc_traj_z", (T, B), np.float32)
        self.tr_reward = g("orc_traj_reward", (T, B), np.float32)
        self.tr_done = g("orc_traj_done", (T, B), np.uint8)
        self.tr_value = g("orc_traj_value", (T + 1, B), np.float32)
        self.tr_head = g("orc_traj_head", (T + 1, B, NH), np.float32)
        self.adv = g("orc_adv", (T, B), np.float64)
        self.ret = g("orc_ret", (T, B), np.float64)
        self.loss = g("orc_loss", (4,), np.float64)
        self.cur_head = g("orc_cur_head", (T + 1, B, NH), np.float64)
        self.rho = g("orc_rho", (T, B), np.float64)

    def __del__(self):
        try:
            if self.h:
                self.L.orc_destroy(self.h)
                self.h = None
        except Exception:
            pass

    @property
    def global_step(self):
        return self.L.orc_global_step(self.h)

    @global_step.setter
    def global_step(self, g):
        self.L.orc_set_global_step(self.h, int(g))

    @property
    def adam_t(self):
        return self.L.orc_get_adam_t(self.h)

    @adam_t.setter
    def adam_t(self, t):
        self.L.orc_set_adam_t(self.h, int(t))

    def observe(self, b):
        x = np.zeros(self.D, np.float32)
        self.L.orc_observe(self.h, b, _ptr(x, C.c_float))
        return x

    def forward(self, x, want_acts=False):
        x = np.ascontiguousarray(x, np.float32)
        head = np.zeros(self.NH, np.float32)
        acts = np.zeros(self.AW, np.float32) if want_acts else None
        self.L.orc_forward(self.h, _ptr(x, C.c_float), _ptr(head, C.c_float),
                           _ptr(acts, C.c_float) if want_acts else None)
        return (head, acts) if want_acts else head

    def env_step(self, b, action=0, action_f=0.0, t=0):
        r = C.c_float(); d = C.c_int32()
        self.L.orc_env_step(self.h, b, int(action), float(action_f), int(t), C.byref(r), C.byref(d))
        return r.value, d.value

    def rollout(self, forced_head=None, sel=None):
        """forced_head: [T+1][B][NH] head outputs to sample from instead of the oracle's own forward.
        sel: env indices to roll out (others untouched; learn is then unavailable)."""
        fh = None
        if forced_head is not None:
            fh = np.ascontiguousarray(forced_head, np.float32)
            assert fh.shape == (self.T + 1, self.B, self.NH)
        fhp = _ptr(fh, C.c_float) if fh is not None else None
        if sel is not None:
            ids = np.ascontiguousarray(sel, np.int32)
            self.L.orc_rollout_sel(self.h, fhp, _ptr(ids, C.c_int32), ids.size)
        else:
            self.L.orc_rollout(self.h, fhp)

    def learn(self):
        rc = self.L.orc_learn(self.h)
        if rc != 0:
            raise RuntimeError("learn without a stored trajectory")

    def learn_n(self, n_updates, sequential=False):
        """N Adam updates on the stored unroll, one per consecutive time chunk: gradients at the acting-time
        parameters, or (sequential) chunk k's at the parameters after the k previous updates."""
        fn = self.L.orc_learn_n_sequential if sequential else self.L.orc_learn_n
        rc = fn(self.h, int(n_updates))
        if rc != 0:
            raise RuntimeError("learn_n: no stored trajectory" if rc == -1 else "learn_n: T is not a multiple of n_updates")

    def loss_and_grad(self, begin=None, end=None):
        """loss[] and grad of the stored unroll at the current parameters with the adv / ret now held;
        begin, end: only the samples begin <= t*B + b < end (their own mean)."""
        if begin is None and end is None:
            self.L.orc_loss_and_grad(self.h)
        elif self.L.orc_loss_and_grad_range(self.h, int(begin), int(end)) != 0:
            raise ValueError("sample range outside the unroll")

    def surrogate_loss(self):
        return self.L.orc_surrogate_loss(self.h)

    def step(self):
        self.L.orc_step(self.h)

    def vtrace_targets(self, rho_bar=1.0, c_bar=1.0):
        """Fills ret (v_t), adv (the policy-gradient advantage), rho and cur_head for the stored trajectory
        at the current parameters."""
        self.L.orc_vtrace_targets(self.h, float(rho_bar), float(c_bar))

    def learn_vtrace(self, rho_bar=1.0, c_bar=1.0):
        if self.L.orc_learn_vtrace(self.h, float(rho_bar), float(c_bar)) != 0:
            raise RuntimeError("learn_vtrace without a stored trajectory")

    def pathwise_grad(self):
        """Gradient of L_path = -mean reward of the stored unroll through env and policy (binary64), and
        dL_path/d(mu, log_sigma) per sample."""
        g = np.zeros(self.P); ph = np.zeros((self.T, self.B, 2))
        self.L.orc_pathwise_grad(self.h, _ptr(g, C.c_double), _ptr(ph, C.c_double))
        return g, ph

    def learn_pathwise(self):
        rc = self.L.orc_learn_pathwise(self.h)
        if rc != 0:
            raise RuntimeError("learn_pathwise: no stored trajectory" if rc == -1 else "learn_pathwise: pendulum with the tanh-Gaussian policy only")

    def step_decoupled(self, forced_head=None):
        """Actor unroll with the parameters as they are now, learner update on the previous unroll.
        forced_head: as in rollout (the actor samples from these head outputs)."""
        if forced_head is None:
            self.L.orc_step_decoupled(self.h)
        else:
            fh = np.ascontiguousarray(forced_head, np.float32)
            assert fh.shape == (self.T + 1, self.B, self.NH)
            self.L.orc_step_decoupled_forced(self.h, _ptr(fh, C.c_float))
