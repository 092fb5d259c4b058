"""Thin ctypes binding of libanakin.so: argument marshalling only.

PyTorch is used for exactly two things: allocating the device workspace and
providing the HIP stream.  Every step of the actor-learner path runs inside the
library's HIP kernels; there is no CPU or PyTorch fallback -- if the library is
missing or no GPU is present the constructors raise.
"""
import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("ANAKIN_LIB", os.path.join(_HERE, "libanakin.so"))

OK = 0
E_INVALID_ARG, E_BAD_CONFIG, E_WORKSPACE_TOO_SMALL, E_MISALIGNED, E_HIP, E_NONFINITE, E_STATE = -1, -2, -3, -4, -5, -6, -7
MODE_VALU_GEMM, MODE_CANONICAL_ACTING, MODE_STREAM_WEIGHTS = 1, 2, 4
PG_SCORE_FUNCTION, PG_PATHWISE = 0, 1
CHUNKS_AT_ACTING_PARAMETERS, CHUNKS_SEQUENTIAL = 0, 1
STATIC_SCRATCH_BYTES = 64 << 20

ENV_KINDS = {"catch": 0, "pendulum": 1, "maze": 2}
POLICIES = {"categorical": 0, "tanh_gaussian": 1}
DTYPES = {"fp32": 0, "bf16": 1}


class EnvCfg(C.Structure):
    _fields_ = [("kind", C.c_int32), ("rows", C.c_int32), ("cols", C.c_int32),
                ("max_steps", C.c_int32), ("p_wall", C.c_float)]


class NetCfg(C.Structure):
    _fields_ = [("n_hidden", C.c_int32), ("hidden", C.c_int32 * 4), ("policy", C.c_int32),
                ("dtype", C.c_int32), ("gamma", C.c_float), ("lambda_", C.c_float),
                ("entropy_coef", C.c_float), ("value_coef", C.c_float), ("lr", C.c_float),
                ("beta1", C.c_float), ("beta2", C.c_float), ("eps", C.c_float)]


_TRAJ_FIELDS = ["state_s0", "state_f0", "state_f1", "action", "eps", "action_f", "reward", "done",
                "value", "head", "adv", "ret"]


class TrajView(C.Structure):
    _fields_ = ([("B", C.c_int32), ("T", C.c_int32), ("num_heads", C.c_int32), ("head_stride", C.c_int32),
                 ("n_hidden", C.c_int32), ("hidden", C.c_int32 * 4), ("act_is_bf16", C.c_int32)]
                + [f for name in _TRAJ_FIELDS for f in ((name, C.c_void_p), ("off_" + name, C.c_size_t))]
                + [("act", C.c_void_p * 4), ("off_act", C.c_size_t * 4)])


class Metrics(C.Structure):
    _fields_ = [("loss", C.c_double), ("policy_loss", C.c_double), ("value_loss", C.c_double),
                ("entropy_loss", C.c_double), ("reward_sum", C.c_double), ("episodes", C.c_int64),
                ("nonfinite", C.c_int32)]


class Plan(C.Structure):
    _fields_ = [("n_hidden", C.c_int32), ("splits", C.c_int32 * 5), ("splits_walls", C.c_int32), ("head_fan", C.c_int32),
                ("dx_rows", C.c_int32 * 4), ("bf16_matrix_path", C.c_int32), ("updates_per_unroll", C.c_int32)]


class KernelTime(C.Structure):
    _fields_ = [("name", C.c_char * 48), ("calls", C.c_int64), ("total_ms", C.c_double)]


EXPORTS = ["anakin_workspace_bytes", "anakin_create", "anakin_rollout", "anakin_learn", "anakin_learn_static", "anakin_step", "anakin_step_decoupled", "anakin_set_actor_stream",
           "anakin_destroy", "anakin_param_count", "anakin_get_params", "anakin_set_params", "anakin_get_grads",
           "anakin_get_opt_state", "anakin_set_opt_state", "anakin_get_env_state", "anakin_set_env_state",
           "anakin_get_walls", "anakin_get_global_step", "anakin_set_global_step", "anakin_get_trajectory",
           "anakin_get_metrics", "anakin_get_plan", "anakin_set_mode", "anakin_set_updates_per_unroll", "anakin_set_update_chunk_mode", "anakin_set_policy_gradient", "anakin_profile", "anakin_kernel_times", "anakin_peak_probe",
           "anakin_last_error"]

_lib = None


class AnakinError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"anakin error {code}: {msg}")
        self.code = code


def load():
    """Load libanakin.so (raises if it has not been built) and declare the signatures."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(f"{LIB_PATH} is missing: run `python -m paper_2104_06272_amd.build` first")
    import torch  # noqa: F401  -- loads the HIP runtime this process will share with the library
    L = C.CDLL(LIB_PATH)
    vp, f32p, i32p, u32p = C.c_void_p, C.POINTER(C.c_float), C.POINTER(C.c_int32), C.POINTER(C.c_uint32)
    L.anakin_workspace_bytes.argtypes = [C.POINTER(EnvCfg), C.POINTER(NetCfg), C.c_int32, C.c_int32]
    L.anakin_workspace_bytes.restype = C.c_size_t
    L.anakin_create.argtypes = [C.POINTER(vp), C.POINTER(EnvCfg), C.POINTER(NetCfg), C.c_int32, C.c_int32,
                                C.c_uint64, vp, C.c_size_t, vp]
    for name in ("anakin_rollout", "anakin_learn", "anakin_step", "anakin_step_decoupled", "anakin_set_actor_stream", "anakin_destroy"):
        getattr(L, name).argtypes = [vp]
    L.anakin_param_count.argtypes = [vp, C.POINTER(C.c_int64)]
    L.anakin_get_params.argtypes = [vp, f32p, C.c_size_t]
    L.anakin_set_params.argtypes = [vp, f32p, C.c_size_t]
    L.anakin_get_grads.argtypes = [vp, f32p, C.c_size_t]
    L.anakin_get_opt_state.argtypes = [vp, f32p, f32p, i32p, C.c_size_t]
    L.anakin_set_opt_state.argtypes = [vp, f32p, f32p, C.c_int32, C.c_size_t]
    L.anakin_get_env_state.argtypes = [vp, i32p, f32p]
    L.anakin_set_env_state.argtypes = [vp, i32p, f32p]
    L.anakin_get_walls.argtypes = [vp, u32p]
    L.anakin_get_global_step.argtypes = [vp, C.POINTER(C.c_uint64)]
    L.anakin_set_global_step.argtypes = [vp, C.c_uint64]
    L.anakin_get_trajectory.argtypes = [vp, C.POINTER(TrajView)]
    L.anakin_get_metrics.argtypes = [vp, C.POINTER(Metrics)]
    L.anakin_get_plan.argtypes = [vp, C.POINTER(Plan)]
    L.anakin_set_actor_stream.argtypes = [vp, vp]
    L.anakin_set_mode.argtypes = [vp, C.c_int32]
    L.anakin_set_updates_per_unroll.argtypes = [vp, C.c_int32]
    L.anakin_set_update_chunk_mode.argtypes = [vp, C.c_int32]
    L.anakin_set_policy_gradient.argtypes = [vp, C.c_int32]
    L.anakin_profile.argtypes = [vp, C.c_int32]
    L.anakin_kernel_times.argtypes = [vp, C.POINTER(KernelTime), C.c_int32, C.POINTER(C.c_int32)]
    L.anakin_last_error.argtypes = [vp]
    L.anakin_last_error.restype = C.c_char_p
    L.anakin_peak_probe.argtypes = [C.c_int32, C.c_int32, vp, C.c_size_t, vp, C.POINTER(C.c_double), C.POINTER(C.c_double)]
    for name in EXPORTS:
        if name not in ("anakin_workspace_bytes", "anakin_last_error"):
            getattr(L, name).restype = C.c_int32
    _lib = L
    return L


def make_cfgs(cfg):
    """cfg: a workload dict (env / net sub-dicts)."""
    e, n = cfg["env"], cfg["net"]
    env = EnvCfg(ENV_KINDS[e["kind"]], e.get("rows", 0), e.get("cols", 0), e.get("max_steps", 0),
                 float(e.get("p_wall", 0.0)))
    hid = list(n["hidden"]) + [0] * (4 - len(n["hidden"]))
    net = NetCfg(len(n["hidden"]), (C.c_int32 * 4)(*hid), POLICIES[n["policy"]], DTYPES[n.get("dtype", "fp32")],
                 n["gamma"], n["lambda"], n["entropy_coef"], n["value_coef"], n["lr"], n["beta1"], n["beta2"],
                 n["eps"])
    return env, net


def workspace_bytes(cfg, B=None, T=None):
    env, net = make_cfgs(cfg)
    return load().anakin_workspace_bytes(C.byref(env), C.byref(net), int(B if B is not None else cfg["B"]),
                                         int(T if T is not None else cfg["T"]))


def _fp(a):
    return a.ctypes.data_as(C.POINTER(C.c_float))


class Anakin:
    """One agent on one GPU: anakin_create / rollout / learn / step plus introspection."""

    def __init__(self, cfg, B=None, T=None, seed=0, device="cuda:0", stream=None):
        import torch
        if not torch.cuda.is_available():
            raise RuntimeError("no GPU: the Anakin path has no CPU fallback")
        self.L = load()
        self.cfg = cfg
        self.B = int(B if B is not None else cfg["B"])
        self.T = int(T if T is not None else cfg["T"])
        env, net = make_cfgs(cfg)
        nbytes = self.L.anakin_workspace_bytes(C.byref(env), C.byref(net), self.B, self.T)
        if nbytes == 0:
            h = C.c_void_p()
            rc = self.L.anakin_create(C.byref(h), C.byref(env), C.byref(net), self.B, self.T, seed, None, 0, None)
            raise AnakinError(rc, self.L.anakin_last_error(None).decode())
        self.device = torch.device(device)
        self.ws = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        self.stream = stream if stream is not None else torch.cuda.current_stream(self.device)
        self.h = C.c_void_p()
        rc = self.L.anakin_create(C.byref(self.h), C.byref(env), C.byref(net), self.B, self.T, int(seed),
                                  C.c_void_p(self.ws.data_ptr()), nbytes, C.c_void_p(self.stream.cuda_stream))
        if rc != OK:
            raise AnakinError(rc, self.L.anakin_last_error(None).decode())
        n = C.c_int64()
        self._chk(self.L.anakin_param_count(self.h, C.byref(n)))
        self.P = n.value
        self._view = None

    def _chk(self, rc):
        if rc != OK:
            raise AnakinError(rc, self.L.anakin_last_error(self.h).decode())

    def close(self):
        if getattr(self, "h", None):
            self.L.anakin_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- the path -------------------------------------------------------------
    def rollout(self):
        self._chk(self.L.anakin_rollout(self.h))

    def learn(self):
        self._chk(self.L.anakin_learn(self.h))

    def learn_static(self):
        self._chk(self.L.anakin_learn_static(self.h))

    def step(self):
        self._chk(self.L.anakin_step(self.h))

    def set_policy_gradient(self, kind):
        self._chk(self.L.anakin_set_policy_gradient(self.h, int(kind)))

    def set_actor_stream(self, stream):
        """stream: a torch.cuda.Stream the actor of step_decoupled runs on (kept alive by this object)"""
        self._chk(self.L.anakin_set_actor_stream(self.h, C.c_void_p(stream.cuda_stream if stream is not None else None)))
        self._actor_stream = stream

    def step_decoupled(self):
        self._chk(self.L.anakin_step_decoupled(self.h))

    def set_mode(self, flags):
        self._chk(self.L.anakin_set_mode(self.h, int(flags)))

    def set_updates_per_unroll(self, n, sequential=None):
        """n Adam updates per unroll; sequential: True / False selects at which parameters chunk gradients are taken
        (anakin_set_update_chunk_mode), None leaves the mode as it is."""
        self._chk(self.L.anakin_set_updates_per_unroll(self.h, int(n)))
        if sequential is not None:
            self._chk(self.L.anakin_set_update_chunk_mode(self.h, CHUNKS_SEQUENTIAL if sequential else CHUNKS_AT_ACTING_PARAMETERS))

    # ---- introspection ----------------------------------------------------------
    def get_params(self):
        a = np.empty(self.P, np.float32)
        self._chk(self.L.anakin_get_params(self.h, _fp(a), self.P))
        return a

    def set_params(self, a):
        a = np.ascontiguousarray(a, np.float32)
        self._chk(self.L.anakin_set_params(self.h, _fp(a), a.size))

    def get_grads(self):
        a = np.empty(self.P, np.float32)
        self._chk(self.L.anakin_get_grads(self.h, _fp(a), self.P))
        return a

    def get_opt_state(self):
        m = np.empty(self.P, np.float32); v = np.empty(self.P, np.float32); t = C.c_int32()
        self._chk(self.L.anakin_get_opt_state(self.h, _fp(m), _fp(v), C.byref(t), self.P))
        return m, v, t.value

    def set_opt_state(self, m, v, t):
        m = np.ascontiguousarray(m, np.float32); v = np.ascontiguousarray(v, np.float32)
        self._chk(self.L.anakin_set_opt_state(self.h, _fp(m), _fp(v), int(t), m.size))

    def get_env_state(self):
        si = np.empty((self.B, 4), np.int32); sf = np.empty((self.B, 2), np.float32)
        self._chk(self.L.anakin_get_env_state(self.h, si.ctypes.data_as(C.POINTER(C.c_int32)), _fp(sf)))
        return si, sf

    def set_env_state(self, si, sf):
        si = np.ascontiguousarray(si, np.int32); sf = np.ascontiguousarray(sf, np.float32)
        self._chk(self.L.anakin_set_env_state(self.h, si.ctypes.data_as(C.POINTER(C.c_int32)), _fp(sf)))

    def get_walls(self):
        w = np.empty((self.B, 8), np.uint32)
        self._chk(self.L.anakin_get_walls(self.h, w.ctypes.data_as(C.POINTER(C.c_uint32))))
        return w

    @property
    def global_step(self):
        g = C.c_uint64()
        self._chk(self.L.anakin_get_global_step(self.h, C.byref(g)))
        return g.value

    @global_step.setter
    def global_step(self, g):
        self._chk(self.L.anakin_set_global_step(self.h, int(g)))

    def metrics(self):
        m = Metrics()
        rc = self.L.anakin_get_metrics(self.h, C.byref(m))
        if rc not in (OK, E_NONFINITE):
            self._chk(rc)
        return {k: getattr(m, k) for k, _ in Metrics._fields_}

    def plan(self):
        p = Plan()
        self._chk(self.L.anakin_get_plan(self.h, C.byref(p)))
        return {"n_hidden": p.n_hidden, "splits": list(p.splits)[:p.n_hidden + 1], "splits_walls": p.splits_walls,
                "head_fan": p.head_fan, "dx_rows": list(p.dx_rows)[:p.n_hidden], "bf16_matrix_path": p.bf16_matrix_path,
                "updates_per_unroll": p.updates_per_unroll}

    def trajectory(self):
        """Host copies (numpy) of the stored unroll; synchronises the stream."""
        import torch
        v = TrajView()
        self._chk(self.L.anakin_get_trajectory(self.h, C.byref(v)))
        B, T, NHP, NH = v.B, v.T, v.head_stride, v.num_heads

        def grab(off, count, dtype):
            nbytes = count * torch.empty((), dtype=dtype).element_size()
            return self.ws[off:off + nbytes].view(dtype).cpu().numpy()

        out = {
            "state_s0": grab(v.off_state_s0, (T + 1) * B, torch.int32).view(np.uint32).reshape(T + 1, B),
            "state_f0": grab(v.off_state_f0, (T + 1) * B, torch.float32).reshape(T + 1, B),
            "state_f1": grab(v.off_state_f1, (T + 1) * B, torch.float32).reshape(T + 1, B),
            "action": grab(v.off_action, T * B, torch.uint8).reshape(T, B),
            "eps": grab(v.off_eps, T * B, torch.float32).reshape(T, B),
            "action_f": grab(v.off_action_f, T * B, torch.float32).reshape(T, B),
            "reward": grab(v.off_reward, T * B, torch.float32).reshape(T, B),
            "done": grab(v.off_done, T * B, torch.uint8).reshape(T, B),
            "value": grab(v.off_value, (T + 1) * B, torch.float32).reshape(T + 1, B),
            "head": grab(v.off_head, (T + 1) * B * NHP, torch.float32).reshape(T + 1, B, NHP)[:, :, :NH],
            "adv": grab(v.off_adv, T * B, torch.float32).reshape(T, B),
            "ret": grab(v.off_ret, T * B, torch.float32).reshape(T, B),
        }
        acts = []
        for l in range(v.n_hidden if v.act_is_bf16 >= 0 else 0):
            H = v.hidden[l]
            if v.act_is_bf16:
                a = self.ws[v.off_act[l]:v.off_act[l] + T * B * H * 2].view(torch.bfloat16).float()
                a = a.view(T * B // 8, H, 8).permute(0, 2, 1).contiguous().cpu().numpy()
            else:
                a = grab(v.off_act[l], T * B * H, torch.float32)
            acts.append(a.reshape(T, B, H))
        out["act"] = acts
        return out

    def profile(self, enable):
        self._chk(self.L.anakin_profile(self.h, 1 if enable else 0))

    def kernel_times(self):
        """{kernel name: (calls, total_ms)} since profiling was switched on; synchronises."""
        buf = (KernelTime * 32)()
        n = C.c_int32()
        self._chk(self.L.anakin_kernel_times(self.h, buf, 32, C.byref(n)))
        return {buf[i].name.decode(): (buf[i].calls, buf[i].total_ms) for i in range(min(n.value, 32))}

    def synchronize(self):
        self.stream.synchronize()


def unpack_state_word(kind, s0):
    """The packed state word of the trajectory as the (B,4)-style integer rows."""
    s0 = np.asarray(s0, np.uint32)
    out = np.zeros(s0.shape + (4,), np.int32)
    if kind == "catch":
        out[..., 0] = s0 & 0xFF; out[..., 1] = (s0 >> 8) & 0xFF; out[..., 2] = (s0 >> 16) & 0xFF
    elif kind == "pendulum":
        out[..., 0] = s0
    else:
        out[..., 0] = s0 & 0xFFFF; out[..., 1] = s0 >> 16
    return out


PROBE_MFMA_F32, PROBE_MFMA_BF16, PROBE_COPY, PROBE_ADAM, PROBE_READ, PROBE_L2_TILES = 0, 1, 2, 3, 4, 5


def peak_probe(kind, scratch, stream_ptr, workgroups=0):
    """(amount, milliseconds) of one peak probe; scratch: a uint8 device tensor the probe may overwrite."""
    L = load()
    amount, ms = C.c_double(0.0), C.c_double(0.0)
    rc = L.anakin_peak_probe(kind, workgroups, C.c_void_p(scratch.data_ptr()), scratch.numel(), C.c_void_p(stream_ptr),
                             C.byref(amount), C.byref(ms))
    if rc != 0:
        raise AnakinError(rc, "peak probe failed")
    return amount.value, ms.value
