"""The five synthetic workloads: shapes, sizes and hyper-parameters only.

This module holds no arithmetic of the method.  Every random quantity of a run
(initial env states, maze walls, initial weights, action noise) is drawn by the
consumer itself from its own counter-based generator, keyed by the seed given
here, so the same dict fully defines the inputs for both the GPU library and
the CPU checker used by the tests.
"""
import copy

_HYPER = dict(gamma=0.99, entropy_coef=0.01, value_coef=0.5, lr=3e-4, beta1=0.9, beta2=0.999, eps=1e-8)


def _net(hidden, policy="categorical", dtype="fp32", lam=1.0):
    d = dict(hidden=list(hidden), policy=policy, dtype=dtype)
    d["lambda"] = lam
    d.update(_HYPER)
    return d


_CATCH = dict(kind="catch", rows=10, cols=5, max_steps=9)

CONFIGS = {
    # small Catch: the case the CPU checker finishes in seconds
    "catch_small": dict(env=_CATCH, net=_net([64, 64]), B=64, T=20, updates=100),
    # headline Catch
    "catch_4096": dict(env=_CATCH, net=_net([256, 256]), B=4096, T=20, updates=1000),
    # Pendulum swing-up, tanh-Gaussian policy, lambda-returns
    "pendulum_8192": dict(env=dict(kind="pendulum", rows=0, cols=0, max_steps=200),
                          net=_net([256, 256], policy="tanh_gaussian", lam=0.95), B=8192, T=32, updates=200),
    # 16x16 grid maze, bf16 layers with fp32 master weights
    "maze_16384": dict(env=dict(kind="maze", rows=16, cols=16, max_steps=256, p_wall=0.2),
                       net=_net([512, 512, 512], dtype="bf16", lam=0.95), B=16384, T=32, updates=100),
    # throughput-bound Catch, tiny network
    "catch_262144": dict(env=_CATCH, net=_net([32]), B=262144, T=16, updates=200),
}

ORDER = ["catch_small", "catch_4096", "pendulum_8192", "maze_16384", "catch_262144"]


def get(name, **over):
    """A deep copy of a workload, with optional overrides of B / T / updates."""
    cfg = copy.deepcopy(CONFIGS[name])
    cfg["name"] = name
    for k, v in over.items():
        if v is not None:
            cfg[k] = v
    return cfg
