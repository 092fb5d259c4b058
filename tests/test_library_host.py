"""Host-side checks of the C-ABI library that need no GPU: it loads, exports
every symbol the header declares, sizes workspaces, and rejects bad input
before touching the device."""
import ctypes as C
import os
import re

import pytest

from paper_2104_06272_amd import binding, workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2104_06272_amd import build
        build.build(verbose=False)
    return binding.load()


def test_exports_match_header(lib):
    text = open(os.path.join(ROOT, "include", "anakin.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(anakin_[a-z_]+)\s*\(", text))
    assert declared == set(binding.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name


def test_workspace_sizes(lib):
    sizes = {n: binding.workspace_bytes(W.get(n)) for n in W.ORDER}
    for n, s in sizes.items():
        assert s > 0 and s % 256 == 0, n
    assert sizes["catch_small"] < sizes["catch_4096"] < sizes["maze_16384"]
    assert sizes["maze_16384"] < 64 << 30               # far inside one GPU's 288 GB
    small = W.get("catch_small")
    assert binding.workspace_bytes(small, B=128) > binding.workspace_bytes(small, B=64)


@pytest.mark.parametrize("mutate", [
    lambda c: c.update(B=60),                                   # not a multiple of 16
    lambda c: c.update(B=0),
    lambda c: c.update(T=0),
    lambda c: c["net"].update(hidden=[48]),                     # not a power of two
    lambda c: c["net"].update(hidden=[16]),
    lambda c: c["net"].update(hidden=[64] * 5),
    lambda c: c["net"].update(policy="tanh_gaussian"),          # wrong policy for catch
    lambda c: c["net"].update(lr=0.0),
    lambda c: c["env"].update(rows=1),
    lambda c: c.update(env=dict(kind="maze", rows=32, cols=32, max_steps=10, p_wall=0.2)),
    # no acting tile fits: a 32-wide layer needs tiles of 32 envs (B = 48 is not a multiple), and a 1024-wide last
    # layer with the only tile it allows (16 envs) is 2 KB over the LDS of a workgroup
    lambda c: (c.update(B=48), c["net"].update(hidden=[32, 64])),
    lambda c: (c.update(B=16), c["net"].update(hidden=[1024])),
    lambda c: (c.update(B=16), c["net"].update(hidden=[1024, 1024])),
])
def test_bad_configs_are_rejected_on_the_host(lib, mutate):
    cfg = W.get("catch_small")
    cfg["env"] = dict(cfg["env"])
    mutate(cfg)
    if len(cfg["net"]["hidden"]) > 4:
        cfg["net"]["hidden"] = cfg["net"]["hidden"][:4]
        env, net = binding.make_cfgs(cfg)
        net.n_hidden = 5
    else:
        env, net = binding.make_cfgs(cfg)
    assert lib.anakin_workspace_bytes(C.byref(env), C.byref(net), cfg["B"], cfg["T"]) == 0
    h = C.c_void_p()
    rc = lib.anakin_create(C.byref(h), C.byref(env), C.byref(net), cfg["B"], cfg["T"], 0, None, 0, None)
    assert rc == binding.E_BAD_CONFIG and not h.value
    assert len(lib.anakin_last_error(None)) > 0


def test_create_checks_workspace_before_any_device_call(lib):
    cfg = W.get("catch_small")
    env, net = binding.make_cfgs(cfg)
    h = C.c_void_p()
    assert lib.anakin_create(C.byref(h), C.byref(env), C.byref(net), 64, 20, 0, None, 0, None) == binding.E_INVALID_ARG
    assert lib.anakin_create(C.byref(h), C.byref(env), C.byref(net), 64, 20, 0, C.c_void_p(0x1001), 1 << 30, None) == binding.E_MISALIGNED
    assert lib.anakin_create(C.byref(h), C.byref(env), C.byref(net), 64, 20, 0, C.c_void_p(0x1000), 4096, None) == binding.E_WORKSPACE_TOO_SMALL
    assert b"need" in lib.anakin_last_error(None)
    assert lib.anakin_create(None, C.byref(env), C.byref(net), 64, 20, 0, None, 0, None) == binding.E_INVALID_ARG
    for fn in (lib.anakin_rollout, lib.anakin_learn, lib.anakin_learn_static, lib.anakin_step, lib.anakin_destroy):
        assert fn(None) == binding.E_INVALID_ARG


def test_no_gpu_means_error_not_fallback():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    with pytest.raises(RuntimeError):
        binding.Anakin(W.get("catch_small"))
