"""Builds libanakin.so (HIP, gfx950 only) in-tree with hipcc.

    python -m paper_2104_06272_amd.build

hipcc cross-compiles for gfx950 without a GPU present.  Contraction is off so
that every fused multiply-add in the kernels is an explicit one, and packed
fp32 instructions are disabled.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.environ.get("ANAKIN_OUT", os.path.join(HERE, "libanakin.so"))
SOURCES = ["anakin.hip", "rollout.hip", "rollout_bf16.hip", "learn.hip", "learn_small.hip", "learn_bf16.hip", "gemm.hip", "gemm_mfma.hip", "gemm_resident.hip", "probe.hip", "pathwise.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-function", "-Wno-unknown-warning-option"]
FLAGS += os.environ.get("ANAKIN_EXTRA_HIPCC_FLAGS", "").split()


def torch_lib_dir():
    try:
        import importlib.util
        spec = importlib.util.find_spec("torch")
        return os.path.join(os.path.dirname(spec.origin), "lib") if spec and spec.origin else None
    except Exception:
        return None


def build(verbose=True, jobs=8):
    objs = []
    procs = []
    bdir = os.environ.get("ANAKIN_BUILD_DIR", os.path.join(HERE, "_build"))
    os.makedirs(bdir, exist_ok=True)
    for src in SOURCES:
        obj = os.path.join(bdir, src.replace(".hip", ".o"))
        cmd = [HIPCC, *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stderr=subprocess.PIPE, text=True)))
        objs.append(obj)
    failed = False
    for src, p in procs:
        _, err = p.communicate()
        err = "\n".join(l for l in err.splitlines() if "packed-fp32-ops" not in l)
        if err.strip() and verbose:
            print(err, file=sys.stderr)
        failed |= p.returncode != 0
    if failed:
        raise RuntimeError("hipcc failed")
    # One HIP runtime per process: PyTorch ships its own libamdhip64.so, and a second copy loaded
    # from /opt/rocm would see no device.  Link against the copy PyTorch loads (falling back to the
    # system one by rpath when PyTorch's directory is absent).
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-no-hip-rt", "-o", LIB, *objs]
    tl = torch_lib_dir()
    if tl and os.path.exists(os.path.join(tl, "libamdhip64.so")):
        cmd += ["-L" + tl, "-Wl,-rpath," + tl]
    cmd += ["-L/opt/rocm/lib", "-Wl,-rpath,/opt/rocm/lib", "-lamdhip64"]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    build()
