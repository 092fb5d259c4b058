#!/usr/bin/env python3
"""Throughput of the Anakin actor-learner step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload maze_16384]

A step is one pass of the whole hot path (unroll of T interactions for B envs,
then one update) through the C ABI.  Prints ONE JSON line: env-steps/s over K
steps of the named workload (default: the largest one, the bf16 maze), the
roofline of its dominant kernel (per-kernel durations from HIP events recorded
on the launch stream in a second, instrumented pass of the same K steps), a
"workloads" block with the same measurement of all five workloads, and the CPU
oracle timed on a bounded sample of the named workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
for p in (ROOT,):
    if p not in sys.path:
        sys.path.insert(0, p)

# published MI355X peaks
PEAK_HBM_GBS = 8000.0
PEAK_FP32_TFLOPS = 157.3      # fp32 vector (packed) = fp32 matrix-core peak
PEAK_BF16_TFLOPS = 2500.0

def measured_traffic(workload):
    """HBM bytes per launch (MB) of each kernel of a workload, read from profiles/<workload>_hbm_traffic.md: the
    table under "per bench.py kernel" (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, scaled by a copy-kernel
    calibration; the file names the commands and the commit it was measured at).  Returns ({kernel: MB}, commit)
    -- empty when the workload has no such file."""
    path = os.path.join(ROOT, "profiles", f"{workload}_hbm_traffic.md")
    out, commit, in_table = {}, None, False
    try:
        lines = open(path).read().splitlines()
    except OSError:
        return out, commit
    for line in lines:
        if line.lower().startswith("measured at commit"):
            commit = line.split()[-1].strip("`. ")
        if line.startswith("## "):
            in_table = "per bench.py kernel" in line
            continue
        if in_table and line.startswith("| `"):
            cells = [c.strip() for c in line.strip("|").split("|")]
            try:
                out[cells[0].strip("`")] = float(cells[-1])
            except ValueError:
                pass
    return out, commit


def measured_issue_utilisation(workload):
    """VALU issue utilisation per bench.py kernel, read from profiles/<workload>_shader_counters.md (rocprofv3 --pmc
    SQ_ACTIVE_INST_VALU over SQ_BUSY_CYCLES; the file names the commands and the commit) through the kernel-name
    mapping of profiles/<workload>_hbm_traffic.md.  For kernels bound by plain vector arithmetic this, not a flop
    count, says how busy the vector units were.  Returns ({kernel: utilisation}, commit)."""
    out, commit, by_rocprof = {}, None, {}
    try:
        lines = open(os.path.join(ROOT, "profiles", f"{workload}_shader_counters.md")).read().splitlines()
        names = open(os.path.join(ROOT, "profiles", f"{workload}_hbm_traffic.md")).read().splitlines()
    except OSError:
        return out, commit
    col = None
    for line in lines:
        if line.lower().startswith("measured at commit"):
            commit = line.split()[-1].strip("`. ")
        if line.startswith("| kernel"):
            heads = [c.strip() for c in line.strip("|").split("|")]
            col = heads.index("VALU issue utilisation") if "VALU issue utilisation" in heads else None
        elif col is not None and line.startswith("| `"):
            cells = [c.strip() for c in line.strip("|").split("|")]
            try:
                by_rocprof[cells[0].strip("`")] = float(cells[col])
            except ValueError:
                pass
    in_table = False
    for line in names:
        if line.startswith("## "):
            in_table = "per bench.py kernel" in line
            continue
        if in_table and line.startswith("| `"):
            cells = [c.strip() for c in line.strip("|").split("|")]
            # a listed name matches the profiler's up to its template arguments ("gemm_nt_bf16_res<512, true>" as listed
            # must not also match "...<512, false>"): compare the part the listing gives, from the start
            wanted = []
            for w in cells[1].split(", "):
                if wanted and "<" in wanted[-1] and ">" not in wanted[-1]:
                    wanted[-1] += ", " + w
                else:
                    wanted.append(w)
            vals = [v for k, v in by_rocprof.items() if any(k.split("::")[-1].startswith(w) for w in wanted)]
            if vals:
                out[cells[0].strip("`")] = round(sum(vals) / len(vals), 3)
    return out, commit


def kernel_models(cfg, P, launched=()):
    """Algorithmic work per launch of each kernel: (bound, amount, unit-peak, unit).  `launched`: the kernel names the
    instrumented pass saw (which products a fused kernel took over depends on the plan)."""
    B, T = cfg["B"], cfg["T"]
    M = B * T
    kind = cfg["env"]["kind"]
    hid = cfg["net"]["hidden"]
    D = {"catch": 50, "pendulum": 3, "maze": 768}[kind]
    NH = 3 if kind == "pendulum" else ({"catch": 3, "maze": 4}[kind] + 1)
    dims = [D] + hid
    # effective input count of the first layer: a one-hot board adds only its set rows
    first_rows = {"catch": 2, "pendulum": 3, "maze": 53}[kind]
    w_act = first_rows * dims[1] + sum(dims[i] * dims[i + 1] for i in range(1, len(dims) - 1)) + dims[-1] * NH
    bf16 = cfg["net"].get("dtype") == "bf16"
    mfma_peak = PEAK_BF16_TFLOPS if bf16 else PEAK_FP32_TFLOPS
    snap = {"catch": 4, "pendulum": 8, "maze": 2}[kind]
    dense_act = sum(dims[i] * dims[i + 1] for i in range(1, len(dims) - 1))
    models = {
        # acting: (T+1) forward passes per env; hidden-to-hidden layers run on the matrix cores, the one-hot
        # first layer and the heads on vector ALUs -- all counted as 2 flop per weight actually touched
        "rollout": ("mfma" if dense_act else "alu", 2.0 * w_act * B * (T + 1) / 1e12, mfma_peak if dense_act else PEAK_FP32_TFLOPS, "TFLOP/s"),
        # 17 B per (t,b): read r 4 + done 1 + V 4, write A 4 + G 4
        "returns_scan": ("hbm", 17.0 * M / 1e9, PEAK_HBM_GBS, "GB/s"),
        # 28 B per parameter: read theta,g,m,v, write theta,m,v
        "adam_reduce": ("hbm", 28.0 * P / 1e9, PEAK_HBM_GBS, "GB/s"),
        "head_grad": ("hbm", (NH * 4 + 1 + 8 + NH * 4) * M / 1e9, PEAK_HBM_GBS, "GB/s"),
        # the two above as one launch: r 4 + done 1 + V 4 read, A 4 + G 4 written (for the caller), heads NH*4 and
        # the action 1 read, head gradient NH*4 written
        "scan_loss": ("hbm", (17.0 + NH * 4 + 1 + NH * 4) * M / 1e9, PEAK_HBM_GBS, "GB/s"),
        # read h_L, write dZ_L (bf16: written in two layouts)
        "head_backward": ("hbm", ((6.0 if bf16 else 8.0) * dims[-1] + 4 * NH) * M / 1e9, PEAK_HBM_GBS, "GB/s"),
        # scatter of dZ1 rows into the selected weight rows: one read of dZ1
        "first_layer_grad": ("hbm", 4.0 * dims[1] * M / 1e9, PEAK_HBM_GBS, "GB/s"),
    }
    # bf16 top layer with the heads folded in: its dW product is a launch of its own (gemm_tn_top) that reads
    # h_{L-1}, h_L and the head gradient and forms dZ_L itself
    top_fused = "gemm_tn_top" in launched
    tn_layers = range(1, len(dims) - (2 if top_fused else 1))
    tn = sum(2.0 * dims[i] * dims[i + 1] * M for i in tn_layers)
    nt = sum(2.0 * dims[i] * dims[i + 1] * M for i in range(1, len(dims) - 1))
    models["gemm_tn"] = ("mfma", tn / 1e12, mfma_peak, "TFLOP/s")
    models["gemm_nt_mask"] = ("mfma", nt / 1e12, mfma_peak, "TFLOP/s")
    if bf16:
        # 2-byte operands: 2 K N flop per sample against 2 (N + 2 K) B (dX: dY and the relu mask read, dX written)
        # resp. 2 (K + N) B (dW: both operands read) is 170 resp. 256 flop/B for 512-wide layers, below the
        # machine balance of 2500 / 8 = 312 flop/B: both GEMMs sit on the HBM roof, not the matrix-core one
        # dX of layer i -> i+1: dY read (2 B per entry; not for a fused top layer, which forms it from the head
        # gradient), the ReLU mask of h_i (flag words, 1/4 B per entry, where the acting kernel writes them: every
        # layer but a first one that is not 512 wide; else the 2-byte activations), dX written (2 B per entry)
        def nt_layer_bytes(i):
            top = top_fused and i == len(dims) - 2
            dy = (dims[i + 1] / 4.0 + 4.0 * NH) if top else 2.0 * dims[i + 1]
            mask = dims[i] / 4.0 if (i >= 2 or dims[1] == 512) else 2.0 * dims[i]
            return (dy + mask + 2.0 * dims[i]) * M
        nt_bytes = sum(nt_layer_bytes(i) for i in range(1, len(dims) - 1))
        tn_bytes = sum(2.0 * (dims[i] + dims[i + 1]) * M for i in tn_layers)
        if nt / max(nt_bytes, 1.0) < PEAK_BF16_TFLOPS * 1e12 / (PEAK_HBM_GBS * 1e9):
            models["gemm_nt_mask"] = ("hbm", nt_bytes / 1e9, PEAK_HBM_GBS, "GB/s")
        if tn / max(tn_bytes, 1.0) < PEAK_BF16_TFLOPS * 1e12 / (PEAK_HBM_GBS * 1e9):
            models["gemm_tn"] = ("hbm", tn_bytes / 1e9, PEAK_HBM_GBS, "GB/s")
    if top_fused:
        top_flop = 2.0 * dims[-2] * dims[-1] * M
        top_bytes = (2.0 * (dims[-2] + dims[-1]) + 4.0 * NH) * M
        models["gemm_tn_top"] = ("mfma", top_flop / 1e12, mfma_peak, "TFLOP/s")
        if top_flop / top_bytes < PEAK_BF16_TFLOPS * 1e12 / (PEAK_HBM_GBS * 1e9):
            models["gemm_tn_top"] = ("hbm", top_bytes / 1e9, PEAK_HBM_GBS, "GB/s")
    # a layer whose two products run as one launch (256-wide fp32 layers): both counted
    models["gemm_tn_nt"] = ("mfma", (tn + nt) / 1e12, mfma_peak, "TFLOP/s")
    models["gemm_tn_obs"] = ("mfma", 2.0 * dims[0] * dims[1] * M / 1e12, mfma_peak, "TFLOP/s")
    if kind == "maze":
        cells = cfg["env"]["rows"] * cfg["env"]["cols"]
        # first layer of a bf16 maze net, reduced plane by plane: time sum of dZ1 (one read, B rows written twice),
        # wall plane over 2B time-summed samples, agent plane over all samples
        models["time_sum"] = ("hbm", (2.0 * dims[1] * M + 4.0 * dims[1] * B) / 1e9, PEAK_HBM_GBS, "GB/s")
        models["gemm_tn_walls"] = ("mfma", 2.0 * cells * dims[1] * 2 * B / 1e12, mfma_peak, "TFLOP/s")
        models["gemm_tn_agent"] = ("mfma", 2.0 * cells * dims[1] * M / 1e12, mfma_peak, "TFLOP/s")
        # the X operand is a one-hot built in the kernel from 4 B per sample: what streams is dZ1 (2 B per entry), and at
        # 2 cells flop per byte of it the product sits under the HBM roof for planes of up to 312 cells
        agent_bytes = (2.0 * dims[1] + 4.0) * M + 4.0 * dims[1] * B
        if bf16 and 2.0 * cells * dims[1] * M / agent_bytes < PEAK_BF16_TFLOPS * 1e12 / (PEAK_HBM_GBS * 1e9):
            models["gemm_tn_agent"] = ("hbm", agent_bytes / 1e9, PEAK_HBM_GBS, "GB/s")
    if len(hid) == 1:
        # fused update of a one-hidden-layer net: reads state, head gradient and returns, rebuilds the layer
        models["learn_one_layer"] = ("alu", 2.0 * (2 * first_rows * dims[1] + 3 * dims[1] * NH) * M / 1e12, PEAK_FP32_TFLOPS, "TFLOP/s")
        # the same arithmetic with the scan and the loss in the launch (their flops are not counted)
        models["learn_catch_fused"] = models["learn_one_layer"]
    # small nets, whole update in one launch: the backward products (dZ, dW per layer and head) and 12 flop per
    # parameter of Adam; a latency-bound launch, the model is there for the record
    models["learn_small_fused"] = ("alu", (2.0 * (2 * first_rows * dims[1] + 2 * dense_act + 2 * dims[-1] * NH) * M + 12.0 * P) / 1e12,
                                   PEAK_FP32_TFLOPS, "TFLOP/s")
    return models, snap


def cpu_baseline(cfg, budget_s=20.0):
    """The oracle as it stands, single-threaded and pinned to one core, on a bounded sample: the same network, T and
    hyper-parameters with B cut so that one full step takes roughly the budget (envs are independent, so the
    per-env-step rate of a B-slice is the rate of the workload; labelled as scaled when B is cut)."""
    from oracle import oracle as O
    host_cores = os.cpu_count()
    pinned = None
    try:
        allowed = sorted(os.sched_getaffinity(0))
        os.sched_setaffinity(0, {allowed[-1]})
        pinned = allowed
    except (AttributeError, OSError):
        pass
    try:
        probe_B = 16
        c = dict(cfg); c["B"] = probe_B
        o = O.Oracle(c, seed=0)
        t0 = time.perf_counter(); o.step(); dt = time.perf_counter() - t0
        per_env = max(dt / probe_B, 1e-9)
        B = int(max(16, min(cfg["B"], (budget_s / per_env) // 16 * 16)))
        c["B"] = B
        o = O.Oracle(c, seed=0)
        t0 = time.perf_counter(); o.step(); dt = time.perf_counter() - t0
    finally:
        if pinned is not None:
            os.sched_setaffinity(0, set(pinned))
    rate = B * cfg["T"] / dt
    usable = len(pinned) if pinned is not None else host_cores
    return {"value": rate, "unit": "env steps/s", "cores": 1, "kind": "oracle",
            "host_cores": host_cores, "usable_cores": usable,
            "ideal_all_cores_estimate": rate * usable,
            "ideal_all_cores_note": "value x usable cores: an ideal-scaling estimate (one oracle process per core over "
                                    "disjoint env shards), not a measurement",
            "scaled_from_B_slice": B != cfg["B"],
            "sample": f"1 full step (rollout + update) at B={B} of {cfg['B']} envs, T={cfg['T']}, same network; "
                      f"{dt:.1f} s single-threaded, pinned to one core"}


def measure(binding, torch, name, cfg, steps, warmup, halves=False, valu_gemm=False):
    """K timed steps of one workload (events on the launch stream), then the same K steps instrumented (two events
    around every kernel launch) for the per-kernel table and the dominant kernel's roofline.  Returns (agent, dict)."""
    g = binding.Anakin(cfg, seed=0, device="cuda:0")
    if valu_gemm:
        g.set_mode(binding.MODE_VALU_GEMM)
    for _ in range(max(warmup, 1)):
        g.step()
    torch.cuda.synchronize()
    e0 = torch.cuda.Event(enable_timing=True); e1 = torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record(g.stream)
    for _ in range(steps):
        g.step()
    e1.record(g.stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms = e0.elapsed_time(e1)
    res = {"ms_per_step": ms / steps, "value": cfg["B"] * cfg["T"] * steps / (ms / 1e3), "wall_s": round(wall, 3), "steps": steps}
    metrics = g.metrics()
    res["loss"] = metrics["loss"]
    res["mean_episode_return"] = metrics["reward_sum"] / max(1, metrics["episodes"])
    if halves:
        # the two halves on their own (same K): unrolls only, then the updates of K further steps bracketed by events
        a0 = torch.cuda.Event(enable_timing=True); a1 = torch.cuda.Event(enable_timing=True)
        a0.record(g.stream)
        for _ in range(steps):
            g.rollout()
        a1.record(g.stream)
        torch.cuda.synchronize()
        ms_rollout = a0.elapsed_time(a1) / steps
        pairs = []
        for _ in range(steps):
            g.rollout()
            b0 = torch.cuda.Event(enable_timing=True); b1 = torch.cuda.Event(enable_timing=True)
            b0.record(g.stream)
            g.learn()
            b1.record(g.stream)
            pairs.append((b0, b1))
        torch.cuda.synchronize()
        ms_learn = sum(x.elapsed_time(y) for x, y in pairs) / steps
        res["rollout_only"] = {"ms": round(ms_rollout, 4), "env_steps_per_s": cfg["B"] * cfg["T"] / (ms_rollout * 1e-3)}
        res["learn_only"] = {"ms": round(ms_learn, 4), "env_steps_per_s": cfg["B"] * cfg["T"] / (ms_learn * 1e-3)}
    # instrumented pass: the same K steps with two events around every kernel launch
    g.profile(True)
    for _ in range(steps):
        g.step()
    times = g.kernel_times()
    g.profile(False)
    models, _ = kernel_models(cfg, g.P, launched=tuple(times))
    per_kernel = {}
    for kname, (calls, total) in times.items():
        launches_per_step = calls / steps
        avg_us = total / calls * 1e3
        entry = {"calls_per_step": launches_per_step, "avg_us": round(avg_us, 2),
                 "us_per_step": round(total / steps * 1e3, 2)}
        if kname in models:
            bound, amount, peak, unit = models[kname]
            per_launch = amount / launches_per_step
            ach = per_launch / (avg_us * 1e-6)
            entry.update({"bound": bound, "achieved": round(ach, 3), "peak": peak, "unit": unit,
                          "frac": round(ach / peak, 4)})
        per_kernel[kname] = entry
    issue, issue_commit = measured_issue_utilisation(name)
    for kname, entry in per_kernel.items():
        if entry.get("bound") == "alu" and kname in issue:
            entry["valu_issue_utilisation"] = issue[kname]
    dominant = max(per_kernel, key=lambda k: per_kernel[k]["us_per_step"])
    d = per_kernel[dominant]
    traffic, commit = measured_traffic(name)
    res["roofline"] = {"kernel": dominant, "bound": d.get("bound"), "achieved": d.get("achieved"), "peak": d.get("peak"),
                       "unit": d.get("unit"), "frac": d.get("frac"),
                       "traffic": traffic.get(dominant), "traffic_unit": "MB per launch",
                       "traffic_source": (f"profiles/{name}_hbm_traffic.md" + (f" (measured at commit {commit})" if commit else "")) if dominant in traffic else None,
                       "avg_launch_us": d["avg_us"]}
    if "valu_issue_utilisation" in d:
        # a kernel bound by plain vector arithmetic: the flop fraction above counts only the network's multiply-adds
        # (not Philox, exponentials, sampling, index arithmetic); the issue counters say how busy the vector units were
        res["roofline"]["valu_issue_utilisation"] = d["valu_issue_utilisation"]
        res["roofline"]["valu_issue_source"] = f"profiles/{name}_shader_counters.md" + (f" (measured at commit {issue_commit})" if issue_commit else "")
    res["kernels"] = per_kernel
    res["plan"] = g.plan()
    return g, res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="maze_16384",
                    help="the workload the headline value is measured on (default: the largest single-GPU one)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-sweep", action="store_true",
                    help="skip the \"workloads\" block (the other four workloads, measured the same way with fewer steps)")
    ap.add_argument("--valu-gemm", action="store_true", help="learn-phase GEMMs on vector ALUs")
    ap.add_argument("--pathwise", action="store_true",
                    help="also time K steps with the policy gradient taken through the environment (pendulum "
                         "workloads) and report them under \"pathwise\"")
    ap.add_argument("--decoupled", action="store_true",
                    help="also time K decoupled steps (actor on a second stream with lagging parameters, off-policy "
                         "update on the previous unroll) and report them under \"decoupled\"")
    ap.add_argument("--peak-probe", action="store_true",
                    help="instead of the benchmark, measure what this GPU delivers for the rooflines: register-only "
                         "fp32 and bf16 MFMA loops and a 2 x 1 GiB streaming copy; prints one JSON line")
    ap.add_argument("--copy-probe", type=int, default=0, metavar="MiB",
                    help="instead of the benchmark, run a plain device copy of this many MiB 20 times "
                         "(calibrates the HBM byte counters under rocprofv3 --pmc)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding, no collectives); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    if args.copy_probe:
        n = args.copy_probe * 1024 * 1024 // 4
        src = torch.ones(n, dtype=torch.float32, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(20):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_probe_MiB": args.copy_probe, "copies": 20}))
        return
    from paper_2104_06272_amd import binding, workloads as W
    if args.peak_probe:
        torch.cuda.set_device(0)
        scratch = torch.zeros(2 << 30, dtype=torch.uint8, device="cuda:0")
        stream = torch.cuda.current_stream().cuda_stream
        out = {}
        for name, kind, unit, peak in (("mfma_f32", binding.PROBE_MFMA_F32, "TFLOP/s", PEAK_FP32_TFLOPS),
                                       ("mfma_bf16", binding.PROBE_MFMA_BF16, "TFLOP/s", PEAK_BF16_TFLOPS),
                                       ("copy", binding.PROBE_COPY, "GB/s", PEAK_HBM_GBS),
                                       ("read_only", binding.PROBE_READ, "GB/s", PEAK_HBM_GBS),
                                       ("l2_weight_stream", binding.PROBE_L2_TILES, "GB/s", None),
                                       ("adam_2^26_params", binding.PROBE_ADAM, "GB/s", PEAK_HBM_GBS)):
            best, best_wg = 0.0, 0
            for wg in ((1024, 4096, 16384, 65536) if name in ("copy", "read_only") else (0,) if kind == binding.PROBE_ADAM
                       else (256,) if kind == binding.PROBE_L2_TILES else (256, 512, 768, 1024, 2048)):
                for _ in range(2):
                    amount, ms = binding.peak_probe(kind, scratch, stream, wg)
                    rate = amount / (ms * 1e-3) / (1e12 if unit == "TFLOP/s" else 1e9)
                    if rate > best:
                        best, best_wg = rate, wg
            out[name] = {"measured": round(best, 1), "published": peak, "unit": unit,
                         "frac": round(best / peak, 3) if peak else None, "workgroups": best_wg}
        print(json.dumps({"peak_probe": out}))
        return
    cfg = W.get(args.workload)
    torch.cuda.set_device(0)
    g, r = measure(binding, torch, args.workload, cfg, args.steps, args.warmup, halves=True, valu_gemm=args.valu_gemm)
    value, ms_per_step = r["value"], r["ms_per_step"]
    out = {
        "metric": "env steps/sec (rollout+learn) on 1 MI355X", "value": value, "unit": "env steps/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if cfg["net"].get("dtype") == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": args.workload, "env": cfg["env"]["kind"], "B": cfg["B"], "T": cfg["T"],
                   "hidden": cfg["net"]["hidden"], "params": g.P},
        "roofline": r["roofline"],
        "kernels": r["kernels"],
        "plan": r["plan"],
        "rollout_only": r["rollout_only"],
        "learn_only": r["learn_only"],
        "wall_s": r["wall_s"],
        "loss": r["loss"], "mean_episode_return": r["mean_episode_return"],
    }
    if args.pathwise:
        if cfg["env"]["kind"] != "pendulum":
            out["pathwise"] = None                        # differentiable dynamics only
        else:
            g.set_policy_gradient(binding.PG_PATHWISE)
            for _ in range(max(args.warmup, 2)):
                g.step()
            torch.cuda.synchronize()
            p0 = torch.cuda.Event(enable_timing=True); p1 = torch.cuda.Event(enable_timing=True)
            p0.record(g.stream)
            for _ in range(args.steps):
                g.step()
            p1.record(g.stream)
            torch.cuda.synchronize()
            ms_pw = p0.elapsed_time(p1) / args.steps
            g.profile(True)
            for _ in range(args.steps):
                g.step()
            pk = g.kernel_times()
            g.profile(False)
            g.set_policy_gradient(binding.PG_SCORE_FUNCTION)
            c, tms = pk["pathwise_sweep"]
            sweep_us = tms / c * 1e3
            # the sweep's matrix-core work: dZ1 = dZ2 W2^T for every sample
            hid = cfg["net"]["hidden"]
            tf = 2.0 * hid[0] * hid[1] * cfg["B"] * cfg["T"] / 1e12 / (sweep_us * 1e-6)
            out["pathwise"] = {"ms_per_step": round(ms_pw, 4), "env_steps_per_s": cfg["B"] * cfg["T"] / (ms_pw * 1e-3),
                               "pathwise_sweep": {"avg_us": round(sweep_us, 2), "bound": "mfma", "achieved": round(tf, 3),
                                                  "peak": PEAK_FP32_TFLOPS, "unit": "TFLOP/s", "frac": round(tf / PEAK_FP32_TFLOPS, 4)}}
    if args.decoupled:
        if True:
            for _ in range(max(args.warmup, 2)):
                g.step_decoupled()
            torch.cuda.synchronize()
            d0 = torch.cuda.Event(enable_timing=True); d1 = torch.cuda.Event(enable_timing=True)
            d0.record(g.stream)
            for _ in range(args.steps):
                g.step_decoupled()
            d1.record(g.stream)                           # the handle's stream waits for the actor's at the end of every step
            torch.cuda.synchronize()
            ms_dec = d0.elapsed_time(d1) / args.steps
            g.profile(True)
            for _ in range(args.steps):
                g.step_decoupled()
            dk = {k: {"calls_per_step": c / args.steps, "avg_us": round(t / c * 1e3, 2)} for k, (c, t) in g.kernel_times().items()}
            g.profile(False)
            out["decoupled"] = {"ms_per_step": round(ms_dec, 4), "env_steps_per_s": cfg["B"] * cfg["T"] / (ms_dec * 1e-3),
                                "kernels": dk}
    g.close()
    del g
    if not args.no_sweep:
        # the other workloads, each measured the same way in this same run (shorter K): one line covers all five
        sweep = {}
        for name in W.ORDER:
            if name == args.workload:
                sweep[name] = {"ms_per_step": round(ms_per_step, 5), "env_steps_per_s": value, "steps": args.steps,
                               "dtype": out["dtype"], "dominant_kernel": r["roofline"]["kernel"], "bound": r["roofline"]["bound"],
                               "frac": r["roofline"]["frac"], "avg_launch_us": r["roofline"]["avg_launch_us"]}
                continue
            c = W.get(name)
            k = max(10, min(args.steps, 100))
            torch.cuda.empty_cache()
            gg, rr = measure(binding, torch, name, c, k, max(3, min(args.warmup, 10)))
            gg.close()
            del gg
            sweep[name] = {"ms_per_step": round(rr["ms_per_step"], 5), "env_steps_per_s": rr["value"], "steps": k,
                           "dtype": "bf16" if c["net"].get("dtype") == "bf16" else "f32",
                           "dominant_kernel": rr["roofline"]["kernel"], "bound": rr["roofline"]["bound"],
                           "frac": rr["roofline"]["frac"], "avg_launch_us": rr["roofline"]["avg_launch_us"],
                           "traffic": rr["roofline"]["traffic"],
                           **({"valu_issue_utilisation": rr["roofline"]["valu_issue_utilisation"]} if "valu_issue_utilisation" in rr["roofline"] else {}),
                           "kernels_us_per_step": {kn: kv["us_per_step"] for kn, kv in rr["kernels"].items()}}
        out["workloads"] = sweep
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
