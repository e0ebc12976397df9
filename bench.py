#!/usr/bin/env python3
"""Benchmark of the quantized Adam step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME]

A "step" is one pass of the whole hot path over every tensor of the workload: the fused
dequant -> Adam -> requant kernel (plus, for the workloads that have them, statistics read-back,
the bit-width decision and the re-pack of changed states).  Inputs are resident in HBM before the
timed region.  Prints ONE JSON line: params/s, the roofline of the dominant kernel from HIP-event
durations measured around every launch, and the CPU oracle timed on a bounded sample.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X HBM3E, published
ALU_PEAK_TLANE = 256 * 4 * 16 * 2.4e9 / 1e12  # vector lanes x peak clock: 39.3 T lane-instructions/s


def block_slices(n, K, parts):
    """Cut [0, n) into at most `parts` contiguous ranges whose boundaries are multiples of K (the
    quantization blocks are independent of one another, so the step of a range is the step of its blocks)."""
    blocks = (n + K - 1) // K
    parts = max(1, min(parts, blocks))
    per = (blocks + parts - 1) // parts
    return [(b * K, min(n, (b + per) * K)) for b in range(0, blocks, per)]


def state_slice(oracle, st, lo, hi):
    """The oracle's state of elements [lo, hi) of a tensor (lo a multiple of K): views, no copies."""
    K = st.K
    return oracle.State(hi - lo, K, st.bm, st.bv, um=st.um[lo:hi], sm=st.sm[lo // K:(hi + K - 1) // K],
                        cv=st.cv[lo:hi], sv=st.sv[lo // K:(hi + K - 1) // K])


def host_description():
    model = ""
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                model = line.split(":", 1)[1].strip()
                break
    except OSError:
        pass
    return {"os_cpu_count": os.cpu_count(), "cpu_model": model}


def cpu_baseline(w, plan, budget_elems=60_000_000, steps=2, max_threads=16):
    """The oracle as it stands on the first `budget_elems` parameters of the workload: once on one
    thread, once with every core of the box's share (a thread per contiguous range of blocks, each
    calling the same C routine; ctypes releases the interpreter lock).  `value` is the all-cores rate."""
    import numpy as np
    import torch
    from concurrent.futures import ThreadPoolExecutor
    from oracle import stq_oracle as oracle
    oracle.lib()
    sample, acc = [], 0
    for l, (_, n) in enumerate(w.tensors):
        take = min(n, budget_elems - acc)
        if take <= 0:
            break
        sample.append((l, take))
        acc += take

    def fresh():
        data = []
        for l, n in sample:
            th = w.gen_param(l)[:n].numpy().copy()
            g = w.gen_grad(l, 1)[:n]
            g = g.view(torch.int16).numpy().view(np.uint16).copy() if w.grad_dtype == "bf16" else g.numpy().copy()
            data.append((th, g, oracle.State.zeros(n, w.K, *plan[l])))
        return data

    data = fresh()
    t0 = time.perf_counter()
    for t in range(1, steps + 1):
        for th, g, st in data:
            oracle.step(th, g, st, **w.hparams, t=t)
    dt1 = time.perf_counter() - t0

    threads = max(1, min(max_threads, os.cpu_count() or 1))
    data = fresh()
    jobs = [(th[lo:hi], g[lo:hi], state_slice(oracle, st, lo, hi))
            for th, g, st in data for lo, hi in block_slices(st.numel, st.K, threads)]
    par_steps = steps * 4
    with ThreadPoolExecutor(max_workers=threads) as ex:
        t0 = time.perf_counter()
        for t in range(1, par_steps + 1):
            list(ex.map(lambda j: oracle.step(j[0], j[1], j[2], **w.hparams, t=t), jobs))
        dtn = time.perf_counter() - t0
    out = {"value": acc * par_steps / dtn, "unit": "params/s", "cores": threads, "kind": "oracle",
           "sample": "first %d parameters of the workload (%d tensors): %d steps on %d threads over contiguous "
                     "ranges of blocks in %.1f s; %d steps on one thread in %.1f s"
                     % (acc, len(sample), par_steps, threads, dtn, steps, dt1),
           "one_thread_value": acc * steps / dt1}
    out.update(host_description())
    return out


def kernel_source_hash():
    """SHA-256 over the sources of the step kernel: stamps the counter-derived figures under profiles/,
    so that figures taken from another version of the kernel are not reported as this one's."""
    import hashlib
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2604_06836_amd", "csrc")
    for name in ("stq_step.hip", "stq_device.h", "stq_tables.h", "stq_tables.cpp"):
        h.update(open(os.path.join(csrc, name), "rb").read())
    return h.hexdigest()[:16]


def copy_calibration(torch, n=1 << 28, launches=5):
    """dst = src + 1 over 2^28 fp32 elements: each launch reads n*4 bytes and writes n*4 bytes.
    A profiler's HBM byte counters for this kernel give the factor that scales them to bytes.
    Also times three plain streaming kernels of torch, as a measured ceiling for this box."""
    src = torch.zeros(n, dtype=torch.float32, device="cuda:0")
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    for _ in range(launches):
        torch.add(src, 1.0, out=dst)
    torch.cuda.synchronize()

    def rate(fn, bytes_per_launch, reps=20):
        fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return bytes_per_launch * reps / (e0.elapsed_time(e1) * 1e-3) / 1e9

    print(json.dumps({"copy_calibration": True, "kernel": "elementwise add", "launches": launches,
                      "read_bytes_per_launch": n * 4, "write_bytes_per_launch": n * 4,
                      "streaming_GBps": {"in_place_add (read+write 1 GiB each)": rate(lambda: dst.add_(1.0), 8 * n),
                                         "out_of_place_add (read 1 GiB, write 1 GiB)": rate(lambda: torch.add(src, 1.0, out=dst), 8 * n),
                                         "fill (write 1 GiB)": rate(lambda: dst.fill_(0.0), 4 * n)}}))


def calibrate_ladder(scores, probs):
    """Thresholds at the score quantiles that give the widths the target frequencies."""
    import numpy as np
    cum = np.cumsum(probs)[:-1]
    return tuple(float(x) for x in np.quantile(np.asarray(scores)[np.isfinite(scores)], cum))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="llama7b-slice")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--transition", choices=("repack", "fused", "engine", "engine-alg1"), default="repack",
                    help="how a new bit plan takes effect: stq_repack_many before the step (the configurations' "
                         "wording), inside the step with stq_step_transition, or (workloads that decide every "
                         "step) the device-resident loop stq_engine_step, which never waits for the GPU (engine-alg1: in "
                         "Algorithm 1's written order, with a pass over the gradients before the step)")
    ap.add_argument("--stats", choices=("full", "grad"), default="full",
                    help="workloads that decide every step: collect every statistic of stq_layer_stats (the "
                         "configuration's wording) or only the gradient's, which is all the decision reads "
                         "(the engine always does the latter)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="run only a plain elementwise kernel of known size (scale reference for HBM counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (no collectives, no sharding); --gpus %d is not supported" % args.gpus)

    import numpy as np
    import torch

    import paper_2604_06836_amd as stq
    from paper_2604_06836_amd import binding
    from workloads import configs
    from workloads.harness import DeviceModel, hparams

    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU (and libstq.so built for gfx950)")
    if args.copy_calibration:
        return copy_calibration(torch)
    stq.load_library()  # fails loudly if the HIP library is missing
    w = configs.get_workload(args.workload)
    # default: the configuration's own step count, repeated on the small workloads so that the timed
    # region lasts a few hundred milliseconds
    steps = args.steps if args.steps is not None else max(w.steps, min(200, int(1.5e11 // w.numel)))
    L = len(w.tensors)
    plan = w.initial_plan()
    ctx = stq.Context(0, max(L, 16))
    dm = DeviceModel(ctx, w, plan, spare_width=8 if w.transitions != "none" else 0)
    stream = torch.cuda.current_stream()

    # two resident gradient sets, alternated, so consecutive steps see different gradients
    grads = [dm.grad, [torch.empty_like(g) for g in dm.grad]]
    for k in (0, 1):
        for l in range(L):
            grads[k][l].copy_(w.gen_grad(l, k + 1, dm.device))
    tensor_sets = []
    for k in (0, 1):
        dm.grad = grads[k]
        dm._rebuild()
        tensor_sets.append(dm.tensors)

    decide_every_step = w.transitions == "decide_every_step"
    stats_arg = ("grad" if args.stats == "grad" else True) if decide_every_step else False
    ema = binding.DecideState(0, 0, 0)
    ladder = None
    kernel_ms, repacked = [], 0

    fused = args.transition == "fused"
    pending = None  # fused mode: the plan that the next step adopts
    use_engine = args.transition in ("engine", "engine-alg1")
    if use_engine and not decide_every_step:
        sys.exit("bench.py: --transition engine is for the workloads that decide every step (gpt2-xl)")
    if use_engine and args.warmup < 1:
        sys.exit("bench.py: --transition engine needs --warmup >= 1 (the first step calibrates the ladder on the host)")
    engine = None   # engine mode: created after the first step has calibrated the ladder
    import ctypes
    grad_ptrs = [(ctypes.c_void_p * L)(*[g.data_ptr() for g in grads[k]]) for k in (0, 1)]

    # The kernel's duration is taken with HIP events around the launches of at most 32 of the timed steps,
    # evenly spaced: every record of a timing event draws on a pool of the runtime that refills in steps of
    # tens of milliseconds (seen after about 160 records), which would stall the host inside the timed region.
    stride = max(1, (steps + 31) // 32)
    timed_steps = 0

    def one_step(t, timed):
        nonlocal plan, ladder, repacked, pending, engine, timed_steps
        events = timed and timed_steps % stride == 0
        if timed:
            timed_steps += 1
        k = t % 2
        dm.grad = grads[k]
        dm.tensors = tensor_sets[k]
        if w.transitions == "switch10pct_every5":
            new_plan = w.switch_plan(plan, t)
            if new_plan != plan:
                if fused:
                    pending = new_plan
                else:
                    repacked += dm.apply_plan(new_plan, also_patch=(tensor_sets[1 - k],))
                    plan = new_plan
        if events:
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
        if engine is not None:
            engine.step(hparams(w, t), 1, grad_ptrs[k], dm.stream)
            if events:
                e1.record(stream)
                kernel_ms.append((e0, e1))
            return
        if pending is not None:
            repacked += dm.step_transition(t, pending, stats=stats_arg, also_patch=(tensor_sets[1 - k],))
            plan, pending = pending, None
        else:
            dm.step(t, stats=stats_arg)
        if events:
            e1.record(stream)
            kernel_ms.append((e0, e1))
        if decide_every_step:
            st = ctx.stats(L, dm.stream)
            if ladder is None:
                _, sc = stq.decide(binding.DecideState(0, 0, 0), st, t, alpha=0.3, tau=4.0, thr=(), bits=(4,))
                ladder = calibrate_ladder(sc, w.p_m)
            new_plan, _ = stq.decide(ema, st, t, alpha=0.3, tau=4.0, v_offset=-0.5, thr=ladder, bits=w.bits_m)
            if fused:
                pending = new_plan if new_plan != plan else None
            else:
                repacked += dm.apply_plan(new_plan, also_patch=(tensor_sets[1 - k],))
                plan = new_plan
            if use_engine:
                # hand the loop over to the device: same ladder, the EMAs as they are now
                second = [(dm._spare[(l, 0)].data_ptr(), dm._spare[(l, 1)].data_ptr()) for l in range(L)]
                engine = ctx.engine(dm.tensors, second, dm.cplan, 8, w.K, alpha=0.3, tau=4.0, v_offset=-0.5,
                                    thr=ladder, bits=w.bits_m, ema=ema, alg1_order=args.transition == "engine-alg1",
                                    stream=dm.stream)

    t = 0
    for _ in range(args.warmup):
        t += 1
        one_step(t, False)
    torch.cuda.synchronize()
    repacked = 0
    dm.repack_bytes = 0
    t0 = time.perf_counter()
    for _ in range(steps):
        t += 1
        one_step(t, True)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0

    if engine is not None:
        plan = engine.read(dm.stream)["stored"]
        engine.close()
        repacked = None  # the host never sees the individual decisions
    n = w.numel
    ms_per_step = dt * 1e3 / steps
    kms = [a.elapsed_time(b) for a, b in kernel_ms]
    k_avg_ms = sum(kms) / len(kms)
    bpp = w.bytes_per_param(plan)
    alg_bytes = bpp * n
    achieved = alg_bytes / (k_avg_ms * 1e-3) / 1e9
    out = {
        "metric": "quantized-Adam step params/sec",
        "value": n * steps / dt,
        "unit": "params/s",
        "n_gpus": 1, "steps": steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": w.name, "configs_index": w.cfg, "params": n, "tensors": L, "block": w.K,
                   "grad_dtype": w.grad_dtype, "avg_state_bits": round(w.avg_bits(plan), 3),
                   "transition": args.transition, "changed_states_in_timed_region": repacked,
                   "repack_bytes_in_timed_region": dm.repack_bytes,
                   "statistics": ("gradient" if (args.stats == "grad" or use_engine) else "all")
                   if decide_every_step else "none"},
        "roofline": {"bound": "hbm", "kernel": "step_kernel", "achieved": achieved, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": None,
                     "kernel_ms_avg": k_avg_ms, "algorithmic_bytes_per_param": bpp,
                     "algorithmic_bytes_per_launch": alg_bytes},
    }
    # Counter-derived figures (HBM bytes per launch, vector-ALU utilisation) come from separate rocprofv3
    # --pmc runs of this same command, stored under profiles/ with the hash of the kernel sources they
    # were taken at; figures of another version of the kernel are not reported.
    src_hash = kernel_source_hash()
    out["roofline"]["kernel_source_sha256"] = src_hash
    traffic_file = os.path.join(ROOT, "profiles", "step_kernel_traffic.json")
    if os.path.exists(traffic_file):
        tr = json.load(open(traffic_file)).get(w.name + ("-engine" if args.transition == "engine" else ("-engine-alg1" if use_engine else "")))
        if tr and tr.get("kernel_source_sha256") == src_hash:
            out["roofline"]["traffic"] = tr["hbm_bytes_per_launch"]
            # the same counters over this run's kernel duration: HBM GB/s as the counters see it
            out["roofline"]["traffic_GBps"] = tr["hbm_bytes_per_launch"] / (k_avg_ms * 1e-3) / 1e9
            if "valu_insts_per_param" in tr:
                # The second roof of this kernel: vector instructions.  One fp32 VALU instruction per lane and
                # cycle on 256 CUs x 4 SIMDs x 16 lanes at 2.4 GHz (the published 157.3 TFLOP/s counts packed
                # fused multiply-adds, four flops per lane and cycle, which this arithmetic contract rules out).
                lane_insts = tr["valu_insts_per_param"] * n / (k_avg_ms * 1e-3) / 1e12
                out["roofline"]["alu"] = {"valu_insts_per_param": tr["valu_insts_per_param"], "achieved": lane_insts,
                                          "peak": ALU_PEAK_TLANE, "unit": "T lane-instructions/s",
                                          "frac": lane_insts / ALU_PEAK_TLANE, "valu_busy": tr.get("valu_busy"),
                                          "shader_clock_ghz": tr.get("shader_clock_ghz")}
        elif tr:
            out["roofline"]["traffic_note"] = "profiles/step_kernel_traffic.json holds counters of another version of the kernel (%s)" % tr.get("kernel_source_sha256")
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, w.initial_plan())
    ctx.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
