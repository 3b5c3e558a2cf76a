#!/usr/bin/env python3
"""Benchmark of the DD-EF-SGD hot path on one MI355X.

A "step" is one full iteration of the path through the C-ABI: ddef_grad, ddef_ef_compress,
ddef_aggregate, ddef_apply_delayed, for all n workers, on the GPT-2-small-sized workload
(d = 124e6 fp32, n = 8, delta = 0.001, tau = 8, Student-t3 gradient noise).  Inputs are
synthetic, generated from the workload's seed and resident in HBM before the timed region.

Prints ONE JSON line: whole-step throughput in gradient elements/s (n*d per step), a roofline
object for the dominant kernel (algorithmic bytes per launch / its average duration, measured
here with HIP events on the library's stream), and the CPU oracle timed on this machine's cores on
a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
# Ceiling for vector ALU work, in lane-instructions per second: the chip's fp32 vector peak of
# 157.3 TFLOP/s counts a fused multiply-add as two operations, i.e. 78.6e12 lane-instructions per
# second (256 compute units x 128 fp32 lanes per clock x 2.4 GHz).  Integer, 64-bit and correctly
# rounded division / square-root sequences issue no faster, so no kernel can exceed it.
VALU_PEAK_TINSTR = 157.3 / 2.0
# vector lane-instructions k_grad executes per noise draw, by noise kind: SQ_INSTS_VALU x 64 / draws
# (profiles/k_grad_C3_valu.txt)
VALU_PER_DRAW = {2: 162.2}

# algorithmic bytes per (worker, element) of each streaming kernel, per launch over n*d
ALGO_BYTES_PER_ELEM = {
    "k_ef_filter": 12.0,       # read e, read g, write p (the candidate filter rides along)
    "k_ef_filter_split": 12.0,  # the same pass for dense messages (sure / band split of the candidates)
    "k_ef_filter_fused": 8.0,  # read e, write p; the gradient is generated in registers
    "k_ef_randk": 12.0,        # same pass for Random-k (+ 1/8 byte of bitmap)
    "k_grad": 4.0,             # write g (+ 12/n shared reads, not counted)
    "k_digit_hist": 4.0, "k_chunk_count": 4.0, "k_chunk_emit": 4.0,   # whole-row search passes
}


class HipEvents:
    """HIP events on a stream of this process's own, through the HIP runtime's C API: the time the
    GPU spends between two points of the stream, without the host's waits in it."""

    def __init__(self):
        import ctypes as C
        self.C = C
        self.hip = C.CDLL("libamdhip64.so")
        self.stream = C.c_void_p()
        self._ok(self.hip.hipStreamCreateWithFlags(C.byref(self.stream), C.c_uint(1)), "hipStreamCreateWithFlags")  # non-blocking
        self.events = []

    def _ok(self, rc, what):
        if rc != 0:
            raise RuntimeError(f"{what} failed with HIP error {rc}")

    def mark(self):
        ev = self.C.c_void_p()
        self._ok(self.hip.hipEventCreate(self.C.byref(ev)), "hipEventCreate")
        self._ok(self.hip.hipEventRecord(ev, self.stream), "hipEventRecord")
        self.events.append(ev)
        return len(self.events) - 1

    def ms(self, a, b):
        out = self.C.c_float()
        self._ok(self.hip.hipEventSynchronize(self.events[b]), "hipEventSynchronize")
        self._ok(self.hip.hipEventElapsedTime(self.C.byref(out), self.events[a], self.events[b]), "hipEventElapsedTime")
        return float(out.value)

    def close(self):
        for ev in self.events:
            self.hip.hipEventDestroy(ev)
        self.events = []
        self.hip.hipStreamDestroy(self.stream)


def source_digest():
    """sha256 over the library's sources (csrc/ and the public header), in a fixed order: names the
    code a hardware-counter summary under profiles/ was measured on."""
    import hashlib
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2507_17346_amd", "csrc")
    for path in sorted(os.path.join(csrc, f) for f in os.listdir(csrc)) + [os.path.join(ROOT, "include", "ddef.h")]:
        h.update(os.path.basename(path).encode())
        with open(path, "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def counter_summary(kernel, workload_name):
    """The committed hardware-counter summary of `kernel` on a workload (rocprofv3 --pmc FETCH_SIZE /
    WRITE_SIZE, scaled by the copy yardstick) as a dict of its `key: value` lines, or None."""
    path = os.path.join(ROOT, "profiles", f"{kernel}_{workload_name}_pmc.txt")
    out = {}
    try:
        for line in open(path):
            if ":" in line and not line.startswith((" ", "#", "\t")):
                key, value = line.split(":", 1)
                if key.replace("_", "").isalnum():
                    out[key] = value.strip()
    except OSError:
        return None
    return out


def measured_traffic(kernel, workload_name, key="traffic_bytes_per_launch"):
    """(bytes, provenance): HBM bytes the counters saw, from the committed summary -- but only if that
    summary was measured on the very sources this run was built from (its source_digest line equals
    source_digest()); otherwise (None, provenance), so that a figure from older code is never
    passed off as this run's."""
    summary = counter_summary(kernel, workload_name)
    if not summary or key not in summary:
        return None, None
    prov = {"file": f"profiles/{kernel}_{workload_name}_pmc.txt", "commit": summary.get("commit"),
            "box": summary.get("box"), "source_digest": summary.get("source_digest"),
            "current_source_digest": source_digest()}
    prov["matches_this_build"] = prov["source_digest"] == prov["current_source_digest"]
    if not prov["matches_this_build"]:
        return None, prov
    return float(summary[key]), prov


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def cpu_baseline(w, lam, xstar, x0, sample_d, budget_note, max_threads=None, compressor=0, rand_ratio=0.2, zeta=0.0):
    """The oracle, as it stands, on a bounded sample: one non-empty iteration over the first
    sample_d coordinates of the workload (all n workers, one thread per worker unless capped)."""
    import oracle
    cores = os.cpu_count() or 1
    try:
        cores = len(os.sched_getaffinity(0))
    except Exception:
        pass
    env_cap = os.environ.get("OMP_NUM_THREADS")
    if env_cap and env_cap.isdigit():
        cores = min(cores, int(env_cap))
    threads = max(1, min(w.n, cores))
    if max_threads:
        threads = min(threads, max_threads)
    o = oracle.Oracle(sample_d, w.n, 0, threads=threads)
    o.set_problem(lam[:sample_d], xstar[:sample_d], x0[:sample_d], w.seed, w.noise_kind, w.noise_scale)
    o.set_tau(0)
    o.set_compressor(compressor)
    o.set_composed(rand_ratio)
    o.set_heterogeneity(zeta)
    t0 = time.perf_counter()
    o.step(w.deltas[0], w.lr)
    dt = time.perf_counter() - t0
    o.close()
    return {"value": w.n * sample_d / dt, "unit": "elements/s", "cores": threads, "kind": "oracle",
            "host": host_description(),
            "sample": f"1 non-empty iteration, all {w.n} workers, first {sample_d} of {w.d} coordinates "
                      f"({dt:.1f} s wall, {threads} threads){budget_note}"}


def host_description():
    """CPU model and the number of logical CPUs this process may use."""
    model = "unknown"
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.lower().startswith("model name"):
                    model = line.split(":", 1)[1].strip()
                    break
    except OSError:
        pass
    try:
        usable = len(os.sched_getaffinity(0))
    except Exception:
        usable = os.cpu_count() or 1
    return {"cpu_model": model, "logical_cpus": os.cpu_count() or 1, "usable_cpus": usable}


def describe(w, sched, k_of):
    noise = {0: "no noise", 1: f"Gaussian noise x{w.noise_scale}", 2: f"Student-t3 noise x{w.noise_scale}"}[w.noise_kind]
    if w.adaptive_period > 0:
        pairs = sorted({sched(t) for t in range(0, w.steps, w.adaptive_period)})
        ratio = f"(tau, delta) re-chosen by DeCo every {w.adaptive_period} iterations from the seeded trace: {pairs}"
    elif len(w.deltas) > 1:
        ratio = f"delta swept over {list(w.deltas)} in segments of {w.steps} iterations, tau={w.tau}"
    else:
        ratio = f"delta={w.deltas[0]} (k={k_of(w.deltas[0])}), tau={w.tau}"
    return f"{w.name}: d={w.d} fp32, n={w.n} workers, {ratio}, lr={w.lr}, {noise}, seed {w.seed}"


def make_schedule(w, binding, workloads):
    """(tau, delta) for iteration t.  Fixed for C1-C3; C4 sweeps its three ratios in segments of
    `steps` iterations after the empty start-up; C5 re-chooses both from the seeded network trace
    with DeCo (Algorithm 3) every `adaptive_period` iterations, clamped to the workload's bounds."""
    if w.adaptive_period > 0:
        tr = workloads.network_trace(w)
        pairs = []
        for a, b in zip(tr.bandwidth_bps, tr.latency_s):
            tau, delta = binding.deco(tr.v_g_bits, a, b, tr.t_comp_s)
            pairs.append((int(min(max(tau, tr.tau_bounds[0]), tr.tau_bounds[1])),
                          float(min(max(delta, tr.delta_bounds[0]), tr.delta_bounds[1]))))
        return lambda t: pairs[(t // w.adaptive_period) % len(pairs)]
    if len(w.deltas) > 1:
        return lambda t: (w.tau, w.deltas[(max(t - w.tau, 0) // w.steps) % len(w.deltas)])
    return lambda t: (w.tau, w.deltas[0])


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="C3")
    ap.add_argument("--d", type=int, default=None, help="shrink d (debug only; not a valid bench)")
    ap.add_argument("--delta", type=float, default=None,
                    help="fix the compression ratio (study runs only; the default follows the workload)")
    ap.add_argument("--rand-ratio", type=float, default=0.2,
                    help="composed compressor: share of the coordinates its Random-k stage keeps")
    ap.add_argument("--compressor", choices=["topk", "randk", "composed"], default="topk",
                    help="sparsifier: the paper's default Top-k, or its appendix's Random-k")
    ap.add_argument("--prefetch", type=int, default=0,
                    help="1: generate the next iteration's gradient on a second stream meanwhile")
    ap.add_argument("--fuse-grad", type=int, default=0,
                    help="1: generate the gradient inside the accumulate pass (never stored)")
    ap.add_argument("--graph", type=int, default=0,
                    help="1: steady iterations are replayed from one recorded HIP graph (ddef_step)")
    ap.add_argument("--queue-form", type=int, default=0,
                    help="1: server state as a message queue (one model, tau_max+1 queued messages) "
                         "instead of the snapshot ring; same iterates for constant tau")
    ap.add_argument("--zeta", type=float, default=0.0,
                    help="heterogeneous local objectives: worker i's optimum is x* + zeta u_i (0: IID, the default)")
    ap.add_argument("--dense-split", type=int, default=1,
                    help="0: dense messages go through the selection whole (study runs; default 1: candidates "
                         "sure to be sent bypass it)")
    ap.add_argument("--full-select", type=int, default=0,
                    help="1: every selection searches its whole row (no candidate filter; study runs only)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-probe", type=int, default=0,
                    help="launch the plain copy yardstick this many times (for hardware byte counters)")
    ap.add_argument("--cpu-sample-d", type=int, default=None)
    ap.add_argument("--print-source-digest", action="store_true",
                    help="print the digest of the library's sources (for a counter summary under profiles/) and exit")
    args = ap.parse_args()
    if args.print_source_digest:
        print(source_digest())
        return
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (all workers' shares resident in one HBM); "
                 "--gpus N with N > 1 is not supported")

    import numpy as np
    from paper_2507_17346_amd import binding, workloads

    w = workloads.get(args.workload, d=args.d)
    if args.delta is not None:
        w = workloads.replace(w, deltas=(args.delta,), adaptive_period=0, tau=w.tau if w.adaptive_period == 0 else 8)
    sched = make_schedule(w, binding, workloads)
    delta = sched(0)[1]
    log(f"workload {w.name}: d={w.d} n={w.n} delta={delta} (Top-k of the whole row: k={binding.k_from_delta(delta, w.d)}) tau={sched(0)[0]} lr={w.lr} "
        f"noise kind {w.noise_kind} scale {w.noise_scale} seed {w.seed}")
    t0 = time.perf_counter()
    lam, xstar, x0 = workloads.make_problem(w)
    log(f"inputs generated in {time.perf_counter() - t0:.1f} s")
    ctx = binding.Context(w.d, w.n, w.tau_max, queue_form=bool(args.queue_form))
    ctx.set_problem(lam, xstar, x0, w.seed, w.noise_kind, w.noise_scale)
    compressor = {"topk": binding.COMPRESSOR_TOPK, "randk": binding.COMPRESSOR_RANDK,
                  "composed": binding.COMPRESSOR_COMPOSED}[args.compressor]
    ctx.set_compressor(compressor)
    if args.compressor == "composed":
        ctx.set_composed(args.rand_ratio)
    if args.zeta:
        ctx.set_heterogeneity(args.zeta)

    def sent_ratio(dl):
        """entries per worker in a message, as a share of d"""
        if args.compressor == "composed":
            return binding.k_from_delta(dl, binding.k_from_delta(args.rand_ratio, w.d)) / w.d
        return binding.k_from_delta(dl, w.d) / w.d
    ctx.set_option(binding.OPT_PREFETCH_GRAD, 1 if args.prefetch else 0)
    ctx.set_option(binding.OPT_FUSE_GRAD, 1 if args.fuse_grad else 0)
    ctx.set_option(binding.OPT_GRAPH, 1 if args.graph else 0)
    ctx.set_option(binding.OPT_DENSE_SPLIT, 1 if args.dense_split else 0)
    if args.full_select:
        ctx.set_option(binding.OPT_FORCE_FULL_SELECT, 1)

    state = {"tau": None}

    def begin_iteration():
        tau, dl = sched(ctx.t)
        if tau != state["tau"]:
            ctx.set_tau(tau)
            state["tau"] = tau
        return dl

    def whole_step():
        dl = begin_iteration()
        ctx.step(dl, w.lr)

    # warm-up: the empty iterations before anything arrives, then W real ones so that the error
    # buffers are populated and the selection runs in its steady state
    for _ in range(sched(0)[0] + args.warmup):
        whole_step()
    ctx.sync()

    # ---- timed region: exactly K whole steps ------------------------------------------------
    t0 = time.perf_counter()
    for _ in range(args.steps):
        whole_step()
    ctx.sync()
    elapsed = time.perf_counter() - t0
    ms_per_step = 1e3 * elapsed / args.steps
    elems = w.n * w.d
    value = elems * args.steps / elapsed

    # ---- the same K steps again, once with a wait after each call (time per call), once with
    # HIP events around every kernel launch on the library's stream (time per kernel) -----------
    phase = {"grad": 0.0, "ef_compress": 0.0, "aggregate": 0.0, "apply_delayed": 0.0}
    samples = {k: [] for k in phase}
    floor_bytes_sum = 0.0
    for _ in range(args.steps):
        delta = begin_iteration()
        floor_bytes_sum += (12.0 + 24.0 * sent_ratio(delta) + 16.0 / w.n) * w.n * w.d
        for name, call in (("grad", ctx.grad), ("ef_compress", lambda: ctx.ef_compress(delta, w.lr)),
                           ("aggregate", ctx.aggregate), ("apply_delayed", lambda: ctx.apply_delayed(w.lr))):
            ctx.sync()
            p0 = time.perf_counter()
            call()
            ctx.sync()
            dt = time.perf_counter() - p0
            phase[name] += dt
            samples[name].append(1e3 * dt)
    phase_ms = {k: 1e3 * v / args.steps for k, v in phase.items()}
    phase_median = {k: sorted(v)[len(v) // 2] for k, v in samples.items()}
    phase_min = {k: min(v) for k, v in samples.items()}

    # ---- and once more with HIP events around each call on the stream, no host wait in between:
    # the time the GPU needs per call, launch gaps between its kernels included
    ctx.sync()
    hev = HipEvents()
    ctx.set_stream(hev.stream.value)
    marks = []
    floor_bytes_sum = 0.0
    for _ in range(args.steps):
        delta = begin_iteration()
        floor_bytes_sum += (12.0 + 24.0 * sent_ratio(delta) + 16.0 / w.n) * w.n * w.d
        row = [hev.mark()]
        for call in (ctx.grad, lambda: ctx.ef_compress(delta, w.lr), ctx.aggregate, lambda: ctx.apply_delayed(w.lr)):
            call()
            row.append(hev.mark())
        marks.append(row)
    ctx.sync()
    gpu_samples = {name: [hev.ms(r[i], r[i + 1]) for r in marks]
                   for i, name in enumerate(("grad", "ef_compress", "aggregate", "apply_delayed"))}
    gpu_ms = {name: sum(v) / args.steps for name, v in gpu_samples.items()}
    gpu_median = {name: sorted(v)[len(v) // 2] for name, v in gpu_samples.items()}
    gpu_min = {name: min(v) for name, v in gpu_samples.items()}
    ctx.set_stream(None)
    hev.close()
    log("  per call, GPU time between HIP events (ms): " + ", ".join(f"{k} {v:.3f}" for k, v in gpu_ms.items()))
    full0 = ctx.full_select_count()
    ctx.profile_enable(True)
    for _ in range(args.steps):
        whole_step()
    prof = ctx.profile_read()
    ctx.profile_enable(False)
    full_selects = ctx.full_select_count() - full0
    kernels = {k: {"launches": c, "avg_ms": ms / c, "ms_per_step": ms / args.steps}
               for k, (c, ms) in prof.items() if c}
    for k, v in sorted(kernels.items(), key=lambda kv: -kv[1]["ms_per_step"]):
        log(f"  {k:18s} launches/step {v['launches'] / args.steps:6.1f}  avg {v['avg_ms']:.4f} ms  "
            f"per step {v['ms_per_step']:.4f} ms")
    log("  per call (ms): " + ", ".join(f"{k} {v:.3f}" for k, v in phase_ms.items()))

    # what a plain copy reaches on this box (read + write of one row each way), for "% of achievable"
    ctx.profile_enable(True)
    for _ in range(max(5, args.copy_probe)):
        probe_bytes = ctx.copy_probe()
    copy_cnt, copy_ms = ctx.profile_read()["k_copy_f4"]
    ctx.profile_enable(False)
    copy_gbps = 2.0 * probe_bytes / (copy_ms / copy_cnt * 1e-3) / 1e9
    log(f"  copy yardstick k_copy_f4: {probe_bytes} bytes each way, {copy_ms / copy_cnt:.4f} ms, {copy_gbps:.0f} GB/s")

    # the dominant kernel of the path is its accumulate pass (12 B per worker and element; 8 B with the
    # gradient fused in), in whichever form this workload runs it most
    passes = [k for k in ("k_ef_filter", "k_ef_filter_split", "k_ef_filter_fused", "k_ef_randk") if k in kernels]
    dominant = max(passes, key=lambda k: kernels[k]["ms_per_step"])
    per_elem = ALGO_BYTES_PER_ELEM[dominant]
    algo_bytes = per_elem * elems
    achieved = algo_bytes / (kernels[dominant]["avg_ms"] * 1e-3) / 1e9
    roofline = {"bound": "hbm", "kernel": dominant, "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": achieved / HBM_PEAK_GBS, "copy_kernel_GBps": copy_gbps,
                "frac_of_copy_kernel": achieved / copy_gbps,
                "traffic": None, "traffic_source": None,
                "algorithmic_bytes_per_launch": algo_bytes,
                "avg_launch_ms": kernels[dominant]["avg_ms"]}
    if args.d is None:
        roofline["traffic"], roofline["traffic_source"] = measured_traffic(dominant, w.name)

    if dominant == "k_ef_filter_fused" and w.noise_kind in VALU_PER_DRAW:
        # with the generator fused in, the pass is bound by vector issue like k_grad: lane-instructions
        # per element = k_grad's per draw + k_ef_filter's 82 wave instructions per 256 coordinates
        per_elem_instr = VALU_PER_DRAW[w.noise_kind] + 82.1 * 64.0 / 256.0
        rate = per_elem_instr * elems / (kernels[dominant]["avg_ms"] * 1e-3) / 1e12
        roofline = {"bound": "alu", "kernel": dominant, "achieved": rate, "peak": VALU_PEAK_TINSTR,
                    "unit": "T lane-instr/s", "frac": rate / VALU_PEAK_TINSTR, "traffic": None,
                    "lane_instr_per_element": per_elem_instr, "avg_launch_ms": kernels[dominant]["avg_ms"],
                    "hbm_GBps": 4.0 * elems * 2 / (kernels[dominant]["avg_ms"] * 1e-3) / 1e9}

    # the gradient generator is bound by vector ALU work (Philox + Box-Muller), not by HBM: report
    # its rate in draws and in vector lane-instructions (count per draw from the hardware counter
    # SQ_INSTS_VALU, profiles/k_grad_C3_valu.txt) next to the nominal plain-VALU issue rate
    grad_info = None
    if "k_grad" in kernels:
        g_s = kernels["k_grad"]["avg_ms"] * 1e-3
        grad_info = {"kernel": "k_grad", "bound": "alu", "avg_launch_ms": kernels["k_grad"]["avg_ms"],
                     "draws_per_s": elems / g_s, "written_GBps": 4.0 * elems / g_s / 1e9}
        if w.noise_kind in VALU_PER_DRAW:
            grad_info["valu_lane_instr_per_draw"] = VALU_PER_DRAW[w.noise_kind]
            grad_info["valu_T_lane_instr_per_s"] = VALU_PER_DRAW[w.noise_kind] * elems / g_s / 1e12
            grad_info["peak_valu_T_lane_instr_per_s"] = VALU_PEAK_TINSTR
            grad_info["frac_of_valu_peak"] = grad_info["valu_T_lane_instr_per_s"] / VALU_PEAK_TINSTR

    # metric of the path proper (EF + top-k + aggregate + apply), gradient generation aside
    path_ms = gpu_ms["ef_compress"] + gpu_ms["aggregate"] + gpu_ms["apply_delayed"]
    floor_bytes = floor_bytes_sum / args.steps
    path = {"ms": path_ms, "ms_with_host_waits": phase_ms["ef_compress"] + phase_ms["aggregate"] + phase_ms["apply_delayed"],
            "elements_per_s": elems / (path_ms * 1e-3),
            "floor_bytes_per_step": floor_bytes,
            "floor_GBps": floor_bytes / (path_ms * 1e-3) / 1e9,
            "floor_frac_of_peak": floor_bytes / (path_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
            # the same rate over ddef_ef_compress + ddef_aggregate alone; on the GPU the sum of the
            # messages is formed inside ddef_apply_delayed (fused with the model update), so this
            # figure leaves the summation out as well and is not a rate of the whole server side
            "elements_per_s_without_apply_delayed":
                elems / ((gpu_ms["ef_compress"] + gpu_ms["aggregate"]) * 1e-3)}
    # bytes the hardware counters saw for all kernels of the path in one iteration (default
    # configuration of this workload only), and the rate and share of the peak they give
    counted = None
    if args.d is None and args.delta is None and args.compressor == "topk" and not (
            args.fuse_grad or args.prefetch or args.queue_form or args.full_select):
        counted, _ = measured_traffic("k_ef_filter", w.name, key="path_traffic_bytes_per_step")
    if counted:
        path["measured_bytes_per_step"] = counted
        path["measured_bytes_per_worker_element"] = counted / elems
        path["measured_GBps"] = counted / (path_ms * 1e-3) / 1e9
        path["measured_frac_of_peak"] = counted / (path_ms * 1e-3) / 1e9 / HBM_PEAK_GBS

    out = {
        "metric": "EF+top-k+aggregate step: gradient elements/s and achieved HBM GB/s (% of peak)",
        "value": value, "unit": "elements/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": describe(w, sched, lambda dl: round(sent_ratio(dl) * w.d)),
                   "d": w.d, "n": w.n, "k": round(sent_ratio(sched(ctx.t)[1]) * w.d), "tau": sched(ctx.t)[0],
                   "compressor": args.compressor, **({"rand_ratio": args.rand_ratio} if args.compressor == "composed" else {}), **({"zeta": args.zeta} if args.zeta else {}), "prefetch_grad": bool(args.prefetch), "fuse_grad": bool(args.fuse_grad), "server_state": "queue" if args.queue_form else "ring", "hip_graph": bool(args.graph), "dense_split": bool(args.dense_split), **({"full_select": True} if args.full_select else {}),
                   "step": "grad + ef_compress + aggregate + apply_delayed, all workers"},
        "roofline": roofline,
        "grad": grad_info,
        "ef_topk_aggregate_apply": path,
        "ms_per_call_gpu_events": gpu_ms,
        "ms_per_call_gpu_events_median": gpu_median,
        "ms_per_call_gpu_events_min": gpu_min,
        "ms_per_call": phase_ms,
        "ms_per_call_median": phase_median,
        "ms_per_call_min": phase_min,
        "device": ctx.device_info(),
        "kernels_ms_per_step": {k: round(v["ms_per_step"], 5) for k, v in kernels.items()},
        "full_row_selects_per_step": full_selects / args.steps,
    }

    if not args.no_cpu_baseline:
        sample_d = args.cpu_sample_d or min(w.d, 124_000_000)
        note = ""
        try:
            out["cpu_baseline"] = cpu_baseline(w, lam, xstar, x0, sample_d, note, compressor=compressor, rand_ratio=args.rand_ratio, zeta=args.zeta)
        except MemoryError:
            out["cpu_baseline"] = cpu_baseline(w, lam, xstar, x0, w.d // 8, "; reduced: host memory",
                                               compressor=compressor, rand_ratio=args.rand_ratio, zeta=args.zeta)
        # the same oracle on one thread, on an eighth of the coordinates to keep the run short
        out["cpu_baseline_single_thread"] = cpu_baseline(w, lam, xstar, x0, max(1, sample_d // 8), "",
                                                         max_threads=1, compressor=compressor, rand_ratio=args.rand_ratio, zeta=args.zeta)
    ctx.close()
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
