#!/usr/bin/env python3
"""Benchmark of the checkpoint-selection hot path on one MI355X.

One step = one pass of the whole path over one configuration's input.  The default is the stress
configuration (5): ckpt_eval_peak (static, then dynamic objective) and ckpt_solve_linear on a batch
of 1,048,576 chains of n = 256 layers, and ckpt_solve_cubic on one chain of n = 4096 layers; sizes
are 4 KiB multiples in [1 MiB, 128 MiB], seed 2.  Inputs are generated on the host once, copied to
HBM, and stay there; the timed region contains only library calls.  Prints one JSON line.

Other modes:
  --config 1..4          time that configuration's step instead (small ones are launch-bound)
  --peaks                only the measurement probes (HBM read/copy, vector issue rate, LDS rate)
  --counter-probes       after the steps, one launch each of the copy and the vector-issue probe
                         (kernels of known work, to scale the profiler's counters)
  --summarize DIR..      no GPU work: fold rocprofv3 CSV output directories into
                         profiles/counters.json (per-kernel counter values per dispatch, with
                         the hash of the kernel sources they were measured on)
"""
import argparse
import csv
import glob
import hashlib
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
# 32-bit vector lane-operations per second: 256 CUs x 4 SIMDs x 32 lanes per clock x 2.4 GHz, the rate
# behind the part's 157.3 TFLOP/s of fp32 vector FMA.  Add, logic and shift-right instructions are
# measured near it (profiles/peaks.json); compare, select, min and max issue at half of it.
INT32_PEAK_TOPS = 256 * 4 * 32 * 2.4e9 / 1e12
INT32_SELECT_CLASS_TOPS = INT32_PEAK_TOPS / 2
CUBIC_OPS_PER_CELL = 3  # one add and two compare-selects (queue push / pop) per recurrence cell
COUNTERS_JSON = os.path.join(ROOT, "profiles", "counters.json")
PEAKS_JSON = os.path.join(ROOT, "profiles", "peaks.json")
COPY_PROBE_BYTES = 1048576 * 257 * 8          # the copy probe run by --counter-probes
VALU_PROBE_WAVES, VALU_PROBE_ITERS = 256 * 4 * 8, 256  # and the vector-issue probe (256 instructions per iteration)
PAPER_CONTEXT = "Python on a Xeon Gold 6226R, VGG-19 (n=24): Algorithm 4 20 ms, Algorithm 6 1.1 ms per chain (Section 5.6)"


def log(*a):
    print(*a, file=sys.stderr, flush=True)


# ---------------------------------------------------------------------------------------------
# counters measured with rocprofv3, kept under profiles/ together with the hash of the sources
# ---------------------------------------------------------------------------------------------

def source_hash():
    """sha256 over the kernel sources and headers: counter values taken on other sources are stale."""
    h = hashlib.sha256()
    files = sorted(glob.glob(os.path.join(ROOT, "paper_2502_12499_amd", "csrc", "*.hip")) +
                   glob.glob(os.path.join(ROOT, "paper_2502_12499_amd", "csrc", "*.h")) +
                   glob.glob(os.path.join(ROOT, "include", "*.h")))
    for f in files:
        h.update(os.path.basename(f).encode())
        h.update(open(f, "rb").read())
    return h.hexdigest()


def short_kernel_name(name):
    """'void ckpt::(anonymous namespace)::cubic_shared_kernel<16, 64, false>(int, ...)' ->
    'cubic_shared_kernel<16, 64, false>'."""
    name = name.strip().strip('"')
    if name.startswith("void "):
        name = name[5:]
    depth = 0
    for i, ch in enumerate(name):       # cut the argument list: the first '(' outside <...> that is
        if ch == "<":                   # not the "(anonymous namespace)"
            depth += 1
        elif ch == ">":
            depth -= 1
        elif ch == "(" and depth == 0 and not name.startswith("(anonymous namespace)", i):
            name = name[:i]
            break
    return name.split("::")[-1]


def summarize(dirs, workload, profiled_steps):
    """Folds rocprofv3 output directories (CSV: *_counter_collection.csv, *_kernel_stats.csv) into
    one record: per kernel the mean counter value per dispatch, the mean duration and the number
    of dispatches per step (dispatches in the trace / steps the profiled command ran)."""
    kernels = {}
    for d in dirs:
        for f in glob.glob(os.path.join(d, "**", "*counter_collection.csv"), recursive=True):
            acc = {}
            for r in csv.DictReader(open(f)):
                acc.setdefault((short_kernel_name(r["Kernel_Name"]), r["Counter_Name"]), []).append(
                    float(r["Counter_Value"]))
            for (k, cn), v in acc.items():
                kernels.setdefault(k, {})[cn] = sum(v) / len(v)
        for f in glob.glob(os.path.join(d, "**", "*kernel_stats.csv"), recursive=True):
            for r in csv.DictReader(open(f)):
                k = kernels.setdefault(short_kernel_name(r["Name"]), {})
                k["avg_us"] = float(r["AverageNs"]) / 1e3
                k["per_step"] = int(r["Calls"]) / float(profiled_steps)
    return {"profiled_steps": profiled_steps, "source_hash": source_hash(), "workload": workload, "kernels": kernels,
            "note": "mean per dispatch; FETCH_SIZE and WRITE_SIZE in KiB; SQ_* summed over the chip; "
                    "written by `bench.py --summarize`"}


def load_counters(workload):
    """The counter record if it was taken on these sources and this workload, else None."""
    try:
        rec = json.load(open(COUNTERS_JSON))
    except (OSError, ValueError):
        return None
    if rec.get("source_hash") != source_hash() or rec.get("workload") != workload:
        return None
    return rec


def kernel_lane_ops(k, probe=None):
    """Executed 32-bit lane-operations of one dispatch: vector instructions x 64 lanes x the mean
    fraction of lanes active (thread-cycles over instruction-cycles x 64).  `probe` is the record of
    the vector-issue probe, whose instruction count and full lanes are known: both factors are
    scaled by what the counters read for it."""
    if k is None or "SQ_INSTS_VALU" not in k:
        return None
    inst_scale, lane_scale = 1.0, 1.0
    if probe and probe.get("SQ_INSTS_VALU"):
        inst_scale = VALU_PROBE_WAVES * VALU_PROBE_ITERS * 256.0 / probe["SQ_INSTS_VALU"]
        if probe.get("SQ_THREAD_CYCLES_VALU") and probe.get("SQ_ACTIVE_INST_VALU"):
            lane_scale = probe["SQ_ACTIVE_INST_VALU"] * 64.0 / probe["SQ_THREAD_CYCLES_VALU"]
    active = 1.0
    if k.get("SQ_THREAD_CYCLES_VALU") and k.get("SQ_ACTIVE_INST_VALU"):
        active = min(1.0, lane_scale * k["SQ_THREAD_CYCLES_VALU"] / (k["SQ_ACTIVE_INST_VALU"] * 64.0))
    return k["SQ_INSTS_VALU"] * inst_scale * 64.0 * active


def kernels_of(rec, prefix):
    """The kernels of one call: those whose name starts with `prefix` and that ran in the step."""
    return [k for n, k in sorted(rec["kernels"].items()) if n.startswith(prefix) and k.get("per_step")]


def call_lane_ops(rec, prefix):
    """Executed lane-operations of one call of the step: sum over its kernels, or None."""
    if rec is None:
        return None
    total = 0.0
    ks = kernels_of(rec, prefix)
    for k in ks:
        v = kernel_lane_ops(k, rec["kernels"].get("probe_valu_kernel<2>"))
        if v is None:
            return None
        total += v * k["per_step"]
    return total if ks else None


def traffic_bytes(rec, prefix):
    """HBM bytes per call of the kernels named `prefix`* (FETCH_SIZE + WRITE_SIZE per dispatch, each
    scaled by what the same counter reads for the copy probe of known size), or None."""
    if rec is None:
        return None
    probe = rec["kernels"].get("probe_copy_kernel")
    copy_bytes = rec.get("copy_probe_bytes")
    if not probe or not copy_bytes or "FETCH_SIZE" not in probe or "WRITE_SIZE" not in probe:
        return None
    f_scale = copy_bytes / (probe["FETCH_SIZE"] * 1024.0)
    w_scale = copy_bytes / (probe["WRITE_SIZE"] * 1024.0)
    total = 0.0
    ks = kernels_of(rec, prefix)
    for k in ks:
        if "FETCH_SIZE" not in k or "WRITE_SIZE" not in k:
            return None
        total += (k["FETCH_SIZE"] * 1024.0 * f_scale + k["WRITE_SIZE"] * 1024.0 * w_scale) * k["per_step"]
    return total if ks else None


# ---------------------------------------------------------------------------------------------
# timing helpers
# ---------------------------------------------------------------------------------------------

def timed_ms(torch, fn, reps, warm=1):
    """Median (and all) of `reps` HIP-event timings of fn() on the current stream, in ms."""
    for _ in range(warm):
        fn()
    torch.cuda.synchronize()
    ts = []
    for _ in range(reps):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        fn()
        b.record()
        torch.cuda.synchronize()
        ts.append(a.elapsed_time(b))
    return float(np.median(ts)), ts


def measure_peaks(reps=5):
    """What the part delivers on kernels of known work (include/ckpt_probe.h): HBM read and copy
    rates on the stress batch's 2.16 GB, the issue rate of 32-bit integer vector instructions and
    the LDS instruction rate.  Median of `reps` launches each, HIP events on the launch stream."""
    import torch
    from paper_2502_12499_amd import binding as B
    dev = torch.device("cuda:0")
    sink = torch.zeros(8, dtype=torch.int64, device=dev)
    out = {}
    nbytes = 1048576 * 257 * 8
    src = torch.empty(nbytes // 8, dtype=torch.int64, device=dev).random_()
    dst = torch.empty_like(src)
    t, _ = timed_ms(torch, lambda: B.ckpt_probe_hbm_read(src, sink), reps)
    out["hbm_read_GBs"] = nbytes / (t * 1e-3) / 1e9
    t, _ = timed_ms(torch, lambda: B.ckpt_probe_hbm_copy(src, dst), reps)
    out["hbm_copy_GBs_moved"] = 2 * nbytes / (t * 1e-3) / 1e9
    del src, dst
    waves = 256 * 4 * 8  # eight waves per SIMD
    for name, which in B.PROBE_VALU.items():
        ops = [0]

        def fn():
            ops[0] = B.ckpt_probe_valu(which, waves, 256, sink)
        t, _ = timed_ms(torch, fn, reps)
        out[name + "_TOPs"] = ops[0] / (t * 1e-3) / 1e12
    for name, which in B.PROBE_LDS.items():
        acc = [0]

        def fn():
            acc[0] = B.ckpt_probe_lds(which, 256 * 16, 2048, sink)
        t, _ = timed_ms(torch, fn, reps)
        out[name + "_bytes_per_clk_per_cu"] = acc[0] * 4 / (t * 1e-3) / 256 / 2.4e9
    out["nominal"] = {"hbm_GBs": HBM_PEAK_GBS, "int32_TOPs": INT32_PEAK_TOPS,
                      "int32_select_class_TOPs": INT32_SELECT_CLASS_TOPS}
    return out


def measured_peaks():
    try:
        return json.load(open(PEAKS_JSON))["peaks"]
    except (OSError, ValueError, KeyError):
        return None


def transfer_rates(torch, sample_bytes=1 << 28):
    """Host-to-device and device-to-host rates over pinned memory, on a 256 MiB sample."""
    dev = torch.device("cuda:0")
    host = torch.empty(sample_bytes, dtype=torch.uint8, pin_memory=True)
    devt = torch.empty(sample_bytes, dtype=torch.uint8, device=dev)
    t_h2d, _ = timed_ms(torch, lambda: devt.copy_(host, non_blocking=True), 3)
    t_d2h, _ = timed_ms(torch, lambda: host.copy_(devt, non_blocking=True), 3)
    return {"h2d_GBs": sample_bytes / (t_h2d * 1e-3) / 1e9, "d2h_GBs": sample_bytes / (t_d2h * 1e-3) / 1e9,
            "sample_bytes": sample_bytes}


# ---------------------------------------------------------------------------------------------
# workloads
# ---------------------------------------------------------------------------------------------

def config_name(cfg, seed, batch=None, n_batch=None, n_cubic=None):
    """The workload string of a configuration (no arrays are made)."""
    if cfg == 1:
        return "config 1: 1 chain n=12, 4 KiB x U{256..16384}, seed %d" % (0 if seed is None else seed)
    if cfg == 2:
        return "config 2: ResNet-152-shaped chain n=152, B=64 fp32"
    if cfg == 3:
        return "config 3: %d chains n=64, log-uniform 64 KiB..256 MiB, seed %d" % (batch or 65536,
                                                                                 1 if seed is None else seed)
    if cfg == 4:
        return "config 4: ResNet-1001-shaped chain n=1001, B=32 fp32"
    return ("stress: 1 chain n=%d (cubic) + %d chains n=%d (linear, eval_peak under both objectives), sizes 4 KiB x U{256..32768}, "
            "seed %d" % (n_cubic or 4096, batch or 1048576, n_batch or 256, 2 if seed is None else seed))


def make_config(cfg, seed, batch=None, n_batch=None, n_cubic=None):
    """Host arrays of configuration `cfg`: (name, batched sizes, their masks, the cubic solver's chains)."""
    from paper_2502_12499_amd import inputs
    name = config_name(cfg, seed, batch, n_batch, n_cubic)
    if cfg == 1:
        s = 0 if seed is None else seed
        d = inputs.uniform_aligned_chains(s, 12, 1, 256, 16384)
        return name, d, inputs.bernoulli_masks(s, 12, 1), d
    if cfg == 2:
        d = inputs.config2()
        return name, d, inputs.bernoulli_masks(0, 152, 1), d
    if cfg == 3:
        s = 1 if seed is None else seed
        d = inputs.log_uniform_chains(s, 64, batch or 65536)
        return name, d, inputs.bernoulli_masks(s, 64, batch or 65536), d
    if cfg == 4:
        d = inputs.config4()
        return name, d, inputs.bernoulli_masks(0, 1001, 1), d
    s = 2 if seed is None else seed
    b, nb, nc = batch or 1048576, n_batch or 256, n_cubic or 4096
    d = inputs.uniform_aligned_chains(s, nb, b, 256, 32768, chain0=1)
    m = inputs.bernoulli_masks(s, nb, b, chain0=1)
    return name, d, m, inputs.uniform_aligned_chains(s, nc, 1, 256, 32768)


class Workload:
    """One configuration resident in HBM, with the step that runs its calls."""

    def __init__(self, torch, B, cfg, seed, args=None):
        dev = torch.device("cuda:0")
        self.torch, self.B, self.cfg = torch, B, cfg
        a = args
        self.name, self.d_np, self.m_np, self.d1_np = make_config(
            cfg, seed, a.batch if a else None, a.n_batch if a else None, a.n_cubic if a else None)
        self.d = torch.from_numpy(self.d_np).to(dev)
        self.m = torch.from_numpy(self.m_np).to(dev)
        self.d1 = self.d if self.d1_np is self.d_np else torch.from_numpy(self.d1_np).to(dev)
        self.batch, self.n = self.d.shape[1], self.d.shape[0] - 1
        self.cbatch, self.nc = self.d1.shape[1], self.d1.shape[0] - 1
        self.ws_lin = torch.empty(B.workspace_bytes(B.CALL_SOLVE_LINEAR, B.layout_of(self.d)), dtype=torch.uint8,
                                  device=dev)
        self.ws_cub = torch.empty(B.workspace_bytes(B.CALL_SOLVE_CUBIC, B.layout_of(self.d1)), dtype=torch.uint8,
                                  device=dev)
        self.calls = [
            # the sets' peaks under both objectives, from one pass over the chains
            ("eval_both", lambda: B.ckpt_eval_peak(self.d, self.m, B.OBJ_BOTH, want_status=False)),
            ("solve_linear", lambda: B.ckpt_solve_linear(self.d, workspace=self.ws_lin, want_status=False)),
            ("solve_cubic", lambda: B.ckpt_solve_cubic(self.d1, workspace=self.ws_cub, want_status=False)),
        ]
        if cfg in (2, 4):   # the configurations that name no evaluation
            self.calls = self.calls[1:]
        self.linear_cells = self.batch * self.n
        self.cubic_cells = self.cbatch * B.cubic_cells(self.nc)
        self.chain_bytes = 9 * (self.n + 1) + 8  # sizes in, mask in or out, 8-byte peak

    def step(self, events=None):
        marks = []
        for _, fn in self.calls:
            if events is not None:
                e = self.torch.cuda.Event(enable_timing=True)
                e.record()
                marks.append(e)
            fn()
        if events is not None:
            e = self.torch.cuda.Event(enable_timing=True)
            e.record()
            marks.append(e)
            events.append(marks)

    def run(self, steps, warmup):
        """(ms per step by the wall clock, {call: median ms by HIP events on the launch stream})."""
        for _ in range(warmup):
            self.step()
        self.torch.cuda.synchronize()
        events = []
        t0 = time.perf_counter()
        for _ in range(steps):
            self.step(events)
        self.torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        per_call = {}
        for i, (name, _) in enumerate(self.calls):
            per_call[name] = float(np.median([marks[i].elapsed_time(marks[i + 1]) for marks in events]))
        return wall * 1e3 / steps, per_call

    def report(self, ms):
        """Per-call rates and roofline fractions from the per-call times."""
        out = {}
        for name, t in ms.items():
            sec = t * 1e-3
            r = {"ms": t, "launch_bound": bool(t < 0.05)}
            if name == "solve_cubic":
                r["instances_per_s"] = self.cbatch / sec
                r["cells_resolved_per_s"] = self.cubic_cells / sec
                r["cells_nominal_n3_per_s"] = self.cbatch * float(self.nc) ** 3 / sec
                r["algorithmic_TOPs"] = self.cubic_cells * CUBIC_OPS_PER_CELL / sec / 1e12
            else:
                per_chain = self.chain_bytes + (8 if name == "eval_both" else 0)  # a second peak out
                r["instances_per_s"] = self.batch / sec
                r["algorithmic_bytes"] = self.batch * per_chain
                r["hbm_GBs"] = self.batch * per_chain / sec / 1e9
                r["hbm_frac"] = r["hbm_GBs"] / HBM_PEAK_GBS
                if name == "solve_linear":
                    r["cells_per_s"] = self.linear_cells / sec
            out[name] = r
        return out


def cpu_baseline(W, threads):
    """The oracle, as it stands, on a bounded sample of the same workload: with all host threads
    (or --oracle-threads) and once with one thread."""
    import oracle
    from paper_2502_12499_amd import inputs
    out = {}
    default = oracle.max_threads()  # what the environment grants (OMP_NUM_THREADS or the processors)
    for label, t in (("all", threads or default), ("one", 1)):
        oracle.set_threads(t)
        used = oracle.max_threads()
        scale = used
        # linear: Algorithm 5 on the first chains of the batch
        sample_chains = min(W.batch, (65536 if W.n <= 256 else 64) * scale)
        dc = inputs.chain_major(W.d_np[:, :sample_chains])
        t0 = time.perf_counter()
        oracle.batch_solve_dynamic(dc, want_mask=True)
        t_lin = time.perf_counter() - t0
        lin_rate = sample_chains * W.n / t_lin
        # cubic: Algorithm 4's queue on slices of the budget list spread over all range lengths
        K = oracle.num_budgets(W.nc)
        slices, per = 16, 16384 * scale
        d1 = W.d1_np[:, 0]
        t0 = time.perf_counter()
        done = 0
        for i in range(slices):
            first = (K // slices) * i
            num = min(per, K - first)
            if num > 0:
                oracle.solve_static_range(d1, first, num)
                done += num
        t_cub = time.perf_counter() - t0
        cub_rate = done * W.nc / t_cub
        est_step_s = W.linear_cells / lin_rate + W.cubic_cells / cub_rate
        out[label] = {
            "value": (W.linear_cells + W.cubic_cells) / est_step_s, "cores": used,
            "sample": (f"Algorithm 5 on {sample_chains} chains of the batch ({t_lin:.2f} s, {lin_rate:.3e} cells/s); "
                       f"Algorithm 4 on {done} of {K} budgets of the n={W.nc} chain in {slices} slices "
                       f"({t_cub:.2f} s, {cub_rate:.3e} cells/s); value = step cells / (cells/rate summed)"),
            "linear_cells_per_s": lin_rate, "cubic_cells_per_s": cub_rate}
    oracle.set_threads(default)
    base = dict(out["all"])
    base.update({"unit": "recurrence cells resolved/s", "kind": "oracle",
                 "single_thread": {k: out["one"][k] for k in ("value", "linear_cells_per_s", "cubic_cells_per_s")}})
    return base


def time_extras(torch, B, inputs, W, reps=3):
    """The calls that are not part of the timed step, each timed on its own: the per-phase memory
    timeline and the sqrt(n) sets on the same batch, the cubic solver without the budgets that
    cannot be optimal on the step's long chain, the quadratic-time solver."""
    out = {}
    Bn, n = W.batch, W.n
    tl_bytes = Bn * 25 * (n + 1)  # 9(n+1) in, 8(2n+2) out per chain
    for name, obj in (("eval_peak_static", B.OBJ_STATIC), ("eval_peak_dynamic", B.OBJ_DYNAMIC)):
        t, _ = timed_ms(torch, lambda: B.ckpt_eval_peak(W.d, W.m, obj, want_status=False), reps)
        by = Bn * (9 * (n + 1) + 8)
        out[name] = {"ms": t, "instances_per_s": Bn / (t * 1e-3), "hbm_GBs": by / (t * 1e-3) / 1e9,
                     "hbm_frac": by / (t * 1e-3) / 1e9 / HBM_PEAK_GBS}
    for name, obj in (("eval_timeline_static", B.OBJ_STATIC), ("eval_timeline_dynamic", B.OBJ_DYNAMIC)):
        t, _ = timed_ms(torch, lambda: B.ckpt_eval_timeline(W.d, W.m, obj, want_status=False), reps)
        out[name] = {"ms": t, "instances_per_s": Bn / (t * 1e-3), "hbm_GBs": tl_bytes / (t * 1e-3) / 1e9,
                     "hbm_frac": tl_bytes / (t * 1e-3) / 1e9 / HBM_PEAK_GBS}
    t, _ = timed_ms(torch, lambda: B.ckpt_select_baseline(W.d, B.SELECT_SQRT), reps)
    out["select_baseline_sqrt"] = {"ms": t, "instances_per_s": Bn / (t * 1e-3),
                                   "hbm_GBs": Bn * (n + 1) / (t * 1e-3) / 1e9,
                                   "hbm_frac": Bn * (n + 1) / (t * 1e-3) / 1e9 / HBM_PEAK_GBS}
    n1 = W.nc
    t, _ = timed_ms(torch, lambda: B.ckpt_solve_cubic_pruned(W.d1, workspace=W.ws_cub, want_status=False), reps)
    run = int(B.ckpt_solve_cubic_pruned(W.d1, workspace=W.ws_cub, want_status=False)[3][0])
    out[f"solve_cubic_pruned_n{n1}"] = {"ms": t, "instances_per_s": 1.0 / (t * 1e-3), "budgets_run": run,
                                        "budgets": n1 * (n1 - 1) // 2 + 1,
                                        "cells_evaluated_per_s": run * n1 / (t * 1e-3)}
    # the longest chain the cubic solver takes, sizes as the step's chain
    d8 = torch.from_numpy(inputs.config5_single(8191)).to(W.d.device)
    ws8 = torch.empty(B.workspace_bytes(B.CALL_SOLVE_CUBIC, B.layout_of(d8)), dtype=torch.uint8, device=W.d.device)
    t, _ = timed_ms(torch, lambda: B.ckpt_solve_cubic(d8, workspace=ws8, want_status=False), reps)
    out["solve_cubic_n8191"] = {"ms": t, "instances_per_s": 1.0 / (t * 1e-3),
                                "cells_resolved_per_s": B.cubic_cells(8191) / (t * 1e-3)}
    del d8, ws8
    d4 = torch.from_numpy(inputs.config4()).to(W.d.device)
    n4 = d4.shape[0] - 1
    t, _ = timed_ms(torch, lambda: B.ckpt_solve_quadratic(d4, want_values=False, want_status=False), reps)
    out["solve_quadratic_n1001"] = {"ms": t, "instances_per_s": 1.0 / (t * 1e-3),
                                    "candidates_per_s": n4 * (n4 + 1) / 2 / (t * 1e-3)}
    # ragged: the depths of the paper's networks mixed in one call; a small batch (a call is then
    # bound by its launches and by the latency of its small groups) and a large one
    for tag, copies, long_every in (("ragged", 16384, 4096), ("ragged_large", 131072, 0)):
        lengths = np.tile(np.array([15, 24, 152, 257], dtype=np.int64), copies)
        if long_every:
            lengths[::long_every] = 1001
        rd, rm, off = inputs.ragged_batch(3, lengths)
        rdd, rmd = torch.from_numpy(rd).to(W.d.device), torch.from_numpy(rm).to(W.d.device)
        offd = torch.from_numpy(off).to(W.d.device)  # the caller keeps the offsets on the device as well
        rbytes = 9 * len(rd) + 8 * len(lengths)
        for name, which, fn in (
                (tag + "_solve_linear", B.CALL_SOLVE_LINEAR,
                 lambda ws: B.ckpt_ragged_solve_linear(rdd, off, workspace=ws, offsets_dev=offd)),
                (tag + "_eval_peak_dynamic", B.CALL_EVAL_PEAK,
                 lambda ws: B.ckpt_ragged_eval_peak(rdd, rmd, off, B.OBJ_DYNAMIC, workspace=ws, offsets_dev=offd))):
            ws = torch.empty(B.load().ckpt_ragged_workspace_bytes(which, off.ctypes.data, len(lengths)),
                             dtype=torch.uint8, device=W.d.device)
            t, _ = timed_ms(torch, lambda: fn(ws), reps)
            out[name] = {"ms": t, "chains": len(lengths),
                         "lengths": "15, 24, 152, 257 in turn" + (", sixteen of 1001" if long_every else ""),
                         "instances_per_s": len(lengths) / (t * 1e-3), "hbm_GBs": rbytes / (t * 1e-3) / 1e9,
                         "hbm_frac": rbytes / (t * 1e-3) / 1e9 / HBM_PEAK_GBS,
                         "note": "offsets on the device: the lengths are counted there; includes the call's one "
                                 "wait on the stream (for the totals that size its launches)"}
            del ws
        del rdd, rmd
    small = min(Bn, 4096)
    ds = W.d[:, :small].contiguous()
    t, _ = timed_ms(torch, lambda: B.ckpt_solve_quadratic(ds, want_values=False, want_status=False), reps)
    out[f"solve_quadratic_{small}x{n}"] = {"ms": t, "instances_per_s": small / (t * 1e-3),
                                           "candidates_per_s": small * n * (n + 1) / 2 / (t * 1e-3)}
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=5, choices=(1, 2, 3, 4, 5),
                    help="the configuration the timed step runs (default 5, the stress configuration)")
    ap.add_argument("--seed", type=int, default=None, help="seed of the random configurations (default: theirs)")
    ap.add_argument("--oracle-threads", type=int, default=0, help="threads of the CPU baseline (0: all)")
    ap.add_argument("--batch", type=int, default=None, help="chains in the batched part (configs 3 and 5)")
    ap.add_argument("--n-batch", type=int, default=None)
    ap.add_argument("--n-cubic", type=int, default=None)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip what lies outside the timed step: the other configurations, the calls beside the "
                         "path, the transfer rates")
    ap.add_argument("--counter-probes", action="store_true")
    ap.add_argument("--peaks", action="store_true")
    ap.add_argument("--summarize", nargs="+", metavar="DIR")
    args = ap.parse_args()
    if args.summarize:
        wl = config_name(args.config, args.seed, args.batch, args.n_batch, args.n_cubic)
        rec = summarize(args.summarize, wl, args.steps + args.warmup)
        rec["copy_probe_bytes"] = COPY_PROBE_BYTES
        json.dump(rec, open(COUNTERS_JSON, "w"), indent=1, sort_keys=True)
        print(f"wrote {COUNTERS_JSON}: {len(rec['kernels'])} kernels, sources {rec['source_hash'][:12]}")
        return
    if args.peaks:
        print(json.dumps({"peaks": measure_peaks()}), flush=True)
        return
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this path runs on one GPU only (independent chains and budgets would be split "
              "across GPUs without communication; no multi-GPU figure is produced). Use --gpus 1.",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2502_12499_amd import binding as B
    from paper_2502_12499_amd import inputs

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    B.load()
    t0 = time.perf_counter()
    W = Workload(torch, B, args.config, args.seed, args)
    log(f"inputs generated and resident in {time.perf_counter() - t0:.1f} s: {W.name}")
    ms_step, ms = W.run(args.steps, args.warmup)
    kernels = W.report(ms)
    names = [k for k, _ in W.calls]

    # ---- rooflines ----
    default_workload = args.config == 5 and (W.batch, W.n, W.nc) == (1048576, 256, 4096) and args.seed is None
    rec_counters = load_counters(W.name) if default_workload else None
    peaks = measured_peaks()
    dominant = max(names, key=lambda k: ms[k])
    if "solve_cubic" in kernels:
        c = kernels["solve_cubic"]
        c["algorithmic_frac_of_int32_peak"] = c["algorithmic_TOPs"] / INT32_PEAK_TOPS
        ops = call_lane_ops(rec_counters, "cubic_")
        c["executed_lane_ops"] = ops
        c["executed_TOPs"] = ops / (ms["solve_cubic"] * 1e-3) / 1e12 if ops else None
        c["work_avoided_x"] = W.cubic_cells * CUBIC_OPS_PER_CELL / ops if ops else None
        c["traffic"] = traffic_bytes(rec_counters, "cubic_")
    for k, prefix in (("eval_both", "eval_peak_kernel<2>"),):
        if k in kernels:
            kernels[k]["traffic"] = traffic_bytes(rec_counters, prefix)
    if "solve_linear" in kernels:
        kernels["solve_linear"]["traffic"] = traffic_bytes(rec_counters, "linear_")
        ops = call_lane_ops(rec_counters, "linear_")
        kernels["solve_linear"]["executed_TOPs"] = ops / (ms["solve_linear"] * 1e-3) / 1e12 if ops else None
    if peaks:
        for k in ("eval_both", "solve_linear"):
            if k in kernels:
                kernels[k]["frac_of_measured_read_rate"] = kernels[k]["hbm_GBs"] / peaks["hbm_read_GBs"]

    if dominant == "solve_cubic":
        c = kernels["solve_cubic"]
        shared = [k for k in (kernels_of(rec_counters, "cubic_shared_kernel") if rec_counters else [])]
        main_k = max(shared, key=lambda k: k.get("avg_us", 0.0)) if shared else None
        main_ops = kernel_lane_ops(main_k, rec_counters["kernels"].get("probe_valu_kernel<2>")) if main_k else None
        roofline = {
            "kernel": "ckpt_solve_cubic (all its kernels; cubic_shared_kernel takes most of the time)",
            "bound": "alu", "unit": "TOP/s", "peak": INT32_PEAK_TOPS,
            "achieved": c["executed_TOPs"],
            "frac": c["executed_TOPs"] / INT32_PEAK_TOPS if c["executed_TOPs"] else None,
            "traffic": c["traffic"],
            "how": "executed 32-bit lane-operations of the call's kernels (rocprofv3 SQ_INSTS_VALU x 64 x mean active "
                   "lane fraction, profiles/counters.json) / the call's time by HIP events in this run / peak; null "
                   "when the counters were taken on other kernel sources or another workload",
            "main_kernel_frac_by_profile": (main_ops / (main_k["avg_us"] * 1e-6) / 1e12 / INT32_PEAK_TOPS
                                            if main_ops and main_k.get("avg_us") else None),
            "algorithmic_TOPs": c["algorithmic_TOPs"],
            "work_avoided_x": c["work_avoided_x"],
        }
        if c["executed_TOPs"]:
            roofline["frac_of_select_class_rate"] = c["executed_TOPs"] / INT32_SELECT_CLASS_TOPS
            if peaks:
                roofline["frac_of_measured_v_max_u32_rate"] = c["executed_TOPs"] / peaks["v_max_u32_TOPs"]
                roofline["frac_of_measured_v_add_u32_rate"] = c["executed_TOPs"] / peaks["v_add_u32_TOPs"]
    else:
        k = kernels[dominant]
        roofline = {"kernel": "ckpt_" + dominant if not dominant.startswith("eval") else "ckpt_eval_peak",
                    "bound": "hbm", "achieved": k["hbm_GBs"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": k["hbm_frac"], "traffic": k.get("traffic")}
    rec = {
        "metric": "DP cells/sec over one pass of the checkpoint-selection path (cubic + linear recurrence cells "
                  "resolved, whether visited one by one or passed over)",
        "value": (W.linear_cells + W.cubic_cells) / (ms_step * 1e-3),
        "unit": "recurrence cells resolved/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int64 in/out, int32 arithmetic after dividing by the common power of two",
        "data": "synthetic",
        "config": {"workload": W.name, "layout": "position-major int64", "timing": "median of the steps per call"},
        "instances_per_sec": {k: kernels[k]["instances_per_s"] for k in names},
        "kernels": kernels,
        "roofline": roofline,
        "paper_context": PAPER_CONTEXT,
    }
    if "solve_linear" in kernels:
        L = kernels["solve_linear"]
        rec["roofline_linear"] = {"kernel": "ckpt_solve_linear", "bound": "hbm", "achieved": L["hbm_GBs"],
                                  "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": L["hbm_frac"],
                                  "traffic": L.get("traffic"),
                                  "frac_of_measured_read_rate": L.get("frac_of_measured_read_rate")}
    if peaks:
        rec["measured_peaks"] = {k: peaks[k] for k in ("hbm_read_GBs", "hbm_copy_GBs_moved", "v_add_u32_TOPs",
                                                       "v_max_u32_TOPs") if k in peaks}

    if args.counter_probes:
        sink = torch.zeros(8, dtype=torch.int64, device=W.d.device)
        src = torch.empty(COPY_PROBE_BYTES // 8, dtype=torch.int64, device=W.d.device).random_()
        dst = torch.empty_like(src)
        B.ckpt_probe_hbm_copy(src, dst)
        lane_ops = B.ckpt_probe_valu(B.PROBE_VALU["v_max_u32"], VALU_PROBE_WAVES, VALU_PROBE_ITERS, sink)
        torch.cuda.synchronize()
        log(f"counter probes: copy of {COPY_PROBE_BYTES} bytes; v_max_u32 probe of {lane_ops} lane-operations")
        del src, dst

    if not args.no_extras:
        others = {}
        for cfg in (1, 2, 3, 4, 5):
            if cfg == args.config:
                continue
            Wc = Workload(torch, B, cfg, None)
            step_ms, ms_c = Wc.run(5, 2)
            others[str(cfg)] = {"workload": Wc.name, "ms_per_step": step_ms, "calls": Wc.report(ms_c)}
            del Wc
        rec["configs"] = others
        rec["other_calls"] = time_extras(torch, B, inputs, W)
        tr = transfer_rates(torch)
        in_bytes = W.d.numel() * 8 + W.m.numel()
        out_bytes = W.batch * (W.n + 1 + 8)
        tr["note"] = ("pinned host memory; the step's inputs are %d bytes and its batched outputs %d bytes: "
                      "%.1f ms in and %.1f ms out at these rates, against %.2f ms for the step itself"
                      % (in_bytes, out_bytes, in_bytes / tr["h2d_GBs"] / 1e6, out_bytes / tr["d2h_GBs"] / 1e6, ms_step))
        rec["transfer"] = tr
    if not args.no_cpu_baseline:
        rec["cpu_baseline"] = cpu_baseline(W, args.oracle_threads)
    print(json.dumps(rec), flush=True)


if __name__ == "__main__":
    main()
