#!/usr/bin/env python3
"""Benchmark of the checkpoint-selection hot path on one MI355X.

One step = one pass of the whole path over the stress workload:
  ckpt_eval_peak (static, then dynamic objective) and ckpt_solve_linear on a
  batch of 1,048,576 chains of n = 256 layers, and ckpt_solve_cubic on one chain
  of n = 4096 layers; sizes are 4 KiB multiples in [1 MiB, 128 MiB], seed 2.
Inputs are generated on the host once, copied to HBM, and stay there; the timed
region contains only library calls.  Prints one JSON line.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
# 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz: one 32-bit integer lane-op per lane per clock
INT32_PEAK_TOPS = 256 * 64 * 2.4e9 / 1e12
CUBIC_VALU_INSTS = 5.05e8  # per launch at n = 4096
CUBIC_OPS_PER_CELL = 3  # one add and two compare-selects (queue push / pop) per recurrence cell


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def cpu_baseline(d_batch_np, d_single_np, n_cubic, linear_cells, cubic_cells):
    """The oracle, as it stands, on a bounded sample of the same workload."""
    import oracle
    from paper_2502_12499_amd import inputs
    threads = oracle.max_threads()
    # linear: Algorithm 5 on the first chains of the batch
    sample_chains = min(d_batch_np.shape[1], 65536 * max(1, threads // 4))
    dc = inputs.chain_major(d_batch_np[:, :sample_chains])
    t0 = time.perf_counter()
    oracle.batch_solve_dynamic(dc, want_mask=True)
    t_lin = time.perf_counter() - t0
    lin_rate = sample_chains * (dc.shape[1] - 1) / t_lin
    # cubic: Algorithm 4's queue on slices of the budget list spread over all range lengths
    K = oracle.num_budgets(n_cubic)
    slices, per = 16, 16384 * max(1, threads // 4)
    d1 = d_single_np[:, 0]
    t0 = time.perf_counter()
    done = 0
    for i in range(slices):
        first = (K // slices) * i
        num = min(per, K - first)
        oracle.solve_static_range(d1, first, num)
        done += num
    t_cub = time.perf_counter() - t0
    cub_rate = done * n_cubic / t_cub
    est_step_s = linear_cells / lin_rate + cubic_cells / cub_rate
    return {
        "value": (linear_cells + cubic_cells) / est_step_s,
        "unit": "cells/s",
        "cores": threads,
        "kind": "oracle",
        "sample": (f"Algorithm 5 on {sample_chains} chains of the batch ({t_lin:.2f} s, {lin_rate:.3e} cells/s); "
                   f"Algorithm 4 on {done} of {K} budgets of the n={n_cubic} chain in {slices} slices "
                   f"({t_cub:.2f} s, {cub_rate:.3e} cells/s); value = step cells / (cells/rate summed)"),
        "linear_cells_per_s": lin_rate,
        "cubic_cells_per_s": cub_rate,
    }


def time_extras(torch, B, inputs, d, m, d1, ws_cub, Bn, n, reps=3):
    """The calls that are not part of the timed step, each timed on its own with HIP events on
    the stream it runs on: the per-phase memory timeline and the sqrt(n) sets on the same batch,
    the cubic solver without the budgets that cannot be optimal on the step's long chain, the
    quadratic-time solver on the ResNet-1001-shaped chain and on the first 4096 chains."""
    def timed(fn):
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
        return float(np.mean(ts))

    out = {}
    tl_bytes = Bn * 25 * (n + 1)  # 9(n+1) in, 8(2n+2) out per chain
    for name, obj in (("eval_timeline_static", B.OBJ_STATIC), ("eval_timeline_dynamic", B.OBJ_DYNAMIC)):
        t = timed(lambda: B.ckpt_eval_timeline(d, m, obj, want_status=False))
        out[name] = {"ms": t, "instances_per_s": Bn / (t * 1e-3), "hbm_GBs": tl_bytes / (t * 1e-3) / 1e9,
                     "hbm_frac": tl_bytes / (t * 1e-3) / 1e9 / HBM_PEAK_GBS}
    t = timed(lambda: B.ckpt_select_baseline(d, B.SELECT_SQRT))
    out["select_baseline_sqrt"] = {"ms": t, "instances_per_s": Bn / (t * 1e-3),
                                   "hbm_GBs": Bn * (n + 1) / (t * 1e-3) / 1e9,
                                   "hbm_frac": Bn * (n + 1) / (t * 1e-3) / 1e9 / HBM_PEAK_GBS}
    n1 = d1.shape[0] - 1
    t = timed(lambda: B.ckpt_solve_cubic_pruned(d1, workspace=ws_cub, want_status=False))
    run = int(B.ckpt_solve_cubic_pruned(d1, workspace=ws_cub, want_status=False)[3][0])
    out[f"solve_cubic_pruned_n{n1}"] = {"ms": t, "instances_per_s": 1.0 / (t * 1e-3), "budgets_run": run,
                                        "budgets": n1 * (n1 - 1) // 2 + 1,
                                        "cells_evaluated_per_s": run * n1 / (t * 1e-3)}
    d4 = torch.from_numpy(inputs.config4()).to(d.device)
    n4 = d4.shape[0] - 1
    t = timed(lambda: B.ckpt_solve_quadratic(d4, want_values=False, want_status=False))
    out["solve_quadratic_n1001"] = {"ms": t, "instances_per_s": 1.0 / (t * 1e-3),
                                    "candidates_per_s": n4 * (n4 + 1) / 2 / (t * 1e-3)}
    small = min(Bn, 4096)
    ds = d[:, :small].contiguous()
    t = timed(lambda: B.ckpt_solve_quadratic(ds, want_values=False, want_status=False))
    out[f"solve_quadratic_{small}x{n}"] = {"ms": t, "instances_per_s": small / (t * 1e-3),
                                           "candidates_per_s": small * n * (n + 1) / 2 / (t * 1e-3)}
    return out


def measure_peaks(reps=5):
    """What the part delivers on kernels of known work (include/ckpt_probe.h): HBM read and copy
    rates on the stress batch's 2.16 GB, the issue rate of 32-bit integer vector instructions and
    the LDS instruction rate.  Median of `reps` launches each, HIP events on the launch stream."""
    import torch
    from paper_2502_12499_amd import binding as B
    dev = torch.device("cuda:0")
    sink = torch.zeros(8, dtype=torch.int64, device=dev)

    def timed(fn):
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
        return float(np.median(ts)) * 1e-3

    out = {}
    nbytes = 1048576 * 257 * 8
    src = torch.empty(nbytes // 8, dtype=torch.int64, device=dev).random_()
    dst = torch.empty_like(src)
    t = timed(lambda: B.ckpt_probe_hbm_read(src, sink))
    out["hbm_read_GBs"] = nbytes / t / 1e9
    t = timed(lambda: B.ckpt_probe_hbm_copy(src, dst))
    out["hbm_copy_GBs_moved"] = 2 * nbytes / t / 1e9
    del src, dst
    waves = 256 * 4 * 8  # eight waves per SIMD
    for name, which in B.PROBE_VALU.items():
        ops = [0]

        def fn():
            ops[0] = B.ckpt_probe_valu(which, waves, 256, sink)
        t = timed(fn)
        out[name + "_TOPs"] = ops[0] / t / 1e12
    for name, which in B.PROBE_LDS.items():
        acc = [0]

        def fn():
            acc[0] = B.ckpt_probe_lds(which, 256 * 16, 2048, sink)
        t = timed(fn)
        out[name + "_T_lane_accesses_per_s"] = acc[0] / t / 1e12
        out[name + "_bytes_per_clk_per_cu"] = acc[0] * 4 / t / 256 / 2.4e9
    out["nominal"] = {"hbm_GBs": HBM_PEAK_GBS, "int32_TOPs": INT32_PEAK_TOPS}
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--batch", type=int, default=1048576, help="chains in the batched part")
    ap.add_argument("--n-batch", type=int, default=256)
    ap.add_argument("--n-cubic", type=int, default=4096)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the calls outside the timed step (timeline, baseline sets, quadratic solver)")
    ap.add_argument("--copy-probe", action="store_true",
                    help="after the timed steps, copy the batch of sizes once (a plain copy kernel of known size, "
                         "to scale the profiler's memory counters)")
    ap.add_argument("--peaks", action="store_true",
                    help="run only the measurement probes (HBM read/copy, integer vector issue rate, LDS rate) "
                         "and print their JSON line")
    args = ap.parse_args()
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
    dev = torch.device("cuda:0")
    B.load()

    t0 = time.perf_counter()
    d_np, m_np = inputs.config5_batch(batch=args.batch, n_layers=args.n_batch)
    d1_np = inputs.config5_single(args.n_cubic)
    log(f"inputs generated in {time.perf_counter() - t0:.1f} s")
    d = torch.from_numpy(d_np).to(dev)
    m = torch.from_numpy(m_np).to(dev)
    d1 = torch.from_numpy(d1_np).to(dev)

    L = B.layout_of(d)
    L1 = B.layout_of(d1)
    ws_lin = torch.empty(B.workspace_bytes(B.CALL_SOLVE_LINEAR, L), dtype=torch.uint8, device=dev)
    ws_cub = torch.empty(B.workspace_bytes(B.CALL_SOLVE_CUBIC, L1), dtype=torch.uint8, device=dev)

    names = ["eval_static", "eval_dynamic", "solve_linear", "solve_cubic"]

    def step(events=None):
        marks = []

        def mark():
            if events is not None:
                e = torch.cuda.Event(enable_timing=True)
                e.record()
                marks.append(e)
        mark()
        r0 = B.ckpt_eval_peak(d, m, B.OBJ_STATIC, want_status=False)
        mark()
        r1 = B.ckpt_eval_peak(d, m, B.OBJ_DYNAMIC, want_status=False)
        mark()
        r2 = B.ckpt_solve_linear(d, workspace=ws_lin, want_status=False)
        mark()
        r3 = B.ckpt_solve_cubic(d1, workspace=ws_cub, want_status=False)
        mark()
        if events is not None:
            events.append(marks)
        return r0, r1, r2, r3

    for _ in range(args.warmup):
        out = step()
    torch.cuda.synchronize()
    events = []
    t0 = time.perf_counter()
    for _ in range(args.steps):
        out = step(events)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    extras = None if args.no_extras else time_extras(torch, B, inputs, d, m, d1, ws_cub, args.batch, args.n_batch)
    if args.copy_probe:
        probe = torch.empty_like(d)
        probe.copy_(d)
        torch.cuda.synchronize()
        print(f"copy probe: {d.numel() * 8} bytes read, as many written", file=sys.stderr, flush=True)

    per_call = {k: [] for k in names}
    for marks in events:
        for i, k in enumerate(names):
            per_call[k].append(marks[i].elapsed_time(marks[i + 1]))
    ms = {k: float(np.mean(v)) for k, v in per_call.items()}
    ms_step = wall * 1e3 / args.steps

    n, Bn, nc = args.n_batch, args.batch, args.n_cubic
    linear_cells = Bn * n
    cubic_cells = B.cubic_cells(nc)
    chain_bytes = 9 * (n + 1) + 8  # sizes in (or out: the mask) + 8-byte peak
    kernels = {
        "eval_static": {"ms": ms["eval_static"], "instances_per_s": Bn / (ms["eval_static"] * 1e-3),
                        "hbm_GBs": Bn * chain_bytes / (ms["eval_static"] * 1e-3) / 1e9},
        "eval_dynamic": {"ms": ms["eval_dynamic"], "instances_per_s": Bn / (ms["eval_dynamic"] * 1e-3),
                         "hbm_GBs": Bn * chain_bytes / (ms["eval_dynamic"] * 1e-3) / 1e9},
        "solve_linear": {"ms": ms["solve_linear"], "instances_per_s": Bn / (ms["solve_linear"] * 1e-3),
                         "cells_per_s": linear_cells / (ms["solve_linear"] * 1e-3),
                         "hbm_GBs": Bn * chain_bytes / (ms["solve_linear"] * 1e-3) / 1e9},
        "solve_cubic": {"ms": ms["solve_cubic"], "instances_per_s": 1.0 / (ms["solve_cubic"] * 1e-3),
                        "cells_per_s": cubic_cells / (ms["solve_cubic"] * 1e-3),
                        "cells_nominal_n3_per_s": float(nc) ** 3 / (ms["solve_cubic"] * 1e-3),
                        "int32_TOPs": cubic_cells * CUBIC_OPS_PER_CELL / (ms["solve_cubic"] * 1e-3) / 1e12},
    }
    for k in ("eval_static", "eval_dynamic", "solve_linear"):
        kernels[k]["hbm_frac"] = kernels[k]["hbm_GBs"] / HBM_PEAK_GBS
        kernels[k]["algorithmic_bytes"] = Bn * chain_bytes
    kernels["solve_cubic"]["int32_frac"] = kernels["solve_cubic"]["int32_TOPs"] / INT32_PEAK_TOPS

    # HBM bytes per launch of the kernels the rooflines are about, from the rocprofv3 FETCH_SIZE /
    # WRITE_SIZE runs summarised in profiles/bench_stress_hbm_counters.md (valid for the default
    # workload only; to be set to None when those kernels change)
    default_workload = (Bn, n, nc) == (1048576, 256, 4096)
    traffic_cubic = 40.0e6 + 8.4e6 if default_workload else None
    traffic_linear = 2.487e9 + 0.584e9 if default_workload else None
    traffic_eval = 2.54e9 + 8.4e6 if default_workload else None
    kernels["eval_static"]["traffic"] = kernels["eval_dynamic"]["traffic"] = traffic_eval
    kernels["solve_linear"]["traffic"] = traffic_linear
    kernels["solve_cubic"]["traffic"] = traffic_cubic
    dominant = max(names, key=lambda k: ms[k])
    # Vector instructions that one launch of cubic_shared_kernel executes (rocprofv3 SQ_INSTS_VALU,
    # profiles/bench_stress_kernel_stats.md; default workload only, None when the kernel changes): with 64
    # lanes each they give the rate the hardware ran at, beside the algorithmic one.
    valu_insts_cubic = CUBIC_VALU_INSTS if default_workload else None
    kernels["solve_cubic"]["executed_TOPs"] = (valu_insts_cubic * 64 / (ms["solve_cubic"] * 1e-3) / 1e12
                                               if valu_insts_cubic else None)
    if dominant == "solve_cubic":
        roofline = {"kernel": "cubic_shared_kernel (timed as the whole ckpt_solve_cubic call)", "bound": "alu",
                    "achieved": kernels["solve_cubic"]["int32_TOPs"], "peak": INT32_PEAK_TOPS, "unit": "TOP/s",
                    "frac": kernels["solve_cubic"]["int32_frac"], "traffic": traffic_cubic,
                    "executed_frac": (kernels["solve_cubic"]["executed_TOPs"] / INT32_PEAK_TOPS
                                      if valu_insts_cubic else None),
                    "note": "achieved/frac count 3 operations for every cell of the recurrence (the algorithmic "
                            "rate); the kernel passes over groups of eight cells in which nothing can happen, so "
                            "it executes fewer and frac can exceed 1; executed_frac = vector instructions "
                            "executed x 64 lanes / time / peak"}
    else:
        roofline = {"kernel": dominant, "bound": "hbm", "achieved": kernels[dominant]["hbm_GBs"],
                    "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": kernels[dominant]["hbm_frac"], "traffic": None}
    roofline_linear = {"kernel": "ckpt_solve_linear", "bound": "hbm", "achieved": kernels["solve_linear"]["hbm_GBs"],
                       "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": kernels["solve_linear"]["hbm_frac"],
                       "traffic": traffic_linear}

    rec = {
        "metric": "DP cells/sec over one pass of the checkpoint-selection path (cubic + linear recurrence cells)",
        "value": (linear_cells + cubic_cells) / (ms_step * 1e-3),
        "unit": "cells/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int64 in/out, int32 arithmetic after dividing by the common power of two",
        "data": "synthetic",
        "config": {"workload": f"stress: 1 chain n={nc} (cubic) + {Bn} chains n={n} (linear, eval_peak x2), "
                               "sizes 4 KiB x U{256..32768}, seed 2",
                   "layout": "position-major int64"},
        "instances_per_sec": {k: kernels[k]["instances_per_s"] for k in names},
        "kernels": kernels,
        "roofline": roofline,
        "roofline_linear": roofline_linear,
        "paper_context": "Python on a Xeon Gold 6226R, VGG-19 (n=24): Algorithm 4 20 ms, Algorithm 6 1.1 ms per chain",
    }
    if extras is not None:
        rec["other_calls"] = extras
    if not args.no_cpu_baseline:
        rec["cpu_baseline"] = cpu_baseline(d_np, d1_np, nc, linear_cells, cubic_cells)
    print(json.dumps(rec), flush=True)


if __name__ == "__main__":
    main()
