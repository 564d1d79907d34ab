"""Host-side pieces of bench.py: folding rocprofv3 CSV output into the counter record, the
source hash that guards it, the lane-operation arithmetic, and the refusal of more than one GPU."""
import json
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import bench  # noqa: E402


def test_kernel_names_are_cut_to_the_function_and_its_template_arguments():
    long = ('"void ckpt::(anonymous namespace)::cubic_shared_kernel<16, 64, false>(int, long, int, int, '
            'ckpt::(anonymous namespace)::CubicWs)"')
    assert bench.short_kernel_name(long) == "cubic_shared_kernel<16, 64, false>"
    assert bench.short_kernel_name("ckpt::(anonymous namespace)::linear_reset_kernel(ckpt::(anonymous namespace)::LinearWs)") \
        == "linear_reset_kernel"
    assert bench.short_kernel_name("void ckpt::(anonymous namespace)::eval_peak_kernel<1>(long const*, int)") \
        == "eval_peak_kernel<1>"


def write_csvs(d):
    os.makedirs(d)
    head = ('"Correlation_Id","Dispatch_Id","Agent_Id","Queue_Id","Process_Id","Thread_Id","Grid_Size","Kernel_Id",'
            '"Kernel_Name","Workgroup_Size","LDS_Block_Size","Scratch_Size","VGPR_Count","Accum_VGPR_Count","SGPR_Count",'
            '"Counter_Name","Counter_Value","Start_Timestamp","End_Timestamp"\n')
    rows = []
    def row(kernel, counter, value):
        rows.append(f'1,1,"Agent 1",1,1,1,64,1,"{kernel}",64,0,0,16,0,48,"{counter}",{value},1,2\n')
    k = "void ckpt::(anonymous namespace)::cubic_shared_kernel<16, 64, false>(int)"
    p = "void ckpt::(anonymous namespace)::probe_valu_kernel<2>(int, unsigned int*)"
    for v in (100.0, 300.0):                     # two dispatches: the mean is kept
        row(k, "SQ_INSTS_VALU", v)
    row(k, "SQ_ACTIVE_INST_VALU", 400.0)
    row(k, "SQ_THREAD_CYCLES_VALU", 400.0 * 64 * 0.5)   # half of the lanes active
    issued = bench.VALU_PROBE_WAVES * bench.VALU_PROBE_ITERS * 256
    row(p, "SQ_INSTS_VALU", issued * 2.0)        # a counter that reads double: everything is scaled by 1/2
    row(p, "SQ_ACTIVE_INST_VALU", 10.0)
    row(p, "SQ_THREAD_CYCLES_VALU", 640.0)
    open(os.path.join(d, "p_counter_collection.csv"), "w").write(head + "".join(rows))
    open(os.path.join(d, "p_kernel_stats.csv"), "w").write(
        '"Name","Calls","TotalDurationNs","AverageNs","Percentage","MinNs","MaxNs","StdDev"\n'
        f'"{k}",8,8000,1000.0,50.0,900,1100,1.0\n"{p}",1,500,500.0,50.0,500,500,0.0\n')


def test_summarize_and_the_lane_operation_arithmetic(tmp_path):
    d = str(tmp_path / "prof")
    write_csvs(d)
    rec = bench.summarize([d], "some workload", 8)
    ks = rec["kernels"]
    k = ks["cubic_shared_kernel<16, 64, false>"]
    assert k["SQ_INSTS_VALU"] == 200.0 and k["avg_us"] == 1.0 and k["per_step"] == 1.0
    assert ks["probe_valu_kernel<2>"]["per_step"] == 0.125
    assert rec["source_hash"] == bench.source_hash() and rec["workload"] == "some workload"
    # 200 instructions x 64 lanes x 0.5 active, halved by the probe's scale
    assert bench.kernel_lane_ops(k, ks["probe_valu_kernel<2>"]) == 200.0 * 64 * 0.5 * 0.5
    assert bench.kernel_lane_ops(k, None) == 200.0 * 64 * 0.5
    assert bench.kernel_lane_ops({"avg_us": 1.0}, None) is None
    assert bench.call_lane_ops(rec, "cubic_") == 200.0 * 64 * 0.5 * 0.5
    assert bench.call_lane_ops(rec, "linear_") is None and bench.traffic_bytes(rec, "cubic_") is None


def test_counters_of_other_sources_or_workloads_are_not_used(tmp_path, monkeypatch):
    path = str(tmp_path / "counters.json")
    monkeypatch.setattr(bench, "COUNTERS_JSON", path)
    assert bench.load_counters("w") is None                      # no file
    json.dump({"source_hash": bench.source_hash(), "workload": "w", "kernels": {}}, open(path, "w"))
    assert bench.load_counters("w") is not None
    assert bench.load_counters("another workload") is None
    json.dump({"source_hash": "0" * 64, "workload": "w", "kernels": {}}, open(path, "w"))
    assert bench.load_counters("w") is None                      # kernels have changed since


def test_the_committed_counters_belong_to_the_committed_sources():
    rec = json.load(open(bench.COUNTERS_JSON))
    assert rec["source_hash"] == bench.source_hash(), "profiles/counters.json is stale: profile again and --summarize"
    assert rec["workload"] == bench.config_name(5, None)


def test_more_than_one_gpu_is_refused():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], stdout=subprocess.PIPE,
                       stderr=subprocess.PIPE, text=True)
    assert p.returncode == 2 and "one GPU" in p.stderr and p.stdout == ""
