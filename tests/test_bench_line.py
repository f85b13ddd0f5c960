"""The benchmark's last stdout line must stay a short, self-contained JSON object: a harness that keeps only the
tail of the log has to find `value`, `roofline` and `cpu_baseline` in it.  (CPU only: canned numbers, no launch.)"""
import json

import pytest

import bench


def canned(n_ops=34, n_extra=93):
    row = {"op": "scatter_reduce_amax_f32_elem_index[131072,256]", "row": "f3", "path": "scatter-reduce-sort",
           "kernel": "seg_reduce_kernel", "us": 1463.73, "GB/s": 458.5, "frac_of_peak": 0.0573, "Gelem/s": 22.92,
           "bytes": 671088640}
    return {
        "metric": "achieved HBM GB/s (algorithmic bytes / time) over one pass of all operator classes on one GPU",
        "value": 5751.3, "unit": "GB/s", "n_gpus": 1, "steps": 20, "warmup": 5, "ms_per_step": 7.512,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "all five workloads at full size: add [4096,1]+[1,4096]; elementwise [8192,8192]; "
                               "reductions [64,4096,1024]; softmax [32768,4096]; cumsum [4096,65536]; "
                               "indexing on src[1048576,256]", "ops_per_step": n_ops},
        "frac_of_peak": 0.7189, "elements_per_s": 1.234567890123e12,
        "roofline": {"bound": "hbm", "kernel": "index_select_rows_kernel", "op": "index_select_f32", "achieved": 6383.9,
                     "peak": 8000.0, "unit": "GB/s", "frac": 0.798, "traffic": 8642587648,
                     "algorithmic_bytes": 8623489024, "avg_us": 1350.79},
        "side_file": "gpurun_out/bench_per_op.json",
        "per_op": [dict(row) for _ in range(n_ops)],
        "per_op_outside_step": [dict(row) for _ in range(n_extra)],
        "measurement_detail": {"x": "y" * 4000},
        "cpu_baseline": {"value": 5.992, "unit": "GB/s", "cores": 16, "kind": "oracle", "value_1_thread": 0.612,
                         "seconds": 21.3, "nproc": 224, "cpu": "AMD EPYC 9575F 64-Core Processor (a long model string)",
                         "sample": "oracle over 1/8-1/16 slices of workloads 2-5 and all of workload 1, about 2 s each at "
                                   "16 threads and at 1 thread; per-workload table in the side file"},
        "cpu_baseline_per_workload": [{"workload": "1", "sample": "s" * 100}] * 5,
    }


def test_headline_is_short_parseable_and_complete():
    line = bench.headline(canned())
    assert "\n" not in line and len(line) <= 1500
    # what a log that keeps the last 2000 characters still holds, with noise after the line
    log = "x" * 5000 + "\n" + line + "\n"
    tail = log[-2000:]
    obj = json.loads(tail[tail.index("\n") + 1:].strip())
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in obj, key
    assert obj["config"]["workload"] and "model" not in obj["config"]
    for key in ("bound", "achieved", "peak", "unit", "frac", "traffic"):
        assert key in obj["roofline"], key
    for key in ("value", "unit", "cores", "kind", "sample"):
        assert key in obj["cpu_baseline"], key
    assert "per_op" not in obj and "per_op_outside_step" not in obj      # the tables live in the side file


def test_headline_refuses_to_grow():
    r = canned()
    r["config"]["workload"] = "w" * 2000
    with pytest.raises(ValueError):
        bench.headline(r)


def test_more_than_one_gpu_is_refused():
    import subprocess
    import sys
    p = subprocess.run([sys.executable, bench.__file__, "--gpus", "2"], capture_output=True, text=True)
    assert p.returncode != 0 and "one" in p.stderr and p.stdout.strip() == ""
