"""bench.py end to end on the smallest workload: one JSON line with the fields the driver reads,
the roofline and hybrid-stack records included (the attention time of a layer stack with some
layers dense, section 4.2)."""

import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.gpu
def test_bench_line_with_hybrid_stack():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--workload", "tiny", "--steps", "3",
                        "--warmup", "1", "--no-extra", "--no-ceilings", "--hybrid-stack", "6:1",
                        "--cpu-sample-tokens", "512"], capture_output=True, text=True, timeout=600, cwd=ROOT)
    assert r.returncode == 0, r.stderr[-2000:]
    out = json.loads(r.stdout.strip().splitlines()[-1])
    for k in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
              "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert k in out, k
    assert out["n_gpus"] == 1 and out["steps"] == 3 and out["config"]["workload"] == "tiny"
    assert out["roofline"]["bound"] == "mfma" and 0 < out["roofline"]["frac"] < 1
    assert out["cpu_baseline"]["kind"] == "oracle" and out["cpu_baseline"]["value"] > 0
    hs = out["hybrid_stack"]
    assert hs["layers"] == 6 and hs["dense_layers"] == [0] and hs["ms"] > 0 and hs["all_dense_ms"] > 0
    par = out["parity_on_cpu_sample"]
    assert par["o_max_excess_over_bound"] <= 0 and par["lse_max_abs"] <= 1e-3


@pytest.mark.gpu
def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True,
                       text=True, timeout=120, cwd=ROOT)
    assert r.returncode != 0 and "one GPU" in (r.stderr + r.stdout)


@pytest.mark.gpu
def test_bench_times_both_forms_of_the_backward():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--workload", "1p3b_8k", "--steps", "3",
                        "--warmup", "1", "--no-extra", "--no-ceilings", "--no-dense", "--no-cpu-baseline"],
                       capture_output=True, text=True, timeout=600, cwd=ROOT)
    assert r.returncode == 0, r.stderr[-2000:]
    d = json.loads(r.stdout.strip().splitlines()[-1])["detail"]
    rec, keep = d["backward_recomputing"], d["backward_keeping_ds"]
    assert keep["workspace_bytes"] > rec["workspace_bytes"] and rec["ms"] > 0 and keep["ms"] > 0
    assert d["backward_path"] == ("keeping dS" if keep["ms"] < rec["ms"] else "recomputing")


@pytest.mark.gpu
@pytest.mark.parametrize("workload,kernel,unit", [("7b_prefill_varlen", "fwd_pipe_kernel", "TFLOP/s"),
                                                  ("7b_decode", "decode_split_kernel", "GB/s")])
def test_bench_lines_of_the_serving_workloads(workload, kernel, unit):
    # the packed prefill batch (two launches per call: their traffic figures are summed) and the decode batch
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--workload", workload, "--steps", "2",
                        "--warmup", "1", "--no-cpu-baseline"], capture_output=True, text=True, timeout=600, cwd=ROOT)
    assert r.returncode == 0, r.stderr[-2000:]
    out = json.loads(r.stdout.strip().splitlines()[-1])
    assert out["unit"] == unit and out["value"] > 0 and out["n_gpus"] == 1 and out["steps"] == 2
    roof = out["roofline"]
    assert kernel in roof["kernel"] and 0 < roof["frac"] < 1
    # the committed counter summary, when it was taken on these kernel sources; else null, never a stale figure
    assert roof["traffic"] is None or roof["traffic"] > 1e8
    if workload == "7b_prefill_varlen":
        assert out["config"]["tflops_fwd_bwd"] > 0 and out["config"]["speedup_vs_padded"] > 1
