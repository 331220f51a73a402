"""Host-side logic of bench.py that needs no GPU: the CPU-baseline legs on a tiny workload, the
traffic file reader, and the refusal of more than one GPU."""
import os
import subprocess
import sys
import types

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

import bench
from paper_2204_04179_amd import workloads as wl


def test_cpu_baseline_legs_report_rates_samples_and_the_measured_ratio():
    w = wl.get("tiny")
    r = types.SimpleNamespace(w=w, X_np=wl.features(w), W_np=wl.weights(w),
                              ids_np=[wl.ids(w, k).reshape(-1) for k in range(w.K)],
                              dH_np=[wl.upstream_grad(w, k) for k in range(w.K)])
    out = bench.cpu_baseline(r, target_s=0.2)
    assert out["kind"] == "oracle" and out["unit"] == "occurrences/s" and out["value"] > 0
    assert out["cores"] >= 1 and "histories" in out["sample"]
    for leg in ("single_thread", "oracle_e2e", "oracle_e2e_single_thread"):
        assert out[leg]["value"] > 0 and out[leg]["histories"] >= 1
    assert out["single_thread"]["cores"] == 1 and out["oracle_e2e_single_thread"]["cores"] == 1
    ratio = out["e2e_over_gram"]
    assert ratio["measured"] > 0
    # R of Eq. 10: interactions per unique item, at least one
    assert ratio["boost_ratio_R_per_step"] >= 1.0 and ratio["boost_ratio_R_per_window"] >= 1.0
    # the thread count is restored for whoever uses the oracle next
    from oracle import gram_oracle as orc
    assert orc.num_threads() == out["cores"]


def test_traffic_file_gives_bytes_and_the_commit_of_the_counter_run(tmp_path, monkeypatch):
    prof = tmp_path / "profiles"
    prof.mkdir()
    (prof / "pmc_traffic.txt").write_text("# workload kernel bytes\n# commit abc1234   (note)\nstress seg_reduce 1144718833\n")
    monkeypatch.setattr(bench, "ROOT", str(tmp_path))
    assert bench.read_traffic("stress", "seg_reduce") == (1144718833.0, "abc1234")
    assert bench.read_traffic("stress", "no_such_kernel") == (None, "abc1234")
    monkeypatch.setattr(bench, "ROOT", str(tmp_path / "nowhere"))
    assert bench.read_traffic("stress", "seg_reduce") == (None, None)


def test_committed_traffic_file_names_its_commit():
    value, commit = bench.read_traffic("stress", "seg_reduce")
    assert value and value > 1e9 and commit


def test_more_than_one_gpu_is_refused_with_a_message():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert p.returncode != 0 and "one GPU" in p.stderr
