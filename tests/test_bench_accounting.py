"""The byte accounting bench.py reports against the roofline: the algorithmic bytes of a
step and of the dominant kernels, checked against the closed forms and the figures the
design quotes for the two headline workloads.  CPU only."""
import json
import os
import subprocess
import sys

import bench
from paper_1901_01544_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_step_bytes_of_the_headline_workloads():
    alex, r50 = wl.make_config(2), wl.make_config(3)
    assert (alex.P, alex.K, r50.P, r50.K) == (61_100_840, 954_701, 25_557_032, 434_735)
    # (12 W + 4) P + (20 + 8 W) K with W = 8: 100 P + 84 K
    assert bench.step_bytes(alex, 8, 8) == 100 * alex.P + 84 * alex.K == 6_190_278_884
    assert bench.step_bytes(r50, 8, 8) == 100 * r50.P + 84 * r50.K == 2_592_220_940
    # the follower pass: 7 workers accumulate, hand over and clear at K pairs; index read once
    assert bench.dominant_kernel_bytes(alex, 8, 8, "whole_step") == 84 * alex.P + 32 * alex.K
    assert bench.dominant_kernel_bytes(alex, 8, 8, "three_calls") == 84 * alex.P
    # a single accumulating worker: the leader pass (r, g, w in, r out)
    flat = wl.make_config(5, scale_down=1000)
    assert bench.dominant_kernel_bytes(flat, 1, 9, "whole_step") == 16 * flat.P
    # threshold mode: every worker accumulates, each chosen node also reads w, the mask goes out once
    assert bench.threshold_step_bytes(alex, 8, 8, 1, 1000) == (96 + 4) * alex.P + alex.P / 8 + 84 * 1000
    assert bench.threshold_step_bytes(alex, 8, 8, 2, 0) - bench.threshold_step_bytes(alex, 8, 8, 1, 0) == 4 * alex.P
    assert bench.threshold_dominant_bytes(alex, 8, 8, 1, 1000) == 84 * alex.P + alex.P / 8 + 28 * 1000
    assert bench.layerwise_extra_bytes(alex, 1) == 8 * alex.P


def test_traffic_file_names_kernels_the_bench_times():
    d = json.load(open(os.path.join(ROOT, "profiles", "traffic.json")))
    for workload, entries in d.items():
        if workload.startswith("_"):
            continue
        assert workload in bench.WORKLOADS
        for name, b in entries.items():
            assert name.startswith("step:") or name in set(bench.DOMINANT_KERNEL.values()) | {"k_leader_pass"}
            assert isinstance(b, int) and b > 0
    assert bench.traffic_from_profiles("alexnet", "k_follow_gather", check_hash=False) == d["alexnet"]["k_follow_gather"]
    assert bench.traffic_from_profiles("alexnet", "no_such_kernel", check_hash=False) is None


def test_traffic_is_reported_only_for_the_kernel_sources_it_was_measured_on(tmp_path, monkeypatch):
    """The counter figures are constants on file; the bench line carries them only while the file's stamp
    equals the hash of the kernel sources in the tree."""
    h = bench.kernel_source_hash()
    assert len(h) == 64 and h == bench.kernel_source_hash()
    d = json.load(open(os.path.join(ROOT, "profiles", "traffic.json")))
    want = d["alexnet"]["k_follow_gather"] if d.get("_csrc_sha256") == h else None
    assert bench.traffic_from_profiles("alexnet", "k_follow_gather") == want
    (tmp_path / "profiles").mkdir()
    for stamp, expect in ((h, 123), ("0" * 64, None)):
        json.dump({"_csrc_sha256": stamp, "alexnet": {"k_follow_gather": 123}},
                  open(tmp_path / "profiles" / "traffic.json", "w"))
        monkeypatch.setattr(bench, "ROOT", str(tmp_path))
        monkeypatch.setattr(bench, "kernel_source_hash", lambda: h)
        assert bench.traffic_from_profiles("alexnet", "k_follow_gather") == expect


def test_more_than_one_gpu_is_refused():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert p.returncode != 0 and "one GPU" in p.stderr and not p.stdout.strip()
