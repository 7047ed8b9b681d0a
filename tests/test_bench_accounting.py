"""The byte and flop accounting bench.py reports against, checked on the CPU: the figures of the
32K-token configuration follow from its shapes alone."""
import bench
import wkv_synth as S


def test_c4_algorithmic_bytes():
    w = S.make_workload("c4")
    ab = bench.algorithmic_bytes(w)
    row = 128 * 2                                           # one bf16 row of a KV head
    k_first = 32768 * 8 * row * 8                           # scored keys: 8 KV heads, 8 groups, read once
    q = 32 * 32 * row * 8
    kept = 256 * 16 + 32                                    # rows kept per KV head
    gather_one_way = 32 * 2 * kept * 8 * row                # 32 layers, K and V
    assert ab["gather"] == 2 * gather_one_way == 1082130432
    assert ab["score_stats"] == ab["score_stage"] == k_first + q          # Eq. 1-2 as a stage: the keys once
    assert ab["score"] == k_first + q + 8 * 8 * 2046 * 4                  # + the window scores it writes
    assert ab["pipeline"] == k_first + q + 2 * gather_one_way == 1621098496
    # per layer group: 67.1 MB of keys + 67.6 MB gathered in + 67.6 MB out
    assert round(ab["pipeline"] / 8 / 1e6, 1) == 202.6
    assert bench.score_flops(w) == 2 * 32 * 32 * 128 * 32768 * 8
    # 60 % of the 8 TB/s peak on these bytes is the step time the target asks for
    assert abs(ab["pipeline"] / (0.6 * 8e12) * 1e6 - 337.7) < 0.1


def test_traffic_figures_are_tied_to_the_kernel_sources(tmp_path, monkeypatch):
    # a traffic profile counts only for the kernel sources it was measured on
    import json, os
    monkeypatch.setattr(bench, "ROOT", str(tmp_path))
    os.makedirs(tmp_path / "profiles")
    rec = {"workloads": {"c4": {"kernel_sources_sha256": bench.kernel_sources_sha256(), "bytes_per_launch": {"gather": 1.0e9}}}}
    (tmp_path / "profiles" / "traffic.json").write_text(json.dumps(rec))
    assert bench.measured_traffic("c4") == {"gather": 1.0e9}
    assert bench.measured_traffic("c2") == {}
    rec["workloads"]["c4"]["kernel_sources_sha256"] = "0" * 64
    (tmp_path / "profiles" / "traffic.json").write_text(json.dumps(rec))
    assert bench.measured_traffic("c4") == {}


def test_only_one_gpu_is_accepted():
    import subprocess, sys, os
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "one GPU" in r.stderr
