"""bench.py's command line, as far as it goes without a GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode == 2
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_help_lists_the_contract_flags():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--help"], capture_output=True, text=True)
    assert r.returncode == 0
    for flag in ("--gpus", "--steps", "--warmup", "--workload"):
        assert flag in r.stdout


def test_traffic_table_is_readable_and_names_its_commit():
    """roofline.traffic comes from the tracked counter summary, not from constants in bench.py."""
    import sys
    sys.path.insert(0, ROOT)
    import bench
    # the dominant kernel of the default path, of the same with separate passes, and of the single wide pass
    for key, kernel, out_bytes in (("config4", "combine<bf16,f32,R=16>+gram4", 4 * 4), ("config4_separate", "combine<bf16,f32,R=16>", 4 * 4),
                                   ("config4_radix64", "combine<bf16,bf16,R=64>", 2)):
        t = bench.measured_traffic(key, kernel)
        assert t is not None and t["source"] == "profiles/hbm_traffic_table.md", (key, kernel)
        # 64 bf16 leaves read and the nodes (or the result) written over N = 335 141 888, give or take a few per cent
        assert 0.99 < t["bytes"] / (64 * 335141888 * 2 + 335141888 * out_bytes) < 1.05
        assert len(t["measured_at_commit"]) >= 7
    assert bench.measured_traffic("config4", "no such kernel") is None
    assert bench.pair_per_level_bytes(64, 335141888, 2, 2) == 1002 * 335141888
