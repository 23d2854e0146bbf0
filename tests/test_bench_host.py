"""bench.py's host-side contract that needs no GPU: more than one GPU is refused with a message, the record lines of
the committed profiles parse, and they name the kernel sources they were measured on."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode == 2
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_profile_records_parse_and_carry_a_source_hash():
    sys.path.insert(0, ROOT)
    import bench
    recs = bench.profile_records()
    assert recs, "profiles/ holds no bench-record lines"
    sha = bench.kernels_sha()
    assert len(sha) == 12 and int(sha, 16) >= 0
    for key, rec in recs.items():
        workload, pipeline, eps, kernel = key
        assert workload in ("C1", "C2", "C3", "C4", "C5", "KV7", "KV13") and pipeline in ("fused", "staged")
        assert isinstance(eps, float) and kernel.startswith("k_")
        assert len(rec["kernels_sha"]) == 12 and rec["source"].endswith(".txt")
        assert os.path.exists(os.path.join(ROOT, "profiles", rec["source"]))
        assert any(k in rec for k in ("hbm_bytes", "valu_wave_insts"))


def test_launch_modes_are_offered():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--help"], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0
    for word in ("--launch", "two-streams", "--workload", "--steps", "--warmup", "--gpus"):
        assert word in r.stdout
