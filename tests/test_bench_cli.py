"""Host-side behaviour of bench.py that needs no GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)


def test_more_than_one_gpu_is_refused_with_a_message():
    # this build runs on exactly one GPU: bench.py says so and exits before it imports torch
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=60)
    assert r.returncode == 2
    assert "one GPU" in r.stderr
    assert r.stdout.strip() == ""


def test_committed_profiles_carry_the_figures_the_roofline_block_reads():
    # roofline.traffic and gather_path.issued_16B_loads_per_launch are read from the rocprofv3 summaries under profiles/
    import bench
    for cfg in (1, 2, 3, 4, 5):
        hbm = bench.profile_value(cfg, "hbm_bytes_per_launch")
        l1 = bench.profile_value(cfg, "l1_accesses_per_launch")
        assert hbm is not None and hbm > 0, cfg
        assert l1 is not None and l1 > 0, cfg
    assert bench.profile_value(5, "no_such_key") is None
    assert bench.profile_value(9, "hbm_bytes_per_launch") is None
