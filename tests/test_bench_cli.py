"""bench.py's command line, as far as it can be checked without a GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_phase_timing_variant_is_declared_by_the_build_script():
    sys.path.insert(0, ROOT)
    from paper_2103_14949_amd import build as hip_build
    assert hip_build.PHASE_LIB.endswith("libhago_phase.so")
    assert any(s.endswith("qgemm_dma.hip") for s in hip_build.sources())
