"""Host-side checks of bench.py's contract that need no GPU: a run on more than one GPU is refused
with a message, and the default step counts / oracle samples stay bounded."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode == 2 and "ONE GPU" in r.stderr and r.stdout.strip() == ""
    env = dict(os.environ, WORLD_SIZE="4")
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py")], capture_output=True, text=True, env=env)
    assert r.returncode == 2


def test_default_sizes_are_bounded():
    sys.path.insert(0, ROOT)
    import bench
    from workloads import CONFIGS
    assert set(bench.DEFAULT_STEPS) == set(bench.ORACLE_SAMPLE_POP) == set(CONFIGS)
    for name, c in CONFIGS.items():
        assert 1 <= bench.DEFAULT_STEPS[name] <= 1000
        pop = bench.ORACLE_SAMPLE_POP[name]
        assert 2 <= pop <= c.pop and pop % 2 == 0
        assert name in bench.MEASURED_TRAFFIC_BYTES
    assert bench.PEAK_HBM_GBS == 8000.0 and bench.PEAK_MFMA_F32_TF == 157.3 and bench.PEAK_MFMA_BF16_TF == 2500.0
