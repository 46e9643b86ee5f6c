"""Host-only checks of the measurement contract: bench.py refuses more than one GPU, the
tracked summaries under profiles/ are the ones it reads, and each summary names its command."""
import glob
import importlib.util
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def load_bench():
    spec = importlib.util.spec_from_file_location("bench", os.path.join(ROOT, "bench.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0 and "ONE GPU" in r.stderr and r.stdout.strip() == ""
    env = dict(os.environ, WORLD_SIZE="2")
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py")], env=env,
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0 and "ONE GPU" in r.stderr


def test_tracked_traffic_and_peaks_are_read():
    b = load_bench()
    # the dominant kernels of the workloads with a committed counter run
    fused = b.traffic_bytes("c3_fine_128x4", "ffn_fused")
    assert fused is not None and 3.8e9 < fused < 6e9         # algorithmic bytes: 3.81e9
    assert b.traffic_bytes("c2_mixtral_8x4", "ffn_gate_up") > 2.2e9
    assert b.traffic_bytes("c3_fine_128x4", "no_such_kernel") is None
    peaks = b.measured_peaks()
    assert set(peaks) == {"lds_fed_random_data", "registers_random_data"}
    assert all(1000.0 < v < 2500.0 for v in peaks.values())   # TFLOP/s, below the datasheet figure


def test_every_profile_summary_names_its_command():
    files = sorted(glob.glob(os.path.join(ROOT, "profiles", "*")))
    assert files
    for f in files:
        assert f.endswith((".md", ".txt")), f
        text = open(f).read()
        assert "python3 bench.py" in text or "python3 -m paper_2510_19366_amd" in text, f
        assert os.path.getsize(f) < 64 * 1024, f
