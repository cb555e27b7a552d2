"""CPU-only checks of bench.py's contract: it refuses more than one GPU with a message, its
roofline.traffic comes from the committed profile, and every committed profile names its command."""
import glob
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    proc = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert proc.returncode == 2
    assert "one GPU" in proc.stderr
    env = dict(os.environ, WORLD_SIZE="2")
    proc = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py")], capture_output=True, text=True, env=env)
    assert proc.returncode == 2


def test_traffic_is_read_from_the_committed_profile():
    sys.path.insert(0, ROOT)
    import bench
    from workloads import CONFIGS
    for name in ("c1", "c2", "c3", "c4"):
        traffic = bench.read_profiled_traffic(name)
        assert isinstance(traffic, int)
        # measured traffic cannot be below what the call must move, nor absurdly above it
        assert 0.95 * CONFIGS[name].attn_bytes_per_layer() <= traffic <= 4 * CONFIGS[name].attn_bytes_per_layer()
    assert bench.read_profiled_traffic("c9") is None


def test_every_profile_names_the_command_that_made_it():
    files = sorted(glob.glob(os.path.join(ROOT, "profiles", "*.txt")))
    assert files
    for path in files:
        text = open(path).read()
        assert "command" in text and "bench.py" in text, path
        assert len(text) < 40_000, path     # summaries, not raw output
