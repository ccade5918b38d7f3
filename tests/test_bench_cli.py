"""Host-side behaviour of bench.py that needs no GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    """This build runs on one GPU: --gpus N > 1 (or a multi-rank launch) exits at once and says so."""
    for argv, env in ((["--gpus", "2"], {}), ([], {"WORLD_SIZE": "4"})):
        r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py")] + argv, capture_output=True, text=True,
                           env={**os.environ, **env}, timeout=60)
        assert r.returncode == 2
        assert "ONE GPU" in r.stderr and r.stdout == ""
