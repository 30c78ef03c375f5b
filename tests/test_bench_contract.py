"""What can be checked of bench.py without a GPU: more than one GPU is refused with a message, before anything
touches a device."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused():
    for extra_env, args in (({}, ["--gpus", "2"]), ({"WORLD_SIZE": "2"}, [])):
        env = dict(os.environ)
        env.update(extra_env)
        r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True, text=True, env=env, timeout=120)
        assert r.returncode == 2
        assert "ONE GPU" in r.stderr and r.stdout.strip() == ""
