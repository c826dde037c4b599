"""bench.py's command line on a machine without a GPU: more than one GPU is refused with a message, and
the options the profiles' commands use exist."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def run(*args):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True, text=True, timeout=120)


def test_more_than_one_gpu_is_refused():
    r = run("--gpus", "2")
    assert r.returncode != 0
    assert "one GPU" in r.stderr + r.stdout


def test_options_of_the_profile_commands_exist():
    r = run("--help")
    assert r.returncode == 0
    for opt in ("--steps", "--warmup", "--gpus", "--probe", "--decode-steps", "--no-cpu-baseline"):
        assert opt in r.stdout, opt
