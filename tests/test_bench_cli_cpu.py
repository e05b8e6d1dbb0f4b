"""bench.py's command line on a machine without a GPU: the single-GPU contract and the options."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def run(*args, env=None):
    e = dict(os.environ)
    e.update(env or {})
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], cwd=ROOT, env=e,
                          capture_output=True, text=True, timeout=300)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = run("--gpus", "2")
    assert r.returncode != 0 and "one GPU" in r.stderr
    r = run(env={"WORLD_SIZE": "4"})
    assert r.returncode != 0 and "one GPU" in r.stderr


def test_help_lists_the_workload_and_measurement_options():
    r = run("--help")
    assert r.returncode == 0
    for opt in ("--gpus", "--steps", "--warmup", "--workload", "--tokens", "--ffn-split", "--ep-sim",
                "--predictor-accuracy", "--no-cpu-baseline"):
        assert opt in r.stdout
