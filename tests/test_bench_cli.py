"""bench.py's command line, without a GPU: the one-GPU rule and the missing-library rule."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def run_bench(*args, env=None):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], cwd=ROOT, env=env,
                          stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True, timeout=120)


def test_more_than_one_gpu_is_refused_with_a_message():
    res = run_bench("--gpus", "2")
    assert res.returncode != 0
    assert "one GPU" in res.stderr + res.stdout
    assert "{" not in res.stdout          # no result line


def test_missing_library_fails_loudly():
    """The product path has no fallback: with the library path pointing nowhere the run ends with an error."""
    env = dict(os.environ, KSA_LIB=os.path.join(ROOT, "no_such_dir", "libksa.so"))
    res = run_bench("--steps", "1", "--warmup", "0", env=env)
    assert res.returncode != 0
    assert "{\"metric\"" not in res.stdout
