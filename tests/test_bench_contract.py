"""Host-side checks of the bench.py contract that need no GPU: more than one GPU is refused with
a message, and without a GPU the bench fails loudly instead of falling back to the CPU."""
import os
import subprocess
import sys

from conftest import ROOT


def run_bench(*args, env_extra=None):
    env = dict(os.environ)
    env.pop("WORLD_SIZE", None)
    if env_extra:
        env.update(env_extra)
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], cwd=ROOT, env=env,
                          capture_output=True, text=True, timeout=300)


def test_more_than_one_gpu_is_refused():
    r = run_bench("--gpus", "2", "--steps", "1", "--warmup", "0")
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""
    r = run_bench("--steps", "1", "--warmup", "0", env_extra={"WORLD_SIZE": "4"})
    assert r.returncode != 0 and "ONE GPU" in r.stderr


def test_no_cpu_fallback():
    import torch
    if torch.cuda.is_available():
        return                      # on a GPU machine the bench itself is exercised by the driver
    r = run_bench("--steps", "1", "--warmup", "0")
    assert r.returncode != 0
    assert "no GPU" in r.stderr and r.stdout.strip() == ""
