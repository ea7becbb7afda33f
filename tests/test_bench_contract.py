"""bench.py's contract that can be checked without a GPU: it runs on one GPU only and says so."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run(args, env_extra=None):
    env = dict(os.environ)
    env.pop("WORLD_SIZE", None)
    env.update(env_extra or {})
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True, text=True,
                          env=env, timeout=120)


def test_more_than_one_gpu_is_refused_with_a_message():
    for args, extra in ((["--gpus", "2"], None), (["--gpus", "8", "--steps", "5", "--warmup", "1"], None),
                        ([], {"WORLD_SIZE": "2"})):
        r = _run(args, extra)
        assert r.returncode == 2, (args, extra, r.returncode)
        assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_unknown_flags_and_workloads_are_refused_by_the_parser():
    assert _run(["--workload", "imagenet"]).returncode == 2
    assert _run(["--noise-bits", "12"]).returncode == 2
    assert _run(["--uniform-bits", "9"]).returncode == 2
