"""bench.py's command line contract, on the CPU: more than one GPU is refused with a message (this build
measures one GPU), the flags the driver passes are accepted, the defaults are the documented ones."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run(*args, env=None):
    e = dict(os.environ)
    e.update(env or {})
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True, text=True,
                          env=e, timeout=120)


def test_more_than_one_gpu_is_refused_with_a_message():
    res = _run("--gpus", "2", "--steps", "1", "--warmup", "0")
    assert res.returncode != 0
    assert "one GPU" in res.stderr
    assert res.stdout.strip() == ""
    res = _run(env={"WORLD_SIZE": "4"})
    assert res.returncode != 0 and "one GPU" in res.stderr


def test_flags_of_the_contract_parse_and_defaults_hold():
    sys.path.insert(0, ROOT)
    import bench
    argv = sys.argv
    try:
        sys.argv = ["bench.py"]
        a = bench.parse()
        assert (a.gpus, a.workload, a.reduce) == (1, "stress", "sum") and a.steps >= 1 and a.warmup >= 0
        sys.argv = ["bench.py", "--gpus", "1", "--steps", "7", "--warmup", "2"]
        a = bench.parse()
        assert (a.gpus, a.steps, a.warmup) == (1, 7, 2)
    finally:
        sys.argv = argv
