"""bench.py's command-line contract that can be checked without a GPU: one GPU only."""

import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run(args, env=None):
    e = dict(os.environ)
    e.update(env or {})
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py")] + args, capture_output=True, text=True,
                          timeout=120, env=e, cwd=ROOT)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = _run(["--gpus", "2"])
    assert r.returncode != 0
    assert "not supported" in (r.stderr + r.stdout)
    assert "{" not in r.stdout                      # no result line is printed


def test_a_multi_rank_launch_is_refused_too():
    r = _run([], env={"WORLD_SIZE": "2", "RANK": "0"})
    assert r.returncode != 0 and "not supported" in (r.stderr + r.stdout)
