"""bench.py issues the steps on two streams, with events that carry no system-scope fence and a
count read from pinned memory.  Its --self-check runs that step sequence and the same steps call
by call on one stream from the same tables and requires identical tables; here it is run on the
headline workload (child process: bench.py is a program, not a module)."""
import json
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.parametrize("extra", [[], ["--optimizer", "adagrad"], ["--index32"]], ids=["sgd", "adagrad", "int32"])
def test_timed_step_sequence_gives_the_tables_of_the_call_by_call_sequence(extra):
    print("[bench] self-check", extra, flush=True)
    cmd = [sys.executable, os.path.join(ROOT, "bench.py"), "--config", "3", "--steps", "8", "--warmup", "2",
           "--self-check", "5", "--no-cpu-baseline"] + extra
    r = subprocess.run(cmd, capture_output=True, text=True, timeout=600, cwd=ROOT)
    assert r.returncode == 0, r.stderr[-2000:]
    assert "tables identical" in r.stderr
    line = json.loads(r.stdout.strip().splitlines()[-1])
    assert line["n_gpus"] == 1 and line["steps"] == 8 and line["value"] > 0
    assert line["config"]["workload"].startswith("3:")
    assert "roofline" in line and line["roofline"]["frac"] > 0


def test_free_form_workload_and_trace_locality_flags_run():
    """bench.py on a workload described on the command line, and on workload 1 with trace-generated indices."""
    for extra, tag in (["--tables", "3", "--rows", "5000", "--dim", "32", "--batch", "256", "--bag", "1:9", "--dist",
                        "zipf:1.1", "--dtype", "bf16"], "0:custom"), (["--config", "1", "--locality", "1.1"], "1:tiny_trace"):
        cmd = [sys.executable, os.path.join(ROOT, "bench.py"), "--steps", "6", "--warmup", "2", "--no-cpu-baseline"] + extra
        r = subprocess.run(cmd, capture_output=True, text=True, timeout=600, cwd=ROOT)
        assert r.returncode == 0, r.stderr[-2000:]
        line = json.loads(r.stdout.strip().splitlines()[-1])
        assert line["config"]["workload"].startswith(tag) and line["value"] > 0
        assert line["state_after_run"]["finite"] and line["roofline"]["traffic"] is None
        assert "per_workload" not in line
