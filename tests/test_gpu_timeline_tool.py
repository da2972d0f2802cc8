"""The measuring aid keeps working: the instrumented build of the library (same sources, -DSPECPV_TIMELINE) loads,
its kernels record their time stamps and clock readings, and timeline.py prints them.  Each run is a process of its
own because the binding loads one library per process."""
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2512_02337_amd", "libspecpv_timeline.so")


def _run(args):
    if not os.path.exists(LIB):
        pytest.skip("instrumented library not built (python -m paper_2512_02337_amd.build --timeline)")
    env = dict(os.environ)
    env.pop("SPECPV_LIB", None)
    p = subprocess.run([sys.executable, "-m", "paper_2512_02337_amd.timeline"] + args, cwd=ROOT, env=env,
                       capture_output=True, text=True, timeout=110)
    assert p.returncode == 0, p.stdout[-2000:] + p.stderr[-2000:]
    return p.stdout


def test_partial_step_timeline(gpu_lib):
    out = _run(["--workload", "llama8b_16k", "--layers", "2", "--reps", "3"])
    assert "chunk loop done" in out and "combine kernel" in out and "core clock" in out, out[-1500:]


def test_full_verification_clock_readings(gpu_lib):
    out = _run(["--full", "--workload", "llama8b_16k", "--layers", "1", "--reps", "4"])
    lines = [l for l in out.splitlines() if "core cycles per chunk" in l]
    assert lines, out[-1500:]
    cycles = float(lines[-1].split("chunks per workgroup,")[1].split("core cycles")[0])
    assert 500 < cycles < 20000, lines[-1]   # a plausible figure, i.e. both counters were read
