"""The host half of the library (free list, tickets, id ring, guards, the scheduler) and the
oracle's C file under AddressSanitizer + UndefinedBehaviorSanitizer -- CPU only.

Builds the sanitizer variant (GPU code is not instrumented) and runs the host-logic tests
again with it in a child process that has the sanitizer's runtime preloaded; any report
from either sanitizer ends that process with an error."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_host_logic_under_address_and_undefined_behaviour_sanitizers():
    env = dict(os.environ, LAMPS_SANITIZE="1")
    build = subprocess.run([sys.executable, "-m", "paper_2410_18248_amd.build"], cwd=ROOT, env=env,
                           capture_output=True, text=True)
    assert build.returncode == 0, build.stderr[-2000:]
    run = subprocess.run([sys.executable, "-m", "paper_2410_18248_amd.build", "--run", sys.executable, "-m", "pytest",
                          "-q", "-x", "-p", "no:cacheprovider", "tests/test_boundary_cpu.py", "tests/test_sched_cpu.py",
                          "tests/test_oracle_attention.py", "tests/test_oracle_blocks.py"],
                         cwd=ROOT, env=env, capture_output=True, text=True)
    tail = (run.stdout + run.stderr)[-3000:]
    assert run.returncode == 0, tail
    assert " passed" in run.stdout and "ERROR: AddressSanitizer" not in tail and "runtime error:" not in tail, tail
