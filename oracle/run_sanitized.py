#!/usr/bin/env python3
"""Run the CPU-only tests (oracle pins, host workload logic, boundary argument checks) with the oracle
built under AddressSanitizer + UndefinedBehaviorSanitizer.

    python oracle/run_sanitized.py [extra pytest arguments]

The oracle is compiled a second time (gcc -fsanitize=address,undefined, its own library file) and the
tests run in a child process that has the sanitizer runtime first in LD_PRELOAD (an instrumented
shared object loaded into an uninstrumented python needs it there); whatever LD_PRELOAD already holds is
kept behind it.  Any report aborts the run (-fno-sanitize-recover).  Host code only: nothing here touches
a GPU.  Exit status is pytest's.
"""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def main(argv):
    asan = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    if not os.path.isabs(asan) or not os.path.exists(asan):
        print("run_sanitized: gcc has no libasan.so here", file=sys.stderr)
        return 3
    env = dict(os.environ)
    env["PROBE_ORACLE_SANITIZE"] = "1"
    env["LD_PRELOAD"] = asan + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    # python itself leaks by design at exit; OpenMP's thread pool is reported as a leak too
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=1"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    tests = ["tests/test_oracle_route.py", "tests/test_oracle_permute.py", "tests/test_oracle_ffn_combine.py",
             "tests/test_oracle_planner.py", "tests/test_oracle_gating.py", "tests/test_host_workload.py"]
    cmd = [sys.executable, "-m", "pytest", "-q", "-x", "-m", "not gpu", "-p", "no:cacheprovider"] + tests + argv
    return subprocess.run(cmd, cwd=ROOT, env=env).returncode


if __name__ == "__main__":
    sys.exit(main(sys.argv[1:]))
