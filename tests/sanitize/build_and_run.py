"""AddressSanitizer + UndefinedBehaviorSanitizer build of the host-side code: the C oracle and the library's
host-side scheduler, driven by sanitize_main.c beside this file.  Test infrastructure: the only place where the
oracle and a source file of the library are linked into one program, and only to run them under the sanitizers.

    python tests/sanitize/build_and_run.py        # builds tests/sanitize/_sanitize/host_asan and runs it

Returns / exits 0 when the run is clean.  (The GPU side cannot be sanitized on this system; device code is checked
by the parity tests.)
"""
from __future__ import annotations

import os
import subprocess
import sys
from pathlib import Path

HERE = Path(__file__).resolve().parent
ROOT = HERE.parent.parent
OUT = HERE / "_sanitize"
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1"]


def build() -> Path:
    OUT.mkdir(exist_ok=True)
    exe = OUT / "host_asan"
    objs = []
    for src, cc, std in ((ROOT / "oracle" / "specee_ref.c", "gcc", "-std=c99"), (HERE / "sanitize_main.c", "gcc", "-std=c99"),
                         (ROOT / "paper_2504_08850_amd" / "csrc" / "sched.cpp", "g++", "-std=c++17")):
        obj = OUT / (src.stem + ".o")
        subprocess.run([cc, std, *SAN, "-fopenmp", "-ffp-contract=off", "-Wall", "-c", str(src), "-o", str(obj)], check=True)
        objs.append(str(obj))
    subprocess.run(["g++", *SAN, "-fopenmp", *objs, "-o", str(exe), "-lm"], check=True)
    return exe


def run() -> subprocess.CompletedProcess:
    exe = build()
    # (verify_asan_link_order=0: whatever the environment preloads may stay ahead of the sanitizer runtime)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0",
               UBSAN_OPTIONS="print_stacktrace=1")
    return subprocess.run([str(exe)], capture_output=True, text=True, env=env)


if __name__ == "__main__":
    r = run()
    sys.stdout.write(r.stdout)
    sys.stderr.write(r.stderr)
    sys.exit(r.returncode)
