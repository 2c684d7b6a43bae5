"""Compile oracle/bnn_oracle.c into oracle/libbnn_oracle.so with gcc.

No fast-math and no floating-point contraction: the fp32 accumulation order
written in the C source is the order that runs.

Sanitizer mode (host code only): with BNN_ORACLE_SANITIZE=1 in the environment the oracle is built with
AddressSanitizer and UndefinedBehaviorSanitizer into libbnn_oracle_san.so and that build is the one loaded.  A
sanitized library needs the sanitizer runtime loaded first, so the CPU pins run under it as

    BNN_ORACLE_SANITIZE=1 LD_PRELOAD="$(gcc -print-file-name=libasan.so) $(gcc -print-file-name=libubsan.so)" \
        ASAN_OPTIONS=detect_leaks=0 python -m pytest tests/test_oracle_pins.py tests/test_train_oracle_pins.py -q

(`python oracle/build.py --sanitize-run` builds it and runs exactly that.)
"""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "bnn_oracle.c")
LIB = os.path.join(HERE, "libbnn_oracle.so")
LIB_SAN = os.path.join(HERE, "libbnn_oracle_san.so")

CFLAGS = ["-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off", "-fno-fast-math",
          "-fvisibility=hidden", "-Wall", "-Wextra"]
SAN_FLAGS = ["-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined"]


def sanitize_requested() -> bool:
    return os.environ.get("BNN_ORACLE_SANITIZE", "") not in ("", "0")


def build(force: bool = False, sanitize: bool | None = None) -> str:
    if sanitize is None:
        sanitize = sanitize_requested()
    lib = LIB_SAN if sanitize else LIB
    if force or not os.path.exists(lib) or os.path.getmtime(lib) < os.path.getmtime(SRC):
        flags = [f for f in CFLAGS if f != "-O2"] + SAN_FLAGS if sanitize else CFLAGS
        subprocess.run(["gcc", *flags, SRC, "-o", lib, "-lm"], check=True)
    return lib


def sanitize_run() -> int:
    """Build the sanitized oracle and run the CPU pins of the oracle under it."""
    build(force=True, sanitize=True)
    runtimes = [subprocess.run(["gcc", f"-print-file-name={n}"], capture_output=True, text=True, check=True).stdout.strip()
                for n in ("libasan.so", "libubsan.so")]
    env = dict(os.environ, BNN_ORACLE_SANITIZE="1", LD_PRELOAD=" ".join(runtimes), ASAN_OPTIONS="detect_leaks=0",
               OMP_NUM_THREADS=os.environ.get("OMP_NUM_THREADS", "4"))
    root = os.path.dirname(HERE)
    return subprocess.run([sys.executable, "-m", "pytest", "tests/test_oracle_pins.py", "tests/test_train_oracle_pins.py",
                           "-q", "-x", "-p", "no:cacheprovider"], cwd=root, env=env).returncode


if __name__ == "__main__":
    if "--sanitize-run" in sys.argv:
        sys.exit(sanitize_run())
    print(build(force=True, sanitize="--sanitize" in sys.argv or None))
