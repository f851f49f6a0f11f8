"""Compile the CPU oracle (plain C, gcc) into oracle/libmsd_oracle.so.

The oracle is test infrastructure: nothing in the product library links against it.
-ffp-contract=off keeps gcc from fusing a*b+c on its own, so the only fused operation
is the explicit fmaf() of the residual step.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "msd_oracle.c")
OUT = os.path.join(HERE, "libmsd_oracle.so")
OUT_SAN = os.path.join(HERE, "libmsd_oracle_san.so")


def sanitize_requested() -> bool:
    """MSD_ORACLE_SANITIZE=1 selects the AddressSanitizer + UndefinedBehaviorSanitizer build of the oracle.
    The process must then have been started with the sanitizer runtime preloaded (sanitizer_preload())."""
    return os.environ.get("MSD_ORACLE_SANITIZE", "") not in ("", "0")


def sanitizer_preload():
    """Path of gcc's AddressSanitizer runtime for LD_PRELOAD, or None when this gcc has none."""
    r = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True)
    path = r.stdout.strip()
    return os.path.realpath(path) if r.returncode == 0 and os.path.isabs(path) and os.path.exists(path) else None


def build(force: bool = True, sanitize=None) -> str:
    if sanitize is None:
        sanitize = sanitize_requested()
    out = OUT_SAN if sanitize else OUT
    if not force and os.path.exists(out) and os.path.getmtime(out) >= os.path.getmtime(SRC):
        return out
    cmd = ["gcc", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fno-fast-math", "-Wall", "-Wextra", "-shared", "-fPIC"]
    # the sanitizer build keeps the arithmetic flags (same results) and adds bounds / UB checking with traps on
    cmd += ["-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
            "-fno-sanitize-recover=undefined"] if sanitize else ["-O2"]
    subprocess.run(cmd + [SRC, "-o", out, "-lm"], check=True)
    return out


if __name__ == "__main__":
    print(build(force=True, sanitize="--sanitize" in sys.argv[1:] or None))
    sys.exit(0)
