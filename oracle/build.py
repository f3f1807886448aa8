"""Compile the CPU oracle (test infrastructure) into two shared objects:
liboracle_f64.so (ORC_REAL=double, the parity reference) and liboracle_f32.so
(ORC_REAL=float).  Run as `python oracle/build.py`; also called by the build entry."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
OUT = os.path.join(HERE, "_build")


def lib_path(precision: str) -> str:
    return os.path.join(OUT, f"liboracle_{precision}.so")


def build(force: bool = True) -> None:
    os.makedirs(OUT, exist_ok=True)
    src = os.path.join(HERE, "echo_oracle.c")
    for prec, real in (("f64", "double"), ("f32", "float")):
        out = lib_path(prec)
        if not force and os.path.exists(out) and os.path.getmtime(out) >= os.path.getmtime(src):
            continue
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-fno-fast-math",
               "-ffp-contract=off", f"-DORC_REAL={real}", src, "-o", out, "-lm"]
        subprocess.check_call(cmd)


if __name__ == "__main__":
    build(force=True)
    print("built", lib_path("f64"), lib_path("f32"), file=sys.stderr)
