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


def build_sanitized() -> dict:
    """AddressSanitizer + UndefinedBehaviorSanitizer builds (host code only) of the fp64 oracle and of the library's
    host-only capacity arithmetic: oracle/_build/liboracle_f64_san.so, liboracle_f32_san.so and libecho_capacity_san.so.  A process that loads
    them needs the sanitizer runtime first in its link order (LD_PRELOAD, see asan_runtime)."""
    os.makedirs(OUT, exist_ok=True)
    san = ["-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined"]
    for prec, real in (("f64", "double"), ("f32", "float")):
        orc = os.path.join(OUT, f"liboracle_{prec}_san.so")
        subprocess.check_call(["gcc", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-fno-fast-math", "-ffp-contract=off", *san,
                               f"-DORC_REAL={real}", os.path.join(HERE, "echo_oracle.c"), "-o", orc, "-lm"])
    cap = os.path.join(OUT, "libecho_capacity_san.so")
    src = os.path.join(HERE, "..", "paper_2602_02192_amd", "csrc", "echo_capacity.hip")
    subprocess.check_call(["g++", "-std=c++17", "-fPIC", "-shared", *san, "-x", "c++", src, "-o", cap])
    return {"oracle": os.path.join(OUT, "liboracle_f64_san.so"), "capacity": cap}


def asan_runtime() -> str:
    """Path of the AddressSanitizer runtime of the gcc that built the sanitized libraries."""
    return subprocess.check_output(["gcc", "-print-file-name=libasan.so"], text=True).strip()


if __name__ == "__main__":
    build(force=True)
    print("built", lib_path("f64"), lib_path("f32"), file=sys.stderr)
