"""Build the HIP shared library (gfx950) in-tree: paper_2602_02192_amd/libecho_hip.so.

`python -m paper_2602_02192_amd.build` compiles every source under csrc/ with hipcc and links them.
Objects go to paper_2602_02192_amd/_build/ (ignored by git)."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libecho_hip.so")
CLIENT = os.path.join(HERE, "echo_client")   # the C-ABI client without Python (csrc/echo_client.cpp)

FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-gpu-rdc",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-function", "-Wno-unknown-warning-option", "-Wno-pass-failed",
         "-Wno-unused-result", "-Wno-unused-value"]


def sources():
    return sorted(f for f in os.listdir(CSRC) if f.endswith(".hip"))


def _stale(obj, src):
    if not os.path.exists(obj):
        return True
    t = os.path.getmtime(obj)
    deps = [src] + [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".h")]
    deps.append(os.path.join(HERE, "..", "include", "echo.h"))
    return any(os.path.getmtime(d) > t for d in deps)


def _compile(name, force):
    src = os.path.join(CSRC, name)
    obj = os.path.join(OBJ, name[:-4] + ".o")
    if force or _stale(obj, src):
        r = subprocess.run(["hipcc", *FLAGS, "-c", src, "-o", obj], capture_output=True, text=True)
        err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed on {name}:\n{err}")
        if err.strip():
            print(err, file=sys.stderr)
    return obj


def build(force: bool = True) -> str:
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=6) as ex:
        objs = list(ex.map(lambda n: _compile(n, force), sources()))
    subprocess.check_call(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs])
    subprocess.check_call(["hipcc", "-O2", "-std=c++17", "-fopenmp", "-Wno-unused-result", os.path.join(CSRC, "echo_client.cpp"), "-o", CLIENT,
                           "-L" + HERE, "-lecho_hip", "-Wl,-rpath,$ORIGIN"])
    return LIB


if __name__ == "__main__":
    print(build(force="--incremental" not in sys.argv))
