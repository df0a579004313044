"""Build libbsp.so (the C-ABI library of gfx950 kernels) in-tree with hipcc."""
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
LIB = os.path.join(HERE, "libbsp.so")
OBJ_DIR = os.path.join(HERE, "_build")
SOURCES = ["bsp_api.hip", "bsp_norms.hip", "bsp_mask.hip", "bsp_pack.hip", "bsp_linear.hip", "bsp_linear_tiled.hip", "bsp_linear_steploop.hip", "bsp_linear_stream16.hip",
           "bsp_plan.hip", "bsp_adam.hip", "bsp_linear_t.hip", "bsp_linear_t_dense.hip", "bsp_linear_dvals.hip"]

FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off", "-fno-fast-math",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-function", "-I", INCLUDE, "-I", CSRC]


def _hipcc():
    for c in ("/opt/rocm/bin/hipcc", "hipcc"):
        if c == "hipcc" or os.path.exists(c):
            return c


def _compile(src):
    obj = os.path.join(OBJ_DIR, src.replace(".hip", ".o"))
    subprocess.run([_hipcc(), *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj], check=True)
    return obj


def _inputs():
    return [os.path.join(CSRC, f) for f in sorted(os.listdir(CSRC)) if f.endswith((".hip", ".h"))] + [
        os.path.join(INCLUDE, "bsp.h")]


def stale() -> bool:
    """True when libbsp.so is missing or older than one of its sources."""
    return not os.path.exists(LIB) or any(os.path.getmtime(LIB) < os.path.getmtime(s) for s in _inputs())


def build(force: bool = True) -> str:
    if not force and not stale():
        return LIB
    os.makedirs(OBJ_DIR, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(_compile, SOURCES))
    subprocess.run([_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs, "-ldl"], check=True)
    return LIB


if __name__ == "__main__":
    print(build())
