"""Build libdiloco_mi355.so (gfx950 only) from csrc/ with hipcc, in-tree.

    python -m paper_2412_01152_amd.build
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
BUILD = os.path.join(HERE, "_build")
OUT = os.path.join(HERE, "libdiloco_mi355.so")
EXAMPLE = os.path.join(HERE, "example_outer_sync")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

# -ffp-contract=off: the bucket index is two separately rounded fp32 operations by definition;
#   fused multiply-adds are written explicitly where they are wanted.
# -munsafe-fp-atomics: LDS / global floating-point atomic adds as single hardware instructions.
# packed-fp32 ops are switched off (scalar fp32 code must stay scalar on this target).
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
         "-munsafe-fp-atomics", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-function", "-Wno-unknown-warning-option"]

UNITS = [("abi.o", "abi.hip", []),
         ("reduce_g0.o", "reduce_dispatch.hip", ["-DDILOCO_W_GROUP=0"]),
         ("reduce_g1.o", "reduce_dispatch.hip", ["-DDILOCO_W_GROUP=1"]),
         ("reduce_g2.o", "reduce_dispatch.hip", ["-DDILOCO_W_GROUP=2"]),
         ("reduce_g3.o", "reduce_dispatch.hip", ["-DDILOCO_W_GROUP=3"]),
         ("ring_order.o", "ring_order.cpp", [])]          # host code only


def _compile(unit):
    obj, src, defs = unit
    cmd = [HIPCC, *FLAGS, *defs, "-c", os.path.join(CSRC, src), "-o", os.path.join(BUILD, obj)]
    r = subprocess.run(cmd, capture_output=True, text=True)
    return unit, r


def build(verbose: bool = False) -> str:
    os.makedirs(BUILD, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(UNITS))) as ex:
        results = list(ex.map(_compile, UNITS))
    for unit, r in results:
        noise = "unknown feature specified for -target-feature"
        err = "\n".join(l for l in r.stderr.splitlines() if noise not in l and l.strip())
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed on {unit[1]} {unit[2]}:\n{err}")
        if verbose and err:
            print(err)
    objs = [os.path.join(BUILD, u[0]) for u in UNITS]
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", OUT]
    subprocess.run(cmd, check=True)
    build_example()
    return OUT


def build_example() -> str:
    """The plain-C caller of the ABI (csrc/example_outer_sync.c), linked against the library just built."""
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    cmd = [os.environ.get("CC", "gcc"), "-std=c99", "-O2", "-Wall", "-D__HIP_PLATFORM_AMD__",
           f"-I{rocm}/include", os.path.join(CSRC, "example_outer_sync.c"), f"-L{HERE}", "-ldiloco_mi355",
           f"-L{rocm}/lib", "-lamdhip64", "-lm", "-Wl,-rpath,$ORIGIN", f"-Wl,-rpath,{rocm}/lib", "-o", EXAMPLE]
    subprocess.run(cmd, check=True)
    return EXAMPLE


if __name__ == "__main__":
    print(build(verbose=True))
    sys.exit(0)
