"""Build ``librodimus_hip.so`` (HIP, gfx950 only) in-tree from ``csrc/*.hip`` with hipcc.

The library is the product: the binding in ``rodimus.py`` loads it and nothing else.
hipcc cross-compiles without a GPU, so this also runs on a CPU-only machine.
"""
import glob
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ_DIR = os.path.join(CSRC, "_build")
LIB = os.path.join(HERE, "librodimus_hip.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-Wall", "-Wno-unused-function",
    # packed fp32 VALU forms are kept out of the generated code on this target
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def _compile(src: str, extra) -> str:
    obj = os.path.join(OBJ_DIR, os.path.basename(src)[:-4] + ".o")
    subprocess.run([HIPCC, *FLAGS, *extra, "-c", src, "-o", obj], check=True)
    return obj


# AddressSanitizer + UndefinedBehaviorSanitizer on the HOST side only (argument validation and dispatch in
# csrc/rodimus_api.hip and the launchers); the device code is compiled as usual.  A checking build: run the CPU tests of
# the boundary with LD_PRELOAD set to clang's ASan runtime (`hipcc -print-file-name=libclang_rt.asan-x86_64.so`) and
# ASAN_OPTIONS=detect_leaks=0, then build again without the flag.
HOST_SANITIZE = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-omit-frame-pointer",
                 "-Xarch_host", "-g"]


def build(extra_flags=(), jobs: int = 4, sanitize_host: bool = False) -> str:
    os.makedirs(OBJ_DIR, exist_ok=True)
    extra = list(extra_flags) + (HOST_SANITIZE if sanitize_host else [])
    with ThreadPoolExecutor(max_workers=jobs) as pool:
        objs = list(pool.map(lambda s: _compile(s, extra), sources()))
    link = ["-fsanitize=address", "-fsanitize=undefined", "-shared-libsan"] if sanitize_host else []
    subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", *link, *objs, "-o", LIB], check=True)
    return LIB


if __name__ == "__main__":
    args = sys.argv[1:]
    print(build(extra_flags=[a for a in args if a != "--sanitize-host"], sanitize_host="--sanitize-host" in args))
