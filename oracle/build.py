"""Compile the C oracle into ``oracle/librodimus_oracle.so`` (gcc, no fast-math).

Building the checker is not using it: the product build may call this so the
tests find the library, but nothing in the product path loads the result.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "rodimus_oracle.c")
LIB = os.path.join(HERE, "librodimus_oracle.so")


def build(force: bool = True, sanitize: bool = False) -> str:
    """sanitize: AddressSanitizer + UndefinedBehaviorSanitizer build of the same library (a checking build: load it in a
    Python process started with LD_PRELOAD=$(gcc -print-file-name=libasan.so) ASAN_OPTIONS=detect_leaks=0, run the CPU
    tests, then build again without the flag)."""
    if not force and not sanitize and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fno-fast-math", "-ffp-contract=off",
           "-Wall", "-Wextra", "-shared", "-fPIC", SRC, "-o", LIB, "-lm"]
    if sanitize:
        cmd[1:2] = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer"]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    import sys
    print(build(sanitize="--sanitize" in sys.argv[1:]))
