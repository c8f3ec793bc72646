"""Compile the CPU oracle with AddressSanitizer and UndefinedBehaviorSanitizer (host code only,
gcc) into oracle/libhq_oracle_san.so.  Test infrastructure: the pins' small cases are run against
this build by tests/test_oracle_sanitizers.py, on the CPU; nothing on the GPU side loads it.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "hq_oracle.c")
LIB = os.path.join(HERE, "libhq_oracle_san.so")


def build(force: bool = True) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    cmd = ["gcc", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
           "-fno-omit-frame-pointer", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-ffp-contract=off",
           "-fno-fast-math", "-Wall", "-Wextra", "-o", LIB, SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return LIB


def runtime() -> str:
    """gcc's AddressSanitizer runtime: a process that is not itself instrumented (the Python
    interpreter) has to load it ahead of every other library."""
    out = subprocess.run(["gcc", "-print-file-name=libasan.so"], check=True, capture_output=True, text=True)
    return os.path.realpath(out.stdout.strip())


if __name__ == "__main__":
    print(build())
