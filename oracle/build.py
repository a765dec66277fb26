"""Compile the CPU oracle (plain C, gcc) into oracle/libtutti_oracle.so.

Test infrastructure: the product never calls this library.  `python oracle/build.py` or
`build_oracle()`; the build is skipped when the library is newer than its sources unless
force=True.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SOURCES = [os.path.join(HERE, "tutti_oracle.c")]
HEADERS = [os.path.join(HERE, "tutti_oracle.h")]
LIB = os.path.join(HERE, "libtutti_oracle.so")


def build_oracle(force: bool = False) -> str:
    if not force and os.path.exists(LIB):
        newest = max(os.path.getmtime(p) for p in SOURCES + HEADERS)
        if os.path.getmtime(LIB) >= newest:
            return LIB
    cmd = ["gcc", "-std=c11", "-O2", "-Wall", "-Wextra", "-Werror", "-fPIC", "-shared", "-pthread",
           *SOURCES, "-o", LIB]
    subprocess.run(cmd, check=True, cwd=HERE)
    return LIB


if __name__ == "__main__":
    print(build_oracle(force=True))
