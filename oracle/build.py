"""Compile the CPU oracle (plain C, fp64) into oracle/libsdvg_oracle.so with gcc.

Test infrastructure only: nothing in the product package imports this.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "sdvg_oracle.c")
LIB = os.path.join(HERE, "libsdvg_oracle.so")


def build(force: bool = True, extra_flags=(), out: str = LIB) -> str:
    """Compiles the oracle. SDVG_ORACLE_LIBRARY names an already built variant (e.g. one with
    sanitizers) that is used as it is."""
    override = os.environ.get("SDVG_ORACLE_LIBRARY")
    if override and out == LIB:
        return override
    if not force and os.path.exists(out) and os.path.getmtime(out) >= os.path.getmtime(SRC):
        return out
    cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra", *extra_flags,
           "-o", out, SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return out


if __name__ == "__main__":
    print(build())
