"""Compile the C oracle into oracle/libcprune_oracle.so (gcc, OpenMP)."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "cprune_oracle.c")
OUT = os.path.join(HERE, "libcprune_oracle.so")


OUT_F32ACC = os.path.join(HERE, "libcprune_oracle_f32acc.so")


def _compile(out: str, extra, force: bool) -> str:
    if (not force and os.path.exists(out)
            and os.path.getmtime(out) >= os.path.getmtime(SRC)):
        return out
    cmd = ["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
           "-Wall", "-Wextra"] + list(extra) + ["-o", out, SRC, "-lm"]
    subprocess.check_call(cmd)
    return out


def build(force: bool = False) -> str:
    """The parity build (fp64 accumulation); also refreshes the timing-only build."""
    _compile(OUT_F32ACC, ["-DORACLE_ACC_T=float"], force)
    return _compile(OUT, [], force)


def build_f32acc(force: bool = False) -> str:
    """The same loops with a float accumulator: for the benchmark's CPU timing row only."""
    return _compile(OUT_F32ACC, ["-DORACLE_ACC_T=float"], force)


if __name__ == "__main__":
    print(build(force="--force" in sys.argv))
