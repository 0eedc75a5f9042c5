"""Compile the CPU oracle (plain C, OpenMP over rows) into oracle/liblq_oracle.so."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))


def build(out: str = None, sanitize: bool = False) -> str:
    """sanitize: an instrumented copy for the pin suite (undefined behaviour, array bounds, float-to-integer overflow
    abort the process; no recovery), same arithmetic flags."""
    src = os.path.join(HERE, "lq_oracle.c")
    out = out or os.path.join(HERE, "liblq_oracle.so")
    cmd = ["gcc", "-O1" if sanitize else "-O2", "-fno-fast-math", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC",
           "-Wall", "-Wextra"]
    if sanitize:
        cmd += ["-g", "-fsanitize=undefined,float-cast-overflow,bounds-strict", "-fno-sanitize-recover=all",
                "-fstack-protector-all"]
    subprocess.run(cmd + ["-o", out, src, "-lm"], check=True)
    return out


if __name__ == "__main__":
    print(build())
    sys.exit(0)
