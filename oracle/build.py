"""Builds the CPU oracle (test infrastructure) into oracle/libdistr_attn_oracle.so with gcc."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRCS = [os.path.join(HERE, "distr_attn_oracle.c"), os.path.join(HERE, "distr_attn_oracle_bwd.c")]
OUT = os.path.join(HERE, "libdistr_attn_oracle.so")


def build(verbose: bool = False) -> str:
    # -ffp-contract=off: no multiply-add is fused unless the source says fmaf;
    # -mfma: fmaf is the hardware instruction (correctly rounded either way).
    cmd = ["gcc", "-std=c11", "-O2", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
           "-mfma", "-Wall", "-Wextra", "-o", OUT, *SRCS, "-lm"]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return OUT


if __name__ == "__main__":
    print(build(verbose=True))
    sys.exit(0)
