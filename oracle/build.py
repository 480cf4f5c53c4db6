"""Compile the C oracle into oracle/libax_oracle.so with gcc (no HIP involved)."""

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
LIB = os.path.join(HERE, "libax_oracle.so")


def build(force: bool = True) -> str:
    srcs = [os.path.join(HERE, "ax_oracle.c"), os.path.join(HERE, "ax_oracle_quant.c"),
            os.path.join(HERE, "ax_oracle_grad.c")]
    deps = srcs + [os.path.join(HERE, "ax_oracle.h")]
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= max(os.path.getmtime(d) for d in deps):
        return LIB
    # -ffp-contract=off: the float32 steps of the quantization must stay single IEEE operations.
    cmd = ["gcc", "-std=c11", "-O2", "-ffp-contract=off", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
           "-o", LIB] + srcs + ["-lm"]
    subprocess.run(cmd, check=True, cwd=HERE)
    return LIB


if __name__ == "__main__":
    print(build())
