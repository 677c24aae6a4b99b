"""Compile the oracle's C helper (float32 gate-logit order) with gcc.

TEST INFRASTRUCTURE ONLY.  No contraction, no fast-math: the file's own fmaf
calls are the only fused operations."""
import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))


def build() -> str:
    src = os.path.join(_HERE, "gate_logits.c")
    out = os.path.join(_HERE, "_gate_logits.so")
    cmd = ["gcc", "-O2", "-fPIC", "-shared", "-std=c11", "-ffp-contract=off", "-fno-fast-math",
           "-o", out, src, "-lm"]
    subprocess.run(cmd, check=True)
    return out


if __name__ == "__main__":
    print(build())
