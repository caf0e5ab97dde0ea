"""Compile the CPU oracle (plain C, gcc). TEST INFRASTRUCTURE ONLY — never used by the GPU path."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "ellm_oracle.c")
LIB = os.path.join(HERE, "libellm_oracle.so")


def build(force: bool = True, defines: tuple = (), out: str | None = None) -> str:
    """gcc -O2 -shared. `defines` lets tests build deliberately broken variants of the oracle
    (on the CPU only) to show that the pins notice them."""
    out = out or LIB
    if not force and os.path.exists(out) and os.path.getmtime(out) >= os.path.getmtime(SRC):
        return out
    cmd = ["gcc", "-O2", "-std=gnu11", "-shared", "-fPIC", "-pthread", "-Wall", "-Wextra",
           *[f"-D{d}" for d in defines], SRC, "-o", out, "-lm"]
    subprocess.run(cmd, check=True)
    return out


if __name__ == "__main__":
    print(build())
