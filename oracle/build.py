"""Compile the C oracle into ``oracle/libbigcn_oracle.so`` with gcc (test infrastructure)."""

from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SOURCE = os.path.join(HERE, "bigcn_oracle.c")
LIBRARY = os.path.join(HERE, "libbigcn_oracle.so")


def build(force: bool = True) -> str:
    """Build the shared library; with ``force=False`` an up-to-date library is kept."""
    if (not force and os.path.exists(LIBRARY)
            and os.path.getmtime(LIBRARY) >= os.path.getmtime(SOURCE)):
        return LIBRARY
    cmd = ["gcc", "-O3", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-Wextra",
           "-fno-fast-math", "-o", LIBRARY, SOURCE, "-lm"]
    subprocess.run(cmd, check=True, cwd=HERE)
    return LIBRARY


if __name__ == "__main__":
    print(build())
