"""Build so_probe, a torch-free C++ caller of the library's C ABI, for use under profilers
(python -m paper_2509_21271_amd.probe.build_probe).  Not part of the product build: the
library must have been built first; the binary lands next to it and finds it through its
run path."""
from __future__ import annotations

import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
_PKG = os.path.dirname(_HERE)
PROBE = os.path.join(_PKG, "so_probe")


def build() -> str:
    cmd = ["hipcc", "-O2", "-std=c++17", "--offload-arch=gfx950", "-Wno-unused-command-line-argument",
           "-I", os.path.join(_PKG, "..", "include"), "-o", PROBE, os.path.join(_HERE, "so_probe.cpp"),
           "-L", _PKG, "-lso_adam", "-Wl,-rpath,$ORIGIN"]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc (so_probe) failed:\n" + res.stdout + res.stderr)
    return PROBE


if __name__ == "__main__":
    print(build())
