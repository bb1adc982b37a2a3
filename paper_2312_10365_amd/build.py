"""Build libspt.so from csrc/ with hipcc for gfx950 (in-tree, no JIT cache)."""
from __future__ import annotations

import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
OUT = os.path.join(_HERE, "libspt.so")
SOURCES = ("api.cpp", "profile.cpp", "router.hip", "bucket.hip", "ffn.hip", "ffn_wide.hip", "lora.hip", "mha.hip")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def build_libspt(verbose: bool = False) -> str:
    cmd = ["hipcc", *FLAGS, "-o", OUT, *[os.path.join(CSRC, s) for s in SOURCES]]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + r.stdout + r.stderr)
    if verbose:
        print(r.stderr)
    return OUT


if __name__ == "__main__":
    print(build_libspt(verbose=True))
