"""Build libspt.so from csrc/ with hipcc for gfx950 (in-tree, no JIT cache)."""
from __future__ import annotations

import os
import subprocess
import tempfile
from concurrent.futures import ThreadPoolExecutor

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
OUT = os.path.join(_HERE, "libspt.so")
SOURCES = ("api.cpp", "profile.cpp", "router.hip", "bucket.hip", "ffn.hip", "ffn_scatter.hip", "ffn_wide.hip",
           "lora.hip", "mha.hip", "calibrate.hip")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _run(cmd):
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + " ".join(cmd) + "\n" + r.stdout + r.stderr)
    return r.stderr


def build_libspt(verbose: bool = False, only=None) -> str:
    """Compile every source to an object (in parallel), then link.  Objects live in a temporary
    directory, so each call compiles everything again."""
    with tempfile.TemporaryDirectory() as tmp:
        objs = [os.path.join(tmp, s + ".o") for s in SOURCES]
        cmds = [["hipcc", *FLAGS, "-c", os.path.join(CSRC, s), "-o", o] for s, o in zip(SOURCES, objs)]
        with ThreadPoolExecutor(max_workers=min(8, len(cmds))) as ex:
            logs = list(ex.map(_run, cmds))
        logs.append(_run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", OUT, *objs]))
    if verbose:
        print("".join(logs))
    return OUT


if __name__ == "__main__":
    print(build_libspt(verbose=True))
