"""Build librapid_attn.so (HIP, gfx950 only) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SOURCES = [os.path.join(HERE, "csrc", "rapid_attn.hip"), os.path.join(HERE, "csrc", "rapid_cache.hip"),
           os.path.join(HERE, "csrc", "rapid_mask.hip")]
OUT = os.path.join(HERE, "librapid_attn.so")
# measurement aid used by bench.py only (an MFMA-only loop), kept out of the attention library
PROBE_SOURCES = [os.path.join(HERE, "csrc", "mfma_probe.hip")]
PROBE_OUT = os.path.join(HERE, "libmfma_probe.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-fvisibility=hidden", "-fno-gpu-rdc",
    # no HIP runtime is linked in: the library binds to the libamdhip64 already loaded
    # in the process (PyTorch's), so streams and pointers belong to the same runtime
    "-no-hip-rt",
    # packed fp32 VALU forms are kept off on the test machines
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
    "-I", os.path.join(ROOT, "include"),
]


def build(verbose: bool = False, extra: list[str] | None = None, out: str = OUT) -> str:
    _compile(PROBE_SOURCES, PROBE_OUT, verbose, extra)
    return _compile(SOURCES, out, verbose, extra)


def _compile(sources, out, verbose, extra):
    cmd = [HIPCC] + FLAGS + (extra or []) + ["-o", out] + sources
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "packed-fp32-ops"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed ({res.returncode}):\n{err}")
    if verbose and err.strip():
        print(err, file=sys.stderr)
    return out


if __name__ == "__main__":
    print(build(verbose=True))
