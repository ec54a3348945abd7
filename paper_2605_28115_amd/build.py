"""Builds libcivic.so (HIP, gfx950) in-tree.  `python -m paper_2605_28115_amd.build`."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libcivic.so")
SOURCES = ["api.hip", "score.hip", "select.hip", "compact.hip", "front.hip", "attn.hip", "kv_write.hip", "decode.hip", "rope.hip", "encoder.hip"]

# Packed-fp32 VALU forms are switched off for all device code (compiler flag, not a host flag).
HIPCC_FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
               "-Wall", "-Wno-unused-command-line-argument", "-Wno-unknown-attributes"]


def _run(cmd, verbose: bool) -> None:
    if verbose:
        print(" ".join(cmd), flush=True)
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    # the host pass does not know the packed-fp32 feature and says so; everything else is shown
    noise = ("is not a recognized feature for this target", "warning generated", "warnings generated")
    out = "\n".join(l for l in proc.stdout.splitlines() if not any(n in l for n in noise))
    if out.strip():
        print(out, file=sys.stderr)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed building libcivic.so")


def build(verbose: bool = False) -> str:
    """One object per source, compiled side by side (the translation units share no device code), then one link."""
    import tempfile
    from concurrent.futures import ThreadPoolExecutor
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    common = [f for f in HIPCC_FLAGS if f != "-shared"] + ["-I", os.path.join(ROOT, "include"), "-I", CSRC]
    with tempfile.TemporaryDirectory(prefix="civic_build_") as tmp:
        objs = [os.path.join(tmp, s.replace(".hip", ".o")) for s in SOURCES]
        jobs = [[hipcc, *common, "-c", "-o", o, os.path.join(CSRC, s)] for s, o in zip(SOURCES, objs)]
        with ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as pool:
            list(pool.map(lambda c: _run(c, verbose), jobs))
        _run([hipcc, "--offload-arch=gfx950", "-fPIC", "-shared", "-Wno-unused-command-line-argument", "-o", LIB, *objs], verbose)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
