"""Build the in-tree HIP shared libraries for gfx950 with hipcc (no JIT, no torch extension)."""
from __future__ import annotations

import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
HIP_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
             "-Wall", "-Wno-unused-command-line-argument"]

TARGETS = {
    # output (relative to the repo root): sources
    "paper_2410_22249_amd/libembbag.so": ["paper_2410_22249_amd/csrc/emb_bag.hip"],
    "inputgen/libembgen.so": ["inputgen/csrc/embgen.hip"],
}


def build_all(verbose: bool = True) -> None:
    for out, srcs in TARGETS.items():
        cmd = [HIPCC] + HIP_FLAGS + ["-I", os.path.join(ROOT, "include"), "-o",
                                      os.path.join(ROOT, out)] + [os.path.join(ROOT, s) for s in srcs]
        if verbose:
            print("[build]", " ".join(cmd), flush=True)
        r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        # the host pass does not know the packed-fp32 feature and says so: harmless noise
        log = "\n".join(l for l in r.stdout.splitlines() if "packed-fp32-ops" not in l)
        if log.strip() and (verbose or r.returncode):
            print(log, flush=True)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed for {out}")


def ensure_built(verbose: bool = True) -> None:
    """Build only if a library is missing (tests, smoke() and bench.py load what is there)."""
    if not all(os.path.exists(os.path.join(ROOT, out)) for out in TARGETS):
        build_all(verbose=verbose)


if __name__ == "__main__":
    build_all()
    sys.exit(0)
