"""Build the in-tree HIP shared libraries for gfx950 with hipcc (no JIT, no torch extension)."""
from __future__ import annotations

import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
HIP_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
             "-Wall", "-Wno-unused-command-line-argument"]

TARGETS = {
    # output (relative to the repo root): sources (compiled side by side, then linked)
    "paper_2410_22249_amd/libembbag.so": ["paper_2410_22249_amd/csrc/emb_bag.hip",
                                          "paper_2410_22249_amd/csrc/emb_bag_stream.hip"],
    "inputgen/libembgen.so": ["inputgen/csrc/embgen.hip"],
}
OBJ_DIR = os.path.join(ROOT, "_build")


C_DRIVER_SRC = "tests/c_abi/c_abi_driver.c"
C_DRIVER_BIN = "tests/c_abi/c_abi_driver"


def build_c_driver(verbose: bool = True) -> None:
    """The plain-C caller of the ABI (gcc, HIP runtime API, no torch): proves the boundary is C."""
    cmd = ["gcc", "-std=c99", "-O1", "-Wall", "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include",
           "-I", os.path.join(ROOT, "include"), "-o", os.path.join(ROOT, C_DRIVER_BIN),
           os.path.join(ROOT, C_DRIVER_SRC), "-L", PKG, "-lembbag", "-L/opt/rocm/lib",
           "-lamdhip64", "-lm", "-Wl,-rpath,$ORIGIN/../../paper_2410_22249_amd",
           "-Wl,-rpath,/opt/rocm/lib"]
    if verbose:
        print("[build]", " ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)


def _run(cmd, verbose: bool):
    if verbose:
        print("[build]", " ".join(cmd), flush=True)
    return subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)


def _finish(proc, what: str, verbose: bool) -> None:
    out, _ = proc.communicate()
    # the host pass does not know the packed-fp32 feature and says so: harmless noise
    log = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
    if log.strip() and (verbose or proc.returncode):
        print(log, flush=True)
    if proc.returncode != 0:
        raise RuntimeError(f"hipcc failed for {what}")


def build_all(verbose: bool = True) -> None:
    os.makedirs(OBJ_DIR, exist_ok=True)
    inc = ["-I", os.path.join(ROOT, "include")]
    # every source to an object, all at once; then one link per library
    jobs = []
    for out, srcs in TARGETS.items():
        for src in srcs:
            obj = os.path.join(OBJ_DIR, os.path.basename(src) + ".o")
            jobs.append((src, _run([HIPCC] + HIP_FLAGS + inc + ["-c", "-o", obj,
                                                               os.path.join(ROOT, src)], verbose)))
    for src, proc in jobs:
        _finish(proc, src, verbose)
    for out, srcs in TARGETS.items():
        objs = [os.path.join(OBJ_DIR, os.path.basename(src) + ".o") for src in srcs]
        _finish(_run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o",
                      os.path.join(ROOT, out)] + objs, verbose), out, verbose)
    build_c_driver(verbose)


def ensure_built(verbose: bool = True) -> None:
    """Build only if a library is missing (tests, smoke() and bench.py load what is there)."""
    if not all(os.path.exists(os.path.join(ROOT, out)) for out in list(TARGETS) + [C_DRIVER_BIN]):
        build_all(verbose=verbose)


if __name__ == "__main__":
    build_all()
    sys.exit(0)
