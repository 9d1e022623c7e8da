"""Build the in-tree HIP shared libraries for gfx950 with hipcc (no JIT, no torch extension)."""
from __future__ import annotations

import os
import subprocess
import sys
import time

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
HIP_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
             "-Wall", "-Wno-unused-command-line-argument"]

CSRC = "paper_2410_22249_amd/csrc/"
TARGETS = {
    # output (relative to the repo root): (source, variant or None) pairs, compiled side by side,
    # then linked.  The wave and stream kernel sources are compiled once per lanes-per-row class
    # (-DEMB_LPR=n), as is the fused kernel for one width; the fused kernel for different widths
    # once per element type (-DEMB_ELEM=n).
    "paper_2410_22249_amd/libembbag.so":
        [(CSRC + "emb_bag.hip", None), (CSRC + "emb_bag_plan.cpp", None),
         (CSRC + "emb_bag_hot_rows.hip", None)]
        + [(CSRC + "emb_bag_wave.hip", n) for n in (0, 4, 8, 16, 32, 64)]
        + [(CSRC + "emb_bag_stream.hip", n) for n in (4, 8, 16, 32, 64)]
        + [(CSRC + "emb_bag_fused.hip", n) for n in (0, 1, 2, 3, 4)]
        + [(CSRC + "emb_bag_fused_uniform.hip", n) for n in (4, 8, 16, 32, 64)],
    "inputgen/libembgen.so": [("inputgen/csrc/embgen.hip", None)],
}
MAX_JOBS = max(1, min(int(os.environ.get("MAX_JOBS", "8")), os.cpu_count() or 1))
OBJ_DIR = os.path.join(ROOT, "_build")


C_DRIVER_SRC = "tests/c_abi/c_abi_driver.c"
C_DRIVER_BIN = "tests/c_abi/c_abi_driver"
# plain-C programs over the ABI: the parity check, and the host-path timing bench.py reports
C_PROGRAMS = {C_DRIVER_BIN: C_DRIVER_SRC, "tests/c_abi/c_abi_latency": "tests/c_abi/c_abi_latency.c"}


def build_c_driver(verbose: bool = True) -> None:
    """The plain-C callers of the ABI (gcc, HIP runtime API, no torch): prove the boundary is C."""
    for out, src in C_PROGRAMS.items():
        cmd = ["gcc", "-std=c99", "-O1", "-Wall", "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include",
               "-I", os.path.join(ROOT, "include"), "-o", os.path.join(ROOT, out),
               os.path.join(ROOT, src), "-L", PKG, "-lembbag", "-L/opt/rocm/lib",
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


def _define(src: str) -> str:
    return "EMB_ELEM" if src.endswith("emb_bag_fused.hip") else "EMB_LPR"


def _obj(src: str, variant) -> str:
    tag = "" if variant is None else f".{_define(src)[4:].lower()}{variant}"
    return os.path.join(OBJ_DIR, os.path.basename(src) + tag + ".o")


def build_all(verbose: bool = True) -> None:
    os.makedirs(OBJ_DIR, exist_ok=True)
    inc = ["-I", os.path.join(ROOT, "include")]
    # every (source, class) to an object, MAX_JOBS at a time; then one link per library
    todo = [(src, lpr) for srcs in TARGETS.values() for src, lpr in srcs]
    running = []
    while todo or running:
        while todo and len(running) < MAX_JOBS:
            src, lpr = todo.pop(0)
            defs = [] if lpr is None else [f"-D{_define(src)}={lpr}"]
            cmd = [HIPCC] + HIP_FLAGS + inc + defs + ["-c", "-o", _obj(src, lpr),
                                                      os.path.join(ROOT, src)]
            running.append((f"{src} {' '.join(defs)}", _run(cmd, verbose)))
        done = [i for i, (_, proc) in enumerate(running) if proc.poll() is not None]
        if not done:
            time.sleep(0.2)
            continue
        what, proc = running.pop(done[0])
        _finish(proc, what, verbose)
    for out, srcs in TARGETS.items():
        objs = [_obj(src, lpr) for src, lpr in srcs]
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
