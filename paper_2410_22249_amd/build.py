"""Build the in-tree HIP shared libraries for gfx950 with hipcc (no JIT, no torch extension)."""
from __future__ import annotations

import hashlib
import json
import os
import subprocess
import sys
import tempfile
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
    """Start a compiler; its output goes to a temporary file (a pipe that nobody reads while the
    process runs would stall a compile that prints more than the pipe holds)."""
    if verbose:
        print("[build]", " ".join(cmd), flush=True)
    log = tempfile.TemporaryFile(mode="w+")
    proc = subprocess.Popen(cmd, stdout=log, stderr=subprocess.STDOUT, text=True)
    proc.log = log
    return proc


def _finish(proc, what: str, verbose: bool) -> None:
    proc.wait()
    proc.log.seek(0)
    out = proc.log.read()
    proc.log.close()
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
    with open(MANIFEST, "w") as fh:
        json.dump(_hashes(), fh, indent=0)


def _sources():
    """Every file a library is built from: the listed sources, the headers beside them and the
    C-ABI header."""
    files = {os.path.join(ROOT, "include", "emb_bag.h")}
    for srcs in TARGETS.values():
        for src, _ in srcs:
            files.add(os.path.join(ROOT, src))
            d = os.path.dirname(os.path.join(ROOT, src))
            files.update(os.path.join(d, f) for f in os.listdir(d) if f.endswith(".h"))
    files.update(os.path.join(ROOT, src) for src in C_PROGRAMS.values())
    return files


MANIFEST = os.path.join(PKG, "build_manifest.json")   # content hashes of the sources last built


def _hashes() -> dict:
    out = {}
    for f in sorted(_sources()):
        with open(f, "rb") as fh:
            out[os.path.relpath(f, ROOT)] = hashlib.sha256(fh.read()).hexdigest()
    return out


def stale() -> list:
    """Sources whose content differs from what the libraries were built from (by content hash,
    so that copying the tree to another machine does not make them look old or new)."""
    outs = [os.path.join(ROOT, out) for out in list(TARGETS) + list(C_PROGRAMS)]
    if not all(os.path.exists(o) for o in outs) or not os.path.exists(MANIFEST):
        return ["(a library is missing)"]
    with open(MANIFEST) as fh:
        built = json.load(fh)
    now = _hashes()
    return sorted(f for f in set(now) | set(built) if now.get(f) != built.get(f))


def ensure_built(verbose: bool = True) -> None:
    """Tests, smoke() and bench.py load what is built.  Nothing built: build.  Built from older
    sources than those on disk: build again where a compiler is at hand, otherwise refuse to run
    an out-of-date binary silently."""
    old = stale()
    if not old:
        return
    if os.path.exists(HIPCC):
        if verbose or old != ["(a library is missing)"]:
            print(f"[build] rebuilding: changed since the last build: {', '.join(old[:6])}", flush=True)
        build_all(verbose=verbose)
    else:
        raise RuntimeError("the built libraries do not match " + ", ".join(old[:6]) +
                           " and there is no hipcc here: run __graft_entry__.build()")


if __name__ == "__main__":
    build_all()
    sys.exit(0)
