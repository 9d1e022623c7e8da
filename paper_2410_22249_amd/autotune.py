"""Occupancy x prefetch-depth x cache-policy sweep for one workload shape.

The paper closes with a static profiling recipe (Sec. 7): check whether the kernel is latency- or
bandwidth-bound, sweep the multithreading level, sweep the prefetch station and distance ("low
multithreading => larger distance"), decide on pinning from the reuse of the access pattern, and
combine.  This tool runs that recipe on the MI355X kernels through the public tuning keys:

    python -m paper_2410_22249_amd.autotune --workload cfg3 [--out tuning.json]

It prints one line per setting and a recommendation; `--out` writes the best setting as JSON that
`apply_tuning()` feeds to `emb_bag_set_tuning`.  Inputs are the seeded synthetic workloads of
`inputgen`; timing uses HIP events on the launch stream and rotates index batches.

    python -m paper_2410_22249_amd.autotune --table tuning_table.json [--shapes ...]

runs the recipe per SHAPE instead - for each (row bytes, pooling factor) of a grid it sweeps the
prefetch depth, the bags per wavefront and the kernel (one wavefront per bag / short-bag stream
kernel) on fp32 tables of that shape - and writes the per-shape table that `load_table()` hands to
`emb_bag_set_tuning_table`, which the library's planner then consults for every call.

    python -m paper_2410_22249_amd.autotune pooling ...   (the two kernels over pooling factor x row width)
    python -m paper_2410_22249_amd.autotune mixed ...     (tables of different widths; fused against separate launches)
    python -m paper_2410_22249_amd.autotune hints ...     (where the streaming hint stops paying: the reuse profiler's constants)
"""
from __future__ import annotations

import argparse
import itertools
import json
import os
import sys
from typing import Dict, List

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

DEFAULT_GRID = {
    "blocks_per_cu": [0, 4, 2],        # waves per SIMD: 8 (no cap), 4, 2
    "depth": [1, 2, 4, 8, 16],
    "station": [0, 1],                 # rows in flight land in registers / in LDS (depth 4 and 8)
    "use_hints": [1, 0],
    "xcd_remap": [1, 0],
}
# for short bags add e.g. --grid '{"stream":[0,1],"bags_per_group":[1,2,4,8],"depth":[4,8]}'
NEUTRAL = {"blocks_per_cu": 0, "depth": 0, "use_hints": 1, "xcd_remap": -1, "addressing": 0,
           "stream": -1, "bags_per_group": 0, "xcd_pieces": 0, "per_table_launch": 0, "fuse": 1,
           "bags_per_wave": 0, "hot_split": 0, "station": 0}

# per-shape sweep (--table): rows of 64 B .. 1 KiB, pooling factors from one-hot to the paper's 150
TABLE_ROW_BYTES = [64, 128, 256, 512, 1024]
TABLE_POOLING = [1, 4, 16, 64, 150]
TABLE_GRID = {"stream": [0, 1], "depth": [4, 8], "bags_per_wave": [1, 2, 4]}
TABLE_KEYS = ("depth", "bags_per_wave", "stream", "bags_per_group")


def apply_tuning(settings: Dict[str, int]) -> None:
    """Apply a {key: value} mapping (e.g. loaded from the JSON this tool writes)."""
    from . import emb_bag_set_tuning
    for k, v in settings.items():
        emb_bag_set_tuning(k, int(v))


def choose(results, margin: float = 0.02):
    """Pick a setting from [(seconds, setting), ...]: the fastest, unless the first entry (the
    library's automatic choice, by convention) is within `margin` of it - then nothing is pinned
    and the empty setting is returned, so that a table never freezes noise."""
    best_t, best = min(results, key=lambda r: r[0])
    auto_t, auto = results[0]
    if auto_t <= best_t * (1.0 + margin):
        return auto_t, auto
    return best_t, best


def table_entries(per_shape, row_bytes_list, pooling_list):
    """Turn {(row_bytes, pooling): setting} into the entries of a tuning table, ordered so that
    the FIRST entry that covers a call is the one for the nearest shape at or above it.  A shape
    stands for the band up to the geometric mean with the next pooling factor."""
    entries = []
    for rb in sorted(row_bytes_list):
        pl = sorted(pooling_list)
        for i, L in enumerate(pl):
            setting = per_shape.get((rb, L), {})
            upper = (L * pl[i + 1]) ** 0.5 if i + 1 < len(pl) else 3.0e38
            e = {"max_row_bytes": int(rb), "max_avg_len": float(upper)}
            e.update({k: int(v) for k, v in setting.items() if k in TABLE_KEYS})
            entries.append(e)
    return entries


def load_table(path_or_entries) -> int:
    """Load a table written by --table (a path, or its list of entries) into the library."""
    from . import emb_bag_set_tuning_table
    entries = path_or_entries
    if isinstance(path_or_entries, str):
        with open(path_or_entries) as f:
            entries = json.load(f)["entries"]
    emb_bag_set_tuning_table(entries)
    return len(entries)


def sweep_table(row_bytes_list, pooling_list, grid, lookups: int, steps: int, warmup: int,
                timer=None, log=print):
    """The per-shape sweep.  `timer(row_bytes, pooling, setting) -> seconds` replaces the GPU
    measurement (tests pass a stub); the first setting tried per shape is the automatic one."""
    per_shape, report = {}, []
    keys = list(grid)
    combos = [dict(zip(keys, c)) for c in itertools.product(*[grid[k] for k in keys])]
    for rb in row_bytes_list:
        for L in pooling_list:
            measure = timer or _shape_timer(rb, L, lookups, steps, warmup)
            results = [(measure(rb, L, {}), {})]
            for setting in combos:
                if setting.get("stream") == 1 and setting.get("bags_per_wave", 1) != 1:
                    continue        # bags per wavefront belong to the other kernel
                if setting.get("depth", 0) > rb // 16 and setting.get("stream") == 1:
                    continue        # the stream kernel's depth is bounded by the lanes per row
                results.append((measure(rb, L, setting), setting))
            t, setting = choose(results)
            per_shape[(rb, L)] = setting
            report.append({"row_bytes": rb, "pooling": L, "auto_us": results[0][0] * 1e6,
                           "best_us": min(r[0] for r in results) * 1e6, "chosen": setting})
            log(f"row {rb:5d} B  pooling {L:4d}: automatic {results[0][0] * 1e6:9.1f} us, best "
                f"{min(r[0] for r in results) * 1e6:9.1f} us -> {json.dumps(setting) if setting else 'automatic'}")
    return per_shape, report


def _shape_timer(row_bytes: int, pooling: int, lookups: int, steps: int, warmup: int):
    """A timer for one shape on the GPU: 26 fp32 tables of 1,000,000 rows, uniform ids, fixed
    pooling, batch chosen so that a launch holds about `lookups` lookups."""
    from inputgen import gen
    T = 26
    B = max(64, lookups // (T * pooling))
    wl = gen.Workload(name=f"shape_{row_bytes}_{pooling}", T=T, rows=(1_000_000,) * T,
                      D=row_bytes // 4, dtype="f32", B=B, pooling=("fixed", pooling),
                      dists=(("uniform",),) * T, seed=0x5EED0E00 + row_bytes + pooling)
    state = _setup_wl(wl, 2)

    def measure(_rb, _L, setting):
        apply_tuning({**NEUTRAL, **setting})
        try:
            return _time(state, steps, warmup)
        finally:
            apply_tuning(NEUTRAL)
    return measure


def _setup(name: str, n_batches: int):
    from inputgen import gen
    return _setup_wl(gen.workload(name), n_batches)


def _setup_wl(wl, n_batches: int):
    import torch
    import paper_2410_22249_amd as emb
    from inputgen import gen

    dev = "cuda:0"
    tdtype = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16,
              "u8row": torch.uint8, "fp8row": torch.uint8}[wl.dtype]
    width = wl.D + 8 if wl.dtype in gen.QUANTISED else wl.D   # quantised rows end with scale and bias
    arena = torch.empty((wl.total_rows, width), dtype=tdtype, device=dev)
    gen.fill_arena_device(arena.data_ptr(), 0, wl.total_rows, wl.D, wl.dtype, wl.seed, wl.kind,
                          torch.cuda.current_stream().cuda_stream)
    batches = gen.make_batches(wl, n_batches)
    toff = torch.from_numpy(wl.table_offsets()).to(dev)
    dev_batches = [(torch.from_numpy(b.indices).to(dev), torch.from_numpy(b.offsets).to(dev),
                    None if b.weights is None else torch.from_numpy(b.weights).to(dev))
                   for b in batches]
    edt = emb.DTYPES[wl.dtype]
    emode = emb.MODES[wl.mode]
    hints = torch.zeros(wl.T, dtype=torch.uint8, device=dev)
    d0 = emb.make_desc(wl.T, wl.B, wl.D, edt, emode, batches[0].num_lookups, 0, max(wl.rows))
    emb.emb_bag_profile_reuse(d0, dev_batches[0][0], dev_batches[0][1], 16384, -1, None, None, hints)
    descs = [emb.make_desc(wl.T, wl.B, wl.D, edt, emode, b.num_lookups, 0, max(wl.rows), hints)
             for b in batches]
    out = torch.empty((wl.B, wl.T * wl.D), dtype=torch.float32, device=dev)
    torch.cuda.synchronize()
    return wl, arena, toff, dev_batches, descs, out, batches, hints


def _time(state, steps: int, warmup: int) -> float:
    """Average kernel time in seconds over `steps` launches."""
    import torch
    import paper_2410_22249_amd as emb
    wl, arena, toff, dev_batches, descs, out, batches, _ = state
    n = len(dev_batches)
    for i in range(warmup):
        k = i % n
        emb.emb_bag_forward(descs[k], arena, toff, dev_batches[k][0], dev_batches[k][1],
                            dev_batches[k][2], out)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(steps):
        k = (warmup + i) % n
        emb.emb_bag_forward(descs[k], arena, toff, dev_batches[k][0], dev_batches[k][1],
                            dev_batches[k][2], out)
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / steps / 1e3


def main(argv: List[str] = None) -> int:
    argv = list(sys.argv[1:] if argv is None else argv)
    if argv and argv[0] == "pooling":
        from . import autotune_pooling
        return autotune_pooling.main(argv[1:])
    if argv and argv[0] == "mixed":
        from . import autotune_mixed
        return autotune_mixed.main(argv[1:])
    if argv and argv[0] == "hints":
        from . import autotune_hints
        return autotune_hints.main(argv[1:])
    ap = argparse.ArgumentParser(description=__doc__.split("\n\n")[0])
    ap.add_argument("--workload", default="cfg3")
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--batches", type=int, default=4)
    ap.add_argument("--grid", default=None, help='JSON, e.g. \'{"depth":[2,8],"blocks_per_cu":[0,2]}\'')
    ap.add_argument("--out", default=None)
    ap.add_argument("--table", default=None, metavar="PATH",
                    help="per-shape sweep: write the tuning table for emb_bag_set_tuning_table")
    ap.add_argument("--shapes", default=None,
                    help='JSON, e.g. \'{"row_bytes":[256,512],"pooling":[1,20,80]}\'')
    ap.add_argument("--lookups", type=int, default=4_000_000, help="lookups per launch (--table)")
    a = ap.parse_args(argv)

    if a.table:
        shapes = json.loads(a.shapes) if a.shapes else {}
        rbs = shapes.get("row_bytes", TABLE_ROW_BYTES)
        pls = shapes.get("pooling", TABLE_POOLING)
        grid = json.loads(a.grid) if a.grid else TABLE_GRID
        per_shape, report = sweep_table(rbs, pls, grid, a.lookups, a.steps, a.warmup)
        entries = table_entries(per_shape, rbs, pls)
        with open(a.table, "w") as f:
            json.dump({"entries": entries, "sweep": report, "grid": grid}, f, indent=1)
        pinned = sum(1 for e in entries if len(e) > 2)
        print(f"# {len(entries)} entries written to {a.table}, {pinned} of them pin a key")
        return 0

    import numpy as np
    import paper_2410_22249_amd as emb
    from paper_2410_22249_amd import metrics

    grid = json.loads(a.grid) if a.grid else DEFAULT_GRID
    keys = list(grid)
    state = _setup(a.workload, a.batches)
    wl, batches, hints = state[0], state[6], state[7]
    nl = float(np.mean([b.num_lookups for b in batches]))
    gathered = metrics.gathered_bytes(nl, wl.D, wl.elem_bytes, wl.row_bytes)
    print(f"# {a.workload}: {nl:.0f} lookups/launch, {gathered / 1e9:.3f} GB gathered, "
          f"{int(hints.sum().item())}/{wl.T} tables classified streaming")
    results = []
    try:
        for combo in itertools.product(*[grid[k] for k in keys]):
            setting = dict(zip(keys, combo))
            apply_tuning({**NEUTRAL, **setting})
            t = _time(state, a.steps, a.warmup)
            results.append((t, setting))
            print(f"{json.dumps(setting):70s} {t * 1e6:10.1f} us  {nl / t / 1e9:7.2f} G lookups/s  "
                  f"{gathered / t / 1e9:8.0f} GB/s ({100 * gathered / t / 1e9 / metrics.HBM_PEAK_GBPS:5.1f} % of peak)",
                  flush=True)
    finally:
        apply_tuning(NEUTRAL)
    best_t, best = min(results, key=lambda r: r[0])
    print(f"# best: {json.dumps(best)} at {best_t * 1e6:.1f} us")
    # Sec. 7, first step: latency- or bandwidth-bound?  If lowering occupancy at the largest depth
    # costs nothing, memory-level parallelism is not the limit.
    if "blocks_per_cu" in grid and "depth" in grid and len(grid["blocks_per_cu"]) > 1:
        full = min(t for t, s in results if s["blocks_per_cu"] == grid["blocks_per_cu"][0])
        low = min(t for t, s in results if s["blocks_per_cu"] == grid["blocks_per_cu"][-1])
        verdict = "bandwidth-bound" if low < 1.03 * full else "latency-sensitive"
        print(f"# occupancy cap {grid['blocks_per_cu'][-1]} workgroups/CU costs "
              f"{100 * (low / full - 1):.1f} % at its best depth: {verdict}")
    if a.out:
        with open(a.out, "w") as f:
            json.dump({"workload": a.workload, "tuning": best, "kernel_us": best_t * 1e6}, f, indent=1)
    return 0


if __name__ == "__main__":
    sys.exit(main())
