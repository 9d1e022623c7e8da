"""Tables of different widths in one launch (`emb_bag_forward_mixed`) against one uniform launch per
width, on one MI355X.

    python -m paper_2410_22249_amd.autotune mixed [--steps 20]
    python -m paper_2410_22249_amd.autotune mixed --split-sweep

Workload "mixed_cfg": 60 fp32 tables x 4,000,000 rows, widths cycling 32 / 64 / 128 / 256, batch
4096, pooling 80, uniform indices (the paper's model has one width, Sec. 5; production models mix
them).  The comparison runs the same 15 tables of each width through `emb_bag_forward`, four
launches, and adds their times.  Prints a markdown table.

`--split-sweep`: workload "mixed_onehot" (26 fp32 tables x 1,000,000 rows, widths cycling 16 / 32 /
64 / 128, short bags) at batch sizes from inference (512, 2048: the paper's, Sec. 5) to 131,072.
Short bags split the call by row class; the table compares the fused launch (the classes as
workgroup ranges of one kernel), the separate launches ("fuse" 0) and the one-wavefront-per-bag
kernel alone ("stream" 0).
"""
from __future__ import annotations

import argparse
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def _events(fn, steps, warmup):
    import torch
    for i in range(warmup):
        fn(i)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(steps):
        fn(warmup + i)
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / steps / 1e3


def split_sweep(steps: int, warmup: int) -> int:
    from dataclasses import replace

    import numpy as np
    import torch
    import paper_2410_22249_amd as emb
    from inputgen import gen

    dev = "cuda:0"
    print("| pooling | batch | parts | fused us | separate launches us | wave kernel alone us | "
          "algorithmic GB/s (fused) |")
    print("|---|---|---|---|---|---|---|")
    for pool, label in ((("fixed", 1), "1"), (("uniform", 0, 4), "U[0,4]")):
        for B in (512, 2048, 8192, 32768, 131072):
            wl = replace(gen.mixed_workload("mixed_onehot"), B=B, pooling=pool)
            arena = torch.empty(wl.table_bytes, dtype=torch.uint8, device=dev)
            gen.mixed_fill_device(wl, arena.data_ptr(), torch.cuda.current_stream().cuda_stream)
            batches = gen.make_batches(wl, 2)
            boff = torch.from_numpy(wl.table_byte_offsets()).to(dev)
            ooff = torch.from_numpy(wl.out_offsets()).to(dev)
            dbat = [(torch.from_numpy(b.indices).to(dev), torch.from_numpy(b.offsets).to(dev))
                    for b in batches]
            hints = torch.ones(wl.T, dtype=torch.uint8, device=dev)
            max_bytes = int(np.diff(wl.table_byte_offsets()).max())
            descs = [emb.make_mixed_desc(wl.dims, wl.B, emb.EMB_F32, emb.EMB_SUM, b.num_lookups, 0,
                                         max_bytes, hints) for b in batches]
            out = torch.empty((wl.B, int(sum(wl.dims))), dtype=torch.float32, device=dev)
            torch.cuda.synchronize()

            def call(i):
                k = i % len(dbat)
                emb.emb_bag_forward_mixed(descs[k], arena, boff, ooff, dbat[k][0], dbat[k][1], None, out)

            times = {}
            try:
                plan = emb.emb_bag_plan_forward_mixed(descs[0])
                times["fused"] = _events(call, steps, warmup)
                emb.emb_bag_set_tuning("fuse", 0)
                times["separate"] = _events(call, steps, warmup)
                emb.emb_bag_set_tuning("fuse", 1)
                emb.emb_bag_set_tuning("stream", 0)
                times["wave"] = _events(call, steps, warmup)
            finally:
                emb.emb_bag_set_tuning("fuse", 1)
                emb.emb_bag_set_tuning("stream", -1)
            nl = float(np.mean([b.num_lookups for b in batches]))
            algo = (float(np.mean([wl.gathered_bytes(b) for b in batches])) + 8 * nl
                    + 8 * (wl.T * B + 1) + 4 * B * sum(wl.dims))
            print(f"| {label} | {B} | {plan.num_launches}{'' if plan.fused else ' (not fused)'} | "
                  f"{times['fused'] * 1e6:.1f} | {times['separate'] * 1e6:.1f} | "
                  f"{times['wave'] * 1e6:.1f} | {algo / times['fused'] / 1e9:.0f} |", flush=True)
            del arena, out
            torch.cuda.empty_cache()
    return 0


def main(argv=None) -> int:
    ap = argparse.ArgumentParser(description=__doc__.split("\n\n")[0])
    ap.add_argument("--split-sweep", action="store_true",
                    help="fused launch against separate launches over batch sizes (mixed_onehot)")
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--batches", type=int, default=4)
    ap.add_argument("--tune", action="append", default=[], metavar="KEY=VALUE",
                    help="emb_bag_set_tuning override, e.g. --tune xcd_remap=0")
    a = ap.parse_args(argv)
    if a.split_sweep:
        return split_sweep(max(a.steps, 50), max(a.warmup, 5))

    import numpy as np
    import torch
    import paper_2410_22249_amd as emb
    from inputgen import gen

    dev = "cuda:0"
    for kv in a.tune:
        k, v = kv.split("=")
        emb.emb_bag_set_tuning(k, int(v))
    wl = gen.mixed_workload("mixed_cfg")
    arena = torch.empty(wl.table_bytes, dtype=torch.uint8, device=dev)
    gen.mixed_fill_device(wl, arena.data_ptr(), torch.cuda.current_stream().cuda_stream)
    batches = gen.make_batches(wl, a.batches)
    boff = torch.from_numpy(wl.table_byte_offsets()).to(dev)
    ooff = torch.from_numpy(wl.out_offsets()).to(dev)
    dbat = [(torch.from_numpy(b.indices).to(dev), torch.from_numpy(b.offsets).to(dev)) for b in batches]
    hints = torch.ones(wl.T, dtype=torch.uint8, device=dev)      # uniform indices: every table streams
    max_bytes = int(np.diff(wl.table_byte_offsets()).max())
    descs = [emb.make_mixed_desc(wl.dims, wl.B, emb.EMB_F32, emb.EMB_SUM, b.num_lookups, 0, max_bytes,
                                 hints) for b in batches]
    out = torch.empty((wl.B, int(sum(wl.dims))), dtype=torch.float32, device=dev)
    torch.cuda.synchronize()

    def mixed(i):
        k = i % len(dbat)
        emb.emb_bag_forward_mixed(descs[k], arena, boff, ooff, dbat[k][0], dbat[k][1], None, out)

    t_mixed = _events(mixed, a.steps, a.warmup)
    nl = float(np.mean([b.num_lookups for b in batches]))
    gathered = float(np.mean([wl.gathered_bytes(b) for b in batches]))
    written = wl.B * sum(wl.dims) * 4
    rows = [("mixed, one launch", t_mixed, nl, gathered, written)]
    del arena, out
    torch.cuda.empty_cache()

    # the same tables grouped by width: one uniform launch per width
    t_sum = 0.0
    for D in sorted(set(wl.dims)):
        nT = sum(1 for d in wl.dims if d == D)
        uw = gen.Workload(name=f"w{D}", T=nT, rows=(wl.rows[0],) * nT, D=D, dtype="f32", B=wl.B,
                          pooling=wl.pooling, dists=(("uniform",),) * nT, seed=wl.seed + D)
        ar = torch.empty((uw.total_rows, D), dtype=torch.float32, device=dev)
        gen.fill_arena_device(ar.data_ptr(), 0, uw.total_rows, D, "f32", uw.seed, uw.kind,
                              torch.cuda.current_stream().cuda_stream)
        ub = gen.make_batches(uw, a.batches)
        toff = torch.from_numpy(uw.table_offsets()).to(dev)
        db = [(torch.from_numpy(b.indices).to(dev), torch.from_numpy(b.offsets).to(dev)) for b in ub]
        h = torch.ones(nT, dtype=torch.uint8, device=dev)
        ds = [emb.make_desc(nT, uw.B, D, emb.EMB_F32, emb.EMB_SUM, b.num_lookups, 0, uw.rows[0], h)
              for b in ub]
        o = torch.empty((uw.B, nT * D), dtype=torch.float32, device=dev)
        torch.cuda.synchronize()

        def uni(i):
            k = i % len(db)
            emb.emb_bag_forward(ds[k], ar, toff, db[k][0], db[k][1], None, o)

        t = _events(uni, a.steps, a.warmup)
        n = float(np.mean([b.num_lookups for b in ub]))
        rows.append((f"uniform, {nT} tables of width {D}", t, n, n * D * 4, uw.B * nT * D * 4))
        t_sum += t
        del ar, o
        torch.cuda.empty_cache()
    rows.append(("uniform, four launches added", t_sum, nl, gathered, written))

    print("| launch | kernel ms | G lookups/s | gathered GB/s | gathered+indices+output GB/s |")
    print("|---|---|---|---|---|")
    for name, t, n, g, w in rows:
        algo = g + 8 * n + w
        print(f"| {name} | {t * 1e3:.3f} | {n / t / 1e9:.2f} | {g / t / 1e9:.0f} | {algo / t / 1e9:.0f} |")
    return 0


if __name__ == "__main__":
    sys.exit(main())
