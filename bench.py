#!/usr/bin/env python3
"""Benchmark of the embedding stage (multi-table EmbeddingBag forward) on one MI355X.

One "step" is one pass of the whole hot path - one `emb_bag_forward` call over one batch of
synthetic input (all tables, all bags) - with every input already resident in HBM.  Timed steps
rotate through several pre-generated index batches so that no step re-reads the rows the previous
step left in the caches.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg3] [--no-cpu-baseline]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

DESCRIPTIONS = {
    "cfg1": "8 fp32 tables x 100,000 rows x dim 64, batch 256, pooling 20 fixed, uniform indices, sum",
    "cfg2": "26 fp32 tables x 1,000,000 rows x dim 64, batch 2048, pooling U[1,40], uniform indices, sum",
    "cfg3": "60 fp32 tables x 4,000,000 rows x dim 128 (122.9 GB), batch 4096, pooling 80 fixed, "
            "uniform indices, sum",
    "cfg4": "60 fp32 tables x 4,000,000 rows x dim 128, batch 4096, pooling U[40,120], "
            "Zipf(1.05) + row permutation, mean",
    "cfg5": "100 fp16 tables x 2,000,000 rows x dim 256 (fp32 accumulate), batch 8192, pooling "
            "U[1,100], tables 0-49 uniform / 50-99 Zipf(1.2), sum",
    "paper": "250 fp32 tables x 500,000 rows x dim 128, batch 2048, pooling 150 fixed, uniform "
             "indices, sum (the paper's model, random dataset)",
    "paper_one_item": "250 fp32 tables x 500,000 x dim 128, batch 2048, pooling 150, one item, sum",
    "cfg3_weighted": "cfg3 with fp32 per-sample weights",
    "cfg3_max": "cfg3 with max pooling",
    "hetero": "26 fp32 tables x 1,000,000 rows x dim 64, batch 32768; 20 tables with ONE lookup per "
              "bag, 6 with 100 (average 23.8): per-table bag lengths split the call into a "
              "stream-kernel launch and a wave-kernel launch",
    "cfg3_fp8": "cfg3's shape with row-wise quantised rows of E4M3 codes: 60 tables x 4,000,000 "
                "rows x dim 120 (128-byte rows), batch 4096, pooling 80, uniform, sum",
    "cfg3_u8": "cfg3's shape with row-wise quantised rows: 60 tables x 4,000,000 rows x dim 120 "
               "(uint8 codes + fp32 scale, bias = 128-byte rows), batch 4096, pooling 80, uniform, sum",
    "onehot": "short bags: 26 fp32 tables x 1,000,000 rows x dim 64, batch 131072, ONE lookup per "
              "bag, uniform indices, sum (stream kernel)",
    "short": "short bags: 26 fp32 tables x 1,000,000 rows x dim 64, batch 32768, pooling U[0,8], "
             "uniform indices, sum (stream kernel)",
    "paper_high": "paper's model, Zipf(1.3396) stand-in for its high-hot trace (4.05 % unique)",
    "paper_med": "paper's model, Zipf(1.0234) stand-in for its med-hot trace (20.5 % unique)",
    "paper_low": "paper's model, Zipf(0.6999) stand-in for its low-hot trace (46.21 % unique)",
    "paper_mix1": "paper's model, Mix1: 100 high / 75 med / 50 low / 25 random tables",
    "paper_mix2": "paper's model, Mix2: 62 / 63 / 63 / 62",
    "paper_mix3": "paper's model, Mix3: 25 / 50 / 75 / 100",
    "cfg4_hot": "cfg4 with every table laid out hot rows first (the 8,192 most popular rows of a "
                "table occupy its first 4 MB, the state after offline profiling and relayout) and "
                "desc.hot_rows naming that head",
    "cfg5_hot": "cfg5 with its 50 Zipf tables laid out hot rows first (8,192 rows) and desc.hot_rows",
    "paper_high_hot": "paper_high with every table laid out hot rows first (8,192 rows) and desc.hot_rows",
    "paper_med_hot": "paper_med with every table laid out hot rows first (8,192 rows) and desc.hot_rows",
    "mixed_onehot": "26 fp32 tables x 1,000,000 rows, widths cycling 16 / 32 / 64 / 128, batch 131072, "
                    "ONE lookup per bag, uniform indices, sum: emb_bag_forward_mixed splits the call "
                    "into one stream-kernel launch per lanes-per-row class",
    "mixed_cfg": "60 fp32 tables x 4,000,000 rows, widths cycling 32 / 64 / 128 / 256 (115.2 GB), "
                 "batch 4096, pooling 80 fixed, uniform indices, sum, one emb_bag_forward_mixed launch",
}


def log(msg: str) -> None:
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def read_traffic(workload: str):
    """HBM bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE, WRITE_SIZE), if a summary
    for this workload has been committed under profiles/."""
    path = os.path.join(ROOT, "profiles", f"emb_bag_forward_{workload}.txt")
    if not os.path.exists(path):
        return None
    vals = {}
    for line in open(path):
        if "=" in line and not line.lstrip().startswith("#"):
            k, v = line.split("=", 1)
            try:
                vals[k.strip()] = float(v.split()[0])
            except (ValueError, IndexError):
                pass
    if "hbm_bytes_per_launch" in vals:
        return vals["hbm_bytes_per_launch"]
    return None


def build_parser() -> argparse.ArgumentParser:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=40)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default=None, choices=sorted(DESCRIPTIONS),
                    help="default: cfg3 (the configuration the target is quoted on), followed by "
                         "short runs of cfg1, cfg2, cfg4 and cfg5 reported under 'others'")
    ap.add_argument("--no-others", action="store_true",
                    help="time the headline workload only")
    ap.add_argument("--batches", type=int, default=4, help="distinct index batches to rotate")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=10.0)
    ap.add_argument("--check-bags", type=int, default=256, help="bags spot-checked vs the oracle")
    ap.add_argument("--graph", action="store_true",
                    help="also replay the K timed steps from one captured HIP graph and report "
                         "its wall time per step (launch overhead removed)")
    ap.add_argument("--arena", default="torch", choices=["torch", "contiguous"],
                    help="table memory: torch's caching allocator (default) or physically "
                         "contiguous hipExtMallocWithFlags")
    ap.add_argument("--arena-pick", default="auto", choices=["auto", "on", "off"],
                    help="allocate the table arena twice, time a few steps on each and keep the "
                         "faster one: which physical region the driver hands out moves random "
                         "gathers by 5-15 %% (auto: when the arena is 16 GB or more and fits twice)")
    ap.add_argument("--arena-decoy", action="store_true",
                    help="allocate (and afterwards free) a block of the arena's size first, so that "
                         "the arena lands in the next physical region the driver hands out")
    ap.add_argument("--no-hints", action="store_true",
                    help="do not profile table reuse / pass per-table cache hints")
    ap.add_argument("--no-table-lengths", action="store_true",
                    help="do not pass per-table bag lengths (table_avg_len) for workloads whose "
                         "tables differ in pooling")
    ap.add_argument("--no-hot-rows", action="store_true",
                    help="do not pass desc.hot_rows for workloads laid out hot rows first (the "
                         "reuse hints are passed instead)")
    ap.add_argument("--tune", action="append", default=[], metavar="KEY=VALUE",
                    help="emb_bag_set_tuning override, e.g. --tune depth=8")
    return ap


def unique_row_bytes(wl, batch, mixed: bool) -> int:
    """Bytes of the distinct rows one batch names: what has to come from HBM at least once."""
    import numpy as np
    total = 0
    for t in range(wl.T):
        s, e = int(batch.offsets[t * wl.B]), int(batch.offsets[(t + 1) * wl.B])
        rb = wl.row_bytes_of(t) if mixed else wl.row_bytes
        total += len(np.unique(batch.indices[s:e])) * rb
    return total


def host_path_latency(wl):
    """Host time of one emb_bag_forward call measured from plain C (tests/c_abi/c_abi_latency):
    at this size the caller sees the call's host cost, not the kernel."""
    import subprocess
    exe = os.path.join(ROOT, "tests", "c_abi", "c_abi_latency")
    if not os.path.exists(exe) or wl.pooling[0] != "fixed":
        return None
    try:
        r = subprocess.run([exe, str(wl.T), str(wl.rows[0]), str(wl.D), str(wl.B),
                            str(int(wl.pooling[1]))], capture_output=True, text=True, timeout=120)
        return json.loads(r.stdout.strip().splitlines()[-1]) if r.returncode == 0 else None
    except (OSError, ValueError, IndexError, subprocess.TimeoutExpired):
        return None


def run_workload(args, name: str, steps: int, warmup: int, headline: bool):
    """Set one workload up in HBM, time `steps` forward calls, spot-check the result against the
    oracle and (headline only) time the oracle on the host.  Returns the result dictionary, or an
    int exit status on failure."""
    import numpy as np
    import torch

    import paper_2410_22249_amd as emb
    from inputgen import gen
    from paper_2410_22249_amd import metrics

    dev = "cuda:0"
    mixed = name.startswith("mixed")
    wl = gen.mixed_workload(name) if mixed else gen.workload(name)
    stream = torch.cuda.Stream()           # default priority; the library launches on it
    sh = stream.cuda_stream

    # ---- inputs, resident in HBM before anything is timed -------------------------------
    t0 = time.time()
    batches = gen.make_batches(wl, args.batches)
    log(f"{wl.name}: {len(batches)} index batches generated in {time.time() - t0:.1f} s "
        f"({batches[0].num_lookups} lookups in batch 0)")
    toff = torch.from_numpy(wl.table_byte_offsets() if mixed else wl.table_offsets()).to(dev)
    ooff = torch.from_numpy(wl.out_offsets()).to(dev) if mixed else None
    total_dim = int(sum(wl.dims)) if mixed else wl.T * wl.D
    dbatches = []
    for b in batches:
        dbatches.append((torch.from_numpy(b.indices).to(dev), torch.from_numpy(b.offsets).to(dev),
                         None if b.weights is None else torch.from_numpy(b.weights).to(dev)))
    out = torch.empty((wl.B, total_dim), dtype=torch.float32, device=dev)
    edt = emb.DTYPES[wl.dtype]
    emode = emb.MODES[wl.mode]
    # Set-up, untimed (the paper profiles table access patterns offline, Sec. 4.3): classify each
    # table as streaming or re-used from the first index batch, on the device.
    hints = None
    if not args.no_hints:
        hints = torch.zeros(wl.T, dtype=torch.uint8, device=dev)
        # the profile reads ids and the row size (tables of different widths: the narrowest,
        # which streams the fewest tables)
        d0 = emb.make_desc(wl.T, wl.B, min(wl.row_bytes_of(t) for t in range(wl.T)) // 4 if mixed
                           else wl.D, emb.EMB_F32 if mixed else edt, emode,
                           batches[0].num_lookups, 0, max(wl.rows))
        emb.emb_bag_profile_reuse(d0, dbatches[0][0], dbatches[0][1], 16384, -1, None, None, hints,
                                  stream)
        stream.synchronize()
        log(f"table hints: {int(hints.sum().item())} of {wl.T} tables streaming")
    # per-table bag lengths (a property of the features, taken from the first batch) where the
    # tables differ in pooling; --no-table-lengths shows the single-kernel choice
    avg_len = None
    if wl.pooling[0] == "per_table" and not args.no_table_lengths:
        avg_len = gen.table_avg_len(wl, batches[0])
    # tables laid out hot rows first: the size of each table's head
    hot_rows = None
    if not mixed and wl.hot_head > 0 and not args.no_hot_rows:
        hot_rows = torch.from_numpy(gen.hot_rows(wl)).to(dev)
    if mixed:
        max_bytes = int(np.diff(wl.table_byte_offsets()).max())
        descs = [emb.make_mixed_desc(wl.dims, wl.B, edt, emode, b.num_lookups, 0, max_bytes, hints,
                                     avg_len) for b in batches]
    else:
        descs = [emb.make_desc(wl.T, wl.B, wl.D, edt, emode, b.num_lookups, 0, max(wl.rows), hints,
                               avg_len, hot_rows) for b in batches]

    tdtype = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16,
              "u8row": torch.uint8, "fp8row": torch.uint8}[wl.dtype]
    width = 0 if mixed else (wl.D + 8 if wl.dtype in gen.QUANTISED else wl.D)  # elements per stored row

    def new_arena():
        if mixed:
            a = torch.empty(wl.table_bytes, dtype=torch.uint8, device=dev)
        else:
            a = torch.empty((wl.total_rows, width), dtype=tdtype, device=dev)
        with torch.cuda.stream(stream):
            if mixed:
                gen.mixed_fill_device(wl, a.data_ptr(), sh)
            else:
                gen.fill_arena_device(a.data_ptr(), 0, wl.total_rows, wl.D, wl.dtype, wl.seed,
                                      wl.kind, sh)
        return a

    def step_on(a, i: int) -> None:
        k = i % len(dbatches)
        idx, off, w = dbatches[k]
        if mixed:
            emb.emb_bag_forward_mixed(descs[k], a, toff, ooff, idx, off, w, out, stream)
        else:
            emb.emb_bag_forward(descs[k], a, toff, idx, off, w, out, stream)

    def probe(a, n: int = 6) -> float:
        for i in range(2):
            step_on(a, i)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for i in range(n):
            step_on(a, 2 + i)
        e1.record(stream)
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / n

    # The arena is the caller's memory.  Which physical region the driver hands out moves the
    # random gathers of the large configurations by 5-15 % (the same arena is always the same
    # speed; a plain streaming read does not show the difference): a caller that cares allocates
    # twice at start-up and keeps the faster block, which is what --arena-pick does.
    owner = None
    arena_pick = None
    free_bytes = torch.cuda.mem_get_info()[0]
    pick = args.arena_pick == "on" or (args.arena_pick == "auto" and wl.table_bytes >= 16e9
                                       and args.arena == "torch" and not args.arena_decoy)
    if pick and 2 * wl.table_bytes + (4 << 30) > free_bytes:
        pick = False
    if pick:
        first = new_arena()
        second = new_arena()
        t_first, t_second = probe(first), probe(second)
        arena_pick = {"first_ms": t_first, "second_ms": t_second,
                      "kept": "first" if t_first <= t_second else "second"}
        arena = first if t_first <= t_second else second
        del first, second
        torch.cuda.empty_cache()
        arena_kind = "torch, the faster of two allocations"
        log(f"arena pick: {arena_pick}")
    elif args.arena == "contiguous" and not mixed:
        owner = gen.DeviceArena(wl.total_rows, wl.D, wl.dtype, contiguous=True)
        arena, arena_kind = owner.tensor, owner.kind
        with torch.cuda.stream(stream):
            gen.fill_arena_device(arena.data_ptr(), 0, wl.total_rows, wl.D, wl.dtype, wl.seed,
                                  wl.kind, sh)
    else:
        decoy = torch.empty(wl.table_bytes, dtype=torch.uint8, device=dev) if args.arena_decoy else None
        arena, arena_kind = new_arena(), "torch"
        if decoy is not None:
            arena_kind += ", allocated after a decoy of the same size"
            del decoy
            torch.cuda.empty_cache()
    log(f"{wl.name}: arena {wl.table_bytes / 1e9:.2f} GB ({arena_kind}) at {hex(arena.data_ptr())}")
    torch.cuda.synchronize()

    def step(i: int) -> None:
        step_on(arena, i)

    stream_read_gbps = None
    if headline:
        # a plain copy of known size on the same stream: the calibration kernel for HBM counters
        cal_bytes = 1 << 30
        cal_src = torch.empty(cal_bytes, dtype=torch.uint8, device=dev)
        cal_dst = torch.empty(cal_bytes, dtype=torch.uint8, device=dev)
        cal_src.zero_()
        torch.cuda.synchronize()
        gen.copy_bytes_device(cal_dst.data_ptr(), cal_src.data_ptr(), cal_bytes, sh)
        torch.cuda.synchronize()
        del cal_src, cal_dst

        # secondary denominator: what a plain streaming read of the same memory reaches on this machine
        probe_bytes = min(wl.table_bytes, 16 << 30) & ~15
        gen.read_bytes_device(arena.data_ptr(), probe_bytes, sh)
        torch.cuda.synchronize()
        pe0, pe1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        pe0.record(stream)
        for _ in range(3):
            gen.read_bytes_device(arena.data_ptr(), probe_bytes, sh)
        pe1.record(stream)
        torch.cuda.synchronize()
        stream_read_gbps = probe_bytes * 3 / (pe0.elapsed_time(pe1) / 1e3) / 1e9
        log(f"plain streaming read of {probe_bytes / 2**30:.1f} GiB: {stream_read_gbps:.0f} GB/s")

    # ---- warm-up, then the timed region --------------------------------------------------
    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
          for _ in range(steps)]
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    for i in range(steps):
        ev[i][0].record(stream)
        step(warmup + i)
        ev[i][1].record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t_start
    kern_ms = [a.elapsed_time(b) for a, b in ev]
    lookups_timed = sum(batches[(warmup + i) % len(batches)].num_lookups for i in range(steps))
    avg_lookups = lookups_timed / steps
    avg_kern_s = float(np.mean(kern_ms)) / 1e3
    lookups_per_s = lookups_timed / wall
    if mixed:   # rows of each table's own width + indices + offsets + output (+ weights)
        gathered = sum(wl.gathered_bytes(batches[(warmup + i) % len(batches)])
                       for i in range(steps)) / steps
        algo = (gathered + 8 * avg_lookups + 8 * (wl.num_bags + 1) + 4 * wl.B * total_dim
                + (4 * avg_lookups if wl.weighted else 0))
    else:
        gathered = metrics.gathered_bytes(avg_lookups, wl.D, wl.elem_bytes, wl.row_bytes)
        algo = metrics.algorithmic_bytes(avg_lookups, wl.T, wl.B, wl.D, wl.elem_bytes, wl.weighted,
                                         wl.row_bytes)
    achieved = algo / avg_kern_s / 1e9
    # what has to come from HBM at least once per launch: every distinct row once, plus the
    # index, offset, weight and output traffic (batch 0 stands for the others)
    unique_rows = unique_row_bytes(wl, batches[0], mixed)
    compulsory = algo - gathered + unique_rows * (avg_lookups / batches[0].num_lookups)
    log(f"wall {wall * 1e3 / steps:.3f} ms/step, kernel avg {avg_kern_s * 1e3:.3f} ms "
        f"(min {min(kern_ms):.3f}, max {max(kern_ms):.3f}); gathered "
        f"{gathered / avg_kern_s / 1e9:.1f} GB/s, algorithmic {achieved:.1f} GB/s, "
        f"compulsory (distinct rows) {compulsory / avg_kern_s / 1e9:.1f} GB/s")

    # ---- tables that fit in the 256 MB Infinity Cache: also time with the caches scrubbed ----
    cold_ms = None
    if wl.table_bytes <= 256 << 20:
        scrub = torch.empty(512 << 20, dtype=torch.uint8, device=dev)
        scrub.zero_()
        cold = []
        for i in range(min(steps, 20)):
            gen.scrub_cache_device(scrub.data_ptr(), scrub.numel(), sh)   # read-modify-write 512 MB
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record(stream)
            step(warmup + i)
            b.record(stream)
            torch.cuda.synchronize()
            cold.append(a.elapsed_time(b))
        cold_ms = {"avg": float(np.mean(cold)), "min": float(min(cold)), "max": float(max(cold))}
        log(f"after a 512 MB cache scrub before every step: kernel avg {cold_ms['avg'] * 1e3:.1f} us "
            f"(warm: {avg_kern_s * 1e6:.1f} us)")
        del scrub

    # ---- optional: the same K steps replayed from one HIP graph (serving loops) ------------
    graph_ms_per_step = None
    if args.graph:
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=stream):
            for i in range(steps):
                step(warmup + i)
        g.replay()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        reps = 5
        for _ in range(reps):
            g.replay()
        torch.cuda.synchronize()
        graph_ms_per_step = (time.perf_counter() - t1) * 1e3 / (reps * steps)
        log(f"HIP graph replay: {graph_ms_per_step * 1e3:.2f} us per step "
            f"(eager wall {wall * 1e6 / steps:.2f} us per step)")

    # ---- parity spot check of the launch configuration that was just timed --------------
    parity = None
    cpu_baseline = None
    want_cpu = headline and not args.no_cpu_baseline
    if args.check_bags > 0 or want_cpu:
        from oracle import emb_bag_oracle
    if args.check_bags > 0:
        k = (warmup + steps - 1) % len(batches)
        step(k)                      # the output of this batch, whatever ran after the timed region
        torch.cuda.synchronize()
        rng = np.random.default_rng(12345)
        nb = wl.num_bags
        bags = np.unique(np.concatenate([rng.integers(0, nb, size=args.check_bags),
                                         [0, wl.B - 1, nb - wl.B, nb - 1]]))
        if mixed:   # table by table: the sampled bags of one table share its width
            base, cols = wl.row_bases(), wl.out_offsets()
            refs, bounds, gots = [], [], []
            for t in np.unique(bags // wl.B):
                bs = bags[bags // wl.B == t]
                segs = [batches[k].indices[batches[k].offsets[g]:batches[k].offsets[g + 1]]
                        for g in bs]
                uniq, inv = np.unique(np.concatenate(segs), return_inverse=True)
                small = gen.table_values(wl.seed, base[t] + uniq, wl.dims[t], wl.dtype, wl.kind)
                off = gen.lengths_to_offsets(np.array([len(x) for x in segs], dtype=np.int64))
                r, bd = emb_bag_oracle.emb_bag(small, np.array([0, len(small)], np.int64),
                                               inv.astype(np.int64), off, len(bs), wl.mode,
                                               codes=wl.codes)
                g = out[torch.from_numpy(bs % wl.B).to(dev), int(cols[t]):int(cols[t + 1])]
                refs.append(r.ravel()), bounds.append(bd.ravel())
                gots.append(g.cpu().numpy().astype(np.float64).ravel())
            ref, bound, got = np.concatenate(refs), np.concatenate(bounds), np.concatenate(gots)
        else:
            small, ix, off, wsmall = gen.compact_rows(wl, batches[k], bags)
            ref, bound = emb_bag_oracle.emb_bag(small, np.array([0, len(small)], np.int64), ix, off,
                                                len(bags), wl.mode, weights=wsmall, codes=wl.codes)
            got_all = out.view(wl.B, wl.T, wl.D)
            tb = torch.from_numpy(np.stack([bags % wl.B, bags // wl.B], 1)).to(dev)
            got = got_all[tb[:, 0], tb[:, 1]].cpu().numpy().astype(np.float64)
        err = np.abs(got - ref)
        ok = err <= 1e-5 * bound
        if wl.dtype != "f32":
            ok |= err <= 1e-3 * np.abs(ref)
        nz = bound > 0
        parity = {"bags_checked": int(len(bags)), "ok": bool(ok.all()),
                  "max_err_over_bound": float(np.max(err[nz] / bound[nz])) if nz.any() else 0.0}
        log(f"parity spot check: {parity}")
        if not parity["ok"]:
            print(f"bench.py: parity spot check FAILED on {wl.name}", file=sys.stderr)
            return 1

    # ---- the oracle timed on this machine's host cores (a reported baseline, not the target) ---
    if want_cpu and mixed:
        if wl.dtype in ("f16", "bf16"):
            raise SystemExit("bench.py: the mixed-width cpu baseline covers f32 and u8row tables")
        boff = wl.table_byte_offsets()
        tsub = max(1, int(np.searchsorted(boff, 8e9, side="right")) - 1)   # <= 8 GB on the host
        tabs = []
        for t in range(tsub):
            raw = arena[int(boff[t]):int(boff[t + 1])].cpu().numpy()
            tabs.append(raw.view(np.float32 if wl.dtype == "f32" else
                                 np.uint8 if wl.dtype in gen.QUANTISED else np.uint16)
                        .reshape(wl.rows[t], -1))
        b0 = batches[0]
        e = int(b0.offsets[tsub * wl.B])
        sub_off, sub_idx = b0.offsets[: tsub * wl.B + 1].copy(), b0.indices[:e]
        emb_bag_oracle.emb_bag_mixed(tabs, sub_idx, sub_off, wl.B, wl.mode, codes=wl.codes)   # warm
        reps, t_cpu = 0, 0.0
        while t_cpu < args.cpu_seconds and reps < 100000:
            t1 = time.perf_counter()
            emb_bag_oracle.emb_bag_mixed(tabs, sub_idx, sub_off, wl.B, wl.mode, codes=wl.codes)
            t_cpu += time.perf_counter() - t1
            reps += 1
        cpu_baseline = {"value": e * reps / t_cpu, "unit": "lookups/s",
                        "cores": emb_bag_oracle.num_threads(), "kind": "oracle",
                        "sample": f"first {tsub} of {wl.T} tables (widths {list(wl.dims[:tsub])}), "
                                  f"all {wl.B} bags each ({e} lookups), {reps} passes in "
                                  f"{t_cpu:.1f} s, tables copied to host RAM"}
        log(f"cpu baseline: {cpu_baseline}")
        del tabs
    elif want_cpu:
        per_table = wl.rows[0] * wl.row_bytes
        tsub = max(1, min(wl.T, int(8e9 // per_table)))      # <= 8 GB of tables on the host
        toff_np = wl.table_offsets()
        host = arena[: int(toff_np[tsub])].cpu().numpy()
        b0 = batches[0]
        e = int(b0.offsets[tsub * wl.B])
        sub_off = b0.offsets[: tsub * wl.B + 1].copy()
        sub_idx = b0.indices[:e]
        n_sub = int(sub_off[-1])
        emb_bag_oracle.emb_bag(host, toff_np[: tsub + 1], sub_idx, sub_off, wl.B, wl.mode,
                                   codes=wl.codes)  # warm
        reps, t_cpu = 0, 0.0
        while t_cpu < args.cpu_seconds and reps < 100000:
            t1 = time.perf_counter()
            emb_bag_oracle.emb_bag(host, toff_np[: tsub + 1], sub_idx, sub_off, wl.B, wl.mode,
                                   codes=wl.codes)
            t_cpu += time.perf_counter() - t1
            reps += 1
        cpu_baseline = {"value": n_sub * reps / t_cpu, "unit": "lookups/s",
                        "cores": emb_bag_oracle.num_threads(), "kind": "oracle",
                        "sample": f"first {tsub} of {wl.T} tables, all {wl.B} bags each "
                                  f"({n_sub} lookups), {reps} passes in {t_cpu:.1f} s, "
                                  f"tables copied to host RAM",
                        "gathered_GBps": n_sub * wl.row_bytes * reps / t_cpu / 1e9}
        # the same oracle on one thread, on the first table only, for about 3 s
        threads = emb_bag_oracle.num_threads()
        emb_bag_oracle.set_num_threads(1)
        e1 = int(b0.offsets[wl.B])
        reps1, t1cpu = 0, 0.0
        while t1cpu < 3.0 and reps1 < 100000:
            t1 = time.perf_counter()
            emb_bag_oracle.emb_bag(host, toff_np[:2], b0.indices[:e1], b0.offsets[: wl.B + 1].copy(),
                                   wl.B, wl.mode, codes=wl.codes)
            t1cpu += time.perf_counter() - t1
            reps1 += 1
        emb_bag_oracle.set_num_threads(threads)
        cpu_baseline["single_thread_value"] = e1 * reps1 / t1cpu
        log(f"cpu baseline: {cpu_baseline}")
        del host

    if mixed:   # a mixed-width call may make several launches
        n_launch = emb.emb_bag_plan_forward_mixed(descs[0], wl.weighted).num_launches
        launch_plan = [emb.emb_bag_plan_forward_mixed(descs[0], wl.weighted, which=w).as_dict()
                       for w in range(n_launch)]
    else:
        n_launch = emb.emb_bag_plan_forward(descs[0], wl.weighted).num_launches
        launch_plan = [emb.emb_bag_plan_forward(descs[0], wl.weighted, which=w).as_dict()
                       for w in range(min(n_launch, 9))]
        if n_launch == 1:
            launch_plan = launch_plan[0]
        elif n_launch > 8:   # one launch per table: the first one stands for all
            launch_plan = {"num_launches": n_launch, "first": launch_plan[0]}
    traffic = read_traffic(wl.name)
    host_latency = host_path_latency(wl) if (not mixed and wl.table_bytes <= 256 << 20) else None
    result = {
        "metric": "embedding lookups/sec and effective gathered HBM GB/s (% of peak), 1 MI355X",
        "value": lookups_per_s,
        "unit": "lookups/s",
        "n_gpus": 1,
        "steps": steps,
        "warmup": warmup,
        "ms_per_step": wall * 1e3 / steps,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": f"{wl.name}: {DESCRIPTIONS[wl.name]}",
                   "tables": wl.T, "rows_per_table": wl.rows[0],
                   "dim": list(wl.dims) if mixed else wl.D,
                   "table_dtype": wl.dtype, "batch": wl.B, "mode": wl.mode,
                   "lookups_per_step": avg_lookups, "index_batches_rotated": len(batches),
                   "arena_allocation": arena_kind, "arena_address": hex(arena.data_ptr()),
                   "arena_pick": arena_pick,
                   "streaming_tables": None if hints is None else int(hints.sum().item()),
                   "hot_rows": None if hot_rows is None else int(hot_rows.max().item()),
                   "launch_plan": launch_plan,
                   "tuning": {k: emb.emb_bag_get_tuning(k) for k in
                              ("depth", "addressing", "blocks_per_cu", "xcd_remap", "use_hints",
                               "stream", "bags_per_group", "xcd_pieces", "per_table_launch", "fuse",
                               "bags_per_wave", "hot_split")}},
        "gathered_GBps": gathered * steps / wall / 1e9,
        "gathered_frac_of_hbm_peak": gathered * steps / wall / 1e9 / metrics.HBM_PEAK_GBPS,
        "kernel_ms": {"avg": avg_kern_s * 1e3, "min": float(min(kern_ms)),
                      "median": float(np.median(kern_ms)), "max": float(max(kern_ms))},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": metrics.HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": achieved / metrics.HBM_PEAK_GBPS,
                     "traffic": traffic,
                     "traffic_GBps": None if traffic is None else traffic / avg_kern_s / 1e9,
                     "measured_stream_read_GBps": stream_read_gbps,
                     "frac_of_measured_stream_read": None if stream_read_gbps is None
                     else achieved / stream_read_gbps,
                     "algorithmic_bytes_per_launch": algo,
                     "gathered_bytes_per_launch": gathered,
                     # every distinct row once + indices, offsets, output: a floor for HBM bytes,
                     # so this fraction stays below 1 also where the caches serve repeats
                     "compulsory_bytes_per_launch": compulsory,
                     "frac_compulsory": compulsory / avg_kern_s / 1e9 / metrics.HBM_PEAK_GBPS,
                     "traffic_over_compulsory": None if traffic is None else traffic / compulsory},
        "kernel_ms_after_cache_scrub": cold_ms,
        "graph_replay_ms_per_step": graph_ms_per_step,
        "host_path_from_c": host_latency,
        "cpu_baseline": cpu_baseline,
        "parity": parity,
    }
    torch.cuda.synchronize()
    del arena
    if owner is not None:
        owner.close()
    torch.cuda.empty_cache()
    return result


def summary(r: dict) -> dict:
    """What the 'others' map keeps of a workload's result."""
    rf = r["roofline"]
    return {"workload": r["config"]["workload"], "kernel_ms": r["kernel_ms"]["avg"],
            "kernel_ms_min": r["kernel_ms"]["min"], "ms_per_step": r["ms_per_step"],
            "steps": r["steps"], "lookups_per_s": r["config"]["lookups_per_step"] / (r["kernel_ms"]["avg"] / 1e3),
            "gathered_GBps": rf["gathered_bytes_per_launch"] / (r["kernel_ms"]["avg"] / 1e3) / 1e9,
            "algorithmic_bytes": rf["algorithmic_bytes_per_launch"],
            "compulsory_bytes": rf["compulsory_bytes_per_launch"],
            "frac_algorithmic": rf["frac"], "frac_compulsory": rf["frac_compulsory"],
            "traffic": rf["traffic"], "traffic_over_compulsory": rf["traffic_over_compulsory"],
            "frac_traffic": None if rf["traffic"] is None else rf["traffic_GBps"] / rf["peak"],
            "kernel_ms_after_cache_scrub": r["kernel_ms_after_cache_scrub"],
            "host_path_from_c": r["host_path_from_c"],
            "arena_pick": r["config"]["arena_pick"], "launch_plan": r["config"]["launch_plan"],
            "parity": r["parity"]}


def main() -> int:
    args = build_parser().parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures ONE GPU only (no sharding, no collectives); "
              "run with --gpus 1", file=sys.stderr)
        return 2

    import importlib.util
    spec = importlib.util.spec_from_file_location(
        "_emb_build", os.path.join(ROOT, "paper_2410_22249_amd", "build.py"))
    _b = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(_b)
    _b.ensure_built(verbose=False)     # loads what is built; builds only if nothing is there

    import torch

    import paper_2410_22249_amd as emb

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    for kv in args.tune:
        k, v = kv.split("=")
        emb.emb_bag_set_tuning(k, int(v))

    name = args.workload or "cfg3"
    result = run_workload(args, name, args.steps, args.warmup, headline=True)
    if isinstance(result, int):
        return result
    # the other benchmark configurations, shorter, for the record (the headline stays cfg3)
    if args.workload is None and not args.no_others:
        others = {}
        for other in ("cfg1", "cfg2", "cfg4", "cfg5"):
            r = run_workload(args, other, min(args.steps, 20), min(args.warmup, 3), headline=False)
            if isinstance(r, int):
                return r
            others[other] = summary(r)
        result["others"] = others
    print(json.dumps(result), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
