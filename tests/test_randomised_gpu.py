"""Seeded random problems over everything the forward calls accept: uniform and mixed widths, all
element types, the three pooling modes, weights, short / long / per-table bag lengths (with and
without table_avg_len), hints, padded outputs, and every tuning key (fused and separate launches
of split mixed-width calls alternate), set process-wide or carried by the descriptor.  Each case is checked against
the CPU oracle, and guard rows around the output show that no store leaves it; a failure names its
case, which the seed reproduces."""
import numpy as np
import pytest
import torch

import paper_2410_22249_amd as emb
from inputgen import gen
from gpu_harness import DEV, assert_close_to_oracle, to_dev, tuning

pytestmark = pytest.mark.gpu

DTYPES = ("f32", "f16", "bf16", "u8row", "fp8row")


def _width(rng, dtype, max_bytes):
    """A legal embedding dimension whose row is at most max_bytes."""
    if dtype in gen.QUANTISED:
        return int(16 * rng.integers(0, max_bytes // 16) + 8)          # D + 8 a multiple of 16
    unit, size = (4, 4) if dtype == "f32" else (8, 2)
    return int(unit * rng.integers(1, max_bytes // (unit * size) + 1))


def _pooling(rng, T):
    kind = int(rng.integers(0, 4))
    if kind == 0:
        return ("fixed", int(rng.choice([1, 2, 5, 33])))
    if kind == 1:
        lo = int(rng.integers(0, 3))
        return ("uniform", lo, lo + int(rng.choice([0, 2, 9, 70, 200])))
    specs = tuple(("fixed", 1) if rng.random() < 0.4 else
                  ("uniform", int(rng.integers(0, 3)), int(rng.choice([2, 6, 60, 150])))
                  for _ in range(T))
    return ("per_table", specs)


@pytest.mark.parametrize("block", range(6))
def test_random_problems(oracle, block):
    rng = np.random.default_rng(0xF00D + block)
    for case in range(30):
        dtype = DTYPES[int(rng.integers(0, len(DTYPES)))]
        mixed = rng.random() < 0.45
        T = int(rng.integers(1, 14))
        B = int(rng.integers(1, 200))
        rows = tuple(int(x) for x in rng.integers(1, 2500, size=T))
        mode = ("sum", "mean", "max")[int(rng.integers(0, 3))]
        weighted = mode == "sum" and rng.random() < 0.35
        dists = tuple((("uniform",), ("zipf", 1.1), ("one_item",))[int(rng.integers(0, 3))]
                      for _ in range(T))
        pooling = _pooling(rng, T)
        seed = 0x5EED2000 + 100 * block + case
        kw = dict(addressing=int(rng.choice([0, 0, 1])), depth=int(rng.choice([0, 1, 2, 4, 8, 16])),
                  xcd_remap=int(rng.integers(-1, 2)), blocks_per_cu=int(rng.choice([0, 0, 0, 3])),
                  stream=int(rng.integers(-1, 2)), bags_per_group=int(rng.choice([0, 0, 1, 2, 3, 7])),
                  use_hints=int(rng.integers(0, 2)), fuse=case % 2,
                  station=int(rng.integers(0, 2)), bags_per_wave=int(rng.choice([0, 0, 1, 3, 32])))
        own = rng.random() < 0.5      # the keys travel in the descriptor instead of process-wide
        hints = to_dev(rng.integers(0, 2, size=T).astype(np.uint8)) if rng.random() < 0.5 else None
        pad = int(rng.choice([0, 0, 4, 64]))
        if mixed:
            dims = tuple(_width(rng, dtype, 1024) for _ in range(T))
            wl = gen.MixedWorkload(name=f"r{case}", T=T, rows=rows, dims=dims, dtype=dtype, B=B,
                                   pooling=pooling, dists=dists, mode=mode, weighted=weighted, seed=seed)
            total = int(sum(dims))
        else:
            D = _width(rng, dtype, 1024 if dtype in gen.QUANTISED else 1280)
            wl = gen.Workload(name=f"r{case}", T=T, rows=rows, D=D, dtype=dtype, B=B,
                              pooling=pooling, dists=dists, mode=mode, weighted=weighted, seed=seed)
            total = T * D
        batch = gen.make_batches(wl, 1)[0]
        avg = gen.table_avg_len(wl, batch) if rng.random() < 0.5 else None
        ld = total + pad
        what = (f"block {block} case {case}: {'mixed' if mixed else 'uniform'} T={T} B={B} {dtype} "
                f"{mode} w={weighted} pooling={pooling[0]} avg_len={'yes' if avg is not None else 'no'} "
                f"{'desc.tuning' if own else 'process-wide'} {kw}")
        print(what, flush=True)
        idx = to_dev(batch.indices) if batch.num_lookups else None
        off, w = to_dev(batch.offsets), to_dev(batch.weights)
        guard = 3                        # rows before and after `out` that no store may touch
        big = torch.full((B + 2 * guard, ld), -3.0, dtype=torch.float32, device=DEV)
        out = big[guard:guard + B]
        if mixed:
            tabs = gen.mixed_host_tables(wl)
            ref, bound = oracle.emb_bag_mixed(tabs, batch.indices, batch.offsets, B, mode,
                                              weights=batch.weights, out_ld=ld, codes=wl.codes)
            arena = torch.from_numpy(np.concatenate([t.view(np.uint8).reshape(-1) for t in tabs])).to(DEV)
            desc = emb.make_mixed_desc(dims, B, emb.DTYPES[dtype], emb.MODES[mode], batch.num_lookups,
                                       ld, int(np.diff(wl.table_byte_offsets()).max()), hints, avg,
                                       tuning=kw if own else None)
            with tuning(**({} if own else kw)):
                emb.emb_bag_forward_mixed(desc, arena, to_dev(wl.table_byte_offsets()),
                                          to_dev(wl.out_offsets()), idx, off, w, out)
        else:
            host = gen.host_arena(wl)
            ref, bound = oracle.emb_bag(host, wl.table_offsets(), batch.indices, batch.offsets, B, mode,
                                        weights=batch.weights, out_ld=ld, codes=wl.codes)
            arena = torch.from_numpy(host.view(np.uint8).reshape(-1)).to(DEV)
            desc = emb.make_desc(T, B, wl.D, emb.DTYPES[dtype], emb.MODES[mode], batch.num_lookups, ld,
                                 max(rows), hints, avg, tuning=kw if own else None)
            with tuning(**({} if own else kw)):
                emb.emb_bag_forward(desc, arena, to_dev(wl.table_offsets()), idx, off, w, out)
        torch.cuda.synchronize()
        whole = big.cpu().numpy()
        assert np.all(whole[:guard] == -3.0) and np.all(whole[guard + B:] == -3.0), what
        got = whole[guard:guard + B]
        assert np.all(got[:, total:] == -3.0), what
        assert_close_to_oracle(got[:, :total], ref[:, :total], bound[:, :total], dtype != "f32", what)
