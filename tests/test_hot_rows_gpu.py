"""GPU parity of the hot / cold split: tables laid out hot rows first (`desc.hot_rows`), whose
lookups the wave kernel regroups per chunk and reads with two cache policies.  The split changes
the order in which a bag's rows are added, nothing else: results equal the oracle within the
usual tolerance, and exactly on integer-valued tables."""
import numpy as np
import pytest
import torch

import paper_2410_22249_amd as emb
from inputgen import gen
from gpu_harness import (DEV, assert_close_to_oracle, device_arena, forward, to_dev, tuning,
                         upload_arena)

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def _split_on():
    """The split is opt-in (tuning key hot_split, default 0): switched on for these tests."""
    with tuning(hot_split=1):
        yield


def _problem(dtype="f32", kind=gen.KIND_NORMAL, weighted=False, **over):
    wl = gen.with_overrides(gen.workload("small_hot"), dtype=dtype, kind=kind, weighted=weighted,
                            **over)
    batch = gen.make_batches(wl, 1)[0]
    return wl, batch, gen.host_arena(wl)


def _plan_says_hot(wl, batch, hot):
    desc = emb.make_desc(wl.T, wl.B, wl.D, emb.DTYPES[wl.dtype], emb.MODES["sum"],
                         batch.num_lookups, 0, max(wl.rows), hot_rows=to_dev(hot))
    return emb.emb_bag_plan_forward(desc).hot_split


@pytest.mark.parametrize("dtype,D", [("f32", 128), ("f32", 64), ("f16", 256), ("bf16", 64),
                                     ("u8row", 120), ("fp8row", 504)])
@pytest.mark.parametrize("mode", ["sum", "mean", "max"])
def test_hot_split_matches_oracle(oracle, dtype, D, mode):
    wl, batch, arena = _problem(dtype, D=D)
    ref, bound = oracle.emb_bag(arena, wl.table_offsets(), batch.indices, batch.offsets, wl.B,
                                mode, codes=wl.codes)
    dev = upload_arena(arena)
    tdt = emb.DTYPES[dtype]
    hot = gen.hot_rows(wl)
    assert _plan_says_hot(wl, batch, hot) == 1
    for depth, split in ((4, 1), (8, 1), (8, 2)):
        for bpw in (1, 3):
            with tuning(depth=depth, bags_per_wave=bpw, stream=0, hot_split=split):
                got = forward(dev, wl.table_offsets(), batch.indices, batch.offsets, wl.B, mode,
                              table_dtype=tdt, hot_rows=hot).cpu().numpy()
            if mode == "max" and dtype not in gen.QUANTISED:
                assert np.array_equal(got.astype(np.float64), ref)
            else:
                assert_close_to_oracle(got, ref, bound, dtype != "f32",
                                       f"hot/{dtype}/{mode}/depth{depth}/bpw{bpw}")


@pytest.mark.parametrize("dtype", ["f32", "f16", "u8row"])
def test_hot_split_is_exact_on_integer_tables_for_any_head(oracle, dtype):
    """Integer-valued rows: every order of summation gives the same bits, so the split must equal
    the oracle and the unsplit kernel exactly, whatever the head sizes are (none, a few rows,
    the whole table, more than the table)."""
    wl, batch, arena = _problem(dtype, kind=gen.KIND_INT, weighted=False,
                                D=120 if dtype == "u8row" else 128)
    ref, _ = oracle.emb_bag(arena, wl.table_offsets(), batch.indices, batch.offsets, wl.B, "sum",
                            codes=wl.codes)
    dev = upload_arena(arena)
    tdt = emb.DTYPES[dtype]
    with tuning(stream=0):
        plain = forward(dev, wl.table_offsets(), batch.indices, batch.offsets, wl.B, "sum",
                        table_dtype=tdt).cpu().numpy()
    assert np.array_equal(plain.astype(np.float64), ref)
    rng = np.random.default_rng(5)
    heads = [np.zeros(wl.T, np.int64), np.asarray(wl.rows, np.int64), np.asarray(wl.rows, np.int64) + 7,
             gen.hot_rows(wl)] + [rng.integers(0, np.asarray(wl.rows) + 1) for _ in range(4)]
    for hot in heads:
        with tuning(stream=0):
            got = forward(dev, wl.table_offsets(), batch.indices, batch.offsets, wl.B, "sum",
                          table_dtype=tdt, hot_rows=hot).cpu().numpy()
        assert np.array_equal(got.view(np.uint32), plain.view(np.uint32)), hot


def test_hot_split_with_weights_and_invalid_ids(oracle):
    """Per-sample weights travel with their lookups through the regrouping; a row id outside the
    table contributes nothing and an id of -1 is not mistaken for a hot row."""
    wl, batch, arena = _problem("f32", weighted=True)
    ref, bound = oracle.emb_bag(arena, wl.table_offsets(), batch.indices, batch.offsets, wl.B,
                                "sum", weights=batch.weights)
    dev = upload_arena(arena)
    hot = gen.hot_rows(wl)
    with tuning(stream=0):
        got = forward(dev, wl.table_offsets(), batch.indices, batch.offsets, wl.B, "sum",
                      weights=batch.weights, hot_rows=hot).cpu().numpy()
    assert_close_to_oracle(got, ref, bound, False, "hot/weights")
    # spoil some ids: the oracle's answer is that of the batch with those lookups given weight 0
    idx = batch.indices.copy()
    rng = np.random.default_rng(9)
    bad = rng.choice(len(idx), size=len(idx) // 7, replace=False)
    idx[bad] = np.where(rng.random(len(bad)) < 0.5, -1, 1 << 40)
    w0 = batch.weights.copy()
    w0[bad] = 0.0
    ref, bound = oracle.emb_bag(arena, wl.table_offsets(), batch.indices, batch.offsets, wl.B,
                                "sum", weights=w0)
    with tuning(stream=0):
        got = forward(dev, wl.table_offsets(), idx, batch.offsets, wl.B, "sum",
                      weights=batch.weights, hot_rows=hot).cpu().numpy()
    assert_close_to_oracle(got, ref, bound, False, "hot/invalid ids")


def test_where_the_hot_split_applies():
    wl, batch, _ = _problem("f32")
    hot = gen.hot_rows(wl)
    assert _plan_says_hot(wl, batch, hot) == 1
    with tuning(hot_split=2):
        assert _plan_says_hot(wl, batch, hot) == 1
    for kw in (dict(hot_split=0), dict(addressing=1), dict(depth=2), dict(depth=16)):
        with tuning(**kw):
            assert _plan_says_hot(wl, batch, hot) == 0, kw
    desc = emb.make_desc(wl.T, wl.B, wl.D, emb.EMB_F32, emb.EMB_SUM, batch.num_lookups, 0, 0,
                         hot_rows=to_dev(hot))              # no row bound: 64-bit addressing
    assert emb.emb_bag_plan_forward(desc).hot_split == 0


@pytest.mark.parametrize("name", ["cfg4_hot", "cfg5_hot"])
def test_full_size_hot_head_sampled_bags(oracle, name):
    """The benchmark's skewed configurations with every Zipf table laid out hot rows first, in the
    launch configuration bench.py times: sampled bags against the oracle, the whole output finite
    and deterministic, and equal within rounding to the launch that ignores the head."""
    print(f"\n[hot] {name}: generating", flush=True)
    wl = gen.workload(name)
    batch = gen.make_batches(wl, 1)[0]
    arena = device_arena(wl)
    toff = to_dev(wl.table_offsets())
    idx, off = to_dev(batch.indices), to_dev(batch.offsets)
    hot = to_dev(gen.hot_rows(wl))
    desc = emb.make_desc(wl.T, wl.B, wl.D, emb.DTYPES[wl.dtype], emb.MODES[wl.mode],
                         batch.num_lookups, 0, max(wl.rows), hot_rows=hot)
    assert emb.emb_bag_plan_forward(desc).hot_split == 1
    out = torch.full((wl.B, wl.T * wl.D), float("nan"), dtype=torch.float32, device=DEV)
    out2 = torch.full_like(out, float("nan"))
    emb.emb_bag_forward(desc, arena, toff, idx, off, None, out)
    emb.emb_bag_forward(desc, arena, toff, idx, off, None, out2)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(out).all()) and torch.equal(out, out2)
    rng = np.random.default_rng(2025)
    edge = np.concatenate([np.arange(wl.T) * wl.B, np.arange(wl.T) * wl.B + wl.B - 1])
    bags = np.unique(np.concatenate([rng.integers(0, wl.num_bags, size=500), edge]))
    small, ix, soff, _ = gen.compact_rows(wl, batch, bags)
    ref, bound = oracle.emb_bag(small, np.array([0, len(small)], np.int64), ix, soff, len(bags),
                                wl.mode)
    sel = torch.from_numpy(np.stack([bags % wl.B, bags // wl.B], 1)).to(DEV)
    got = out.view(wl.B, wl.T, wl.D)[sel[:, 0], sel[:, 1]].cpu().numpy()
    worst = assert_close_to_oracle(got, ref, bound, wl.dtype != "f32", f"{name} sampled")
    with tuning(hot_split=0):
        emb.emb_bag_forward(desc, arena, toff, idx, off, None, out2)
        torch.cuda.synchronize()
    assert torch.allclose(out, out2, rtol=1e-4, atol=1e-5)
    print(f"[hot] {name}: {len(bags)} bags checked, max err/bound {worst:.3e}", flush=True)
