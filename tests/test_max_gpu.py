"""GPU parity for max pooling (EMB_MAX): the element-wise maximum of a bag's rows.  The result is
an element of the table, so for fp32 / fp16 / bf16 rows the comparison with the oracle is exact;
quantised rows are dequantised in fp32 on the device and carry the usual tolerance."""
import numpy as np
import pytest
import torch

import paper_2410_22249_amd as emb
from inputgen import gen
from gpu_harness import DEV, assert_close_to_oracle, forward, to_dev, tuning, upload_arena

pytestmark = pytest.mark.gpu

SMALL = ["tiny", "small_f32_d64", "small_f32_d128", "small_f16_d256", "small_bf16_d256",
         "small_u8_d120", "small_u8_d504"]


def _problem(name, **over):
    wl = gen.with_overrides(gen.workload(name), **over) if over else gen.workload(name)
    return wl, gen.make_batches(wl, 1)[0], gen.host_arena(wl)


def _check(got, ref, bound, dtype, what):
    if dtype == "u8row":
        assert_close_to_oracle(got, ref, bound, True, what)
    else:
        assert np.array_equal(got.astype(np.float64), ref), what


@pytest.mark.parametrize("name", SMALL)
def test_max_pooling_matches_oracle(oracle, name):
    wl, batch, arena = _problem(name)
    ref, bound = oracle.emb_bag(arena, wl.table_offsets(), batch.indices, batch.offsets, wl.B, "max")
    dev = upload_arena(arena)
    for kw in (dict(), dict(addressing=1), dict(depth=1), dict(depth=8), dict(depth=16, xcd_remap=1),
               dict(blocks_per_cu=2), dict(stream=1), dict(stream=1, bags_per_group=1),
               dict(stream=1, bags_per_group=3, depth=8), dict(stream=1, bags_per_group=63, depth=4)):
        with tuning(**kw):
            got = forward(dev, wl.table_offsets(), batch.indices, batch.offsets, wl.B, "max").cpu().numpy()
        _check(got, ref, bound, wl.dtype, f"max/{name}/{kw}")


@pytest.mark.parametrize("name", ["small_f32_d64", "small_f16_d256", "small_u8_d120"])
def test_max_pooling_short_and_empty_bags(oracle, name):
    wl, batch, arena = _problem(name, pooling=("uniform", 0, 3))
    ref, bound = oracle.emb_bag(arena, wl.table_offsets(), batch.indices, batch.offsets, wl.B, "max")
    dev = upload_arena(arena)
    desc = emb.make_desc(wl.T, wl.B, wl.D, emb.DTYPES[wl.dtype], emb.EMB_MAX, batch.num_lookups, 0,
                         max(wl.rows))
    # bags this short take the stream kernel by themselves; the wave kernel must agree
    assert emb.emb_bag_plan_forward(desc).kernel == emb.EMB_KERNEL_STREAM
    for kw in (dict(), dict(stream=0), dict(stream=1, bags_per_group=2), dict(stream=1, bags_per_group=15)):
        with tuning(**kw):
            got = forward(dev, wl.table_offsets(), batch.indices, batch.offsets, wl.B,
                          "max").cpu().numpy()
        _check(got, ref, bound, wl.dtype, f"max short/{name}/{kw}")
        empty = np.repeat(np.diff(batch.offsets).reshape(wl.T, wl.B).T == 0, wl.D, axis=1)
        assert empty.any() and np.all(got[empty] == 0) and not np.signbit(got[empty]).any()


@pytest.mark.parametrize("D,dtype", [(4, "f32"), (12, "f32"), (96, "f32"), (320, "f32"), (24, "f16"),
                                     (520, "bf16"), (24, "u8row"), (1016, "u8row")])
def test_max_pooling_row_widths(oracle, D, dtype):
    """Every lanes-per-row class, rows that leave lanes idle, and rows longer than 1 KiB."""
    wl = gen.Workload(name="w", T=3, rows=(300, 17, 1), D=D, dtype=dtype, B=29,
                      pooling=("uniform", 0, 70), dists=(("uniform",),) * 3, seed=0x5EED1000 + D)
    batch = gen.make_batches(wl, 1)[0]
    arena = gen.host_arena(wl)
    ref, bound = oracle.emb_bag(arena, wl.table_offsets(), batch.indices, batch.offsets, wl.B, "max")
    got = forward(upload_arena(arena), wl.table_offsets(), batch.indices, batch.offsets, wl.B, "max",
                  out_ld=3 * D + 4, fill=-3.0).cpu().numpy()
    assert np.all(got[:, 3 * D:] == -3.0)
    _check(got[:, :3 * D], ref, bound, dtype, f"max widths/{dtype}/D{D}")


def test_max_pooling_skips_invalid_lookups(oracle):
    """A lookup that names no row takes no part in the maximum (it fetched zeros, which would win
    in an all-negative bag); a bag left without a valid lookup gives 0."""
    wl, batch, arena = _problem("small_f32_d128")
    arena = -np.abs(arena) - 1.0                          # every element negative
    toff = wl.table_offsets()
    rng = np.random.default_rng(17)
    idx = batch.indices.copy()
    pos = rng.choice(len(idx), size=80, replace=False)
    table_of = np.repeat(np.arange(wl.T), np.diff(batch.offsets[::wl.B]))
    idx[pos] = np.where(rng.random(80) < 0.5, -1 - rng.integers(0, 5, 80),
                        np.asarray(wl.rows)[table_of[pos]] + rng.integers(0, 3, 80))
    g = int(np.argmax(np.diff(batch.offsets) == 2))       # a bag of two lookups: both invalid
    idx[batch.offsets[g]:batch.offsets[g + 1]] = -7
    keep = np.ones(len(idx), bool)
    keep[pos] = False
    keep[batch.offsets[g]:batch.offsets[g + 1]] = False
    lens = np.add.reduceat(keep.astype(np.int64), batch.offsets[:-1].clip(max=len(idx) - 1))
    lens[np.diff(batch.offsets) == 0] = 0
    ref, bound = oracle.emb_bag(arena, toff, batch.indices[keep], gen.lengths_to_offsets(lens),
                                wl.B, "max")
    dev = upload_arena(arena)
    for kw in (dict(addressing=0), dict(addressing=1), dict(stream=1), dict(stream=1, bags_per_group=4),
               dict(stream=1, addressing=1)):
        with tuning(**kw):
            got = forward(dev, toff, idx, batch.offsets, wl.B, "max").cpu().numpy()
        assert np.array_equal(got.astype(np.float64), ref), kw
        t, b = divmod(g, wl.B)
        assert np.all(got[b, t * wl.D:(t + 1) * wl.D] == 0)


def test_max_pooling_mixed_widths_and_hints(oracle):
    wl = gen.mixed_workload("mixed_small")
    batch = gen.make_batches(wl, 1)[0]
    tabs = gen.mixed_host_tables(wl)
    arena = torch.from_numpy(np.concatenate([t.view(np.uint8).reshape(-1) for t in tabs])).to(DEV)
    ref, bound = oracle.emb_bag_mixed(tabs, batch.indices, batch.offsets, wl.B, "max")
    total = int(sum(wl.dims))
    for hints in (None, to_dev(np.ones(wl.T, np.uint8))):
        for own in (None, dict(stream=1), dict(stream=1, bags_per_group=3, fuse=0)):
            out = torch.full((wl.B, total), float("nan"), dtype=torch.float32, device=DEV)
            desc = emb.make_mixed_desc(wl.dims, wl.B, emb.EMB_F32, emb.EMB_MAX, batch.num_lookups, 0,
                                       int(np.diff(wl.table_byte_offsets()).max()), hints, tuning=own)
            if own:     # one stream launch per lanes-per-row class, never fused for max pooling
                plan = emb.emb_bag_plan_forward_mixed(desc)
                assert plan.kernel == emb.EMB_KERNEL_STREAM and plan.fused == 0
            emb.emb_bag_forward_mixed(desc, arena, to_dev(wl.table_byte_offsets()),
                                      to_dev(wl.out_offsets()), to_dev(batch.indices),
                                      to_dev(batch.offsets), None, out)
            torch.cuda.synchronize()
            assert np.array_equal(out.cpu().numpy().astype(np.float64), ref), own


def test_max_pooling_one_hot_takes_the_stream_kernel_and_returns_the_rows(oracle):
    """One lookup per bag: the maximum of a bag is its row; the short-bag kernel serves it."""
    wl = gen.Workload(name="onehot_max", T=5, rows=(1000, 33, 1, 5000, 64), D=32, dtype="f16", B=700,
                      pooling=("fixed", 1), dists=(("uniform",),) * 5, seed=0x5EED1207)
    batch = gen.make_batches(wl, 1)[0]
    arena = gen.host_arena(wl)
    desc = emb.make_desc(wl.T, wl.B, wl.D, emb.EMB_F16, emb.EMB_MAX, batch.num_lookups, 0, max(wl.rows))
    assert emb.emb_bag_plan_forward(desc).kernel == emb.EMB_KERNEL_STREAM
    got = forward(upload_arena(arena), wl.table_offsets(), batch.indices, batch.offsets, wl.B,
                  "max").cpu().numpy()
    toff = wl.table_offsets()
    for t in range(wl.T):
        rows = arena[toff[t] + batch.indices[t * wl.B:(t + 1) * wl.B]].astype(np.float32)
        assert np.array_equal(got[:, t * wl.D:(t + 1) * wl.D], rows), t
    ref, _ = oracle.emb_bag(arena, toff, batch.indices, batch.offsets, wl.B, "max")
    assert np.array_equal(got.astype(np.float64), ref)
