"""GPU parity for tables of different widths (emb_bag_forward_mixed) against the oracle."""
import numpy as np
import pytest
import torch

import paper_2410_22249_amd as emb
from inputgen import gen
from gpu_harness import DEV, assert_close_to_oracle, to_dev, tuning

pytestmark = pytest.mark.gpu

EDT = emb.DTYPES


def _device_arena(wl):
    arena = torch.empty(wl.table_bytes, dtype=torch.uint8, device=DEV)
    gen.mixed_fill_device(wl, arena.data_ptr(), torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    return arena


def _forward(wl, arena, batch, mode="sum", weights=None, out_ld=0, hints=None, fill=float("nan")):
    total = int(sum(wl.dims))
    ld = out_ld if out_ld else total
    out = torch.full((wl.B, ld), fill, dtype=torch.float32, device=DEV)
    desc = emb.make_mixed_desc(wl.dims, wl.B, EDT[wl.dtype],
                               emb.MODES[mode], batch.num_lookups,
                               out_ld, int(np.diff(wl.table_byte_offsets()).max()), hints)
    emb.emb_bag_forward_mixed(desc, arena, to_dev(wl.table_byte_offsets()), to_dev(wl.out_offsets()),
                              to_dev(batch.indices) if batch.num_lookups else None,
                              to_dev(batch.offsets), to_dev(weights), out)
    torch.cuda.synchronize()
    return out


def _wl(dtype, **kw):
    base = gen.mixed_workload("mixed_small")
    dims = {"f32": base.dims, "f16": (64, 8, 128, 512, 32, 96, 24), "bf16": (64, 8, 128, 512, 32, 96, 24),
            "u8row": (120, 8, 248, 1016, 56, 24, 504)}[dtype]
    from dataclasses import replace
    return replace(base, dtype=dtype, dims=dims, **kw)


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16", "u8row"])
def test_mixed_widths_match_oracle(oracle, dtype):
    for mode, weighted in (("sum", False), ("mean", False), ("sum", True)):
        wl = _wl(dtype, weighted=weighted)
        batch = gen.make_batches(wl, 1)[0]
        tabs = gen.mixed_host_tables(wl)
        arena = _device_arena(wl)
        # the device fill of every table equals the host values
        boff = wl.table_byte_offsets()
        host_bytes = np.concatenate([t.view(np.uint8).reshape(-1) for t in tabs])
        assert np.array_equal(arena.cpu().numpy(), host_bytes)
        ref, bound = oracle.emb_bag_mixed(tabs, batch.indices, batch.offsets, wl.B, mode,
                                          weights=batch.weights)
        first = None
        for kw in (dict(), dict(addressing=1), dict(depth=8), dict(depth=2, xcd_remap=1),
                   dict(blocks_per_cu=3)):
            with tuning(**kw):
                got = _forward(wl, arena, batch, mode, batch.weights).cpu().numpy()
            assert_close_to_oracle(got, ref, bound, dtype != "f32", f"mixed/{dtype}/{mode}/{kw}")
            if first is None:
                first = got
            elif kw.get("depth") is None:
                assert np.array_equal(got, first), kw       # addressing / launch shape: same bits


def test_mixed_equals_uniform_when_widths_agree(oracle):
    wl = gen.workload("small_f32_d128")
    batch = gen.make_batches(wl, 1)[0]
    host = gen.host_arena(wl)
    from gpu_harness import forward, upload_arena
    with tuning(stream=0):   # the mixed path has no short-bag kernel: compare like with like
        uni = forward(upload_arena(host), wl.table_offsets(), batch.indices, batch.offsets, wl.B,
                      "mean")
    mw = gen.MixedWorkload(name="same", T=wl.T, rows=wl.rows, dims=(wl.D,) * wl.T, dtype="f32",
                           B=wl.B, pooling=wl.pooling, dists=wl.dists, seed=wl.seed)
    arena = torch.from_numpy(host.view(np.uint8).reshape(-1)).to(DEV)
    mix = _forward(mw, arena, batch, "mean")
    assert torch.equal(uni, mix)


def test_mixed_padding_hints_and_empty(oracle):
    wl = _wl("f32")
    batch = gen.make_batches(wl, 1)[0]
    tabs = gen.mixed_host_tables(wl)
    arena = _device_arena(wl)
    total = int(sum(wl.dims))
    ref, bound = oracle.emb_bag_mixed(tabs, batch.indices, batch.offsets, wl.B, "sum", out_ld=total + 12)
    hints = to_dev((np.arange(wl.T) % 2).astype(np.uint8))
    got = _forward(wl, arena, batch, "sum", out_ld=total + 12, hints=hints, fill=-5.0).cpu().numpy()
    assert np.all(got[:, total:] == -5.0)
    assert_close_to_oracle(got[:, :total], ref[:, :total], bound[:, :total], False, "mixed/padded")
    plain = _forward(wl, arena, batch, "sum").cpu().numpy()
    assert np.array_equal(plain, got[:, :total])
    # every bag empty
    empty = gen.Batch(offsets=np.zeros(wl.T * wl.B + 1, np.int64), indices=np.zeros(0, np.int64))
    z = _forward(wl, arena, empty, "mean").cpu().numpy()
    assert np.all(z == 0) and not np.signbit(z).any()


def test_mixed_malformed_table_description_is_skipped():
    """out_offsets that contradict the rules (a width that is not a multiple of 4 floats here) make
    the kernel skip that table instead of writing out of place; the others are unaffected."""
    wl = _wl("f32")
    batch = gen.make_batches(wl, 1)[0]
    arena = _device_arena(wl)
    good = _forward(wl, arena, batch, "sum")
    total = int(sum(wl.dims))
    out = torch.full((wl.B, total), -9.0, dtype=torch.float32, device=DEV)
    ooff = wl.out_offsets().copy()
    ooff[3] += 2                      # table 2 gets width 130, table 3 starts unaligned
    desc = emb.make_mixed_desc(wl.dims, wl.B, emb.EMB_F32, emb.EMB_SUM, batch.num_lookups, 0,
                               int(np.diff(wl.table_byte_offsets()).max()))
    emb.emb_bag_forward_mixed(desc, arena, to_dev(wl.table_byte_offsets()), to_dev(ooff),
                              to_dev(batch.indices), to_dev(batch.offsets), None, out)
    torch.cuda.synchronize()
    o, g = out.cpu().numpy(), good.cpu().numpy()
    c = wl.out_offsets()
    assert np.all(o[:, c[2]:c[4]] == -9.0)                         # tables 2 and 3 skipped
    assert np.array_equal(o[:, :c[2]], g[:, :c[2]]) and np.array_equal(o[:, c[4]:], g[:, c[4]:])


def test_mixed_full_size_sampled(oracle):
    """60 tables x 4 M rows with widths 32 / 64 / 128 / 256 (115 GB): sampled bags against the oracle."""
    wl = gen.mixed_workload("mixed_cfg")
    batch = gen.make_batches(wl, 1)[0]
    arena = _device_arena(wl)
    out = _forward(wl, arena, batch, "sum")
    assert bool(torch.isfinite(out).all())
    out2 = _forward(wl, arena, batch, "sum")
    assert torch.equal(out, out2)
    rng = np.random.default_rng(7)
    base, cols = wl.row_bases(), wl.out_offsets()
    worst = 0.0
    for t in range(wl.T):
        bs = np.unique(np.concatenate([rng.integers(0, wl.B, size=6), [0, wl.B - 1]]))
        segs = [batch.indices[batch.offsets[t * wl.B + b]:batch.offsets[t * wl.B + b + 1]] for b in bs]
        uniq, inv = np.unique(np.concatenate(segs), return_inverse=True)
        small = gen.table_values(wl.seed, base[t] + uniq, wl.dims[t], wl.dtype, wl.kind)
        soff = gen.lengths_to_offsets(np.array([len(x) for x in segs]))
        ref, bound = oracle.emb_bag(small, np.array([0, len(small)], np.int64), inv.astype(np.int64),
                                    soff, len(bs), "sum")
        got = out[torch.from_numpy(bs).to(DEV), cols[t]:cols[t + 1]].cpu().numpy()
        worst = max(worst, assert_close_to_oracle(got, ref, bound, False, f"mixed_cfg table {t}"))
    print(f"\n[mixed_cfg] max err/bound {worst:.3e}", flush=True)


@pytest.mark.parametrize("T", [8, 10, 12, 16, 24])
def test_mixed_width_balanced_xcd_order(oracle, T):
    """With the XCD-affine block order forced on, tables of different widths are dealt to the XCDs
    by width (2, 4 or 8 XCD sets depending on T); the result must not depend on the order."""
    rng = np.random.default_rng(100 + T)
    dims = tuple(int(d) for d in rng.choice([4, 8, 16, 32, 64, 96, 128, 192, 256], size=T))
    rows = tuple(int(r) for r in rng.integers(1, 400, size=T))
    wl = gen.MixedWorkload(name=f"order{T}", T=T, rows=rows, dims=dims, dtype="f32", B=37,
                           pooling=("uniform", 0, 70), dists=(("uniform",),) * T, seed=0x5EED0D00 + T)
    batch = gen.make_batches(wl, 1)[0]
    tabs = gen.mixed_host_tables(wl)
    arena = _device_arena(wl)
    ref, bound = oracle.emb_bag_mixed(tabs, batch.indices, batch.offsets, wl.B, "sum")
    with tuning(xcd_remap=0):
        natural = _forward(wl, arena, batch).cpu().numpy()
    with tuning(xcd_remap=1):
        ordered = _forward(wl, arena, batch).cpu().numpy()
    assert_close_to_oracle(ordered, ref, bound, False, f"mixed order T={T}")
    assert np.array_equal(natural, ordered)


def test_mixed_batches_validate_profile_and_replay_from_a_graph(oracle):
    """The checker and the reuse profiler read only ids and bag bounds, so a uniform descriptor of
    any width and the cumulative row counts serve a mixed-width batch; and the mixed launch (its
    table order travels by value in the kernel arguments) replays from a HIP graph."""
    wl = gen.mixed_workload("mixed_small")
    batch = gen.make_batches(wl, 1)[0]
    tabs = gen.mixed_host_tables(wl)
    arena = _device_arena(wl)
    rows = to_dev(wl.row_bases())
    idx, off = to_dev(batch.indices), to_dev(batch.offsets)
    udesc = emb.make_desc(wl.T, wl.B, 4, emb.EMB_F32, emb.EMB_SUM, batch.num_lookups, 0, max(wl.rows))
    bad = torch.zeros(1, dtype=torch.int64, device=DEV)
    emb.emb_bag_validate(udesc, rows, idx, off, bad)
    hints = torch.zeros(wl.T, dtype=torch.uint8, device=DEV)
    emb.emb_bag_profile_reuse(udesc, idx, off, 16384, -1, None, None, hints)
    torch.cuda.synchronize()
    assert int(bad.item()) == 0
    from oracle import reuse_oracle
    assert np.array_equal(hints.cpu().numpy(),
                          reuse_oracle.profile_reuse(batch.indices, batch.offsets, wl.T, wl.B, 16384, 75,
                                                     row_bytes=16)[2])
    bad_idx = idx.clone()
    bad_idx[0] = wl.rows[0]                                 # one past the end of table 0
    bad.zero_()
    emb.emb_bag_validate(udesc, rows, bad_idx, off, bad)
    torch.cuda.synchronize()
    assert int(bad.item()) == 1

    ref, bound = oracle.emb_bag_mixed(tabs, batch.indices, batch.offsets, wl.B, "sum")
    out = torch.empty((wl.B, int(sum(wl.dims))), dtype=torch.float32, device=DEV)
    desc = emb.make_mixed_desc(wl.dims, wl.B, emb.EMB_F32, emb.EMB_SUM, batch.num_lookups, 0,
                               int(np.diff(wl.table_byte_offsets()).max()), hints)
    boff, ooff = to_dev(wl.table_byte_offsets()), to_dev(wl.out_offsets())
    with tuning(xcd_remap=1):
        stream = torch.cuda.Stream()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=stream):
            emb.emb_bag_forward_mixed(desc, arena, boff, ooff, idx, off, None, out, stream)
    for _ in range(3):
        out.fill_(-1.0)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert_close_to_oracle(out.cpu().numpy(), ref, bound, False, "mixed graph replay")


@pytest.mark.parametrize("dtype", ["f32", "f16", "u8row"])
@pytest.mark.parametrize("pooling", [("fixed", 1), ("uniform", 0, 3), ("uniform", 0, 9)])
def test_mixed_widths_with_short_bags_use_the_stream_kernel(oracle, dtype, pooling):
    """Short bags split a mixed-width call into one stream-kernel launch per lanes-per-row class
    and one wave-kernel launch for the remaining tables; every table is still written once."""
    wl = _wl(dtype, pooling=pooling, B=211)
    batch = gen.make_batches(wl, 1)[0]
    tabs = gen.mixed_host_tables(wl)
    arena = _device_arena(wl)
    max_bytes = int(np.diff(wl.table_byte_offsets()).max())
    desc = emb.make_mixed_desc(wl.dims, wl.B, EDT[dtype], emb.EMB_SUM, batch.num_lookups, 0, max_bytes)
    plan = emb.emb_bag_plan_forward_mixed(desc)
    assert plan.num_launches > 1
    for mode in ("sum", "mean"):
        ref, bound = oracle.emb_bag_mixed(tabs, batch.indices, batch.offsets, wl.B, mode)
        first = None
        for kw in (dict(), dict(xcd_remap=1), dict(bags_per_group=3), dict(addressing=1),
                   dict(addressing=1, bags_per_group=2, fuse=0), dict(stream=1, depth=4),
                   dict(stream=1, depth=8, addressing=1)):          # (addressing 1: 64-bit rows)
            with tuning(**kw):
                if kw.get("addressing") == 1:
                    n = emb.emb_bag_plan_forward_mixed(desc).num_launches
                    p64 = [emb.emb_bag_plan_forward_mixed(desc, which=k) for k in range(n)]
                    assert all(p.buffer_addressing == 0 for p in p64)
                    assert any(p.kernel == emb.EMB_KERNEL_STREAM for p in p64)
                got = _forward(wl, arena, batch, mode).cpu().numpy()
            assert_close_to_oracle(got, ref, bound, dtype != "f32", f"mixed short/{dtype}/{mode}/{kw}")
            if first is None:
                first = got
            elif "stream" not in kw:
                assert np.array_equal(got, first), kw
        with tuning(stream=0):                              # the wave kernel alone, for comparison
            wave = _forward(wl, arena, batch, mode).cpu().numpy()
        assert_close_to_oracle(wave, ref, bound, dtype != "f32", "mixed short/wave only")


def test_mixed_short_bags_weights_padding_and_hints(oracle):
    wl = _wl("f32", pooling=("uniform", 0, 4), weighted=True, B=97)
    batch = gen.make_batches(wl, 1)[0]
    tabs = gen.mixed_host_tables(wl)
    arena = _device_arena(wl)
    total = int(sum(wl.dims))
    ref, bound = oracle.emb_bag_mixed(tabs, batch.indices, batch.offsets, wl.B, "sum",
                                      weights=batch.weights, out_ld=total + 8)
    hints = to_dev((np.arange(wl.T) % 2).astype(np.uint8))
    got = _forward(wl, arena, batch, "sum", batch.weights, out_ld=total + 8, hints=hints,
                   fill=-5.0).cpu().numpy()
    assert np.all(got[:, total:] == -5.0)
    assert_close_to_oracle(got[:, :total], ref[:, :total], bound[:, :total], False, "mixed short weighted")


def test_mixed_onehot_full_size_sampled(oracle):
    """26 tables x 1 M rows, widths 16 / 32 / 64 / 128, batch 131,072, one lookup per bag."""
    wl = gen.mixed_workload("mixed_onehot")
    batch = gen.make_batches(wl, 1)[0]
    arena = _device_arena(wl)
    out = _forward(wl, arena, batch, "sum")
    assert bool(torch.isfinite(out).all())
    rng = np.random.default_rng(9)
    base, cols = wl.row_bases(), wl.out_offsets()
    for t in range(wl.T):
        bs = np.unique(np.concatenate([rng.integers(0, wl.B, size=40), [0, wl.B - 1]]))
        rows = batch.indices[batch.offsets[t * wl.B + bs]]
        want = gen.table_values(wl.seed, base[t] + rows, wl.dims[t], wl.dtype, wl.kind)
        got = out[torch.from_numpy(bs).to(DEV), cols[t]:cols[t + 1]].cpu().numpy()
        assert np.array_equal(got, want), t                  # one lookup per bag: the row itself


def test_mixed_widths_with_per_table_bag_lengths(oracle):
    """Short-bag and long-bag tables of several widths in one call: table_avg_len sends each
    short-bag table to the stream launch of its row class and the others to the wave launch."""
    specs = (("fixed", 1), ("uniform", 60, 140), ("uniform", 0, 2), ("fixed", 90), ("fixed", 2))
    wl = _wl("f32", pooling=("per_table", specs), B=130)
    batch = gen.make_batches(wl, 1)[0]
    tabs = gen.mixed_host_tables(wl)
    arena = _device_arena(wl)
    avg = gen.table_avg_len(wl, batch)
    total = int(sum(wl.dims))
    ref, bound = oracle.emb_bag_mixed(tabs, batch.indices, batch.offsets, wl.B, "mean")
    desc = emb.make_mixed_desc(wl.dims, wl.B, emb.EMB_F32, emb.EMB_MEAN, batch.num_lookups, 0,
                               int(np.diff(wl.table_byte_offsets()).max()), None, avg)
    n = emb.emb_bag_plan_forward_mixed(desc).num_launches
    assert n >= 3
    kinds = {emb.emb_bag_plan_forward_mixed(desc, which=w).kernel for w in range(n)}
    assert kinds == {emb.EMB_KERNEL_WAVE, emb.EMB_KERNEL_STREAM}
    out = torch.full((wl.B, total), float("nan"), dtype=torch.float32, device=DEV)
    emb.emb_bag_forward_mixed(desc, arena, to_dev(wl.table_byte_offsets()), to_dev(wl.out_offsets()),
                              to_dev(batch.indices), to_dev(batch.offsets), None, out)
    torch.cuda.synchronize()
    assert_close_to_oracle(out.cpu().numpy(), ref, bound, False, "mixed per-table lengths")


@pytest.mark.parametrize("pooling", [("uniform", 0, 3), ("uniform", 20, 60), ("uniform", 60, 100)])
def test_mixed_widths_with_more_tables_than_one_list_holds(oracle, pooling):
    """2,600 tables of four widths (three lanes-per-row classes, the narrowest with 1,300 tables):
    launches that take their tables from a list are cut into pieces of at most 1,024 tables
    (short bags), and a single wave launch over more tables than that keeps the natural block
    order (long bags)."""
    T = 2600
    dims = tuple((8, 16, 32, 64)[t % 4] for t in range(T))
    wl = gen.MixedWorkload(name="many", T=T, rows=(7,) * T, dims=dims, dtype="f32", B=33,
                           pooling=pooling, dists=(("uniform",),) * T, seed=0x5EED0C10)
    batch = gen.make_batches(wl, 1)[0]
    tabs = gen.mixed_host_tables(wl)
    arena = _device_arena(wl)
    desc = emb.make_mixed_desc(dims, wl.B, emb.EMB_F32, emb.EMB_SUM, batch.num_lookups, 0,
                               int(np.diff(wl.table_byte_offsets()).max()))
    n = emb.emb_bag_plan_forward_mixed(desc).num_launches
    # short bags: classes of 1300 + 650 + 650 tables -> 2 + 1 + 1 stream launches; mid-length bags:
    # the narrowest class streams (2 launches), the other 1300 tables share 2 wave launches
    assert n == (1 if pooling[1] == 60 else 4)
    ref, bound = oracle.emb_bag_mixed(tabs, batch.indices, batch.offsets, wl.B, "sum")
    with tuning(xcd_remap=1):
        got = _forward(wl, arena, batch, "sum").cpu().numpy()
    assert_close_to_oracle(got, ref, bound, False, f"2600 tables/{pooling}")


@pytest.mark.parametrize("dtype", ["f32", "bf16", "u8row"])
@pytest.mark.parametrize("pooling", [("fixed", 1), ("uniform", 0, 5),
                                     ("per_table", (("fixed", 1), ("uniform", 50, 90), ("uniform", 0, 2)))])
def test_fused_launch_equals_the_separate_launches(oracle, dtype, pooling):
    """A split mixed-width call runs as one fused launch (consecutive workgroup ranges run what
    the separate launches would): same bits as the separate launches, in every mode, with and
    without weights, hints and the XCD-affine order, and within tolerance of the oracle."""
    for weighted in (False, True):
        wl = _wl(dtype, pooling=pooling, weighted=weighted, B=389)
        batch = gen.make_batches(wl, 1)[0]
        tabs = gen.mixed_host_tables(wl)
        arena = _device_arena(wl)
        avg = gen.table_avg_len(wl, batch) if pooling[0] == "per_table" else None
        total = int(sum(wl.dims))
        hints = to_dev((np.arange(wl.T) % 2).astype(np.uint8))
        boff, ooff = to_dev(wl.table_byte_offsets()), to_dev(wl.out_offsets())
        idx, off, w = to_dev(batch.indices), to_dev(batch.offsets), to_dev(batch.weights)
        for mode in (("sum",) if weighted else ("sum", "mean")):
            desc = emb.make_mixed_desc(wl.dims, wl.B, EDT[dtype], emb.MODES[mode], batch.num_lookups, 0,
                                       int(np.diff(wl.table_byte_offsets()).max()), hints, avg)
            ref, bound = oracle.emb_bag_mixed(tabs, batch.indices, batch.offsets, wl.B, mode,
                                              weights=batch.weights)

            def run():
                out = torch.full((wl.B, total), float("nan"), dtype=torch.float32, device=DEV)
                emb.emb_bag_forward_mixed(desc, arena, boff, ooff, idx, off, w, out)
                torch.cuda.synchronize()
                return out.cpu().numpy()

            for kw in (dict(), dict(xcd_remap=1), dict(depth=8), dict(depth=4, bags_per_group=2)):
                with tuning(fuse=1, **kw):
                    plan = emb.emb_bag_plan_forward_mixed(desc, weighted)
                    assert plan.num_launches >= 2 and plan.fused == 1
                    blocks = [emb.emb_bag_plan_forward_mixed(desc, weighted, which=k).grid_blocks
                              for k in range(plan.num_launches)]
                    assert plan.fused_grid_blocks == sum(-(-b // 8) * 8 for b in blocks)
                    fused = run()
                with tuning(fuse=0, **kw):
                    assert emb.emb_bag_plan_forward_mixed(desc, weighted).fused == 0
                    separate = run()
                what = f"fused/{dtype}/{pooling[0]}/{mode}/w{int(weighted)}/{kw}"
                assert np.array_equal(fused.view(np.uint32), separate.view(np.uint32)), what
                assert_close_to_oracle(fused, ref, bound, dtype != "f32", what)


def test_fused_launch_replays_from_a_graph_and_respects_the_occupancy_cap(oracle):
    wl = _wl("f32", pooling=("uniform", 0, 4), B=300)
    batch = gen.make_batches(wl, 1)[0]
    tabs = gen.mixed_host_tables(wl)
    arena = _device_arena(wl)
    ref, bound = oracle.emb_bag_mixed(tabs, batch.indices, batch.offsets, wl.B, "sum")
    with tuning(blocks_per_cu=2):
        got = _forward(wl, arena, batch, "sum").cpu().numpy()
    assert_close_to_oracle(got, ref, bound, False, "fused, 2 workgroups per CU")
    total = int(sum(wl.dims))
    desc = emb.make_mixed_desc(wl.dims, wl.B, emb.EMB_F32, emb.EMB_SUM, batch.num_lookups, 0,
                               int(np.diff(wl.table_byte_offsets()).max()))
    assert emb.emb_bag_plan_forward_mixed(desc).fused == 1
    boff, ooff = to_dev(wl.table_byte_offsets()), to_dev(wl.out_offsets())
    idx, off = to_dev(batch.indices), to_dev(batch.offsets)
    out = torch.zeros((wl.B, total), dtype=torch.float32, device=DEV)
    stream = torch.cuda.Stream()
    stream.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(stream):
        emb.emb_bag_forward_mixed(desc, arena, boff, ooff, idx, off, None, out, stream.cuda_stream)
    stream.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=stream):
        emb.emb_bag_forward_mixed(desc, arena, boff, ooff, idx, off, None, out,
                                  torch.cuda.current_stream().cuda_stream)
    for _ in range(3):
        out.fill_(float("nan"))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert np.array_equal(out.cpu().numpy().view(np.uint32), got.view(np.uint32))
