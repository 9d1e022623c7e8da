"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times.

The table arenas of the large configurations (up to 123 GB) do not fit in host memory, so the
oracle evaluates a sample of bags one by one: the generator rebuilds exactly the rows those bags
touch on the host (its values are a pure function of seed, row and column; the device fill is
checked bit for bit against that function in test_parity_gpu.py).  The sample holds random bags
plus the first and last bag of every table (table-boundary mistakes show there).  The smallest
configuration is checked whole, element by element.
"""
import numpy as np
import pytest
import torch

import paper_2410_22249_amd as emb
from inputgen import gen
from gpu_harness import DEV, assert_close_to_oracle, device_arena, forward, to_dev, tuning

pytestmark = pytest.mark.gpu


def _run(wl, batch, arena, toff):
    idx, off = to_dev(batch.indices), to_dev(batch.offsets)
    w = to_dev(batch.weights)
    out = torch.full((wl.B, wl.T * wl.D), float("nan"), dtype=torch.float32, device=DEV)
    # tables that differ in pooling: their bag lengths go in, as in the benchmark
    avg_len = gen.table_avg_len(wl, batch) if wl.pooling[0] == "per_table" else None
    desc = emb.make_desc(wl.T, wl.B, wl.D, emb.DTYPES[wl.dtype],
                         emb.MODES[wl.mode], batch.num_lookups, 0,
                         max(wl.rows), None, avg_len)
    emb.emb_bag_forward(desc, arena, toff, idx, off, w, out)
    bad = torch.zeros(1, dtype=torch.int64, device=DEV)
    emb.emb_bag_validate(desc, toff, idx, off, bad)
    torch.cuda.synchronize()
    assert int(bad.item()) == 0
    return out, (desc, idx, off, w)


def _sample_bags(wl, n, seed=2024):
    """`n` random bags plus the first and last bag of every table; n = "1%" stands for the plan
    of the benchmark configurations: every bag of four tables (the first, the last and two in
    between) plus a seeded 1 % of all bags."""
    rng = np.random.default_rng(seed)
    edge = np.concatenate([np.arange(wl.T) * wl.B, np.arange(wl.T) * wl.B + wl.B - 1])
    if n == "1%":
        whole = sorted({0, wl.T // 3, (2 * wl.T) // 3, wl.T - 1})
        full = np.concatenate([np.arange(t * wl.B, (t + 1) * wl.B) for t in whole])
        rand = rng.integers(0, wl.num_bags, size=max(1, wl.num_bags // 100))
        return np.unique(np.concatenate([full, rand, edge]))
    return np.unique(np.concatenate([rng.integers(0, wl.num_bags, size=n), edge]))


def test_cfg1_whole_output(oracle):
    wl = gen.workload("cfg1")
    batch = gen.make_batches(wl, 1)[0]
    arena = device_arena(wl)
    out, _ = _run(wl, batch, arena, to_dev(wl.table_offsets()))
    host = gen.host_arena(wl)
    assert np.array_equal(arena.cpu().numpy().view(np.uint8), host.view(np.uint8))
    ref, bound = oracle.emb_bag(host, wl.table_offsets(), batch.indices, batch.offsets, wl.B, wl.mode)
    assert_close_to_oracle(out.cpu().numpy(), ref, bound, False, "cfg1 whole")


@pytest.mark.parametrize("name,nsample", [("cfg2", "1%"), ("cfg3", "1%"), ("cfg4", "1%"),
                                          ("cfg5", "1%"), ("paper", 400), ("cfg3_weighted", 300),
                                          ("cfg3_u8", 300), ("onehot", 3000), ("short", 3000),
                                          ("cfg3_max", 300), ("cfg3_fp8", 300),
                                          ("paper_one_item", 300), ("paper_high", 300),
                                          ("paper_med", 300), ("paper_low", 300),
                                          ("paper_mix1", 300), ("paper_mix2", 300),
                                          ("paper_mix3", 300), ("hetero", 2000)])
def test_full_size_sampled_bags(oracle, name, nsample):
    print(f"\n[fullsize] {name}: generating", flush=True)
    wl = gen.workload(name)
    batch = gen.make_batches(wl, 1)[0]
    arena = device_arena(wl)
    toff = to_dev(wl.table_offsets())
    print(f"[fullsize] {name}: {batch.num_lookups} lookups, arena {wl.table_bytes / 1e9:.1f} GB", flush=True)
    out, (desc, idx, off, w) = _run(wl, batch, arena, toff)
    assert bool(torch.isfinite(out).all())                    # every bag was written
    # run-to-run determinism over the whole output
    out2 = torch.full_like(out, float("nan"))
    emb.emb_bag_forward(desc, arena, toff, idx, off, w, out2)
    torch.cuda.synchronize()
    assert torch.equal(out, out2)
    bags = _sample_bags(wl, nsample)
    small, ix, soff, wsmall = gen.compact_rows(wl, batch, bags)
    ref, bound, strict = oracle.emb_bag(small, np.array([0, len(small)], np.int64), ix, soff,
                                        len(bags), wl.mode, weights=wsmall, codes=wl.codes,
                                        strict=True)
    sel = torch.from_numpy(np.stack([bags % wl.B, bags // wl.B], 1)).to(DEV)
    got = out.view(wl.B, wl.T, wl.D)[sel[:, 0], sel[:, 1]].cpu().numpy()
    worst = assert_close_to_oracle(got, ref, bound, wl.dtype != "f32", f"{name} sampled",
                                   strict=strict)
    # hints from the device-side profiler: what the benchmark uses; classification as expected
    from oracle import reuse_oracle
    hints = torch.zeros(wl.T, dtype=torch.uint8, device=DEV)
    dup = torch.zeros(wl.T, dtype=torch.int32, device=DEV)
    used = torch.zeros(wl.T, dtype=torch.int32, device=DEV)
    emb.emb_bag_profile_reuse(desc, idx, off, 16384, -1, dup, used, hints)
    torch.cuda.synchronize()
    rd, ru, rh = reuse_oracle.profile_reuse(batch.indices, batch.offsets, wl.T, wl.B, 16384, 75,
                                            row_bytes=wl.row_bytes)
    assert np.array_equal(dup.cpu().numpy(), rd) and np.array_equal(used.cpu().numpy(), ru)
    assert np.array_equal(hints.cpu().numpy(), rh)
    # skewed tables stay cached; a uniform table streams when its rows outgrow the 256 MiB
    # memory-side cache or the batch draws a small part of it (the estimated share of repeated
    # lookups, draws / 2 rows, reaches the 7.5 % threshold at draws = 0.15 rows), and stays
    # cached when neither holds; tables within a factor of two of a threshold may fall on
    # either side
    per_table = np.diff(batch.offsets[::wl.B])
    for t, d in enumerate(wl.dists):
        table_bytes = wl.rows[t] * wl.row_bytes
        if d[0] != "uniform":
            assert rh[t] == 0, t
        elif table_bytes > (2 << 28) or per_table[t] < 0.075 * wl.rows[t]:
            assert rh[t] == 1, t
        elif table_bytes < (1 << 27) and per_table[t] > 0.3 * wl.rows[t]:
            assert rh[t] == 0, t
    hdesc = emb.make_desc(wl.T, wl.B, wl.D, emb.DTYPES[wl.dtype],
                          emb.MODES[wl.mode], batch.num_lookups,
                          0, max(wl.rows), hints, desc._avg_len_keepalive
                          if hasattr(desc, "_avg_len_keepalive") else None)
    emb.emb_bag_forward(hdesc, arena, toff, idx, off, w, out2)
    torch.cuda.synchronize()
    assert torch.equal(out, out2), "hints must not change results"
    # the alternative launch shapes give the same bits at full size too
    # ("short" runs the stream kernel, which 64-bit addressing would switch off; the wave kernel
    # adds a bag's rows in another order, so there the alternative is another group size)
    if name == "hetero":    # a fused launch of two kernel bodies: the launches taken apart
        alts = (dict(xcd_remap=1), dict(fuse=0))
    else:
        alts = (dict(xcd_remap=1), dict(bags_per_group=3, depth=8) if name == "short"
                else dict(addressing=1, depth=8), dict(station=1))   # (rows through LDS)
    for kw in alts:
        with tuning(**kw):
            emb.emb_bag_forward(desc, arena, toff, idx, off, w, out2)
            torch.cuda.synchronize()
        assert torch.equal(out, out2), kw
    print(f"[fullsize] {name}: {len(bags)} bags checked, max err/bound {worst:.3e}", flush=True)
    del arena, out, out2
    torch.cuda.empty_cache()


def test_many_tiny_bags_whole_output(oracle):
    """16.7 million bags of 0-2 lookups over 16-byte rows: the smallest row the ABI accepts (4 of the
    64 lanes per row, 16 rows per wave load), a launch of 4 million workgroups, whole output checked."""
    wl = gen.Workload(name="tiny_bags", T=64, rows=(50_000,) * 64, D=4, dtype="f32", B=1 << 18,
                      pooling=("uniform", 0, 2), dists=(("uniform",),) * 64, seed=0x5EED0900)
    batch = gen.make_batches(wl, 1)[0]
    arena = device_arena(wl)
    out, _ = _run(wl, batch, arena, to_dev(wl.table_offsets()))
    host = gen.host_arena(wl)
    ref, bound = oracle.emb_bag(host, wl.table_offsets(), batch.indices, batch.offsets, wl.B, "sum")
    assert_close_to_oracle(out.cpu().numpy(), ref, bound, False, "tiny bags")


def test_widest_rows(oracle):
    """64 KiB rows (the ABI's maximum): 64 column slabs per bag."""
    wl = gen.Workload(name="wide", T=2, rows=(300, 50), D=16384, dtype="f32", B=9,
                      pooling=("uniform", 0, 70), dists=(("uniform",), ("zipf", 1.1)), mode="mean",
                      seed=0x5EED0901)
    batch = gen.make_batches(wl, 1)[0]
    arena = device_arena(wl)
    out, _ = _run(wl, batch, arena, to_dev(wl.table_offsets()))
    host = gen.host_arena(wl)
    ref, bound = oracle.emb_bag(host, wl.table_offsets(), batch.indices, batch.offsets, wl.B, "mean")
    assert_close_to_oracle(out.cpu().numpy(), ref, bound, False, "64 KiB rows")
    wl16 = gen.with_overrides(wl, D=32768, dtype="f16", mode="sum")
    batch = gen.make_batches(wl16, 1)[0]
    arena = device_arena(wl16)
    out, _ = _run(wl16, batch, arena, to_dev(wl16.table_offsets()))
    host = gen.host_arena(wl16)
    ref, bound = oracle.emb_bag(host, wl16.table_offsets(), batch.indices, batch.offsets, wl16.B, "sum")
    assert_close_to_oracle(out.cpu().numpy(), ref, bound, True, "64 KiB f16 rows")


def test_more_than_2_pow_32_lookups_in_one_call():
    """Positions in `indices` beyond 2^32: 65,536 bags of 65,552 lookups (34 GB of indices).  The
    table has two rows, +1 and -1 in every element, and position p names row (p mod 32 >= 16),
    so every partial sum any lane group can form stays tiny and the result is exact: a bag that
    starts on a multiple of 32 ends with an unpaired run of +1 (sum 16), the others start with an
    unpaired run of -1 (sum -16)."""
    B, L = 1 << 16, (1 << 16) + 16
    n = B * L
    assert n > 1 << 32
    table = torch.tensor([[1.0] * 4, [-1.0] * 4], dtype=torch.float32, device=DEV)
    idx = torch.empty(n, dtype=torch.int64, device=DEV)
    step = 1 << 28
    for lo in range(0, n, step):                          # in pieces: bounded temporaries
        hi = min(n, lo + step)
        idx[lo:hi] = (torch.arange(lo, hi, device=DEV) % 32) >= 16
    off = to_dev(np.arange(B + 1, dtype=np.int64) * L)
    toff = to_dev(np.array([0, 2], np.int64))
    want_sum = np.where(np.arange(B) % 2 == 0, 16.0, -16.0).astype(np.float32)
    for kw in (dict(), dict(addressing=1), dict(stream=1, bags_per_group=2)):
        for mode in (emb.EMB_SUM, emb.EMB_MAX):
            out = torch.full((B, 4), float("nan"), dtype=torch.float32, device=DEV)
            desc = emb.make_desc(1, B, 4, emb.EMB_F32, mode, n, 0, 2)
            with tuning(**kw):
                emb.emb_bag_forward(desc, table, toff, idx, off, None, out)
            torch.cuda.synchronize()
            got = out.cpu().numpy()
            want = want_sum if mode == emb.EMB_SUM else np.ones(B, np.float32)
            assert np.array_equal(got, np.repeat(want[:, None], 4, axis=1)), (kw, mode)
    bad = torch.zeros(1, dtype=torch.int64, device=DEV)
    emb.emb_bag_validate(desc, toff, idx, off, bad)
    torch.cuda.synchronize()
    assert int(bad.item()) == 0
    idx[n - 3] = 2                                         # one invalid id beyond position 2^32
    emb.emb_bag_validate(desc, toff, idx, off, bad)
    torch.cuda.synchronize()
    assert int(bad.item()) == 1


def test_table_of_more_than_2_pow_31_rows(oracle):
    """Row ids beyond 2^31 and byte offsets beyond 2^35 inside ONE table (64-bit addressing; the
    table is far above the 3.5 GiB that buffer addressing covers)."""
    R = (1 << 31) + 1000
    wl = gen.Workload(name="tall", T=2, rows=(R, 10), D=4, dtype="f32", B=64,
                      pooling=("uniform", 0, 40), dists=(("uniform",), ("uniform",)), seed=0x5EED0A01)
    batch = gen.make_batches(wl, 1)[0]
    assert int(batch.indices.max()) > (1 << 31) - (1 << 27)     # lookups reach the far end
    assert int(batch.offsets[wl.B]) >= 64                        # table 0 owns the first lookups
    idx = batch.indices.copy()
    idx[:64] = np.arange(R - 64, R, dtype=np.int64)              # ... and the very last rows
    batch = gen.Batch(offsets=batch.offsets, indices=idx)
    arena = device_arena(wl)
    out, _ = _run(wl, batch, arena, to_dev(wl.table_offsets()))
    bags = np.arange(wl.num_bags)
    small, ix, soff, _ = gen.compact_rows(wl, batch, bags)
    ref, bound = oracle.emb_bag(small, np.array([0, len(small)], np.int64), ix, soff, len(bags), "sum")
    got = out.view(wl.B, wl.T, wl.D).permute(1, 0, 2).reshape(wl.num_bags, wl.D).cpu().numpy()
    assert_close_to_oracle(got, ref, bound, False, "table of 2^31 + 1000 rows")


@pytest.mark.parametrize("dtype,D,R", [("f32", 128, 7_000_000), ("f16", 64, 28_000_011)])
def test_buffer_addressing_beyond_2_pow_31_bytes(oracle, dtype, D, R):
    """One table between 2 GiB and 3.5 GiB under buffer addressing: 32-bit row offsets at and
    above 2^31 (as unsigned), the very last row, and ids at or beyond R (neutralised by the
    buffer's range check); the same input through 64-bit addressing must give the same bits."""
    wl = gen.Workload(name="buf3g", T=2, rows=(R, 1000), D=D, dtype=dtype, B=512,
                      pooling=("uniform", 1, 150), dists=(("uniform",), ("uniform",)), seed=0x5EED0B0F)
    row_bytes = D * (4 if dtype == "f32" else 2)
    assert (1 << 31) + (1 << 29) < R * row_bytes <= 0xE0000000
    batch = gen.make_batches(wl, 1)[0]
    idx = batch.indices.copy()
    n0 = int(batch.offsets[wl.B])                                # lookups of table 0
    assert n0 > 2000
    first_high = -(-(1 << 31) // row_bytes)                      # first row at byte offset >= 2^31
    idx[:32] = np.arange(R - 32, R)                              # the last rows
    idx[32:64] = np.arange(first_high - 16, first_high + 16)     # across 2^31
    bad = np.array([64, 100, n0 - 1])
    idx[bad] = [R, R + 7, (1 << 40) + 3]                         # at and beyond R: contribute nothing
    assert int((idx[:n0] * row_bytes >= (3 << 30)).sum()) > 100  # the uniform draw reaches past 3 GiB
    arena = device_arena(wl)
    toff = wl.table_offsets()
    with tuning(addressing=0):
        plan = emb.emb_bag_plan_forward(emb.make_desc(wl.T, wl.B, wl.D, emb.DTYPES[dtype],
                                                      emb.MODES["sum"], len(idx), 0, R))
        assert plan.buffer_addressing == 1
        got_buf = forward(arena, toff, idx, batch.offsets, wl.B, max_table_rows=R)
    with tuning(addressing=1):
        got_flat = forward(arena, toff, idx, batch.offsets, wl.B, max_table_rows=R)
    assert torch.equal(got_buf.view(torch.int32), got_flat.view(torch.int32))
    clean, w = idx.copy(), np.ones(len(idx), np.float32)
    clean[bad], w[bad] = 0, 0.0
    bags = np.arange(wl.num_bags)
    small, ix, soff, ws = gen.compact_rows(wl, gen.Batch(offsets=batch.offsets, indices=clean, weights=w), bags)
    ref, bound = oracle.emb_bag(small, np.array([0, len(small)], np.int64), ix, soff, len(bags), "sum",
                                weights=ws)
    got = got_buf.view(wl.B, wl.T, wl.D).permute(1, 0, 2).reshape(wl.num_bags, wl.D).cpu().numpy()
    assert_close_to_oracle(got, ref, bound, dtype == "f16", f"buffer addressing, {dtype} table of {R * row_bytes} bytes")


def test_short_bags_on_a_table_beyond_buffer_addressing(oracle):
    """A 4.1 GB table with one or two lookups per bag: the short-bag kernel with 64-bit row
    addresses (the table is beyond the 3.5 GiB a buffer covers); the last rows, ids at and
    beyond R; the one-wavefront-per-bag kernel must give the same sums to rounding."""
    R = 8_000_000
    wl = gen.Workload(name="big_short", T=2, rows=(R, 1000), D=128, dtype="f32", B=20_000,
                      pooling=("uniform", 0, 2), dists=(("uniform",), ("uniform",)), seed=0x5EED0B10)
    batch = gen.make_batches(wl, 1)[0]
    idx = batch.indices.copy()
    n0 = int(batch.offsets[wl.B])
    idx[:16] = np.arange(R - 16, R)
    bad = np.array([16, 17, n0 - 1])
    idx[bad] = [R, -1, (1 << 40) + 3]
    assert int((idx[:n0] * 512 >= (7 << 29)).sum()) > 100          # lookups beyond 3.5 GiB
    arena = device_arena(wl)
    toff = wl.table_offsets()
    desc = emb.make_desc(wl.T, wl.B, wl.D, emb.EMB_F32, emb.EMB_SUM, len(idx), 0, R)
    plan = emb.emb_bag_plan_forward(desc)
    assert plan.kernel == emb.EMB_KERNEL_STREAM and plan.buffer_addressing == 0
    got_stream = forward(arena, toff, idx, batch.offsets, wl.B, max_table_rows=R)
    with tuning(stream=0):
        got_wave = forward(arena, toff, idx, batch.offsets, wl.B, max_table_rows=R)
    clean, w = idx.copy(), np.ones(len(idx), np.float32)
    clean[bad], w[bad] = 0, 0.0
    bags = np.arange(wl.num_bags)
    small, ix, soff, ws = gen.compact_rows(wl, gen.Batch(offsets=batch.offsets, indices=clean, weights=w), bags)
    ref, bound = oracle.emb_bag(small, np.array([0, len(small)], np.int64), ix, soff, len(bags), "sum",
                                weights=ws)
    for what, out in (("stream", got_stream), ("wave", got_wave)):
        got = out.view(wl.B, wl.T, wl.D).permute(1, 0, 2).reshape(wl.num_bags, wl.D).cpu().numpy()
        assert_close_to_oracle(got, ref, bound, False, f"4.1 GB table, short bags, {what} kernel")


def test_the_largest_grid_a_launch_can_hold(oracle):
    """67,108,800 bags with a wavefront each are 16,777,200 workgroups, the most one dispatch
    takes (its work-items are counted in 32 bits); the XCD-affine order would pad that to 2^24
    and steps back to the natural order.  Nearly all bags are empty; one in 4099 holds 1-3
    lookups.  Integer-valued rows make every sum exact, so the result is compared bit for bit."""
    T, D, R = 64, 4, 1000
    B = ((1 << 24) - 1) * 4 // T
    nb = T * B
    rng = np.random.default_rng(77)
    host = rng.integers(-8, 9, size=(T * R, D)).astype(np.float32)
    arena = to_dev(host)
    toff = np.arange(T + 1, dtype=np.int64) * R
    lengths = torch.zeros(nb, dtype=torch.int64, device=DEV)
    some = torch.arange(0, nb, 4099, device=DEV)
    lengths[some] = some % 3 + 1
    lengths[-1] = 3
    off = torch.zeros(nb + 1, dtype=torch.int64, device=DEV)
    torch.cumsum(lengths, 0, out=off[1:])
    NL = int(off[-1].item())
    idx_host = rng.integers(0, R, size=NL).astype(np.int64)
    idx = to_dev(idx_host)
    desc = emb.make_desc(T, B, D, emb.EMB_F32, emb.EMB_SUM, NL, 0, R)
    out = torch.full((B, T * D), float("nan"), dtype=torch.float32, device=DEV)
    print(f"\n[fullsize] largest grid: {nb} bags, {NL} lookups", flush=True)
    with tuning(stream=0, bags_per_wave=1):
        plan = emb.emb_bag_plan_forward(desc)
        assert plan.kernel == emb.EMB_KERNEL_WAVE and plan.grid_blocks == nb // 4 == (1 << 24) - 16
        assert plan.xcd_pieces == 0
        emb.emb_bag_forward(desc, arena, to_dev(toff), idx, off, None, out)
    bad = torch.zeros(1, dtype=torch.int64, device=DEV)
    emb.emb_bag_validate(desc, to_dev(toff), idx, off, bad)
    torch.cuda.synchronize()
    assert int(bad.item()) == 0
    # the non-empty bags against the oracle (one table of all rows, global row ids)
    bags_dev = lengths.nonzero().flatten()
    bags = bags_dev.cpu().numpy()
    lens = lengths[bags_dev].cpu().numpy()
    soff = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    assert soff[-1] == NL
    gidx = idx_host + np.repeat(toff[bags // B], lens)
    ref, _ = oracle.emb_bag(host, np.array([0, T * R], np.int64), gidx, soff, len(bags), "sum")
    sel_b, sel_t = torch.from_numpy(bags % B).to(DEV), torch.from_numpy(bags // B).to(DEV)
    got = out.view(B, T, D)[sel_b, sel_t]
    assert np.array_equal(got.cpu().numpy().astype(np.float64), ref)
    # ... and exact zeros everywhere else (a bag left unwritten would still hold its NaN)
    assert int(torch.count_nonzero(out).item()) == int(torch.count_nonzero(got).item())
    # the automatic choice (short bags: the stream kernel, far fewer wavefronts) agrees
    out2 = torch.full_like(out, float("nan"))
    plan = emb.emb_bag_plan_forward(desc)
    assert plan.kernel == emb.EMB_KERNEL_STREAM
    emb.emb_bag_forward(desc, arena, to_dev(toff), idx, off, None, out2)
    torch.cuda.synchronize()
    assert torch.equal(out, out2)
    # one bag more per table is refused before anything is launched
    big = emb.make_desc(T, B + 1, D, emb.EMB_F32, emb.EMB_SUM, NL, 0, R)
    with tuning(stream=0, bags_per_wave=1):
        with pytest.raises(emb.EmbBagError) as ex:
            emb.emb_bag_forward(big, arena, to_dev(toff), idx, off, None, out)
    assert ex.value.status == -7
