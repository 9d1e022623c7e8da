"""GPU parity for the short-bag (stream) kernel: a lane group streams several consecutive bags.
Every case forces the kernel on ("stream" = 1) and compares with the CPU oracle; since a bag is
always added up in the order of its lookups, the result must not depend on the bags per group,
the depth or the block order, which is checked bit for bit."""
import numpy as np
import pytest
import torch

from inputgen import gen
from gpu_harness import DEV, assert_close_to_oracle, forward, to_dev, tuning, upload_arena

pytestmark = pytest.mark.gpu

SMALL = ["tiny", "small_f32_d64", "small_f32_d128", "small_f16_d256", "small_bf16_d256",
         "small_u8_d120", "small_u8_d504"]


def _problem(name, **over):
    wl = gen.with_overrides(gen.workload(name), **over) if over else gen.workload(name)
    return wl, gen.make_batches(wl, 1)[0], gen.host_arena(wl)


@pytest.mark.parametrize("name", SMALL)
@pytest.mark.parametrize("mode", ["sum", "mean"])
def test_stream_kernel_matches_oracle(oracle, name, mode):
    wl, batch, arena = _problem(name)
    ref, bound = oracle.emb_bag(arena, wl.table_offsets(), batch.indices, batch.offsets, wl.B, mode)
    dev = upload_arena(arena)
    first = None
    for kw in (dict(), dict(bags_per_group=1), dict(bags_per_group=2), dict(bags_per_group=3),
               dict(bags_per_group=7, depth=4), dict(bags_per_group=63, depth=8),
               dict(bags_per_group=5, xcd_remap=1), dict(bags_per_group=2, blocks_per_cu=2),
               dict(addressing=1), dict(addressing=1, bags_per_group=3, depth=8)):   # 64-bit rows
        with tuning(stream=1, **kw):
            got = forward(dev, wl.table_offsets(), batch.indices, batch.offsets, wl.B,
                          mode).cpu().numpy()
        assert_close_to_oracle(got, ref, bound, wl.dtype != "f32", f"stream/{name}/{mode}/{kw}")
        if first is None:
            first = got
        else:
            assert np.array_equal(got, first), kw


@pytest.mark.parametrize("name", SMALL)
def test_stream_kernel_short_and_empty_bags(oracle, name):
    """Pooling 0..3: most bags hold one or two lookups, a quarter are empty."""
    wl, batch, arena = _problem(name, pooling=("uniform", 0, 3))
    dev = upload_arena(arena)
    for mode in ("sum", "mean"):
        ref, bound = oracle.emb_bag(arena, wl.table_offsets(), batch.indices, batch.offsets, wl.B,
                                    mode)
        for m in (0, 1, 3, 15):
            for addressing in (0, 1):
                with tuning(stream=1, bags_per_group=m, addressing=addressing):
                    got = forward(dev, wl.table_offsets(), batch.indices, batch.offsets, wl.B,
                                  mode).cpu().numpy()
                assert_close_to_oracle(got, ref, bound, wl.dtype != "f32",
                                       f"short/{name}/{mode}/M{m}/addressing {addressing}")


@pytest.mark.parametrize("name", ["small_f32_d64", "small_f32_d128", "small_f16_d256",
                                  "small_bf16_d256", "small_u8_d120"])
def test_stream_kernel_integer_tables_bit_exact_and_equal_to_wave_kernel(oracle, name):
    wl, batch, arena = _problem(name, kind=gen.KIND_INT)
    ref, _ = oracle.emb_bag(arena, wl.table_offsets(), batch.indices, batch.offsets, wl.B, "sum")
    dev = upload_arena(arena)
    with tuning(stream=1):
        s = forward(dev, wl.table_offsets(), batch.indices, batch.offsets, wl.B).cpu().numpy()
    with tuning(stream=0):
        w = forward(dev, wl.table_offsets(), batch.indices, batch.offsets, wl.B).cpu().numpy()
    assert np.array_equal(s.astype(np.float64), ref)
    assert np.array_equal(s, w)


@pytest.mark.parametrize("name", ["small_f32_d64", "small_f16_d256", "small_bf16_d256",
                                  "small_u8_d120"])
def test_stream_kernel_per_sample_weights(oracle, name):
    wl, batch, arena = _problem(name, weighted=True)
    ref, bound = oracle.emb_bag(arena, wl.table_offsets(), batch.indices, batch.offsets, wl.B,
                                "sum", weights=batch.weights)
    for m, addressing in ((0, 0), (2, 0), (6, 0), (0, 1), (5, 1)):
        with tuning(stream=1, bags_per_group=m, addressing=addressing):
            got = forward(upload_arena(arena), wl.table_offsets(), batch.indices, batch.offsets,
                          wl.B, weights=batch.weights).cpu().numpy()
        assert_close_to_oracle(got, ref, bound, wl.dtype != "f32",
                               f"stream weighted/{name}/M{m}/addressing {addressing}")


@pytest.mark.parametrize("D,dtype", [(4, "f32"), (12, "f32"), (32, "f32"), (96, "f32"), (200, "f32"),
                                     (256, "f32"), (8, "f16"), (24, "f16"), (264, "f16"),
                                     (512, "bf16"), (8, "u8row"), (24, "u8row"), (248, "u8row"),
                                     (1016, "u8row")])
@pytest.mark.parametrize("B", [1, 2, 53])
def test_stream_kernel_row_widths_and_ragged_batches(oracle, D, dtype, B):
    """Every lanes-per-row class, rows that do not fill their lanes, and batches that leave the
    last wavefront and the last group with fewer bags than the others."""
    wl = gen.Workload(name="w", T=3, rows=(300, 17, 1), D=D, dtype=dtype, B=B,
                      pooling=("uniform", 0, 9), dists=(("uniform",),) * 3, seed=0x5EED0E00 + D)
    batch = gen.make_batches(wl, 1)[0]
    arena = gen.host_arena(wl)
    dev = upload_arena(arena)
    for mode in ("sum", "mean"):
        ref, bound = oracle.emb_bag(arena, wl.table_offsets(), batch.indices, batch.offsets, wl.B,
                                    mode)
        for m, addressing in ((0, 0), (1, 0), (3, 0), (2, 1)):
            with tuning(stream=1, bags_per_group=m, addressing=addressing):
                got = forward(dev, wl.table_offsets(), batch.indices, batch.offsets, wl.B, mode,
                              out_ld=3 * D + 8, fill=-3.0).cpu().numpy()
            assert np.all(got[:, 3 * D:] == -3.0)
            assert_close_to_oracle(got[:, :3 * D], ref, bound, dtype != "f32",
                                   f"widths/{dtype}/D{D}/B{B}/{mode}/M{m}/addressing {addressing}")


def test_stream_kernel_all_bags_empty_and_single_lookup():
    wl = gen.workload("small_f32_d64")
    arena = upload_arena(gen.host_arena(wl))
    off = np.zeros(wl.T * wl.B + 1, np.int64)
    with tuning(stream=1):
        z = forward(arena, wl.table_offsets(), np.zeros(0, np.int64), off, wl.B, "mean").cpu().numpy()
    assert np.all(z == 0) and not np.signbit(z).any()
    off[-1] = 1                                            # one lookup, in the very last bag
    with tuning(stream=1):
        one = forward(arena, wl.table_offsets(), np.array([5], np.int64), off, wl.B).cpu().numpy()
    host = gen.host_arena(wl)
    row = host[wl.table_offsets()[wl.T - 1] + 5]
    assert np.array_equal(one[wl.B - 1, (wl.T - 1) * wl.D:], row)
    one[wl.B - 1, (wl.T - 1) * wl.D:] = 0
    assert np.all(one == 0)


def test_stream_kernel_bad_indices_and_malformed_offsets(oracle):
    """Invalid row ids contribute zero; a wavefront that sees bag bounds out of order treats its
    bags one by one like the wave kernel.  Integer tables make every sum exact, so the two
    kernels must agree bit for bit whatever the order of the additions."""
    wl, batch, arena = _problem("small_f32_d128", kind=gen.KIND_INT)
    toff = wl.table_offsets()
    rng = np.random.default_rng(11)
    idx = batch.indices.copy()
    pos = rng.choice(len(idx), size=60, replace=False)
    table_of = np.repeat(np.arange(wl.T), np.diff(batch.offsets[::wl.B]))
    idx[pos] = np.where(rng.random(60) < 0.5, -1 - rng.integers(0, 5, 60),
                        np.asarray(wl.rows)[table_of[pos]] + rng.integers(0, 3, 60))
    w = np.ones(len(idx), np.float32)
    w[pos] = 0.0
    ref, bound = oracle.emb_bag(arena, toff, batch.indices, batch.offsets, wl.B, "sum", weights=w)
    dev = upload_arena(arena)
    for addressing in (0, 1):     # (64-bit rows: a row that does not exist is not read at all)
        with tuning(stream=1, addressing=addressing):
            got = forward(dev, toff, idx, batch.offsets, wl.B).cpu().numpy()
        assert_close_to_oracle(got, ref, bound, False, f"stream/bad indices/addressing {addressing}")
    off = batch.offsets.copy()
    for g in (10, 11, 200, len(off) - 3):
        off[g + 1] = max(off[g] - 3, 0)                   # decreasing pairs
    off[3] = -(1 << 40)
    off[-1] = 1 << 40
    for m, addressing in ((0, 0), (1, 0), (4, 0), (2, 1)):
        with tuning(stream=1, bags_per_group=m, addressing=addressing):
            s = forward(dev, toff, batch.indices, off, wl.B).cpu().numpy()
        with tuning(stream=0):
            v = forward(dev, toff, batch.indices, off, wl.B).cpu().numpy()
        assert np.isfinite(s).all() and np.array_equal(s, v), (m, addressing)


def test_stream_kernel_group_of_2_pow_25_lookups_takes_the_slow_path(oracle):
    """A lane group whose bags hold 2^25 lookups or more cannot use 26-bit relative positions."""
    n = (1 << 25) + 5
    R, D = 1000, 4
    rng = np.random.default_rng(3)
    host = rng.integers(-3, 4, size=(R, D)).astype(np.float32)
    idx = rng.integers(0, R, size=n + 3).astype(np.int64)
    off = np.array([0, n, n + 3, n + 3], np.int64)
    ref, bound = oracle.emb_bag(host, np.array([0, R], np.int64), idx, off, 3, "mean")
    with tuning(stream=1):
        got = forward(upload_arena(host), np.array([0, R], np.int64), idx, off, 3, "mean").cpu().numpy()
    err = np.abs(got - ref)
    assert np.all(err[0] <= 1e-3 * np.maximum(bound[0], 1e-30))       # 33 M fp32 additions
    assert_close_to_oracle(got[1:], ref[1:], bound[1:], False, "after the long bag")


def test_stream_kernel_is_chosen_by_average_bag_length(oracle):
    """Automatic choice for 512-byte rows (two rows per wave load): the stream kernel below an
    average of 6 lookups per bag, the wave kernel from there on.  The two kernels round
    differently on non-integer tables, which is how the choice is observed."""
    runs = {}
    for L, expect in ((5, "stream"), (6, "wave"), (40, "wave")):
        wl, batch, arena = _problem("small_f32_d128", pooling=("fixed", L))
        dev = upload_arena(arena)
        for key, kw in (("auto", dict()), ("stream", dict(stream=1)), ("wave", dict(stream=0))):
            with tuning(**kw):
                runs[key] = forward(dev, wl.table_offsets(), batch.indices, batch.offsets,
                                    wl.B).cpu().numpy()
        assert not np.array_equal(runs["stream"], runs["wave"])
        assert np.array_equal(runs["auto"], runs[expect]), (L, expect)


def test_stream_kernel_replays_from_a_hip_graph(oracle):
    wl, batch, arena = _problem("small_f32_d64")
    ref, bound = oracle.emb_bag(arena, wl.table_offsets(), batch.indices, batch.offsets, wl.B)
    import paper_2410_22249_amd as emb
    dev = upload_arena(arena)
    toff, idx, off = to_dev(wl.table_offsets()), to_dev(batch.indices), to_dev(batch.offsets)
    out = torch.empty((wl.B, wl.T * wl.D), dtype=torch.float32, device=DEV)
    desc = emb.make_desc(wl.T, wl.B, wl.D, emb.EMB_F32, emb.EMB_SUM, batch.num_lookups, 0, max(wl.rows))
    with tuning(stream=1):
        stream = torch.cuda.Stream()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=stream):
            emb.emb_bag_forward(desc, dev, toff, idx, off, None, out, stream)
    for _ in range(3):
        out.fill_(-1.0)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert_close_to_oracle(out.cpu().numpy(), ref, bound, False, "stream graph replay")


@pytest.mark.parametrize("name", ["small_f32_d64", "small_f16_d256", "small_u8_d120"])
def test_per_table_bag_lengths_give_two_launches_and_the_same_result(oracle, name):
    """Tables with one lookup per bag next to tables with long bags: with table_avg_len the call
    is planned as a stream launch plus a wave launch; the result still matches the oracle."""
    import paper_2410_22249_amd as emb
    specs = (("fixed", 1), ("uniform", 60, 140), ("uniform", 0, 2), ("fixed", 90))
    wl, batch, arena = _problem(name, pooling=("per_table", specs), B=150)
    avg = gen.table_avg_len(wl, batch)
    dev = upload_arena(arena)
    toff, idx, off = to_dev(wl.table_offsets()), to_dev(batch.indices), to_dev(batch.offsets)
    for mode in ("sum", "mean"):
        ref, bound = oracle.emb_bag(arena, wl.table_offsets(), batch.indices, batch.offsets, wl.B, mode)
        desc = emb.make_desc(wl.T, wl.B, wl.D, emb.DTYPES[wl.dtype], emb.MODES[mode],
                             batch.num_lookups, 0, max(wl.rows), None, avg)
        assert emb.emb_bag_plan_forward(desc).num_launches == 2
        for kw in (dict(), dict(xcd_remap=1), dict(depth=8)):
            out = torch.full((wl.B, wl.T * wl.D), float("nan"), dtype=torch.float32, device=DEV)
            with tuning(**kw):
                emb.emb_bag_forward(desc, dev, toff, idx, off, None, out)
            torch.cuda.synchronize()
            assert_close_to_oracle(out.cpu().numpy(), ref, bound, wl.dtype != "f32",
                                   f"per-table lengths/{name}/{mode}/{kw}")
        # both launches of the call are captured into one HIP graph and replay correctly
        stream = torch.cuda.Stream()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=stream):
            emb.emb_bag_forward(desc, dev, toff, idx, off, None, out, stream)
        for _ in range(2):
            out.fill_(float("nan"))
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            assert_close_to_oracle(out.cpu().numpy(), ref, bound, wl.dtype != "f32",
                                   f"per-table lengths/{name}/{mode}/graph")


def test_per_table_bag_lengths_with_more_tables_than_one_list_holds(oracle):
    """2,600 tables, every other one with one-lookup bags: 1,300 tables per kernel, so each side is
    cut into launches of at most 1,024 listed tables."""
    import paper_2410_22249_amd as emb
    T = 2600
    specs = (("fixed", 1), ("uniform", 40, 80))
    wl = gen.Workload(name="many", T=T, rows=(9,) * T, D=8, dtype="f32", B=21,
                      pooling=("per_table", specs), dists=(("uniform",),) * T, seed=0x5EED0E50)
    batch = gen.make_batches(wl, 1)[0]
    arena = gen.host_arena(wl)
    ref, bound = oracle.emb_bag(arena, wl.table_offsets(), batch.indices, batch.offsets, wl.B, "sum")
    desc = emb.make_desc(T, wl.B, wl.D, emb.EMB_F32, emb.EMB_SUM, batch.num_lookups, 0, 9, None,
                         gen.table_avg_len(wl, batch))
    n = emb.emb_bag_plan_forward(desc).num_launches
    assert n == 4
    sizes = sorted(emb.emb_bag_plan_forward(desc, which=w).tables for w in range(n))
    assert sizes == [276, 276, 1024, 1024]
    out = torch.full((wl.B, T * wl.D), float("nan"), dtype=torch.float32, device=DEV)
    with tuning(xcd_remap=1):
        emb.emb_bag_forward(desc, upload_arena(arena), to_dev(wl.table_offsets()),
                            to_dev(batch.indices), to_dev(batch.offsets), None, out)
    torch.cuda.synchronize()
    assert_close_to_oracle(out.cpu().numpy(), ref, bound, False, "2600 tables, per-table lengths")


def test_one_launch_per_table_gives_the_same_bits(oracle):
    """"per_table_launch" reproduces the paper's launch structure (one kernel per table); the
    result is that of the single launch, bit for bit."""
    for name, pooling in (("small_f32_d128", None), ("small_f32_d64", ("uniform", 0, 4))):
        wl, batch, arena = _problem(name, **({"pooling": pooling} if pooling else {}))
        dev = upload_arena(arena)
        one = forward(dev, wl.table_offsets(), batch.indices, batch.offsets, wl.B).cpu().numpy()
        with tuning(per_table_launch=1):
            many = forward(dev, wl.table_offsets(), batch.indices, batch.offsets, wl.B).cpu().numpy()
        assert np.array_equal(one, many), name


@pytest.mark.parametrize("name", ["small_f32_d64", "small_f32_d128", "small_f16_d256",
                                  "small_bf16_d256", "small_u8_d120", "small_fp8_d120"])
def test_fused_launch_of_a_uniform_call_equals_its_two_launches(oracle, name):
    """With table_avg_len a call with short-bag and long-bag tables is one fused launch (wave
    body, then stream body); it gives the bits of the two separate launches."""
    import paper_2410_22249_amd as emb
    specs = (("fixed", 1), ("uniform", 60, 140), ("uniform", 0, 2), ("fixed", 90), ("fixed", 2))
    for weighted in (False, True):
        wl, batch, arena = _problem(name, pooling=("per_table", specs), B=333, weighted=weighted)
        avg = gen.table_avg_len(wl, batch)
        dev = upload_arena(arena)
        hints = to_dev((np.arange(wl.T) % 2).astype(np.uint8))
        toff, idx, off = to_dev(wl.table_offsets()), to_dev(batch.indices), to_dev(batch.offsets)
        w = to_dev(batch.weights)
        for mode in (("sum",) if weighted else ("sum", "mean")):
            ref, bound = oracle.emb_bag(arena, wl.table_offsets(), batch.indices, batch.offsets,
                                        wl.B, mode, weights=batch.weights, codes=wl.codes)
            desc = emb.make_desc(wl.T, wl.B, wl.D, emb.DTYPES[wl.dtype], emb.MODES[mode],
                                 batch.num_lookups, 0, max(wl.rows), hints, avg)

            def run():
                out = torch.full((wl.B, wl.T * wl.D), float("nan"), dtype=torch.float32, device=DEV)
                emb.emb_bag_forward(desc, dev, toff, idx, off, w, out)
                torch.cuda.synchronize()
                return out.cpu().numpy()

            for kw in (dict(), dict(xcd_remap=1), dict(depth=8), dict(depth=4, bags_per_group=2)):
                with tuning(fuse=1, **kw):
                    plan = emb.emb_bag_plan_forward(desc, weighted)
                    assert plan.num_launches == 2 and plan.fused == 1
                    fused = run()
                with tuning(fuse=0, **kw):
                    assert emb.emb_bag_plan_forward(desc, weighted).fused == 0
                    separate = run()
                what = f"fused uniform/{name}/{mode}/w{int(weighted)}/{kw}"
                assert np.array_equal(fused.view(np.uint32), separate.view(np.uint32)), what
                assert_close_to_oracle(fused, ref, bound, wl.dtype != "f32", what)
            with tuning(depth=2):           # no fused kernel at this depth: two launches
                assert emb.emb_bag_plan_forward(desc, weighted).fused == 0
                assert_close_to_oracle(run(), ref, bound, wl.dtype != "f32", "depth 2")
