"""Host logic of the forward calls, observed through emb_bag_plan_forward* (no GPU needed): which
kernel is chosen, with which depth and group size, and how the grid maps workgroups to (table,
wavefront) - simulated here from the plan, following the description in include/emb_bag.h."""
import numpy as np
import pytest

import paper_2410_22249_amd as emb
from tuning_ctx import tuning


def _plan(T, B, D, L, dtype=emb.EMB_F32, mode=emb.EMB_SUM, rows=1_000_000, weights=False, order=False):
    desc = emb.make_desc(T, B, D, dtype, mode, int(T * B * L), 0, rows)
    return emb.emb_bag_plan_forward(desc, weights, order)


def test_plan_of_the_benchmark_configurations():
    p = _plan(60, 4096, 128, 80, rows=4_000_000).as_dict()           # cfg3
    assert p["kernel"] == emb.EMB_KERNEL_WAVE and p["lanes_per_row"] == 32 and p["depth"] == 8
    assert p["buffer_addressing"] == 1 and p["wavefronts"] == 60 * 4096
    assert p["xcd_pieces"] == 2 and p["grid_blocks"] == 60 * 2 * 512
    p = _plan(26, 2048, 64, 20.5).as_dict()                          # cfg2: average 20.5 >= 12
    assert p["kernel"] == emb.EMB_KERNEL_WAVE and p["lanes_per_row"] == 16 and p["depth"] == 4
    p = _plan(8, 256, 64, 20, rows=100_000).as_dict()                # cfg1: small launch
    assert p["xcd_pieces"] == 0 and p["grid_blocks"] == 8 * 256 // 4
    p = _plan(100, 8192, 256, 50.5, dtype=emb.EMB_F16, rows=2_000_000).as_dict()   # cfg5
    assert p["kernel"] == emb.EMB_KERNEL_WAVE and p["lanes_per_row"] == 32 and p["depth"] == 4


@pytest.mark.parametrize("D,threshold", [(32, 24), (64, 12), (128, 6), (256, 3)])
def test_stream_kernel_threshold_is_three_row_loads_per_bag(D, threshold):
    B = 40_000
    below = _plan(26, B, D, threshold - 0.01)
    at = _plan(26, B, D, threshold)
    assert below.kernel == emb.EMB_KERNEL_STREAM and at.kernel == emb.EMB_KERNEL_WAVE
    assert below.bags_per_group >= 1 and at.bags_per_group == 0
    # every pooling mode streams short bags
    assert _plan(26, B, D, 1, mode=emb.EMB_MAX).kernel == emb.EMB_KERNEL_STREAM
    assert _plan(26, B, D, threshold, mode=emb.EMB_MAX).kernel == emb.EMB_KERNEL_WAVE
    # ... with either addressing (no row bound, or tables beyond 3.5 GiB: 64-bit)
    for kw in (dict(rows=0), dict(rows=1 << 40)):
        p = _plan(26, B, D, 1, **kw)
        assert p.kernel == emb.EMB_KERNEL_STREAM and p.buffer_addressing == 0
    with tuning(addressing=1):
        p = _plan(26, B, D, 1)
        assert p.kernel == emb.EMB_KERNEL_STREAM and p.buffer_addressing == 0
    # what rules the stream kernel out whatever the bag length
    with tuning(stream=0):
        assert _plan(26, B, D, 1).kernel == emb.EMB_KERNEL_WAVE
    with tuning(stream=1):
        assert _plan(26, B, D, 500).kernel == emb.EMB_KERNEL_STREAM
    assert _plan(26, B, 320, 1).kernel == emb.EMB_KERNEL_WAVE                   # rows above 1 KiB


def test_bags_per_group_rule():
    big = 200_000
    assert _plan(26, big, 64, 1).bags_per_group == 4
    assert _plan(26, big, 64, 2).bags_per_group == 2
    assert _plan(26, big, 64, 3).bags_per_group == 1
    assert _plan(26, big, 64, 8).bags_per_group == 1
    assert _plan(26, big, 4, 1).bags_per_group == 3           # 4 lanes per row hold 4 bag bounds
    # a launch that would fall below 1024 wavefronts halves the group instead
    p = _plan(2, 3000, 64, 1)
    assert p.bags_per_group in (1, 2) and p.wavefronts >= 2 * 3000 // (4 * 2)
    with tuning(stream=1, bags_per_group=63):
        assert _plan(26, big, 64, 30).bags_per_group == 15    # capped at lanes per row - 1
        assert _plan(26, big, 256, 30).bags_per_group == 63
    # waves: ceil(B / (groups * M)) per table
    p = _plan(26, 1001, 64, 1)
    g = 64 // p.lanes_per_row
    assert p.waves_per_table == -(-1001 // (g * p.bags_per_group))
    assert p.wavefronts == 26 * p.waves_per_table


def test_depth_rules():
    assert _plan(4, 5000, 128, 80).depth == 8                 # fp32 rows of 512 B and more
    assert _plan(4, 5000, 64, 80).depth == 4
    assert _plan(4, 5000, 256, 80, dtype=emb.EMB_F16).depth == 4
    with tuning(depth=16):
        assert _plan(4, 5000, 64, 80).depth == 16
        assert _plan(4, 5000, 64, 80, mode=emb.EMB_MAX).depth == 8     # max pooling: 4 or 8
        assert _plan(4, 5000, 64, 1).depth == 8                        # stream kernel: 4 or 8
        assert _plan(4, 5000, 4, 1).depth == 4                         # ... and at most lanes per row
    with tuning(depth=1):
        assert _plan(4, 5000, 64, 80).depth == 1
        assert _plan(4, 5000, 64, 80, mode=emb.EMB_MAX).depth == 4


def test_plan_reports_descriptor_errors_like_forward():
    def status(**kw):
        base = dict(num_tables=2, batch=4, dim=64, table_dtype=emb.EMB_F32, mode=emb.EMB_SUM,
                    num_lookups=10)
        try:
            emb.emb_bag_plan_forward(emb.make_desc(**{**base, **kw}), kw.pop("_w", False))
        except emb.EmbBagError as ex:
            return ex.status
        return 0
    assert status() == 0 and status(table_dtype=9) == -3 and status(mode=3) == -4
    assert status(dim=6) == -2 and status(out_ld=100) == -2 and status(batch=-1) == -7
    plan = emb.emb_bag_plan_forward(emb.make_desc(2, 0, 64, emb.EMB_F32, emb.EMB_SUM, 0))
    assert all(v == 0 for v in plan.as_dict().values())                # batch 0: nothing to launch
    with pytest.raises(emb.EmbBagError):
        emb.emb_bag_plan_forward(emb.make_desc(2, 4, 64, emb.EMB_F32, emb.EMB_MEAN, 10), True)
    with tuning(depth=16, stream=0):                                   # no such mixed kernel? mapped
        m = emb.make_mixed_desc([64, 32], 4, emb.EMB_F32, emb.EMB_SUM, 10, 0, 1 << 20)
        assert emb.emb_bag_plan_forward_mixed(m).depth == 8


def _simulate(plan, T, order=None):
    """(table, wavefront-in-table) of every wavefront of the grid that has work, and the XCD it
    runs on, from the fields of the plan alone."""
    p = plan.as_dict()
    g = np.arange(p["grid_blocks"], dtype=np.int64)
    w = np.arange(4, dtype=np.int64)
    if p["xcd_pieces"] == 0:
        n = (g[:, None] * 4 + w[None, :]).ravel()
        keep = n < p["wavefronts"]
        n = n[keep]
        pos = n // p["waves_per_table"]
        table = np.asarray(order, dtype=np.int64)[pos] if order is not None else pos
        return table, n % p["waves_per_table"], np.repeat(g % 8, 4)[keep]
    xcd, slot = g % 8, g // 8
    unit = (slot // p["blocks_per_piece"]) * 8 + xcd
    piece, pos = unit % p["xcd_pieces"], unit // p["xcd_pieces"]
    in_piece = ((slot % p["blocks_per_piece"]) * 4)[:, None] + w[None, :]
    in_table = piece[:, None] * p["waves_per_piece"] + in_piece
    keep = ((in_piece < p["waves_per_piece"]) & (in_table < p["waves_per_table"])
            & (unit < T * p["xcd_pieces"])[:, None])
    pos = np.minimum(pos, T - 1)          # units beyond the last table have no work (masked above)
    table = np.asarray(order, dtype=np.int64)[pos] if order is not None else pos
    return (np.broadcast_to(table[:, None], keep.shape)[keep], in_table[keep],
            np.broadcast_to(xcd[:, None], keep.shape)[keep])


@pytest.mark.parametrize("T", [1, 2, 3, 4, 5, 7, 8, 12, 13, 16, 26, 60, 100, 250])
@pytest.mark.parametrize("B,L", [(1000, 30), (4097, 30), (333, 1), (70_001, 1)])
def test_every_wavefront_of_every_table_is_launched_exactly_once(T, B, L):
    with tuning(xcd_remap=1):
        plan = _plan(T, B, 64, L)
    if -(-plan.wavefronts // 4) >= 64:      # smaller launches keep the natural order
        assert plan.xcd_pieces in (1, 2, 4, 8) and (T * plan.xcd_pieces) % 8 == 0
    else:
        assert plan.xcd_pieces == 0
    table, wave, xcd = _simulate(plan, T)
    assert len(table) == plan.wavefronts == T * plan.waves_per_table
    flat = table * plan.waves_per_table + wave
    assert np.array_equal(np.sort(flat), np.arange(T * plan.waves_per_table))
    # a table runs on exactly xcd_pieces XCDs, and every XCD gets the same number of pieces
    for t in range(min(T, 9) if plan.xcd_pieces else 0):
        assert len(np.unique(xcd[table == t])) == plan.xcd_pieces
    with tuning(xcd_remap=0):
        nat = _plan(T, B, 64, L)
    table, wave, _ = _simulate(nat, T)
    assert np.array_equal(table * nat.waves_per_table + wave, np.arange(T * nat.waves_per_table))


def _mixed_plan(dims, B=4096, L=80, dtype=emb.EMB_F32, which=0, mode=emb.EMB_SUM):
    desc = emb.make_mixed_desc(list(dims), B, dtype, mode, int(len(dims) * B * L), 0, 1 << 30)
    return emb.emb_bag_plan_forward_mixed(desc, False, True, which)


@pytest.mark.parametrize("seed", range(8))
def test_tables_of_different_widths_are_dealt_to_the_xcds_by_bytes(seed):
    rng = np.random.default_rng(seed)
    T = int(rng.choice([4, 10, 12, 20, 60, 100, 250, 1000]))
    dims = rng.choice([4, 8, 16, 32, 64, 96, 128, 192, 256], size=T)
    plan, order = _mixed_plan(dims)
    assert plan.num_launches == 1 and plan.tables == T and sorted(order) == list(range(T))
    if plan.xcd_pieces in (1, 2, 4):
        assert plan.listed == 1
    table, wave, xcd = _simulate(plan, T, order)
    flat = table * plan.waves_per_table + wave
    assert np.array_equal(np.sort(flat), np.arange(T * plan.waves_per_table))
    # bytes per XCD: within one widest table's piece of each other (greedy, widest first)
    load = np.bincount(xcd, weights=dims[table].astype(np.float64), minlength=8)
    assert load.max() - load.min() <= dims.max() * plan.waves_per_piece + 1e-9
    # the caller's own order would have been worse or equal
    naive = np.bincount(_simulate(plan, T)[2], weights=dims[_simulate(plan, T)[0]].astype(np.float64),
                        minlength=8)
    assert load.max() <= naive.max() + 1e-9


def test_mixed_plan_special_cases():
    plan, order = _mixed_plan([64] * 60)                       # equal widths: the caller's order
    assert plan.listed == 0 and order == list(range(60)) and plan.xcd_pieces == 2
    plan, order = _mixed_plan([64, 32] * 600)                  # more tables than the order holds
    assert plan.xcd_pieces == 0 and plan.listed == 0      # natural order instead
    plan, _ = _mixed_plan([64] * 1200)                         # ... which equal widths do not need
    assert plan.xcd_pieces == 1                                # 1200 is a multiple of 8
    plan, order = _mixed_plan([64, 32, 128] * 5)               # odd T: every table on all 8 XCDs
    assert plan.xcd_pieces == 8 and plan.listed == 0
    plan, order = _mixed_plan([(32, 64, 128, 256)[t % 4] for t in range(60)])
    assert order[:15] == list(range(3, 60, 4))                 # widest tables first


@pytest.mark.parametrize("L", [0.5, 1, 2, 5, 10, 20])
@pytest.mark.parametrize("seed", range(3))
def test_short_bags_split_a_mixed_call_into_one_launch_per_row_class(seed, L):
    """Below three row loads per bag a lanes-per-row class goes to the stream kernel, the other
    tables to one wave-kernel launch; together the launches cover every table exactly once."""
    rng = np.random.default_rng(100 + seed)
    T = int(rng.choice([7, 40, 333]))
    dims = rng.choice([4, 8, 16, 32, 64, 96, 128, 192, 256], size=T)
    B = 5000
    first, _ = _mixed_plan(dims, B, L)
    lanes = np.maximum(4, 2 ** np.ceil(np.log2(dims * 4 / 16)).astype(int))      # lanes per row
    want_stream = L < 3 * (64 // lanes)
    seen = np.zeros(T, dtype=int)
    kinds = []
    for w in range(first.num_launches):
        plan, order = _mixed_plan(dims, B, L, which=w)
        assert plan.num_launches == first.num_launches and plan.tables == len(order) > 0
        kinds.append((plan.kernel, plan.lanes_per_row))
        order = np.asarray(order)
        seen[order] += 1
        if plan.kernel == emb.EMB_KERNEL_STREAM:
            assert np.all(lanes[order] == plan.lanes_per_row) and np.all(want_stream[order])
            g = 64 // plan.lanes_per_row
            assert 1 <= plan.bags_per_group <= plan.lanes_per_row - 1
            assert plan.waves_per_table == -(-B // (g * plan.bags_per_group))
        else:
            assert plan.lanes_per_row == 0 and plan.bags_per_wave >= 1
            assert plan.waves_per_table == -(-B // plan.bags_per_wave)
            if first.num_launches > 1:
                assert not np.any(want_stream[order])
        table, wave, _ = _simulate(plan, plan.tables, order)
        flat = table * plan.waves_per_table + wave
        assert len(np.unique(flat)) == len(flat) == plan.tables * plan.waves_per_table
        assert set(np.unique(table)) == set(order.tolist())
    assert np.all(seen == 1)
    assert len(set(kinds)) == len(kinds)                       # one launch per kernel and class
    with pytest.raises(emb.EmbBagError):
        _mixed_plan(dims, B, L, which=first.num_launches)


def test_mixed_plan_streams_with_either_addressing_and_never_fuses_max_pooling_or_64_bit_rows():
    dims = [32, 64, 128, 256] * 5
    first = _mixed_plan(dims, 5000, 1, mode=emb.EMB_MAX)[0]
    assert first.num_launches == 4 and first.kernel == emb.EMB_KERNEL_STREAM and first.fused == 0
    assert _mixed_plan(dims, 5000, 1)[0].fused == 1
    with tuning(stream=0):
        assert _mixed_plan(dims, 5000, 1)[0].num_launches == 1
    # 64-bit addressing (forced, or no bound on the table sizes): the same launches, not fused
    with tuning(addressing=1):
        first = _mixed_plan(dims, 5000, 1)[0]
        assert (first.num_launches, first.kernel, first.buffer_addressing, first.fused) == \
            (4, emb.EMB_KERNEL_STREAM, 0, 0)
    desc = emb.make_mixed_desc(dims, 5000, emb.EMB_F32, emb.EMB_SUM, 20 * 5000, 0, 0)   # no size bound
    first = emb.emb_bag_plan_forward_mixed(desc)
    assert (first.num_launches, first.kernel, first.buffer_addressing, first.fused) == \
        (4, emb.EMB_KERNEL_STREAM, 0, 0)
    with tuning(stream=1):                                      # forced on: every class streams
        first, _ = _mixed_plan(dims, 5000, 100)
        assert first.num_launches == 4 and first.kernel == emb.EMB_KERNEL_STREAM
    # more tables than a list holds: pieces of at most 1024 tables
    first, _ = _mixed_plan([32, 64] * 1500, 2000, 1)
    assert first.num_launches == 4
    sizes = [_mixed_plan([32, 64] * 1500, 2000, 1, which=w)[0].tables for w in range(4)]
    assert sorted(sizes) == [476, 476, 1024, 1024]


def test_per_table_bag_lengths_split_a_uniform_call_in_two():
    """With table_avg_len the choice of kernel is made per table: short-bag tables in a stream
    launch, the others in a wave launch, each with its table list."""
    T, B = 26, 32768
    lens = [100.0 if t % 4 == 3 and t < 24 else 1.0 for t in range(T)]
    nl = int(sum(lens) * B)

    def plans(avg=lens, **kw):
        desc = emb.make_desc(T, B, 64, emb.EMB_F32, kw.pop("mode", emb.EMB_SUM), nl, 0, 1_000_000,
                             table_avg_len=avg)
        first = emb.emb_bag_plan_forward(desc)
        return [emb.emb_bag_plan_forward(desc, False, True, w) for w in range(first.num_launches)]

    assert len(plans(avg=None)) == 1 and plans(avg=None)[0][0].kernel == emb.EMB_KERNEL_WAVE  # average 23.8
    both = plans()
    assert [p.kernel for p, _ in both] == [emb.EMB_KERNEL_WAVE, emb.EMB_KERNEL_STREAM]
    short = [t for t in range(T) if lens[t] == 1.0]
    assert both[1][1] == short and both[0][1] == [t for t in range(T) if lens[t] == 100.0]
    assert both[1][0].bags_per_group == 4 and both[0][0].listed == 1 and both[1][0].listed == 1
    # ... as the two workgroup ranges of one fused launch (depth 4 or 8, at most 1024 tables)
    assert all(p.fused == 1 for p, _ in both)
    assert both[0][0].fused_grid_blocks == sum(-(-p.grid_blocks // 8) * 8 for p, _ in both)
    with tuning(fuse=0):
        assert all(p.fused == 0 for p, _ in plans())
    with tuning(depth=2):
        assert all(p.fused == 0 for p, _ in plans()) and len(plans()) == 2
    with tuning(depth=8):
        assert all(p.fused == 1 for p, _ in plans())
    for plan, order in both:
        table, wave, _ = _simulate(plan, plan.tables, order)
        flat = table * plan.waves_per_table + wave
        assert len(np.unique(flat)) == len(flat) == plan.tables * plan.waves_per_table
    # everything on one side: one launch, no list
    one = plans(avg=[1.0] * T)
    assert len(one) == 1 and one[0][0].kernel == emb.EMB_KERNEL_STREAM and one[0][0].listed == 0
    one = plans(avg=[50.0] * T)
    assert len(one) == 1 and one[0][0].kernel == emb.EMB_KERNEL_WAVE and one[0][0].listed == 0
    # the explicit settings override the per-table choice
    with tuning(stream=0):
        assert len(plans()) == 1 and plans()[0][0].kernel == emb.EMB_KERNEL_WAVE
    with tuning(stream=1):
        assert len(plans()) == 1 and plans()[0][0].kernel == emb.EMB_KERNEL_STREAM
    # max pooling splits the same way, as two launches (the fused kernels are built for sums)
    split = plans(mode=emb.EMB_MAX)
    assert [p.kernel for p, _ in split] == [emb.EMB_KERNEL_WAVE, emb.EMB_KERNEL_STREAM]
    assert all(p.fused == 0 for p, _ in split)
    with pytest.raises(ValueError):
        emb.make_desc(T, B, 64, emb.EMB_F32, emb.EMB_SUM, nl, 0, 0, table_avg_len=[1.0])


def test_per_table_bag_lengths_in_a_mixed_call():
    dims = [32, 64, 128, 256] * 3
    lens = [1.0, 50.0, 1.0, 50.0, 2.0, 2.0, 50.0, 50.0, 1.0, 1.0, 1.0, 1.0]
    desc = emb.make_mixed_desc(dims, 4096, emb.EMB_F32, emb.EMB_SUM, int(sum(lens) * 4096), 0, 1 << 30,
                               table_avg_len=lens)
    n = emb.emb_bag_plan_forward_mixed(desc).num_launches
    got = {}
    for w in range(n):
        plan, order = emb.emb_bag_plan_forward_mixed(desc, False, True, w)
        got[(plan.kernel, plan.lanes_per_row)] = sorted(order)   # (the wave launch orders by width)
    # short tables by class: widths 32 -> 8 lanes, 64 -> 16, 128 -> 32, 256 -> 64
    assert got == {(emb.EMB_KERNEL_WAVE, 0): [1, 3, 6, 7],
                   (emb.EMB_KERNEL_STREAM, 8): [0, 4, 8],
                   (emb.EMB_KERNEL_STREAM, 16): [5, 9],
                   (emb.EMB_KERNEL_STREAM, 32): [2, 10],
                   (emb.EMB_KERNEL_STREAM, 64): [11]}


@pytest.mark.parametrize("T,pieces", [(60, 1), (7, 2), (250, 1), (13, 4), (5, 8)])
def test_forced_pieces_per_table_still_cover_every_wavefront_once(T, pieces):
    """With "xcd_pieces" forced the XCDs may differ by one piece; nothing is lost or doubled."""
    with tuning(xcd_remap=1, xcd_pieces=pieces):
        plan = _plan(T, 4096, 64, 30)
    assert plan.xcd_pieces == pieces and plan.grid_blocks == -(-T * pieces // 8) * 8 * plan.blocks_per_piece
    table, wave, xcd = _simulate(plan, T)
    flat = table * plan.waves_per_table + wave
    assert np.array_equal(np.sort(flat), np.arange(T * plan.waves_per_table))
    counts = np.bincount(xcd, minlength=8)
    assert counts.max() - counts.min() <= plan.waves_per_piece


def test_a_launch_holds_at_most_2_pow_24_minus_1_workgroups():
    """A dispatch counts work-items in 32 bits: 2^24 - 1 workgroups of 256 threads.  Calls beyond
    that are refused with EMB_ERR_BAD_SIZE; the XCD-affine order, whose grid is padded, steps back
    to the natural order when only the padding would not fit."""
    limit = (1 << 24) - 1
    def status(T, B, D=4, L=30.0, **kw):
        try:
            return _plan(T, B, D, L, **kw)
        except emb.EmbBagError as ex:
            return ex.status
    with tuning(stream=0, bags_per_wave=1):                   # a wavefront per bag
        ok = status(64, limit * 4 // 64)                      # 67,108,800 wavefronts
        assert ok.grid_blocks <= limit and ok.wavefronts == 64 * (limit * 4 // 64)
        assert status(64, limit * 4 // 64 + 1) == -7          # 67,108,864: one workgroup too many
        assert status(1, 1 << 31) == -7 and status(3, 1 << 30) == -7
        assert status(64, 600_000, D=512) == -7               # two slabs per row double the count
        # 7 tables: 8 pieces each; the padding of the last workgroup of each piece tips it over
        B = limit * 4 // 7
        with tuning(xcd_remap=1):
            p = status(7, B)
        assert p.xcd_pieces in (0, 8) and p.grid_blocks <= limit and p.wavefronts == 7 * B
    # the short-bag kernel needs fewer wavefronts for the same bags
    p = status(64, 4_000_000, L=1.0)
    assert p.kernel == emb.EMB_KERNEL_STREAM and p.grid_blocks <= limit
    # tables of different widths
    m = emb.make_mixed_desc([4, 8] * 32, limit * 4 // 64 + 1, emb.EMB_F32, emb.EMB_SUM, 10, 0, 1 << 20)
    with tuning(stream=0, bags_per_wave=1):
        with pytest.raises(emb.EmbBagError) as ex:
            emb.emb_bag_plan_forward_mixed(m)
        assert ex.value.status == -7
    # several bags per wavefront (the automatic choice for short bags) make room for more bags
    with tuning(stream=0):
        p = status(64, limit * 4 // 64 + 1)
        assert p.bags_per_wave > 1 and p.waves_per_table == -(-(limit * 4 // 64 + 1) // p.bags_per_wave)


def test_split_mixed_calls_are_fused_into_one_launch():
    """The launches of a split mixed-width call become consecutive workgroup ranges of one launch
    when every body occurs once and the table lists fit one list of 1024."""
    dims = [(16, 32, 64, 128)[t % 4] for t in range(26)]
    first, _ = _mixed_plan(dims, 2048, 1)
    assert first.num_launches == 4 and first.fused == 1
    parts = [_mixed_plan(dims, 2048, 1, which=w)[0] for w in range(4)]
    assert all(p.fused == 1 and p.fused_grid_blocks == first.fused_grid_blocks for p in parts)
    assert first.fused_grid_blocks == sum(-(-p.grid_blocks // 8) * 8 for p in parts)
    with tuning(fuse=0):
        assert _mixed_plan(dims, 2048, 1)[0].fused == 0
    assert _mixed_plan(dims, 2048, 80)[0].fused == 0                    # one launch: nothing to fuse
    # a wave launch and stream launches together (per-table lengths)
    lens = [1.0 if t % 2 else 80.0 for t in range(26)]
    desc = emb.make_mixed_desc(dims, 2048, emb.EMB_F32, emb.EMB_MEAN, int(sum(lens) * 2048), 0, 1 << 30,
                               table_avg_len=lens)
    plans = [emb.emb_bag_plan_forward_mixed(desc, False, False, w)
             for w in range(emb.emb_bag_plan_forward_mixed(desc).num_launches)]
    assert {p.kernel for p in plans} == {emb.EMB_KERNEL_WAVE, emb.EMB_KERNEL_STREAM}
    assert all(p.fused == 1 for p in plans)
    # more tables than one list holds: separate launches
    assert _mixed_plan([32, 64] * 1500, 2000, 1)[0].fused == 0
    assert _mixed_plan([32, 64] * 600, 2000, 1)[0].fused == 0           # 1200 tables in two lists
    assert _mixed_plan([32, 64] * 500, 2000, 1)[0].fused == 1           # 1000 tables
    # a uniform-width call with more than 1024 tables keeps its two launches
    d = emb.make_desc(1100, 512, 64, emb.EMB_F32, emb.EMB_SUM, 1100 * 512 * 10, 0, 1000,
                      table_avg_len=[1.0] * 550 + [100.0] * 550)
    assert emb.emb_bag_plan_forward(d).num_launches == 2 and emb.emb_bag_plan_forward(d).fused == 0


def test_the_hot_head_is_opt_in():
    """desc.hot_rows is used only when the hot_split tuning key asks for it (measured: no gain),
    and only by the wave kernel with buffer addressing and a depth of 4 or 8."""
    import torch
    hot = torch.zeros(60, dtype=torch.int64)                 # (the plan only tests the pointer)
    desc = emb.make_desc(60, 4096, 128, emb.EMB_F32, emb.EMB_MEAN, 60 * 4096 * 80, 0, 4_000_000,
                         hot_rows=hot)
    assert emb.emb_bag_plan_forward(desc).hot_split == 0
    for mode in (1, 2):
        with tuning(hot_split=mode):
            assert emb.emb_bag_plan_forward(desc).hot_split == 1
            with tuning(depth=2):
                assert emb.emb_bag_plan_forward(desc).hot_split == 0
            with tuning(addressing=1):
                assert emb.emb_bag_plan_forward(desc).hot_split == 0
    plain = emb.make_desc(60, 4096, 128, emb.EMB_F32, emb.EMB_MEAN, 60 * 4096 * 80, 0, 4_000_000)
    with tuning(hot_split=1):
        assert emb.emb_bag_plan_forward(plain).hot_split == 0


def test_a_descriptor_can_carry_its_own_tuning():
    """emb_bag_desc.tuning replaces the process-wide keys for that descriptor (two models in one
    process can hold different settings); a value out of range is an error of the call."""
    shape = (60, 4096, 128, emb.EMB_F32, emb.EMB_SUM, 60 * 4096 * 80, 0, 4_000_000)
    plain = emb.make_desc(*shape)
    own = emb.make_desc(*shape, tuning=dict(depth=2, bags_per_wave=3, xcd_remap=0))
    other = emb.make_desc(*shape, tuning=dict(station=1, depth=4))
    with tuning(depth=16, bags_per_wave=1):
        a, b, c = (emb.emb_bag_plan_forward(d) for d in (plain, own, other))
        assert (a.depth, a.bags_per_wave, a.station) == (16, 1, 0) and a.xcd_pieces > 0
        assert (b.depth, b.bags_per_wave, b.station, b.xcd_pieces) == (2, 3, 0, 0)
        assert (c.depth, c.station) == (4, 1) and c.bags_per_wave == 1 and c.xcd_pieces > 0
        assert emb.emb_bag_get_tuning("depth") == 16          # nothing process-wide was touched
    # the defaults are those of a fresh process
    t = emb.emb_bag_tuning_defaults()
    for key, _ in emb.emb_bag_tuning._fields_:
        if key != "reserved":
            assert getattr(t, key) == emb.emb_bag_get_tuning(key), key
    with tuning(depth=8, stream=0):
        assert emb.emb_bag_plan_forward(emb.make_desc(*shape, tuning={})).depth == 8   # automatic: 8
        short = (60, 4096, 128, emb.EMB_F32, emb.EMB_SUM, 60 * 4096, 0, 4_000_000)
        assert emb.emb_bag_plan_forward(emb.make_desc(*short)).kernel == emb.EMB_KERNEL_WAVE
        assert emb.emb_bag_plan_forward(emb.make_desc(*short, tuning={})).kernel == emb.EMB_KERNEL_STREAM
    for bad in (dict(depth=3), dict(station=2), dict(bags_per_wave=33), dict(xcd_pieces=3),
                dict(stream=-2), dict(blocks_per_cu=9)):
        with pytest.raises(emb.EmbBagError) as e:
            emb.emb_bag_plan_forward(emb.make_desc(*shape, tuning=bad))
        assert e.value.status == -9, bad
    with pytest.raises(ValueError):
        emb.make_desc(*shape, tuning=dict(no_such_key=1))
    # tables of different widths: the same field
    lens = [1.0] * 4 + [60.0] * 4
    mshape = ([32, 64] * 4, 2048, emb.EMB_F32, emb.EMB_SUM, 8 * 2048 * 30, 0, 1 << 30)
    fused = emb.make_mixed_desc(*mshape, table_avg_len=lens)
    apart = emb.make_mixed_desc(*mshape, table_avg_len=lens, tuning=dict(fuse=0))
    assert emb.emb_bag_plan_forward_mixed(fused).fused == 1
    assert emb.emb_bag_plan_forward_mixed(apart).fused == 0
    with pytest.raises(emb.EmbBagError):
        emb.emb_bag_plan_forward_mixed(emb.make_mixed_desc(*mshape, tuning=dict(depth=5)))


def test_the_lds_station_is_opt_in():
    """Row loads land in LDS only when the station tuning key asks for it (measured: never
    faster), and only in the wave kernel with buffer addressing, unweighted sum or mean pooling,
    a depth of 4 or 8, tables of one width, no hot / cold split and no fused launch."""
    import torch

    def station(mode=emb.EMB_SUM, rows=4_000_000, weights=False, dtype=emb.EMB_F32, D=128, L=80, **kw):
        desc = emb.make_desc(60, 4096, D, dtype, mode, 60 * 4096 * L, 0, rows, **kw)
        return emb.emb_bag_plan_forward(desc, weights).station

    assert station() == 0
    with tuning(station=1):
        assert station() == 1 and station(emb.EMB_MEAN) == 1
        for dtype, D in ((emb.EMB_F16, 128), (emb.EMB_BF16, 64), (emb.EMB_U8ROW, 120),
                         (emb.EMB_FP8ROW, 56), (emb.EMB_F32, 4), (emb.EMB_F32, 1024)):
            assert station(dtype=dtype, D=D, rows=500_000) == 1, (dtype, D)
        assert station(emb.EMB_MAX) == 0
        assert station(weights=True) == 0
        assert station(rows=1 << 40) == 0                      # 64-bit addressing
        assert station(L=1) == 0                               # the stream kernel
        with tuning(stream=0):
            assert station(L=1) == 1
        for depth, want in ((1, 0), (2, 0), (4, 1), (8, 1), (16, 0)):
            with tuning(depth=depth):
                assert station() == want, depth
        with tuning(addressing=1):
            assert station() == 0
        hot = torch.zeros(60, dtype=torch.int64)
        assert station(hot_rows=hot) == 1                      # the head is ignored by default
        with tuning(hot_split=1):
            assert station(hot_rows=hot) == 0
        # a split call that is fused keeps its rows in registers; taken apart, the wave part
        # of it uses the station
        lens = [1.0] * 30 + [100.0] * 30
        d = emb.make_desc(60, 4096, 128, emb.EMB_F32, emb.EMB_SUM, 60 * 4096 * 50, 0, 4_000_000,
                          table_avg_len=lens)
        assert emb.emb_bag_plan_forward(d).fused == 1 and emb.emb_bag_plan_forward(d).station == 0
        with tuning(fuse=0):
            plans = [emb.emb_bag_plan_forward(d, which=k) for k in range(2)]
            assert sorted(pl.station for pl in plans) == [0, 1]
        mixed = emb.make_mixed_desc([32, 64] * 4, 2048, emb.EMB_F32, emb.EMB_SUM, 8 * 2048 * 40, 0,
                                    1 << 30)
        assert emb.emb_bag_plan_forward_mixed(mixed).station == 0
    with pytest.raises(emb.EmbBagError):
        emb.emb_bag_set_tuning("station", 2)


def test_bags_per_wave_rule():
    """Automatic bags per wavefront: more for short bags, one for long bags, for rows beyond one
    slab, and whenever the launch would drop below 32,768 wavefronts."""
    assert _plan(60, 16384, 64, 20).bags_per_wave == 3        # 5 row loads per bag -> 16 / 5
    assert _plan(60, 4096, 128, 80).bags_per_wave == 1        # 40 row loads per bag
    assert _plan(26, 2048, 64, 20.5).bags_per_wave == 1       # 53,248 bags: too few wavefronts
    assert _plan(8, 256, 64, 20).bags_per_wave == 1
    assert _plan(4, 100_000, 512, 4).bags_per_wave == 1       # 2 KiB rows: one slab per wavefront
    with tuning(bags_per_wave=5):
        p = _plan(8, 256, 64, 20)
        assert p.bags_per_wave == 5 and p.waves_per_table == -(-256 // 5)
