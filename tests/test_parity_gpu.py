"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element, on
seeded inputs small enough for the oracle to finish in seconds yet spanning several 64-lookup
chunks, ragged tails, empty bags, several tables and every addressing / depth variant."""
import numpy as np
import pytest
import torch

from inputgen import gen
from gpu_harness import (DEV, EMB_DTYPE, TORCH_DTYPE, arena_bytes, assert_close_to_oracle,
                         device_arena, forward, to_dev, tuning, upload_arena)

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    assert torch.cuda.is_available(), "GPU tests need a GPU (run with -m 'not gpu' otherwise)"


def _problem(name, **over):
    wl = gen.with_overrides(gen.workload(name), **over) if over else gen.workload(name)
    batch = gen.make_batches(wl, 1)[0]
    arena = gen.host_arena(wl)
    return wl, batch, arena


@pytest.mark.parametrize("name", ["tiny", "small_f32_d64", "small_f32_d128", "small_f16_d256",
                                  "small_bf16_d256", "small_u8_d120", "small_u8_d504"])
@pytest.mark.parametrize("mode", ["sum", "mean"])
@pytest.mark.parametrize("addressing", [0, 1])
def test_small_workloads_match_oracle(oracle, name, mode, addressing):
    wl, batch, arena = _problem(name)
    ref, bound, strict = oracle.emb_bag(arena, wl.table_offsets(), batch.indices, batch.offsets,
                                        wl.B, mode, strict=True)
    with tuning(addressing=addressing):
        got = forward(upload_arena(arena), wl.table_offsets(), batch.indices, batch.offsets, wl.B,
                      mode).cpu().numpy()
    assert_close_to_oracle(got, ref, bound, wl.dtype != "f32", f"{name}/{mode}/addr{addressing}",
                           strict=strict)


@pytest.mark.parametrize("depth", [1, 2, 4, 8, 16])
@pytest.mark.parametrize("name", ["small_f32_d64", "small_f32_d128", "small_f16_d256",
                                  "small_bf16_d256", "small_u8_d120", "small_u8_d504"])
def test_every_depth(oracle, name, depth):
    wl, batch, arena = _problem(name)
    ref, bound = oracle.emb_bag(arena, wl.table_offsets(), batch.indices, batch.offsets, wl.B)
    dev = upload_arena(arena)
    for addressing in (0, 1):
        with tuning(depth=depth, addressing=addressing):
            got = forward(dev, wl.table_offsets(), batch.indices, batch.offsets, wl.B).cpu().numpy()
        assert_close_to_oracle(got, ref, bound, wl.dtype != "f32", f"{name}/depth{depth}")


@pytest.mark.parametrize("name", ["small_f32_d64", "small_f32_d128", "small_f16_d256",
                                  "small_bf16_d256", "small_u8_d120", "small_u8_d504"])
def test_integer_tables_are_bit_exact(oracle, name):
    """Integer-valued tables: every partial sum is exact in fp32, so any order gives the same bits."""
    wl, batch, arena = _problem(name, kind=gen.KIND_INT)
    for mode in ("sum",):
        ref, _ = oracle.emb_bag(arena, wl.table_offsets(), batch.indices, batch.offsets, wl.B, mode)
        for addressing in (0, 1):
            with tuning(addressing=addressing):
                got = forward(upload_arena(arena), wl.table_offsets(), batch.indices,
                              batch.offsets, wl.B, mode).cpu().numpy()
            assert np.array_equal(got.astype(np.float64), ref)


@pytest.mark.parametrize("name", ["small_f32_d64", "small_f32_d128", "small_f16_d256",
                                  "small_bf16_d256", "small_u8_d120", "small_u8_d504"])
def test_per_sample_weights(oracle, name):
    wl, batch, arena = _problem(name, weighted=True)
    assert batch.weights is not None
    ref, bound = oracle.emb_bag(arena, wl.table_offsets(), batch.indices, batch.offsets, wl.B,
                                "sum", weights=batch.weights)
    dev = upload_arena(arena)
    for addressing in (0, 1):
        with tuning(addressing=addressing):
            got = forward(dev, wl.table_offsets(), batch.indices, batch.offsets, wl.B, "sum",
                          weights=batch.weights).cpu().numpy()
        assert_close_to_oracle(got, ref, bound, wl.dtype != "f32", f"{name}/weights")


# rows of 16 B .. 4 KiB: non-power-of-two widths, several 1-KiB column slabs, both dtypes
@pytest.mark.parametrize("D,dtype", [(4, "f32"), (12, "f32"), (32, "f32"), (96, "f32"),
                                     (256, "f32"), (320, "f32"), (1024, "f32"), (8, "f16"),
                                     (24, "f16"), (128, "f16"), (520, "f16"), (2048, "f16"),
                                     (8, "bf16"), (72, "bf16"), (512, "bf16"), (1032, "bf16"),
                                     (8, "u8row"), (24, "u8row"), (56, "u8row"), (88, "u8row"),
                                     (248, "u8row"), (312, "u8row"), (1016, "u8row")])
def test_general_row_widths(oracle, D, dtype):
    wl = gen.Workload(name=f"w{D}{dtype}", T=3, rows=(300, 17, 64), D=D, dtype=dtype, B=21,
                      pooling=("uniform", 0, 90), dists=(("uniform",),) * 3, seed=0x5EED0100 + D)
    batch = gen.make_batches(wl, 1)[0]
    arena = gen.host_arena(wl)
    dev = upload_arena(arena)
    for mode in ("sum", "mean"):
        ref, bound = oracle.emb_bag(arena, wl.table_offsets(), batch.indices, batch.offsets, wl.B, mode)
        for addressing in (0, 1):
            with tuning(addressing=addressing):
                got = forward(dev, wl.table_offsets(), batch.indices, batch.offsets, wl.B,
                              mode).cpu().numpy()
            assert_close_to_oracle(got, ref, bound, dtype != "f32", f"D{D}/{dtype}/{mode}")


def test_padded_output_leading_dimension(oracle):
    wl, batch, arena = _problem("small_f32_d64")
    ld = wl.T * wl.D + 8
    ref, bound = oracle.emb_bag(arena, wl.table_offsets(), batch.indices, batch.offsets, wl.B,
                                "sum", out_ld=ld)
    got = forward(upload_arena(arena), wl.table_offsets(), batch.indices, batch.offsets, wl.B,
                  "sum", out_ld=ld, fill=-7.0).cpu().numpy()
    assert np.all(got[:, wl.T * wl.D:] == -7.0)           # padding columns untouched
    assert_close_to_oracle(got[:, :wl.T * wl.D], ref[:, :wl.T * wl.D], bound[:, :wl.T * wl.D], False)


def test_empty_inputs(oracle):
    arena = gen.table_values(1, np.arange(10), 64)
    toff = np.array([0, 4, 10], dtype=np.int64)
    # every bag empty, no indices at all
    got = forward(upload_arena(arena), toff, np.zeros(0, np.int64), np.zeros(2 * 5 + 1, np.int64), 5)
    g = got.cpu().numpy()
    assert g.shape == (5, 128) and np.all(g == 0) and not np.signbit(g).any()
    got = forward(upload_arena(arena), toff, np.zeros(0, np.int64), np.zeros(2 * 5 + 1, np.int64), 5, "mean")
    assert np.all(got.cpu().numpy() == 0)
    # B = 0 is a no-op
    out = forward(upload_arena(arena), toff, np.zeros(0, np.int64), np.zeros(1, np.int64), 0)
    assert out.shape == (0, 128)


def test_single_bag_single_table_and_len1(oracle):
    arena = gen.table_values(2, np.arange(50), 128)
    toff = np.array([0, 50], dtype=np.int64)
    got = forward(upload_arena(arena), toff, np.array([7], np.int64), np.array([0, 1], np.int64), 1)
    assert np.array_equal(got.cpu().numpy()[0], arena[7])            # len 1: the row itself
    got = forward(upload_arena(arena), toff, np.array([7], np.int64), np.array([0, 1], np.int64), 1, "mean")
    assert np.array_equal(got.cpu().numpy()[0], arena[7])


def test_one_item_case(oracle):
    """Paper Sec. 3.2 'one item': all lookups name one row."""
    for kind in (gen.KIND_NORMAL, gen.KIND_INT):
        wl = gen.Workload(name="one", T=2, rows=(500, 300), D=128, dtype="f32", B=40,
                          pooling=("fixed", 64), dists=(("one_item",),) * 2, seed=77, kind=kind)
        batch = gen.make_batches(wl, 1)[0]
        arena = gen.host_arena(wl)
        ref, bound = oracle.emb_bag(arena, wl.table_offsets(), batch.indices, batch.offsets,
                                    wl.B, "mean")
        g = forward(upload_arena(arena), wl.table_offsets(), batch.indices, batch.offsets, wl.B,
                    "mean").cpu().numpy()
        assert_close_to_oracle(g, ref, bound, False, "one item")
        if kind == gen.KIND_INT:  # small integers: 64 * row / 64 is exact
            for t in range(2):
                row = arena[wl.table_offsets()[t] + gen.one_item_row(wl, t)]
                assert np.array_equal(g[:, t * 128:(t + 1) * 128], np.broadcast_to(row, (wl.B, 128)))


def test_long_bags_many_chunks(oracle):
    wl = gen.Workload(name="long", T=2, rows=(5000, 1000), D=128, dtype="f32", B=6,
                      pooling=("uniform", 500, 1500), dists=(("uniform",), ("zipf", 1.05)), seed=91)
    batch = gen.make_batches(wl, 1)[0]
    arena = gen.host_arena(wl)
    ref, bound = oracle.emb_bag(arena, wl.table_offsets(), batch.indices, batch.offsets, wl.B, "mean")
    got = forward(upload_arena(arena), wl.table_offsets(), batch.indices, batch.offsets, wl.B, "mean")
    # 1500 terms: the fp32 bound still holds in practice (errors grow like sqrt(L) * 2^-24)
    assert_close_to_oracle(got.cpu().numpy(), ref, bound, False, "long bags")


def test_launch_shaping_knobs_do_not_change_bits(oracle):
    wl = gen.Workload(name="knobs", T=6, rows=(900,) * 6, D=128, dtype="f32", B=300,
                      pooling=("uniform", 0, 70), dists=(("uniform",),) * 6, seed=0x5EED0200)
    batch = gen.make_batches(wl, 1)[0]
    arena = gen.host_arena(wl)
    ref, bound = oracle.emb_bag(arena, wl.table_offsets(), batch.indices, batch.offsets, wl.B)
    dev = upload_arena(arena)
    base = forward(dev, wl.table_offsets(), batch.indices, batch.offsets, wl.B).cpu().numpy()
    assert_close_to_oracle(base, ref, bound, False, "knobs/base")
    again = forward(dev, wl.table_offsets(), batch.indices, batch.offsets, wl.B).cpu().numpy()
    assert np.array_equal(base, again)                                  # run-to-run deterministic
    for kw in (dict(xcd_remap=1), dict(blocks_per_cu=1), dict(blocks_per_cu=2),
               dict(blocks_per_cu=5), dict(xcd_remap=1, blocks_per_cu=3)):
        with tuning(**kw):
            got = forward(dev, wl.table_offsets(), batch.indices, batch.offsets, wl.B).cpu().numpy()
        assert np.array_equal(got, base), kw


@pytest.mark.parametrize("T,B,D", [(1, 700, 64), (3, 333, 128), (5, 129, 64), (8, 64, 128),
                                   (7, 100, 320), (16, 40, 128), (12, 257, 64)])
def test_xcd_affine_order_covers_every_bag(oracle, T, B, D):
    """The XCD-affine block order cuts tables into 1, 2, 4 or 8 pieces depending on T; whatever
    the split, every bag is written exactly as in the natural order."""
    wl = gen.Workload(name="xcd", T=T, rows=(500,) * T, D=D, dtype="f32", B=B,
                      pooling=("uniform", 0, 30), dists=(("uniform",),) * T, seed=0x5EED0400 + T)
    batch = gen.make_batches(wl, 1)[0]
    arena = gen.host_arena(wl)
    ref, bound = oracle.emb_bag(arena, wl.table_offsets(), batch.indices, batch.offsets, wl.B)
    dev = upload_arena(arena)
    with tuning(xcd_remap=0):
        nat = forward(dev, wl.table_offsets(), batch.indices, batch.offsets, wl.B).cpu().numpy()
    assert_close_to_oracle(nat, ref, bound, False, "natural order")
    with tuning(xcd_remap=1):
        aff = forward(dev, wl.table_offsets(), batch.indices, batch.offsets, wl.B).cpu().numpy()
    assert np.array_equal(nat, aff)
    for pieces in (1, 2, 4, 8):          # forced: the XCDs may then differ by one piece
        with tuning(xcd_remap=1, xcd_pieces=pieces):
            got = forward(dev, wl.table_offsets(), batch.indices, batch.offsets, wl.B).cpu().numpy()
        assert np.array_equal(nat, got), pieces


def test_bad_indices_and_offsets_are_neutralised_and_counted(oracle):
    import paper_2410_22249_amd as emb
    wl, batch, arena = _problem("small_f32_d128")
    toff = wl.table_offsets()
    rng = np.random.default_rng(5)
    idx = batch.indices.copy()
    nbad = 40
    pos = rng.choice(len(idx), size=nbad, replace=False)
    table_of = np.repeat(np.arange(wl.T), np.diff(batch.offsets[::wl.B]))
    bad_vals = np.where(rng.random(nbad) < 0.5, -1 - rng.integers(0, 5, nbad),
                        np.asarray(wl.rows)[table_of[pos]] + rng.integers(0, 3, nbad))
    idx[pos] = bad_vals
    # oracle on the same problem with the bad lookups given zero weight
    w = np.ones(len(idx), np.float32)
    w[pos] = 0.0
    ref, bound = oracle.emb_bag(arena, toff, batch.indices, batch.offsets, wl.B, "sum", weights=w)
    dev = upload_arena(arena)
    for addressing in (0, 1):
        with tuning(addressing=addressing):
            got = forward(dev, toff, idx, batch.offsets, wl.B).cpu().numpy()
        assert_close_to_oracle(got, ref, bound, False, f"bad indices/addr{addressing}")
    desc = emb.make_desc(wl.T, wl.B, wl.D, emb.EMB_F32, emb.EMB_SUM, len(idx), 0, max(wl.rows))
    count = torch.zeros(1, dtype=torch.int64, device=DEV)
    emb.emb_bag_validate(desc, to_dev(toff), to_dev(idx), to_dev(batch.offsets), count)
    assert int(count.item()) == nbad
    count.zero_()
    emb.emb_bag_validate(desc, to_dev(toff), to_dev(batch.indices), to_dev(batch.offsets), count)
    assert int(count.item()) == 0
    # offsets: one decreasing pair -> two defects (bag g ends low, bag g+1 starts... stays valid)
    off = batch.offsets.copy()
    g = 10
    off[g + 1] = off[g] - 1 if off[g] > 0 else off[g]
    count.zero_()
    emb.emb_bag_validate(desc, to_dev(toff), to_dev(batch.indices), to_dev(off), count)
    assert int(count.item()) >= 1
    got = forward(dev, toff, batch.indices, off, wl.B).cpu().numpy()   # must not fault
    assert np.isfinite(got).all()
    # offsets that point far outside [0, NL] are clamped
    off2 = batch.offsets.copy()
    off2[-1] = 1 << 40
    off2[3] = -(1 << 40)
    got = forward(dev, toff, batch.indices, off2, wl.B).cpu().numpy()
    assert np.isfinite(got).all()


def test_rows_beyond_max_table_rows_read_as_zero(oracle):
    wl, batch, arena = _problem("small_f32_d128")
    cap = 100
    w = np.ones(len(batch.indices), np.float32)
    w[batch.indices >= cap] = 0.0
    ref, bound = oracle.emb_bag(arena, wl.table_offsets(), batch.indices, batch.offsets, wl.B,
                                "sum", weights=w)
    got = forward(upload_arena(arena), wl.table_offsets(), batch.indices, batch.offsets, wl.B,
                  max_table_rows=cap).cpu().numpy()
    assert_close_to_oracle(got, ref, bound, False, "max_table_rows clamp")


@pytest.mark.parametrize("dtype,kind", [("f32", 0), ("f16", 0), ("bf16", 0), ("u8row", 0), ("f32", 1),
                                        ("f16", 1), ("bf16", 1), ("u8row", 1)])
def test_device_fill_matches_host_values_bit_for_bit(dtype, kind):
    wl = gen.Workload(name="fill", T=2, rows=(7001, 4099),
                      D={"f32": 128, "u8row": 120}.get(dtype, 256),
                      dtype=dtype, B=1, pooling=("fixed", 1), dists=(("uniform",),) * 2,
                      seed=0x5EED0300, kind=kind)
    dev = device_arena(wl)
    torch.cuda.synchronize()
    host = gen.host_arena(wl)
    assert np.array_equal(arena_bytes(dev), host.view(np.uint8))
    # a slab filled from a non-zero first row matches the same rows of the whole
    part = torch.empty((1000, dev.shape[1]), dtype=dev.dtype, device=DEV)
    gen.fill_arena_device(part.data_ptr(), 5000, 1000, wl.D, dtype, wl.seed, kind,
                          torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    assert torch.equal(part, dev[5000:6000])


def test_forward_replays_correctly_from_a_hip_graph(oracle):
    """The forward is one kernel launch with no allocation and no memset, so it can be captured;
    every replay (with eager work and synchronisations in between) must equal the eager result."""
    import paper_2410_22249_amd as emb
    wl = gen.workload("small_f32_d128")
    b0, b1, b2 = gen.make_batches(wl, 3)
    arena = upload_arena(gen.host_arena(wl))
    toff = to_dev(wl.table_offsets())
    cap = max(b.num_lookups for b in (b0, b1, b2))
    idx = torch.zeros(cap, dtype=torch.int64, device=DEV)
    off = torch.zeros(wl.T * wl.B + 1, dtype=torch.int64, device=DEV)
    out = torch.zeros((wl.B, wl.T * wl.D), dtype=torch.float32, device=DEV)
    # the descriptor is read at capture time: size it for the largest batch; the shorter
    # batches simply end earlier in the (clamped) index buffer
    desc = emb.make_desc(wl.T, wl.B, wl.D, emb.EMB_F32, emb.EMB_SUM, cap, 0, max(wl.rows))

    def load(b):
        idx[: b.num_lookups].copy_(torch.from_numpy(b.indices))
        off.copy_(torch.from_numpy(b.offsets))

    load(b0)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        emb.emb_bag_forward(desc, arena, toff, idx, off, None, out)        # warm-up on the side stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        emb.emb_bag_forward(desc, arena, toff, idx, off, None, out)
    for b in (b1, b2, b0, b1):
        load(b)
        out.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = out.cpu().numpy().copy()
        eager = forward(arena, wl.table_offsets(), b.indices, b.offsets, wl.B).cpu().numpy()
        assert np.array_equal(got, eager)
        ref, bound = oracle.emb_bag(gen.host_arena(wl), wl.table_offsets(), b.indices, b.offsets, wl.B)
        assert_close_to_oracle(got, ref, bound, False, "graph replay")


def test_table_hints_change_speed_only(oracle):
    """Streaming hints switch the cache policy of the row loads; results must not move a bit."""
    import paper_2410_22249_amd as emb
    for name in ("small_f32_d64", "small_f32_d128", "small_f16_d256", "small_bf16_d256",
                 "small_u8_d120"):
        wl = gen.workload(name)
        batch = gen.make_batches(wl, 1)[0]
        host = gen.host_arena(wl)
        arena = upload_arena(host)
        toff, idx, off = to_dev(wl.table_offsets()), to_dev(batch.indices), to_dev(batch.offsets)
        ref, bound = oracle.emb_bag(host, wl.table_offsets(), batch.indices, batch.offsets, wl.B)
        outs = []
        for hints_np in (None, np.zeros(wl.T, np.uint8), np.ones(wl.T, np.uint8),
                         (np.arange(wl.T) % 2).astype(np.uint8)):
            hints = None if hints_np is None else to_dev(hints_np)
            for addressing in (0, 1):
                out = torch.full((wl.B, wl.T * wl.D), float("nan"), dtype=torch.float32, device=DEV)
                desc = emb.make_desc(wl.T, wl.B, wl.D, EMB_DTYPE[TORCH_DTYPE[wl.dtype]],
                                     emb.EMB_SUM, batch.num_lookups, 0, max(wl.rows), hints)
                with tuning(addressing=addressing):
                    emb.emb_bag_forward(desc, arena, toff, idx, off, None, out)
                torch.cuda.synchronize()
                outs.append(out.cpu().numpy())
        assert_close_to_oracle(outs[0], ref, bound, wl.dtype != "f32", f"{name}/hints")
        for o in outs[1:]:
            assert np.array_equal(o, outs[0])


def test_reuse_profile_matches_oracle_bit_for_bit():
    import paper_2410_22249_amd as emb
    from oracle import reuse_oracle
    cases = [gen.workload("small_f32_d64"), gen.workload("small_f32_d128"),
             gen.Workload(name="prof", T=9, rows=(4_000_000, 50, 1, 100_000, 7, 4_000_000, 300, 9, 2),
                          D=64, dtype="f32", B=160, pooling=("uniform", 0, 300),
                          dists=(("uniform",), ("uniform",), ("one_item",), ("zipf", 1.05),
                                 ("uniform",), ("zipf", 1.2), ("zipf", 0.7), ("uniform",),
                                 ("one_item",)), seed=0x5EED0500)]
    for wl in cases:
        batch = gen.make_batches(wl, 1)[0]
        idx, off = to_dev(batch.indices), to_dev(batch.offsets)
        # the row size enters the rule only: the same ids are profiled as rows of 16 B .. 4 KiB
        for D in (wl.D, 4, 16, 1024):
            desc = emb.make_desc(wl.T, wl.B, D, emb.EMB_F32, emb.EMB_SUM, batch.num_lookups)
            for window, thr in ((4096, 20), (100, 75), (1, 20), (5000, 500), (333, -1), (16384, -1),
                                (1 << 30, 75), (64, 2_000_000_000), (16384, 0)):
                dup = torch.full((wl.T,), -1, dtype=torch.int32, device=DEV)
                used = torch.full((wl.T,), -1, dtype=torch.int32, device=DEV)
                hints = torch.full((wl.T,), 9, dtype=torch.uint8, device=DEV)
                emb.emb_bag_profile_reuse(desc, idx, off, window, thr, dup, used, hints)
                torch.cuda.synchronize()
                # (a window beyond the interface's range is clamped to it)
                rd, ru, rh = reuse_oracle.profile_reuse(batch.indices, batch.offsets, wl.T, wl.B,
                                                        min(window, reuse_oracle.MAX_WINDOW),
                                                        75 if thr < 0 else thr, row_bytes=D * 4)
                assert np.array_equal(dup.cpu().numpy(), rd), (wl.name, window)
                assert np.array_equal(used.cpu().numpy(), ru)
                assert np.array_equal(hints.cpu().numpy(), rh), (wl.name, D, window, thr)
    # no lookups at all
    desc = emb.make_desc(3, 4, 64, emb.EMB_F32, emb.EMB_SUM, 0)
    hints = torch.full((3,), 9, dtype=torch.uint8, device=DEV)
    emb.emb_bag_profile_reuse(desc, None, torch.zeros(13, dtype=torch.int64, device=DEV), 64, 20,
                              None, None, hints)
    torch.cuda.synchronize()
    assert hints.cpu().tolist() == [1, 1, 1]


def test_randomised_shapes(oracle):
    """Forty seeded random problems: table counts, row counts, widths, batch sizes, pooling ranges,
    dtypes, modes, weights, padded leading dimensions, addressing and launch knobs drawn at random."""
    rng = np.random.default_rng(0xE3B)
    for case in range(40):
        dtype = ("f32", "f16", "bf16", "u8row")[int(rng.integers(0, 4))]
        unit = 4 if dtype == "f32" else 8
        D = int(unit * rng.integers(1, 80))                      # rows of 16 B .. 1264 B
        if dtype == "u8row":
            D = int(16 * rng.integers(0, 63) + 8)                # D + 8 a multiple of 16, <= 1024
        T = int(rng.integers(1, 12))
        rows = tuple(int(x) for x in rng.integers(1, 3000, size=T))
        B = int(rng.integers(1, 90))
        lo = int(rng.integers(0, 4))
        hi = lo + int(rng.choice([0, 3, 40, 150, 400]))
        mode = "mean" if rng.random() < 0.4 else "sum"
        weighted = mode == "sum" and rng.random() < 0.4
        dists = tuple((("uniform",), ("zipf", 1.1), ("one_item",))[int(rng.integers(0, 3))]
                      for _ in range(T))
        wl = gen.Workload(name=f"rnd{case}", T=T, rows=rows, D=D, dtype=dtype, B=B,
                          pooling=("uniform", lo, hi), dists=dists, mode=mode, weighted=weighted,
                          seed=0x5EED0600 + case)
        batch = gen.make_batches(wl, 1)[0]
        host = gen.host_arena(wl)
        pad = int(rng.choice([0, 4, 64]))
        ld = T * D + pad
        ref, bound = oracle.emb_bag(host, wl.table_offsets(), batch.indices, batch.offsets, B,
                                    mode, weights=batch.weights, out_ld=ld)
        kw = dict(addressing=int(rng.integers(0, 2)), depth=int(rng.choice([0, 1, 2, 4, 8, 16])),
                  xcd_remap=int(rng.integers(-1, 2)), blocks_per_cu=int(rng.choice([0, 0, 3])))
        with tuning(**kw):
            got = forward(upload_arena(host), wl.table_offsets(), batch.indices, batch.offsets, B,
                          mode, weights=batch.weights, out_ld=ld, fill=-3.0).cpu().numpy()
        what = f"case {case}: T={T} D={D} {dtype} B={B} L=[{lo},{hi}] {mode} w={weighted} {kw}"
        assert np.all(got[:, T * D:] == -3.0), what
        assert_close_to_oracle(got[:, :T * D], ref[:, :T * D], bound[:, :T * D], dtype != "f32", what)


def test_gpu_invariants_without_the_oracle():
    """The invariants that pin the oracle also hold for the HIP path on its own."""
    rng = np.random.default_rng(41)
    # identity tables: output = histogram of the bag's indices (exact)
    T, D, B = 3, 64, 50
    tables = np.concatenate([np.eye(D, dtype=np.float32)] * T)
    toff = np.arange(T + 1, dtype=np.int64) * D
    lengths = rng.integers(0, 200, size=T * B)
    offsets = gen.lengths_to_offsets(lengths)
    idx = rng.integers(0, D, size=int(offsets[-1])).astype(np.int64)
    dev = upload_arena(tables)
    got = forward(dev, toff, idx, offsets, B).cpu().numpy()
    for t in range(T):
        for b in range(B):
            s, e = offsets[t * B + b], offsets[t * B + b + 1]
            assert np.array_equal(got[b, t * D:(t + 1) * D], np.bincount(idx[s:e], minlength=D))
    # mean = sum / len (one correctly rounded division), empty bags exactly +0
    tables = rng.normal(0, 0.1, size=(T * D, D)).astype(np.float32)
    dev = upload_arena(tables)
    s_out = forward(dev, toff, idx, offsets, B, "sum").cpu().numpy()
    m_out = forward(dev, toff, idx, offsets, B, "mean").cpu().numpy()
    L = lengths.reshape(T, B).T                                         # [B, T]
    Lcol = np.repeat(L, D, axis=1).astype(np.float32)
    want = np.where(Lcol > 0, s_out / np.maximum(Lcol, 1), 0).astype(np.float32)
    assert np.array_equal(m_out, want)
    assert not np.signbit(m_out[Lcol == 0]).any()
    # permutation invariance inside a bag: exact on integer tables, within tolerance otherwise
    itab = rng.integers(-8, 8, size=tables.shape).astype(np.float32)
    idx2 = idx.copy()
    for gbag in range(T * B):
        a, b_ = offsets[gbag], offsets[gbag + 1]
        idx2[a:b_] = rng.permutation(idx2[a:b_])
    di = upload_arena(itab)
    assert np.array_equal(forward(di, toff, idx, offsets, B).cpu().numpy(),
                          forward(di, toff, idx2, offsets, B).cpu().numpy())
    p1 = forward(dev, toff, idx2, offsets, B, "sum").cpu().numpy()
    scale = np.abs(tables).max() * np.maximum(Lcol, 1)
    assert np.all(np.abs(p1 - s_out) <= 2e-5 * scale)
    # linearity on integer tables
    jtab = rng.integers(-8, 8, size=tables.shape).astype(np.float32)
    a1 = forward(di, toff, idx, offsets, B).cpu().numpy()
    a2 = forward(upload_arena(jtab), toff, idx, offsets, B).cpu().numpy()
    a12 = forward(upload_arena(itab + jtab), toff, idx, offsets, B).cpu().numpy()
    assert np.array_equal(a12, a1 + a2)


def test_quantised_rows_reject_bad_shapes():
    import ctypes
    import paper_2410_22249_amd as emb
    fake = ctypes.c_void_p(0x1000)
    for dim, want in ((120, None), (128, -2), (1016, None), (1032, -2), (4, -2)):
        desc = emb.make_desc(2, 4, dim, emb.EMB_U8ROW, emb.EMB_SUM, 10)
        rc = emb.lib().emb_bag_validate(ctypes.byref(desc), None, fake, fake, fake, None)
        assert rc == (want if want is not None else -1), dim    # -1: shape accepted, NULL pointer


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16", "u8row"])
def test_hip_allocated_arena_gives_the_same_result(oracle, dtype):
    """Arenas allocated by the generator straight from HIP (physically contiguous on request)
    are ordinary device memory: same fill, same forward result as a torch allocation."""
    wl = gen.Workload(name="arena", T=3, rows=(900, 40, 333),
                      D={"f32": 128, "u8row": 248}.get(dtype, 256),
                      dtype=dtype, B=37, pooling=("uniform", 0, 70), dists=(("uniform",),) * 3,
                      seed=0x5EED0800)
    batch = gen.make_batches(wl, 1)[0]
    ref_dev = device_arena(wl)
    want = forward(ref_dev, wl.table_offsets(), batch.indices, batch.offsets, wl.B).cpu().numpy()
    for contiguous in (True, False):
        arena = gen.DeviceArena(wl.total_rows, wl.D, dtype, contiguous=contiguous)
        try:
            gen.fill_arena_device(arena.data_ptr(), 0, wl.total_rows, wl.D, dtype, wl.seed, wl.kind,
                                  torch.cuda.current_stream().cuda_stream)
            torch.cuda.synchronize()
            assert np.array_equal(arena_bytes(arena.tensor), arena_bytes(ref_dev))
            got = forward(arena.tensor, wl.table_offsets(), batch.indices, batch.offsets,
                          wl.B).cpu().numpy()
            assert np.array_equal(got, want)
        finally:
            torch.cuda.synchronize()
            arena.close()
    host = gen.host_arena(wl)
    ref, bound = oracle.emb_bag(host, wl.table_offsets(), batch.indices, batch.offsets, wl.B)
    assert_close_to_oracle(want, ref, bound, dtype != "f32", "hip arena")


def test_plain_c_caller_of_the_abi():
    """tests/c_abi/c_abi_driver.c links libembbag.so and the HIP runtime from C (no Python, no
    torch in its process), runs sum and mean on a small problem and checks them itself."""
    import os
    import subprocess
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    exe = os.path.join(root, "tests", "c_abi", "c_abi_driver")
    assert os.path.exists(exe), "build() compiles the C driver"
    r = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=100)
    assert r.returncode == 0 and "C ABI OK" in r.stdout, r.stdout


def test_concurrent_calls_on_two_streams(oracle):
    """The library keeps no state between calls (no scratch, no retained pointers): two calls
    enqueued on different streams with different outputs do not disturb each other."""
    import paper_2410_22249_amd as emb
    wl = gen.Workload(name="streams", T=8, rows=(5000,) * 8, D=128, dtype="f32", B=512,
                      pooling=("uniform", 0, 90), dists=(("uniform",),) * 8, seed=0x5EED0B00)
    b0, b1 = gen.make_batches(wl, 2)
    host = gen.host_arena(wl)
    arena = upload_arena(host)
    toff = to_dev(wl.table_offsets())
    dev = [(to_dev(b.indices), to_dev(b.offsets)) for b in (b0, b1)]
    outs = [torch.full((wl.B, wl.T * wl.D), float("nan"), dtype=torch.float32, device=DEV)
            for _ in range(2)]
    descs = [emb.make_desc(wl.T, wl.B, wl.D, emb.EMB_F32, emb.EMB_SUM, b.num_lookups, 0, max(wl.rows))
             for b in (b0, b1)]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    torch.cuda.synchronize()
    for rep in range(5):
        for k in range(2):
            emb.emb_bag_forward(descs[k], arena, toff, dev[k][0], dev[k][1], None, outs[k], streams[k])
    torch.cuda.synchronize()
    for k, b in enumerate((b0, b1)):
        ref, bound = oracle.emb_bag(host, wl.table_offsets(), b.indices, b.offsets, wl.B)
        assert_close_to_oracle(outs[k].cpu().numpy(), ref, bound, False, f"stream {k}")
        alone = forward(arena, wl.table_offsets(), b.indices, b.offsets, wl.B).cpu().numpy()
        assert np.array_equal(outs[k].cpu().numpy(), alone)


@pytest.mark.parametrize("name", ["small_f32_d64", "small_f32_d128", "small_f16_d256",
                                  "small_u8_d120"])
@pytest.mark.parametrize("mode", ["sum", "mean", "max"])
def test_bags_per_wave_gives_the_same_bits(oracle, name, mode):
    """A wavefront that takes several consecutive bags (bounds with one load, the next bag's row
    ids requested ahead) adds every bag exactly as a wavefront with one bag does."""
    wl, batch, arena = _problem(name)
    ref, bound = oracle.emb_bag(arena, wl.table_offsets(), batch.indices, batch.offsets, wl.B, mode)
    dev = upload_arena(arena)
    weights = None
    for addressing in (0, 1):
        base = None
        for bpw in (1, 2, 3, 5, 8, 32):
            with tuning(bags_per_wave=bpw, addressing=addressing, stream=0):
                got = forward(dev, wl.table_offsets(), batch.indices, batch.offsets, wl.B, mode,
                              weights=weights).cpu().numpy()
            if base is None:
                base = got
                if mode == "max" and wl.dtype not in gen.QUANTISED:
                    assert np.array_equal(got.astype(np.float64), ref)
                else:
                    assert_close_to_oracle(got, ref, bound, wl.dtype != "f32", f"{name}/{mode}")
            assert np.array_equal(got.view(np.uint32), base.view(np.uint32)), (bpw, addressing)


def test_a_descriptor_with_its_own_tuning_runs_as_planned(oracle):
    """emb_bag_desc.tuning: the call runs what the process-wide keys with the same values would
    run (same bits), whatever the process-wide keys say meanwhile."""
    import paper_2410_22249_amd as emb
    wl, batch, arena = _problem("small_f32_d128")
    ref, bound = oracle.emb_bag(arena, wl.table_offsets(), batch.indices, batch.offsets, wl.B, "sum")
    dev, toff = upload_arena(arena), to_dev(wl.table_offsets())
    idx, off = to_dev(batch.indices), to_dev(batch.offsets)
    for own in (dict(depth=2, bags_per_wave=3, stream=0), dict(station=1, depth=4, stream=0, xcd_remap=1),
                dict(stream=1, bags_per_group=5), dict(blocks_per_cu=2, addressing=1)):
        with tuning(**own):
            want = forward(dev, wl.table_offsets(), batch.indices, batch.offsets, wl.B)
            plan_want = emb.emb_bag_plan_forward(emb.make_desc(
                wl.T, wl.B, wl.D, emb.EMB_F32, emb.EMB_SUM, batch.num_lookups, 0, max(wl.rows))).as_dict()
        desc = emb.make_desc(wl.T, wl.B, wl.D, emb.EMB_F32, emb.EMB_SUM, batch.num_lookups, 0,
                             max(wl.rows), tuning=own)
        with tuning(depth=16, stream=-1, bags_per_wave=7):     # must not matter
            assert emb.emb_bag_plan_forward(desc).as_dict() == plan_want
            out = torch.full((wl.B, wl.T * wl.D), float("nan"), dtype=torch.float32, device=DEV)
            emb.emb_bag_forward(desc, dev, toff, idx, off, None, out)
            torch.cuda.synchronize()
        assert torch.equal(out.view(torch.int32), want.view(torch.int32)), own
        assert_close_to_oracle(out.cpu().numpy(), ref, bound, False, f"desc tuning {own}")
    bad = emb.make_desc(wl.T, wl.B, wl.D, emb.EMB_F32, emb.EMB_SUM, batch.num_lookups, 0,
                        max(wl.rows), tuning=dict(depth=5))
    with pytest.raises(emb.EmbBagError):
        emb.emb_bag_forward(bad, dev, toff, idx, off, None, out)


@pytest.mark.parametrize("name", ["small_f32_d64", "small_f32_d128", "small_f16_d256",
                                  "small_u8_d120"])
@pytest.mark.parametrize("mode", ["sum", "mean"])
def test_the_lds_station_gives_the_same_bits(oracle, name, mode):
    """Row loads that land in LDS instead of registers (the shared-memory prefetch station of
    paper Sec. 4.2) feed the same additions in the same order."""
    import paper_2410_22249_amd as emb
    wl, batch, arena = _problem(name)
    ref, bound = oracle.emb_bag(arena, wl.table_offsets(), batch.indices, batch.offsets, wl.B, mode)
    dev = upload_arena(arena)
    desc = emb.make_desc(wl.T, wl.B, wl.D, emb.DTYPES[wl.dtype], emb.MODES[mode], batch.num_lookups,
                         0, max(wl.rows))
    for depth in (4, 8):
        for bpw in (1, 3):
            with tuning(depth=depth, bags_per_wave=bpw, stream=0):
                base = forward(dev, wl.table_offsets(), batch.indices, batch.offsets, wl.B,
                               mode).cpu().numpy()
                with tuning(station=1):
                    assert emb.emb_bag_plan_forward(desc).station == 1
                    got = forward(dev, wl.table_offsets(), batch.indices, batch.offsets, wl.B,
                                  mode).cpu().numpy()
            assert np.array_equal(got.view(np.uint32), base.view(np.uint32)), (depth, bpw)
    assert_close_to_oracle(got, ref, bound, wl.dtype != "f32", f"{name}/{mode} LDS station")


@pytest.mark.parametrize("kernel", ["wave", "stream"])
def test_every_finite_half_is_widened_exactly(kernel):
    """A table that holds every finite binary16 bit pattern (subnormals included), one lookup per
    bag: the output is the exact widening of the element, bit for bit, also through the
    mixed-precision FMA the kernels use for fp16 rows, in sum, mean and weighted form."""
    bits = np.arange(1 << 16, dtype=np.uint16)
    bits = bits[(bits & 0x7C00) != 0x7C00]                      # no infinities, no NaNs
    D = 8
    pad = (-len(bits)) % D
    table = np.concatenate([bits, np.zeros(pad, np.uint16)]).view(np.float16).reshape(-1, D)
    R = len(table)
    dev = torch.from_numpy(table).to(DEV)
    want = table.astype(np.float32) + np.float32(0.0)           # numpy widens exactly; the sum
    idx = np.arange(R, dtype=np.int64)                          # starts at +0, so -0 comes out +0
    off = np.arange(R + 1, dtype=np.int64)
    toff = np.array([0, R], np.int64)
    with tuning(stream=1 if kernel == "stream" else 0):
        for mode, weights in (("sum", None), ("mean", None), ("sum", np.ones(R, np.float32))):
            got = forward(dev, toff, idx, off, R, mode, weights=weights).cpu().numpy()
            assert np.array_equal(got.view(np.uint32), want.view(np.uint32)), (mode, weights is None)
        # a weight of 0.5 halves every element exactly (subnormal halves widen to normal floats)
        got = forward(dev, toff, idx, off, R, "sum", weights=np.full(R, 0.5, np.float32)).cpu().numpy()
        assert np.array_equal(got.view(np.uint32), (want * np.float32(0.5)).view(np.uint32))
        # two lookups per bag: x + (-0.0 or +0.0) keeps x; and x + x doubles it
        idx2 = np.stack([idx, idx], 1).ravel()
        off2 = np.arange(R + 1, dtype=np.int64) * 2
        got = forward(dev, toff, idx2, off2, R, "sum").cpu().numpy()
        assert np.array_equal(got, want * np.float32(2.0))
