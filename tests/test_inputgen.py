"""Checks of the seeded input generator (no GPU): statistics the paper fixes, structure, determinism."""
import json
import math
import os

import numpy as np
import pytest

from inputgen import gen

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "paper_constants.json")))


def test_uniform_unique_fraction_matches_paper():
    """Sec. 3.2: R uniform draws over R rows touch 63.21 % (= 1 - 1/e) of the rows."""
    R = GOLD["unique_access_pct"]["rows"]
    wl = gen.Workload(name="u", T=1, rows=(R,), D=4, dtype="f32", B=R // 100,
                      pooling=("fixed", 100), dists=(("uniform",),), seed=123)
    b = gen.make_batches(wl, 1)[0]
    assert b.num_lookups == R
    pct = 100.0 * len(np.unique(b.indices)) / R
    assert abs(pct - GOLD["unique_access_pct"]["random"]) < 0.2
    assert abs(GOLD["unique_access_pct"]["random"] - 100 * (1 - math.exp(-1))) < 0.005
    assert b.indices.min() >= 0 and b.indices.max() < R


def test_one_item_unique_fraction_matches_paper():
    R = GOLD["unique_access_pct"]["rows"]
    wl = gen.Workload(name="o", T=1, rows=(R,), D=4, dtype="f32", B=R // 100,
                      pooling=("fixed", 100), dists=(("one_item",),), seed=5)
    b = gen.make_batches(wl, 1)[0]
    assert len(np.unique(b.indices)) == 1
    assert abs(100.0 / R - GOLD["unique_access_pct"]["one_item"]) < 1e-9


@pytest.mark.parametrize("alpha", [1.05, 1.2])
def test_zipf_head_mass(alpha):
    R, n = 200_000, 400_000
    rng = np.random.Generator(np.random.Philox(key=np.array([7, 7], dtype=np.uint64)))
    ranks = gen.zipf_ranks(rng, R, alpha, n)
    assert ranks.min() >= 0 and ranks.max() < R
    w = np.arange(1, R + 1, dtype=np.float64) ** -alpha
    for k in (1, 10, 1000, 50_000):
        expect = w[:k].sum() / w.sum()
        got = np.mean(ranks < k)
        assert abs(got - expect) < 4 * math.sqrt(expect * (1 - expect) / n) + 1e-3


def test_zipf_rows_are_permuted_ranks():
    wl = gen.Workload(name="z", T=2, rows=(5000, 3000), D=4, dtype="f32", B=50,
                      pooling=("fixed", 40), dists=(("zipf", 1.2), ("zipf", 1.2)), seed=9)
    for t in range(2):
        p = gen.table_permutation(wl, t)
        assert np.array_equal(np.sort(p), np.arange(wl.rows[t]))
    b = gen.make_batches(wl, 1)[0]
    seg0 = b.indices[: b.offsets[wl.B]]
    hot = np.bincount(seg0, minlength=5000).argmax()
    assert hot == gen.table_permutation(wl, 0)[0]  # the most frequent row is rank 1's image


def test_offsets_structure_and_length_ranges():
    for name in ("cfg1", "cfg2", "small_f32_d64"):
        wl = gen.workload(name)
        L = gen.make_lengths(wl)
        off = gen.lengths_to_offsets(L)
        assert off[0] == 0 and off[-1] == L.sum() and len(off) == wl.T * wl.B + 1
        assert np.all(np.diff(off) >= 0)
        if wl.pooling[0] == "fixed":
            assert np.all(L == wl.pooling[1])
        else:
            assert L.min() >= wl.pooling[1] and L.max() <= wl.pooling[2]
            assert L.min() == wl.pooling[1] and L.max() == wl.pooling[2]  # inclusive ends occur
    L2 = gen.make_lengths(gen.workload("cfg2"))
    assert abs(L2.mean() - 20.5) < 0.2


def test_indices_in_range_per_table_and_deterministic():
    wl = gen.workload("small_f32_d64")
    a, a2 = gen.make_batches(wl, 2)
    b = gen.make_batches(wl, 1)[0]
    assert np.array_equal(a.indices, b.indices) and np.array_equal(a.offsets, b.offsets)
    assert not np.array_equal(a.offsets, a2.offsets)
    again = gen.make_batches(wl, 1, first_batch=1)[0]
    assert np.array_equal(again.indices, a2.indices)
    for t in range(wl.T):
        s, e = a.offsets[t * wl.B], a.offsets[(t + 1) * wl.B]
        seg = a.indices[s:e]
        assert seg.min() >= 0 and seg.max() < wl.rows[t]


def test_table_values_distribution_and_determinism():
    v = gen.table_values(0x5EED0003, np.arange(4096), 128, "f32")
    assert v.dtype == np.float32 and v.shape == (4096, 128)
    assert abs(v.mean()) < 1e-3 and abs(v.std() - 0.1) < 1e-3      # N(0, 0.1^2), sigma = 0.1
    assert np.array_equal(v[100:200], gen.table_values(0x5EED0003, np.arange(100, 200), 128))
    assert not np.array_equal(v, gen.table_values(0x5EED0004, np.arange(4096), 128))
    h = gen.table_values(0x5EED0003, np.arange(4096), 128, "f16")
    assert h.dtype == np.float16 and np.array_equal(h, v.astype(np.float16))
    bf = gen.table_values(0x5EED0003, np.arange(4096), 128, "bf16")
    assert bf.dtype == np.uint16
    back = (bf.astype(np.uint32) << np.uint32(16)).view(np.float32)
    assert np.all(np.abs(back - v) <= np.abs(v) * 2.0 ** -8)               # 8 significant bits
    torch_bf = __import__("torch").from_numpy(v).to(__import__("torch").bfloat16)
    assert np.array_equal(torch_bf.view(__import__("torch").int16).numpy().view(np.uint16), bf)
    k = gen.table_values(1, np.arange(512), 64, "f32", gen.KIND_INT)
    assert k.min() == -8 and k.max() == 7 and np.array_equal(k, np.round(k))
    # rows and columns are not interchangeable and no two rows coincide
    assert len({r.tobytes() for r in v}) == 4096
    r = gen.table_values_range(0x5EED0003, 10, 300, 128, chunk_rows=64)
    assert np.array_equal(r, v[10:310])


def test_compact_rows_reproduces_full_problem(oracle):
    wl = gen.workload("small_f32_d128")
    batch = gen.make_batches(wl, 1)[0]
    arena = gen.host_arena(wl)
    ref, _ = oracle.emb_bag(arena, wl.table_offsets(), batch.indices, batch.offsets, wl.B)
    bags = [0, 5, wl.B, 2 * wl.B + 17, wl.T * wl.B - 1]
    small, ix, off, wsmall = gen.compact_rows(wl, batch, bags)
    assert wsmall is None
    r2, _ = oracle.emb_bag(small, np.array([0, len(small)], np.int64), ix, off, len(bags))
    for i, g in enumerate(bags):
        t, b = divmod(g, wl.B)
        assert np.array_equal(r2[i], ref[b, t * wl.D:(t + 1) * wl.D])


def test_compact_rows_carries_weights(oracle):
    wl = gen.with_overrides(gen.workload("small_f32_d64"), weighted=True)
    batch = gen.make_batches(wl, 1)[0]
    arena = gen.host_arena(wl)
    ref, _ = oracle.emb_bag(arena, wl.table_offsets(), batch.indices, batch.offsets, wl.B,
                            weights=batch.weights)
    bags = [1, wl.B + 3, wl.T * wl.B - 2]
    small, ix, off, wsmall = gen.compact_rows(wl, batch, bags)
    r2, _ = oracle.emb_bag(small, np.array([0, len(small)], np.int64), ix, off, len(bags), weights=wsmall)
    for i, g in enumerate(bags):
        t, b = divmod(g, wl.B)
        assert np.array_equal(r2[i], ref[b, t * wl.D:(t + 1) * wl.D])


def test_config_sizes_match_the_stated_shapes():
    c3 = gen.workload("cfg3")
    assert c3.table_bytes == 122_880_000_000 and c3.row_bytes == 512
    assert c3.num_bags * 80 == 19_660_800
    c5 = gen.workload("cfg5")
    assert c5.table_bytes == 102_400_000_000 and c5.row_bytes == 512
    assert sum(d[0] == "zipf" for d in c5.dists) == 50
    p = gen.workload("paper")
    g = GOLD["bytes_per_table"]
    assert (p.B, p.pooling[1], p.D, p.elem_bytes) == (g["batch"], g["lookups_per_sample"], g["dim"], g["elem_bytes"])


def test_hotness_ladder_matches_the_papers_unique_access_table():
    """Sec. 3.2 table: unique access % 4.05 / 20.50 / 46.21 for high / med / low hot."""
    R = GOLD["unique_access_pct"]["rows"]
    want = {"paper_high": 4.05, "paper_med": 20.50, "paper_low": 46.21}
    for name, pct in want.items():
        alpha = gen.PAPER_HOTNESS_ALPHA[name]
        assert abs(100 * gen.expected_unique_fraction(R, alpha, R) - pct) < 0.05
    # and by sampling, for one of them
    rng = np.random.Generator(np.random.Philox(key=np.array([3, 4], dtype=np.uint64)))
    ranks = gen.zipf_ranks(rng, R, gen.PAPER_HOTNESS_ALPHA["paper_med"], R)
    assert abs(100 * len(np.unique(ranks)) / R - 20.50) < 0.3
    for name, counts in gen.PAPER_MIXES.items():
        wl = gen.workload(name)
        assert wl.T == sum(counts) == 250
        assert sum(d[0] == "uniform" for d in wl.dists) == counts[3]


def test_quantised_row_generators():
    """Row-wise quantised rows from the generator: layout, code ranges, scale and bias rules."""
    rows = np.arange(5000, dtype=np.uint64)
    for dtype in ("u8row", "fp8row"):
        for kind in (gen.KIND_NORMAL, gen.KIND_INT):
            t = gen.table_values(0x5EED, rows, 24, dtype, kind)
            assert t.dtype == np.uint8 and t.shape == (5000, 32)
            assert np.array_equal(t, gen.table_values(0x5EED, rows, 24, dtype, kind))
            scale = t[:, 24:28].copy().view(np.float32).ravel()
            bias = t[:, 28:32].copy().view(np.float32).ravel()
            codes = t[:, :24]
            if kind == gen.KIND_INT:
                assert np.all(scale == 1.0)
                assert np.all(bias == (-128.0 if dtype == "u8row" else -1.0))
            else:
                assert np.all(scale > 0) and len(np.unique(scale)) > 100
                assert np.allclose(bias, scale * (-128.0 if dtype == "u8row" else -32.0), rtol=1e-6)
            if dtype == "fp8row":
                assert not np.any((codes & 0x7F) == 0x7F)            # the two NaN codes never occur
                if kind == gen.KIND_INT:
                    assert not np.any(codes & 0x40)                  # exponent below 8: |value| < 2
                else:
                    assert len(np.unique(codes)) == 254
            else:
                assert len(np.unique(codes)) == 256
    # a different table seed gives different codes
    assert not np.array_equal(gen.table_values(1, rows[:50], 24, "fp8row"),
                              gen.table_values(2, rows[:50], 24, "fp8row"))
