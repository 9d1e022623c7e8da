"""Pins for the CPU oracle: it is checked against things other than itself.

The paper (Sec. 3.1, Algorithm 1) defines the embedding stage as a per-bag gather + sum of
table rows; it prints no output value of the operator.  So the oracle is pinned by
  * exact rational brute force on hand-sized inputs,
  * closed forms (identity tables -> index histograms, one-item case, len 1, empty bags),
  * invariants (mean = sum/len, permutation, linearity, weights),
  * library special cases (sparse incidence matrix x table; torch's CPU embedding_bag),
each chosen so that a dropped term, wrong index/offset, transposed operand or wrong table base
fails at least one of them.
"""
from fractions import Fraction

import numpy as np
import pytest

from inputgen import gen


def _rand_problem(rng, T, rows, D, B, max_len, dtype=np.float32, integer=False):
    toff = np.concatenate([[0], np.cumsum(rows)]).astype(np.int64)
    if integer:
        tables = rng.integers(-8, 8, size=(int(toff[-1]), D)).astype(dtype)
    else:
        tables = rng.normal(0, 0.1, size=(int(toff[-1]), D)).astype(dtype)
    lengths = rng.integers(0, max_len + 1, size=T * B)
    offsets = gen.lengths_to_offsets(lengths)
    idx = np.empty(int(offsets[-1]), dtype=np.int64)
    for t in range(T):
        s, e = offsets[t * B], offsets[(t + 1) * B]
        idx[s:e] = rng.integers(0, rows[t], size=e - s)
    return tables, toff, idx, offsets


def _brute_force_fraction(tables, toff, idx, offsets, B, mode, weights=None):
    """Exact rational arithmetic, pure Python loops, written straight from the definition."""
    T = len(toff) - 1
    D = tables.shape[1]
    out = [[Fraction(0)] * (T * D) for _ in range(B)]
    mag = [[Fraction(0)] * (T * D) for _ in range(B)]
    for t in range(T):
        for b in range(B):
            lo, hi = int(offsets[t * B + b]), int(offsets[t * B + b + 1])
            for d in range(D):
                a = Fraction(0)
                m = Fraction(0)
                for j in range(lo, hi):
                    x = Fraction(float(tables[int(toff[t]) + int(idx[j]), d]))
                    w = Fraction(float(weights[j])) if weights is not None else Fraction(1)
                    a += w * x
                    m += abs(w * x)
                if mode == "mean":
                    a = a / (hi - lo) if hi > lo else Fraction(0)
                    m = m / (hi - lo) if hi > lo else Fraction(0)
                out[b][t * D + d] = a
                mag[b][t * D + d] = m
    return out, mag


@pytest.mark.parametrize("mode", ["sum", "mean"])
@pytest.mark.parametrize("dtype", [np.float32, np.float16])
def test_brute_force_exact_rational(oracle, mode, dtype):
    rng = np.random.default_rng(11)
    T, rows, D, B = 3, [8, 5, 7], 4, 4
    tables, toff, idx, offsets = _rand_problem(rng, T, rows, D, B, 5, dtype)
    ref, bound = oracle.emb_bag(tables, toff, idx, offsets, B, mode)
    exact, mag = _brute_force_fraction(tables, toff, idx, offsets, B, mode)
    for b in range(B):
        for c in range(T * D):
            # fp64 accumulation of <= 5 fp32-exact terms: error <= 5 ulp(fp64) of the magnitude
            tol = 8 * 2.0 ** -53 * float(mag[b][c]) + 1e-300
            assert abs(ref[b, c] - float(exact[b][c])) <= tol
            assert abs(bound[b, c] - float(mag[b][c])) <= tol


def test_brute_force_weighted(oracle):
    rng = np.random.default_rng(12)
    T, rows, D, B = 2, [6, 3], 4, 3
    tables, toff, idx, offsets = _rand_problem(rng, T, rows, D, B, 4)
    w = rng.uniform(-1, 1, size=len(idx)).astype(np.float32)
    ref, bound = oracle.emb_bag(tables, toff, idx, offsets, B, "sum", weights=w)
    exact, mag = _brute_force_fraction(tables, toff, idx, offsets, B, "sum", w)
    for b in range(B):
        for c in range(T * D):
            tol = 16 * 2.0 ** -53 * float(mag[b][c]) + 1e-300
            assert abs(ref[b, c] - float(exact[b][c])) <= tol
            assert abs(bound[b, c] - float(mag[b][c])) <= tol


def test_hand_worked_example(oracle):
    """A case small enough to do on paper; values typed in, not computed."""
    # table 0 has 3 rows, table 1 has 2 rows, D = 2
    tables = np.array([[1, 2], [10, 20], [100, 200],      # table 0
                       [-1, 5], [3, -7]], dtype=np.float32)  # table 1
    toff = np.array([0, 3, 5], dtype=np.int64)
    B = 2
    # bags (t,b): (0,0)=[2,0,2]  (0,1)=[]  (1,0)=[1]  (1,1)=[0,1,1,0]
    idx = np.array([2, 0, 2, 1, 0, 1, 1, 0], dtype=np.int64)
    offsets = np.array([0, 3, 3, 4, 8], dtype=np.int64)
    ref, bound = oracle.emb_bag(tables, toff, idx, offsets, B, "sum")
    assert ref.tolist() == [[201.0, 402.0, 3.0, -7.0], [0.0, 0.0, 4.0, -4.0]]
    assert bound.tolist() == [[201.0, 402.0, 3.0, 7.0], [0.0, 0.0, 8.0, 24.0]]
    ref, bound = oracle.emb_bag(tables, toff, idx, offsets, B, "mean")
    assert ref.tolist() == [[67.0, 134.0, 3.0, -7.0], [0.0, 0.0, 1.0, -1.0]]
    assert bound.tolist() == [[67.0, 134.0, 3.0, 7.0], [0.0, 0.0, 2.0, 6.0]]
    # out_ld wider than T*D: extra columns untouched (zero), layout is [b, t*D + d]
    ref, _ = oracle.emb_bag(tables, toff, idx, offsets, B, "sum", out_ld=6)
    assert ref.tolist() == [[201.0, 402.0, 3.0, -7.0, 0.0, 0.0], [0.0, 0.0, 4.0, -4.0, 0.0, 0.0]]


def test_identity_tables_give_index_histograms(oracle):
    """With table_t = I (R = D) the output row of bag (t,b) counts how often each index occurs."""
    rng = np.random.default_rng(13)
    T, D, B = 3, 16, 9
    tables = np.concatenate([np.eye(D, dtype=np.float32)] * T)
    toff = np.arange(T + 1, dtype=np.int64) * D
    lengths = rng.integers(0, 40, size=T * B)
    offsets = gen.lengths_to_offsets(lengths)
    idx = rng.integers(0, D, size=int(offsets[-1]))
    ref, bound = oracle.emb_bag(tables, toff, idx, offsets, B, "sum")
    for t in range(T):
        for b in range(B):
            s, e = offsets[t * B + b], offsets[t * B + b + 1]
            hist = np.bincount(idx[s:e], minlength=D).astype(np.float64)
            assert np.array_equal(ref[b, t * D:(t + 1) * D], hist)
            assert np.array_equal(bound[b, t * D:(t + 1) * D], hist)


def test_table_base_is_respected(oracle):
    """Tables holding a constant equal to their number: a wrong table base shows at once."""
    T, D, B, R = 4, 8, 5, [3, 9, 2, 6]
    toff = np.concatenate([[0], np.cumsum(R)]).astype(np.int64)
    tables = np.concatenate([np.full((R[t], D), t + 1, dtype=np.float32) for t in range(T)])
    rng = np.random.default_rng(14)
    lengths = rng.integers(0, 7, size=T * B)
    offsets = gen.lengths_to_offsets(lengths)
    idx = np.concatenate([rng.integers(0, R[t], size=int(offsets[(t + 1) * B] - offsets[t * B]))
                          for t in range(T)]).astype(np.int64)
    ref, _ = oracle.emb_bag(tables, toff, idx, offsets, B, "sum")
    for t in range(T):
        for b in range(B):
            assert np.all(ref[b, t * D:(t + 1) * D] == (t + 1) * lengths[t * B + b])


def test_one_item_case(oracle):
    """Paper Sec. 3.2 'one item': every index names the same row -> sum = len*row, mean = row."""
    rng = np.random.default_rng(15)
    R, D, B = 50, 12, 6
    table = rng.normal(0, 0.1, size=(R, D)).astype(np.float32)
    toff = np.array([0, R], dtype=np.int64)
    lengths = np.array([1, 2, 4, 8, 16, 64])  # powers of two: len*row is exact in fp64
    offsets = gen.lengths_to_offsets(lengths)
    idx = np.full(int(offsets[-1]), 17, dtype=np.int64)
    s, _ = oracle.emb_bag(table, toff, idx, offsets, B, "sum")
    m, _ = oracle.emb_bag(table, toff, idx, offsets, B, "mean")
    for b in range(B):
        assert np.array_equal(s[b], table[17].astype(np.float64) * lengths[b])
        assert np.array_equal(m[b], table[17].astype(np.float64))


def test_mean_is_sum_over_len_and_edge_lengths(oracle):
    rng = np.random.default_rng(16)
    T, rows, D, B = 2, [40, 9], 8, 12
    tables, toff, idx, offsets = _rand_problem(rng, T, rows, D, B, 30)
    lengths = np.diff(offsets)
    assert (lengths == 0).any() and (lengths > 1).any()
    s, sb = oracle.emb_bag(tables, toff, idx, offsets, B, "sum")
    m, mb = oracle.emb_bag(tables, toff, idx, offsets, B, "mean")
    for t in range(T):
        for b in range(B):
            L = lengths[t * B + b]
            sl = slice(t * D, (t + 1) * D)
            if L == 0:
                assert np.all(s[b, sl] == 0) and np.all(m[b, sl] == 0) and np.all(mb[b, sl] == 0)
                assert not np.signbit(m[b, sl]).any()
            else:
                assert np.array_equal(m[b, sl], s[b, sl] / L)
                assert np.array_equal(mb[b, sl], sb[b, sl] / L)


def test_empty_and_len1_bags(oracle):
    table = np.arange(12, dtype=np.float32).reshape(3, 4) - 5
    toff = np.array([0, 3], dtype=np.int64)
    offsets = np.array([0, 0, 1, 1, 2], dtype=np.int64)  # lengths 0,1,0,1
    idx = np.array([2, 0], dtype=np.int64)
    for mode in ("sum", "mean"):
        r, b = oracle.emb_bag(table, toff, idx, offsets, 4, mode)
        assert np.array_equal(r, np.array([[0] * 4, table[2], [0] * 4, table[0]], dtype=np.float64))
        assert np.array_equal(b, np.abs(r))
    # all bags empty, no indices at all
    r, b = oracle.emb_bag(table, toff, np.zeros(0, np.int64), np.zeros(5, np.int64), 4, "sum")
    assert not r.any() and not b.any()
    # B = 0
    r, b = oracle.emb_bag(table, toff, np.zeros(0, np.int64), np.zeros(1, np.int64), 0, "sum")
    assert r.shape == (0, 4)


def test_permutation_invariance(oracle):
    rng = np.random.default_rng(17)
    T, rows, D, B = 3, [20, 11, 64], 8, 10
    for integer in (True, False):
        tables, toff, idx, offsets = _rand_problem(rng, T, rows, D, B, 25, integer=integer)
        r0, b0 = oracle.emb_bag(tables, toff, idx, offsets, B, "sum")
        idx2 = idx.copy()
        for g in range(T * B):
            s, e = offsets[g], offsets[g + 1]
            idx2[s:e] = rng.permutation(idx2[s:e])
        r1, b1 = oracle.emb_bag(tables, toff, idx2, offsets, B, "sum")
        if integer:
            assert np.array_equal(r0, r1) and np.array_equal(b0, b1)
        else:
            assert np.all(np.abs(r0 - r1) <= 1e-14 * b0 + 1e-300)


def test_weights(oracle):
    rng = np.random.default_rng(18)
    T, rows, D, B = 2, [30, 12], 8, 7
    tables, toff, idx, offsets = _rand_problem(rng, T, rows, D, B, 9)
    r0, b0 = oracle.emb_bag(tables, toff, idx, offsets, B, "sum")
    r1, b1 = oracle.emb_bag(tables, toff, idx, offsets, B, "sum",
                            weights=np.ones(len(idx), np.float32))
    assert np.array_equal(r0, r1) and np.array_equal(b0, b1)
    # a selector weight picks out one row of each non-empty bag
    w = np.zeros(len(idx), np.float32)
    pick = {}
    for g in range(T * B):
        s, e = offsets[g], offsets[g + 1]
        if e > s:
            j = int(rng.integers(s, e))
            w[j] = 2.0
            pick[g] = j
    r2, _ = oracle.emb_bag(tables, toff, idx, offsets, B, "sum", weights=w)
    for g, j in pick.items():
        t, b = divmod(g, B)
        assert np.array_equal(r2[b, t * D:(t + 1) * D],
                              2.0 * tables[toff[t] + idx[j]].astype(np.float64))
    with pytest.raises(ValueError):
        oracle.emb_bag(tables, toff, idx, offsets, B, "mean", weights=w)


def test_linearity_on_integer_tables(oracle):
    rng = np.random.default_rng(19)
    T, rows, D, B = 2, [15, 33], 8, 6
    A, toff, idx, offsets = _rand_problem(rng, T, rows, D, B, 12, integer=True)
    Bm = rng.integers(-8, 8, size=A.shape).astype(np.float32)
    ra, _ = oracle.emb_bag(A, toff, idx, offsets, B, "sum")
    rb, _ = oracle.emb_bag(Bm, toff, idx, offsets, B, "sum")
    rab, _ = oracle.emb_bag(A + Bm, toff, idx, offsets, B, "sum")
    assert np.array_equal(rab, ra + rb)


def test_bound_is_sum_of_abs_terms(oracle):
    rng = np.random.default_rng(20)
    T, rows, D, B = 2, [15, 33], 8, 6
    A, toff, idx, offsets = _rand_problem(rng, T, rows, D, B, 12)
    w = rng.uniform(-1, 1, len(idx)).astype(np.float32)
    _, bound = oracle.emb_bag(A, toff, idx, offsets, B, "sum", weights=w)
    r_abs, _ = oracle.emb_bag(np.abs(A), toff, idx, offsets, B, "sum", weights=np.abs(w))
    assert np.allclose(bound, r_abs, rtol=1e-15, atol=0)
    assert np.all(bound >= 0)


def test_strict_bound_equals_the_bound_for_unquantised_rows(oracle):
    """For fp32 / fp16 / bf16 rows an element is one term: the strict scale is the bound itself;
    for max pooling it is the magnitude of the selected element."""
    rng = np.random.default_rng(21)
    T, rows, D, B = 2, [15, 33], 8, 6
    A, toff, idx, offsets = _rand_problem(rng, T, rows, D, B, 12)
    w = rng.uniform(-1, 1, len(idx)).astype(np.float32)
    for mode, weights in (("sum", None), ("sum", w), ("mean", None), ("max", None)):
        ref, bound, strict = oracle.emb_bag(A, toff, idx, offsets, B, mode, weights=weights, strict=True)
        assert np.array_equal(bound, strict)
        if mode == "max":
            assert np.array_equal(strict, np.abs(ref))
    ref, bound, strict = oracle.emb_bag(A.astype(np.float16), toff, idx, offsets, B, "sum", strict=True)
    assert np.array_equal(bound, strict)


def test_second_opinion_sparse_matmul(oracle):
    """Per table, sum pooling is (bag-incidence CSR matrix) x (table): a library SpMM."""
    import scipy.sparse as sp
    wl = gen.workload("small_f32_d64")
    batch = gen.make_batches(wl, 1)[0]
    arena = gen.host_arena(wl)
    toff = wl.table_offsets()
    ref, _ = oracle.emb_bag(arena, toff, batch.indices, batch.offsets, wl.B, "sum")
    for t in range(wl.T):
        o = batch.offsets[t * wl.B:(t + 1) * wl.B + 1]
        ix = batch.indices[o[0]:o[-1]]
        M = sp.csr_matrix((np.ones(len(ix)), ix, o - o[0]), shape=(wl.B, wl.rows[t]))
        want = M @ arena[toff[t]:toff[t + 1]].astype(np.float64)
        got = ref[:, t * wl.D:(t + 1) * wl.D]
        assert np.allclose(got, want, rtol=1e-12, atol=1e-15)


@pytest.mark.parametrize("name,mode", [("small_f32_d128", "sum"), ("small_f32_d128", "mean"),
                                       ("small_f16_d256", "sum")])
def test_second_opinion_torch_cpu(oracle, name, mode):
    import torch
    import torch.nn.functional as F
    wl = gen.workload(name)
    batch = gen.make_batches(wl, 1)[0]
    arena = gen.host_arena(wl)
    toff = wl.table_offsets()
    ref, _ = oracle.emb_bag(arena, toff, batch.indices, batch.offsets, wl.B, mode)
    for t in range(wl.T):
        o = batch.offsets[t * wl.B:(t + 1) * wl.B + 1]
        ix = torch.from_numpy(batch.indices[o[0]:o[-1]])
        W = torch.from_numpy(arena[toff[t]:toff[t + 1]].astype(np.float64))
        want = F.embedding_bag(ix, W, torch.from_numpy(o[:-1] - o[0]), mode=mode).numpy()
        got = ref[:, t * wl.D:(t + 1) * wl.D]
        assert np.allclose(got, want, rtol=1e-12, atol=1e-15)


def test_half_widening_is_exact(oracle):
    """Every finite half bit pattern, looked up alone, must come back as its exact value."""
    bits = np.arange(0, 1 << 16, dtype=np.uint16)
    halves = bits.view(np.float16)
    finite = np.isfinite(halves)
    table = halves.reshape(-1, 8)  # 8192 rows of 8
    R = table.shape[0]
    toff = np.array([0, R], dtype=np.int64)
    idx = np.arange(R, dtype=np.int64)
    offsets = np.arange(R + 1, dtype=np.int64)
    ref, _ = oracle.emb_bag(table, toff, idx, offsets, R, "sum")
    got = ref.reshape(-1)
    want = halves.astype(np.float64)
    assert np.array_equal(got[finite], want[finite])
    assert np.all(np.isnan(got[np.isnan(halves)]))
    assert np.array_equal(got[np.isinf(halves)], want[np.isinf(halves)])


def test_bfloat16_widening_is_exact(oracle):
    """Every bfloat16 bit pattern, looked up alone, comes back as the binary32 with those upper bits."""
    bits = np.arange(0, 1 << 16, dtype=np.uint16)
    with np.errstate(invalid="ignore"):   # signalling NaN patterns are part of the sweep
        want = (bits.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    table = bits.reshape(-1, 8)
    R = table.shape[0]
    ref, _ = oracle.emb_bag(table, np.array([0, R], np.int64), np.arange(R, dtype=np.int64),
                            np.arange(R + 1, dtype=np.int64), R, "sum")
    got = ref.reshape(-1)
    fin = np.isfinite(want)
    assert np.array_equal(got[fin], want[fin])
    assert np.all(np.isnan(got[np.isnan(want)]))
    assert np.array_equal(got[np.isinf(want)], want[np.isinf(want)])
    # and sums of bfloat16 rows agree with the same rows given as float32
    rng = np.random.default_rng(21)
    b16 = rng.integers(0x3C00, 0x4100, size=(40, 8)).astype(np.uint16)
    f32 = (b16.astype(np.uint32) << np.uint32(16)).view(np.float32)
    idx = rng.integers(0, 40, size=30).astype(np.int64)
    off = np.array([0, 7, 7, 30], dtype=np.int64)
    toff = np.array([0, 40], dtype=np.int64)
    ra, ba = oracle.emb_bag(b16, toff, idx, off, 3, "mean")
    rb, bb = oracle.emb_bag(f32, toff, idx, off, 3, "mean")
    assert np.array_equal(ra, rb) and np.array_equal(ba, bb)


def _quantised_table(rng, rows, D):
    """uint8 [rows, D + 8]: D codes, then fp32 scale and fp32 bias (little endian)."""
    t = np.zeros((rows, D + 8), dtype=np.uint8)
    t[:, :D] = rng.integers(0, 256, size=(rows, D))
    scale = rng.uniform(0.001, 0.01, size=rows).astype(np.float32)
    bias = rng.uniform(-1.0, 1.0, size=rows).astype(np.float32)
    t[:, D:D + 4] = scale.view(np.uint8).reshape(rows, 4)
    t[:, D + 4:D + 8] = bias.view(np.uint8).reshape(rows, 4)
    return t, scale, bias


def test_quantised_rows_brute_force(oracle):
    """Row-wise quantised rows: element = scale * code + bias, checked in exact rationals."""
    rng = np.random.default_rng(31)
    R, D, B = 9, 8, 4
    table, scale, bias = _quantised_table(rng, R, D)
    toff = np.array([0, 5, 9], dtype=np.int64)          # two tables of 5 and 4 rows
    lengths = np.array([3, 0, 2, 4, 1, 0, 5, 2])
    offsets = gen.lengths_to_offsets(lengths)
    idx = np.concatenate([rng.integers(0, 5, size=lengths[:4].sum()),
                          rng.integers(0, 4, size=lengths[4:].sum())]).astype(np.int64)
    w = rng.uniform(-1, 1, size=len(idx)).astype(np.float32)
    for mode, weights in (("sum", None), ("mean", None), ("sum", w)):
        ref, bound, strict = oracle.emb_bag(table, toff, idx, offsets, B, mode, weights=weights,
                                            strict=True)
        for t in range(2):
            for b in range(B):
                lo, hi = int(offsets[t * B + b]), int(offsets[t * B + b + 1])
                for d in range(D):
                    a = Fraction(0)
                    m = Fraction(0)
                    sm = Fraction(0)             # the strict scale: |w * element|, one term each
                    for j in range(lo, hi):
                        r = int(toff[t]) + int(idx[j])
                        ww = Fraction(float(weights[j])) if weights is not None else Fraction(1)
                        sc = Fraction(float(scale[r])) * int(table[r, d])
                        a += ww * (sc + Fraction(float(bias[r])))
                        m += abs(ww) * (abs(sc) + abs(Fraction(float(bias[r]))))
                        sm += abs(ww * (sc + Fraction(float(bias[r]))))
                    if mode == "mean" and hi > lo:
                        a, m, sm = a / (hi - lo), m / (hi - lo), sm / (hi - lo)
                    tol = 16 * 2.0 ** -53 * float(m) + 1e-300
                    assert abs(ref[b, t * D + d] - float(a)) <= tol
                    assert abs(bound[b, t * D + d] - float(m)) <= tol
                    assert abs(strict[b, t * D + d] - float(sm)) <= tol
        assert np.all(strict <= bound * (1 + 1e-15)) and np.all(np.abs(ref) <= strict * (1 + 1e-12) + 1e-300)
        assert np.any(strict < 0.9 * bound)       # scale * code and bias have opposite signs here


def test_quantised_rows_equal_their_dequantised_table(oracle):
    """Looking up quantised rows equals looking up the table dequantised in fp64 beforehand
    (here: codes chosen so that scale * code + bias is exact in fp32)."""
    rng = np.random.default_rng(32)
    R, D, B = 40, 24, 6
    table = np.zeros((R, D + 8), dtype=np.uint8)
    table[:, :D] = rng.integers(0, 256, size=(R, D))
    scale = (2.0 ** rng.integers(-6, 2, size=R)).astype(np.float32)      # powers of two
    bias = (scale * rng.integers(-128, 128, size=R)).astype(np.float32)
    table[:, D:D + 4] = scale.view(np.uint8).reshape(R, 4)
    table[:, D + 4:] = bias.view(np.uint8).reshape(R, 4)
    deq = (scale[:, None] * table[:, :D].astype(np.float32) + bias[:, None]).astype(np.float32)
    toff = np.array([0, R], dtype=np.int64)
    lengths = rng.integers(0, 12, size=B)
    offsets = gen.lengths_to_offsets(lengths)
    idx = rng.integers(0, R, size=int(offsets[-1])).astype(np.int64)
    rq, bq = oracle.emb_bag(table, toff, idx, offsets, B, "sum")
    rf, bf = oracle.emb_bag(deq, toff, idx, offsets, B, "sum")
    assert np.array_equal(rq, rf)
    assert np.all(bq >= bf)          # |scale*code| + |bias| >= |scale*code + bias|
    # a single lookup returns the dequantised row itself
    r1, _ = oracle.emb_bag(table, toff, np.array([7], np.int64), np.array([0, 1], np.int64), 1)
    assert np.array_equal(r1[0], deq[7].astype(np.float64))


def test_rejects_bad_inputs(oracle):
    table = np.ones((4, 4), np.float32)
    toff = np.array([0, 4], dtype=np.int64)
    with pytest.raises(ValueError, match="index out of range"):
        oracle.emb_bag(table, toff, np.array([4], np.int64), np.array([0, 1], np.int64), 1)
    with pytest.raises(ValueError, match="index out of range"):
        oracle.emb_bag(table, toff, np.array([-1], np.int64), np.array([0, 1], np.int64), 1)
    with pytest.raises(ValueError, match="offsets"):
        oracle.emb_bag(table, toff, np.array([0, 1], np.int64), np.array([0, 2, 1, 2], np.int64), 3)


def test_thread_count_does_not_change_result(oracle):
    wl = gen.workload("small_f32_d64")
    batch = gen.make_batches(wl, 1)[0]
    arena = gen.host_arena(wl)
    n = oracle.num_threads()
    try:
        oracle.set_num_threads(1)
        r1, b1 = oracle.emb_bag(arena, wl.table_offsets(), batch.indices, batch.offsets, wl.B)
        oracle.set_num_threads(max(2, n))
        r2, b2 = oracle.emb_bag(arena, wl.table_offsets(), batch.indices, batch.offsets, wl.B)
    finally:
        oracle.set_num_threads(n)
    assert np.array_equal(r1, r2) and np.array_equal(b1, b2)


# ---- the reuse-profile oracle (integer work) -------------------------------------------------
def test_reuse_profile_hand_worked():
    from oracle import reuse_oracle
    # T = 2, B = 2.  table 0 lookups: [5,5,7,5 | 9]  table 1 lookups: [ | 1,2,3]; 128-byte rows
    idx = np.array([5, 5, 7, 5, 9, 1, 2, 3], dtype=np.int64)
    off = np.array([0, 4, 5, 5, 8], dtype=np.int64)
    # table 0: w = 5, d = 2, n_t = 5: 5 * 2 * 1000 = 10000 against 75 * 25 = 1875; 25 * 128 < 2 * 2^29
    dup, used, hints = reuse_oracle.profile_reuse(idx, off, 2, 2, 4096, 75, row_bytes=128)
    assert dup.tolist() == [2, 0] and used.tolist() == [5, 3] and hints.tolist() == [0, 1]
    dup, used, hints = reuse_oracle.profile_reuse(idx, off, 2, 2, 2, 75, row_bytes=128)   # window of 2
    assert dup.tolist() == [1, 0] and used.tolist() == [2, 2] and hints.tolist() == [0, 1]
    # the threshold is a strict bound on the share of repeats: 2 of 5 is 400 permille
    assert reuse_oracle.profile_reuse(idx, off, 2, 2, 4096, 400, row_bytes=128)[2].tolist() == [0, 1]
    assert reuse_oracle.profile_reuse(idx, off, 2, 2, 4096, 401, row_bytes=128)[2].tolist() == [1, 1]
    idx9 = np.array([5, 5, 7, 6, 9, 4, 3, 2, 1, 1, 2, 3], dtype=np.int64)    # table 0: 1 repeat in 9
    off9 = np.array([0, 8, 9, 9, 12], dtype=np.int64)
    assert reuse_oracle.profile_reuse(idx9, off9, 2, 2, 4096, 111, row_bytes=128)[2].tolist() == [0, 1]
    assert reuse_oracle.profile_reuse(idx9, off9, 2, 2, 4096, 112, row_bytes=128)[2].tolist() == [1, 1]
    # a table that receives nothing is "streaming"
    dup, used, hints = reuse_oracle.profile_reuse(np.zeros(0, np.int64), np.zeros(3, np.int64), 2, 1, 8,
                                                  row_bytes=128)
    assert used.tolist() == [0, 0] and hints.tolist() == [1, 1]


def test_reuse_profile_closed_forms():
    from oracle import reuse_oracle
    n = 3000
    off = np.array([0, n, 2 * n, 3 * n], dtype=np.int64)
    rng = np.random.default_rng(3)
    uni = rng.integers(0, 4_000_000, size=n)
    idx = np.concatenate([np.arange(n), np.full(n, 42), uni]).astype(np.int64)
    dup, used, hints = reuse_oracle.profile_reuse(idx, off, 3, 1, 4096, row_bytes=512)
    assert used.tolist() == [n, n, n]
    assert dup[0] == 0 and dup[1] == n - 1
    # birthday problem: expected repeats of n uniform draws over R rows is about n^2 / (2R) = 1.1
    assert dup[2] == n - len(np.unique(uni)) and dup[2] < 12
    assert hints.tolist() == [1, 0, 1]


def _one_table_with_repeats(w, d, n):
    """n lookups of one table: the first w hold exactly d repeats, the rest are all new."""
    head = np.concatenate([np.arange(d), np.arange(w - d)]).astype(np.int64)
    idx = np.concatenate([head, np.arange(n - w, dtype=np.int64) + 10_000_000])
    return idx, np.array([0, n], dtype=np.int64)


def test_reuse_profile_counts_the_whole_batch():
    """A table whose window shows few repeats is still re-used when the batch sends it many more
    lookups than the window holds: with d repeats among w examined draws, about n * d / w^2 of
    the table's n lookups repeat, and from the threshold (75 permille) on the table is not
    streaming."""
    from oracle import reuse_oracle
    w = 4096
    # d = 8: n * 8 * 1000 < 75 * 2^24 holds up to n = 157286 (128-byte rows: the cache rule asks for d < 4)
    for n, want in ((157286, 1), (157287, 0)):
        idx, off = _one_table_with_repeats(w, 8, n)
        dup, used, hints = reuse_oracle.profile_reuse(idx, off, 1, 1, w, 75, row_bytes=128)
        assert dup.tolist() == [8] and used.tolist() == [w] and hints.tolist() == [want], n
    # when the window covers the table's lookups the share is the measured one: 14 repeats in 200
    # draws are 70 permille, 15 are 75
    for d, want in ((14, 1), (15, 0)):
        idx = np.concatenate([np.arange(d), np.arange(200 - d)]).astype(np.int64)
        assert reuse_oracle.profile_reuse(idx, np.array([0, 200], np.int64), 1, 1, w, 75,
                                          row_bytes=128)[2].tolist() == [want]
    # rows narrower than a 128-byte line share it: 64-byte rows double the share, 32-byte rows
    # quadruple it (7 repeats in 200 are 35 permille, 3 are 15)
    for d, row_bytes, want in ((7, 64, 1), (8, 64, 0), (3, 32, 1), (4, 32, 0), (14, 256, 1), (15, 256, 0)):
        idx = np.concatenate([np.arange(d), np.arange(200 - d)]).astype(np.int64)
        assert reuse_oracle.profile_reuse(idx, np.array([0, 200], np.int64), 1, 1, w, 75,
                                          row_bytes=row_bytes)[2].tolist() == [want], (d, row_bytes)
    # all 200 draws equal, 16-byte rows: 199 / 200 of the draws repeat and a line holds 8 rows,
    # a share of 7960 permille
    idx, off = np.zeros(200, np.int64), np.array([0, 200], np.int64)
    assert reuse_oracle.profile_reuse(idx, off, 1, 1, w, 7960, row_bytes=16)[2].tolist() == [0]
    assert reuse_oracle.profile_reuse(idx, off, 1, 1, w, 7961, row_bytes=16)[2].tolist() == [1]
    # a threshold beyond 1,000,000 permille counts as 1,000,000: 100,000 lookups whose first 200
    # are all equal give an estimated share of 100000 * 199 / 200^2 = 497.5, i.e. 497,500 permille
    # of 128-byte rows and 995,000 of 64-byte rows
    idx = np.concatenate([np.zeros(200, np.int64), np.arange(99_800, dtype=np.int64) + 5])
    off = np.array([0, 100_000], np.int64)
    assert reuse_oracle.profile_reuse(idx, off, 1, 1, 200, 497_500, row_bytes=128)[2].tolist() == [0]
    assert reuse_oracle.profile_reuse(idx, off, 1, 1, 200, 497_501, row_bytes=128)[2].tolist() == [1]
    assert reuse_oracle.profile_reuse(idx, off, 1, 1, 200, 1_000_000, row_bytes=64)[2].tolist() == [1]
    assert reuse_oracle.profile_reuse(idx, off, 1, 1, 200, 2_000_000_000, row_bytes=32)[2].tolist() == [0]


def test_reuse_profile_rows_in_use_beyond_the_cache():
    """d repeats among w draws put the rows in use at w^2 / 2d.  With w = 4096 and 512-byte rows
    that is 2^33 / 2d bytes: above 256 MiB = 2^28 for d < 16, whatever the batch sends; 256-byte
    rows halve it (d < 8)."""
    from oracle import reuse_oracle
    w, n = 4096, 3_000_000      # n * d / w^2 is far above the share threshold for every d here
    for d, row_bytes, want in ((15, 512, 1), (16, 512, 0), (7, 256, 1), (8, 256, 0), (15, 256, 0),
                               (1, 32, 0), (0, 16, 1)):
        idx, off = _one_table_with_repeats(w, d, n)
        dup, used, hints = reuse_oracle.profile_reuse(idx, off, 1, 1, w, 75, row_bytes=row_bytes)
        assert dup.tolist() == [d] and hints.tolist() == [want], (d, row_bytes)
    # rows narrower than a line: 64-byte rows need twice the cache, 2^28 * 64 > d * 2^30 for d < 16
    for d, row_bytes, want in ((15, 64, 1), (16, 64, 0), (3, 32, 1), (4, 32, 0), (63, 128, 1), (64, 128, 0)):
        idx, off = _one_table_with_repeats(16384, d, n)
        assert reuse_oracle.profile_reuse(idx, off, 1, 1, 16384, 75, row_bytes=row_bytes)[2].tolist() == [want]
    # the largest window: 16384 draws, 1024-byte rows: 2^38 > d * 2^29 for d < 512
    idx, off = _one_table_with_repeats(16384, 511, n)
    assert reuse_oracle.profile_reuse(idx, off, 1, 1, 16384, 75, row_bytes=1024)[2].tolist() == [1]
    idx, off = _one_table_with_repeats(16384, 512, n)
    dup, used, hints = reuse_oracle.profile_reuse(idx, off, 1, 1, 16384, 75, row_bytes=1024)
    assert used.tolist() == [16384] and dup.tolist() == [512] and hints.tolist() == [0]
    # windows outside the interface's range are not defined here (the interface clamps them)
    for bad in (0, 16385, 1 << 20):
        with pytest.raises(ValueError):
            reuse_oracle.profile_reuse(idx, off, 1, 1, bad, 75, row_bytes=1024)


@pytest.mark.parametrize("name,seeds,want", [
    ("cfg1", 6, "1" * 8), ("cfg2", 4, "1" * 26), ("cfg3", 2, "1" * 60), ("cfg4", 1, "0" * 60),
    ("cfg5", 1, "1" * 50 + "0" * 50)])
def test_reuse_classification_of_the_benchmark_configurations(name, seeds, want):
    """The hints of the five benchmark configurations do not depend on the seed: uniform tables
    far larger than what a batch draws stream (cfg1-cfg3, the first half of cfg5), power-law
    tables do not (cfg4, the second half of cfg5).  For each, the repeat count of the window sits
    well away from the two thresholds."""
    import dataclasses
    from oracle import reuse_oracle
    base = gen.workload(name)
    for k in range(seeds):
        wl = dataclasses.replace(base, seed=base.seed + 977 * k)
        batch = gen.make_batches(wl, 1)[0]
        dup, used, hints = reuse_oracle.profile_reuse(batch.indices, batch.offsets, wl.T, wl.B, 16384,
                                                      row_bytes=wl.row_bytes)
        assert "".join(map(str, hints)) == want, (name, k, dup.tolist())


# ---- the hot-row profile oracle (integer work) -------------------------------------------------
def test_hot_rows_hand_worked():
    from oracle import hot_rows_oracle
    # T = 2, B = 2.  table 0 lookups: [5,5,7,5 | 9,7]   table 1 lookups: [ | 3,1,2]
    idx = np.array([5, 5, 7, 5, 9, 7, 3, 1, 2], dtype=np.int64)
    off = np.array([0, 4, 6, 6, 9], dtype=np.int64)
    ids, counts, num = hot_rows_oracle.profile_hot_rows(idx, off, 2, 2, 100, 3)
    assert ids.tolist() == [[5, 7, 9], [1, 2, 3]]            # 5 x3, 7 x2, 9 x1; ties: smaller id first
    assert counts.tolist() == [[3, 2, 1], [1, 1, 1]] and num.tolist() == [3, 3]
    ids, counts, num = hot_rows_oracle.profile_hot_rows(idx, off, 2, 2, 100, 2)   # k cuts the list
    assert ids.tolist() == [[5, 7], [1, 2]] and counts.tolist() == [[3, 2], [1, 1]]
    ids, counts, num = hot_rows_oracle.profile_hot_rows(idx, off, 2, 2, 100, 5)   # k beyond the ids
    assert ids.tolist() == [[5, 7, 9, -1, -1], [1, 2, 3, -1, -1]] and num.tolist() == [3, 3]
    assert counts.tolist() == [[3, 2, 1, 0, 0], [1, 1, 1, 0, 0]]
    ids, counts, num = hot_rows_oracle.profile_hot_rows(idx, off, 2, 2, 3, 2)     # window of 3: [5,5,7]
    assert ids.tolist() == [[5, 7], [1, 2]] and counts.tolist() == [[2, 1], [1, 1]]
    # ids that are no row ids are not counted; a table without lookups has no hot rows
    idx = np.array([-1, 4, 1 << 40, 4, (1 << 40) - 1, (1 << 40) - 2], dtype=np.int64)
    ids, counts, num = hot_rows_oracle.profile_hot_rows(idx, np.array([0, 6, 6]), 2, 1, 100, 3)
    assert ids.tolist() == [[4, (1 << 40) - 2, -1], [-1, -1, -1]] and num.tolist() == [2, 0]
    assert counts.tolist() == [[2, 1, 0], [0, 0, 0]]


def test_hot_rows_closed_forms_and_second_route():
    import collections
    from oracle import hot_rows_oracle
    n = 500
    # table 0: all distinct -> the k smallest ids, once each; table 1: one item -> one hot row;
    # table 2: id i occurs i + 1 times -> ids in descending order with counts id + 1
    tri = np.repeat(np.arange(40), np.arange(40) + 1)
    rng = np.random.default_rng(17)
    rng.shuffle(tri)
    idx = np.concatenate([rng.permutation(n) + 1000, np.full(n, 77), tri]).astype(np.int64)
    off = np.array([0, n, 2 * n, 2 * n + len(tri)], dtype=np.int64)
    ids, counts, num = hot_rows_oracle.profile_hot_rows(idx, off, 3, 1, 1 << 20, 8)
    assert ids[0].tolist() == list(range(1000, 1008)) and counts[0].tolist() == [1] * 8
    assert ids[1].tolist() == [77] + [-1] * 7 and counts[1].tolist() == [n] + [0] * 7
    assert ids[2].tolist() == list(range(39, 31, -1)) and counts[2].tolist() == list(range(40, 32, -1))
    assert num.tolist() == [8, 1, 8]
    # a Zipf sample: the same answer through collections.Counter
    zipf = np.minimum(rng.zipf(1.3, size=5000), 3000).astype(np.int64)
    ids, counts, num = hot_rows_oracle.profile_hot_rows(zipf, np.array([0, 5000]), 1, 1, 4000, 50)
    want = sorted(collections.Counter(zipf[:4000].tolist()).items(), key=lambda kv: (-kv[1], kv[0]))[:50]
    assert ids[0].tolist() == [kv[0] for kv in want] and counts[0].tolist() == [kv[1] for kv in want]
    assert ids[0, 0] == 1                                     # rank 1 is the most frequent


# ---- tables of different widths: the same definition, table by table ---------------------------
def test_mixed_widths_equal_the_uniform_oracle_when_widths_agree(oracle):
    rng = np.random.default_rng(41)
    T, rows, D, B = 3, [20, 7, 33], 8, 6
    tables, toff, idx, offsets = _rand_problem(rng, T, rows, D, B, 9)
    w = rng.uniform(-1, 1, len(idx)).astype(np.float32)
    per_table = [tables[toff[t]:toff[t + 1]] for t in range(T)]
    for mode, weights in (("sum", None), ("mean", None), ("sum", w)):
        r0, b0 = oracle.emb_bag(tables, toff, idx, offsets, B, mode, weights=weights)
        r1, b1 = oracle.emb_bag_mixed(per_table, idx, offsets, B, mode, weights=weights)
        assert np.array_equal(r0, r1) and np.array_equal(b0, b1)


def test_mixed_widths_hand_worked(oracle):
    t0 = np.array([[1, 2], [10, 20], [100, 200]], dtype=np.float32)          # D = 2
    t1 = np.array([[1, 2, 3, 4], [-1, -2, -3, -4]], dtype=np.float32)        # D = 4
    B = 2
    # bags (t,b): (0,0)=[2,0]  (0,1)=[1]  (1,0)=[]  (1,1)=[0,1,0]
    idx = np.array([2, 0, 1, 0, 1, 0], dtype=np.int64)
    offsets = np.array([0, 2, 3, 3, 6], dtype=np.int64)
    ref, bound = oracle.emb_bag_mixed([t0, t1], idx, offsets, B, "sum")
    assert ref.tolist() == [[101.0, 202.0, 0.0, 0.0, 0.0, 0.0], [10.0, 20.0, 1.0, 2.0, 3.0, 4.0]]
    assert bound.tolist() == [[101.0, 202.0, 0.0, 0.0, 0.0, 0.0], [10.0, 20.0, 3.0, 6.0, 9.0, 12.0]]
    ref, _ = oracle.emb_bag_mixed([t0, t1], idx, offsets, B, "mean", out_ld=8)
    assert ref.tolist() == [[50.5, 101.0, 0, 0, 0, 0, 0, 0],
                            [10.0, 20.0, 1 / 3, 2 / 3, 1.0, 4 / 3, 0, 0]]


def test_mixed_widths_brute_force(oracle):
    rng = np.random.default_rng(42)
    dims, rows, B = [4, 12, 8], [6, 3, 9], 5
    tables = [rng.normal(0, 0.1, size=(rows[t], dims[t])).astype(np.float32) for t in range(3)]
    lengths = rng.integers(0, 6, size=3 * B)
    offsets = gen.lengths_to_offsets(lengths)
    idx = np.concatenate([rng.integers(0, rows[t], size=int(offsets[(t + 1) * B] - offsets[t * B]))
                          for t in range(3)]).astype(np.int64)
    ref, bound = oracle.emb_bag_mixed(tables, idx, offsets, B, "sum")
    col = 0
    for t in range(3):
        for b in range(B):
            lo, hi = int(offsets[t * B + b]), int(offsets[t * B + b + 1])
            for d in range(dims[t]):
                a = sum((Fraction(float(tables[t][int(idx[j]), d])) for j in range(lo, hi)), Fraction(0))
                m = sum((abs(Fraction(float(tables[t][int(idx[j]), d]))) for j in range(lo, hi)), Fraction(0))
                assert abs(ref[b, col + d] - float(a)) <= 8 * 2.0 ** -53 * float(m) + 1e-300
                assert abs(bound[b, col + d] - float(m)) <= 8 * 2.0 ** -53 * float(m) + 1e-300
        col += dims[t]


# ------------------------------------------------------------------------------------------
# max pooling (not in the paper: the usual third mode of an embedding-bag operator)
# ------------------------------------------------------------------------------------------
def test_max_hand_worked(oracle):
    """Values typed in.  All-negative bags show that the maximum does not start from zero."""
    tables = np.array([[1, -2], [10, -20], [-100, 200],      # table 0
                       [-1, -5], [-3, -7]], dtype=np.float32)  # table 1
    toff = np.array([0, 3, 5], dtype=np.int64)
    # bags (t,b): (0,0)=[2,0,2]  (0,1)=[]  (1,0)=[1]  (1,1)=[0,1,1,0]
    idx = np.array([2, 0, 2, 1, 0, 1, 1, 0], dtype=np.int64)
    offsets = np.array([0, 3, 3, 4, 8], dtype=np.int64)
    ref, bound = oracle.emb_bag(tables, toff, idx, offsets, 2, "max")
    assert ref.tolist() == [[1.0, 200.0, -3.0, -7.0], [0.0, 0.0, -1.0, -5.0]]
    assert bound.tolist() == [[1.0, 200.0, 3.0, 7.0], [0.0, 0.0, 1.0, 5.0]]


@pytest.mark.parametrize("dtype", [np.float32, np.float16])
def test_max_brute_force(oracle, dtype):
    rng = np.random.default_rng(21)
    T, rows, D, B = 3, [8, 5, 7], 4, 6
    tables, toff, idx, offsets = _rand_problem(rng, T, rows, D, B, 5, dtype)
    ref, bound = oracle.emb_bag(tables, toff, idx, offsets, B, "max")
    for t in range(T):
        for b in range(B):
            lo, hi = int(offsets[t * B + b]), int(offsets[t * B + b + 1])
            for d in range(D):
                vals = [Fraction(float(tables[int(toff[t]) + int(idx[j]), d])) for j in range(lo, hi)]
                want = max(vals) if vals else Fraction(0)
                assert Fraction(ref[b, t * D + d]) == want             # a table element: exact
                assert Fraction(bound[b, t * D + d]) == abs(want)


def test_max_invariants(oracle):
    rng = np.random.default_rng(22)
    T, rows, D, B = 2, [30, 9], 8, 10
    tables, toff, idx, offsets = _rand_problem(rng, T, rows, D, B, 12)
    mx, _ = oracle.emb_bag(tables, toff, idx, offsets, B, "max")
    mean, _ = oracle.emb_bag(tables, toff, idx, offsets, B, "mean")
    assert np.all(mx >= mean - 1e-12)                      # a maximum is at least the average
    # order inside a bag does not matter; duplicating a bag's lookups does not either
    idx2, off2 = [], [0]
    for g in range(T * B):
        seg = idx[offsets[g]:offsets[g + 1]]
        seg = np.concatenate([seg[::-1], seg])
        idx2.append(seg)
        off2.append(off2[-1] + len(seg))
    mx2, _ = oracle.emb_bag(tables, toff, np.concatenate(idx2).astype(np.int64),
                            np.array(off2, np.int64), B, "max")
    assert np.array_equal(mx, mx2)
    # one lookup per bag: the row itself; negated table: max(-x) = -min(x)
    one = np.arange(T * B, dtype=np.int64) % 9
    r1, _ = oracle.emb_bag(tables, toff, one, np.arange(T * B + 1, dtype=np.int64), B, "max")
    for t in range(T):
        for b in range(B):
            assert np.array_equal(r1[b, t * D:(t + 1) * D],
                                  tables[toff[t] + one[t * B + b]].astype(np.float64))
    neg, _ = oracle.emb_bag(-tables, toff, idx, offsets, B, "max")
    mn = np.zeros_like(mx)
    for t in range(T):
        for b in range(B):
            seg = idx[offsets[t * B + b]:offsets[t * B + b + 1]]
            if len(seg):
                mn[b, t * D:(t + 1) * D] = tables[toff[t] + seg].astype(np.float64).min(axis=0)
    assert np.array_equal(neg, -mn)
    with pytest.raises(ValueError):                        # no weights with max pooling
        oracle.emb_bag(tables, toff, idx, offsets, B, "max", weights=np.ones(len(idx), np.float32))


def test_max_second_opinion_torch_cpu(oracle):
    import torch
    import torch.nn.functional as F
    wl = gen.workload("small_f32_d64")
    batch = gen.make_batches(wl, 1)[0]
    arena = gen.host_arena(wl)
    toff = wl.table_offsets()
    ref, _ = oracle.emb_bag(arena, toff, batch.indices, batch.offsets, wl.B, "max")
    for t in range(wl.T):
        o = batch.offsets[t * wl.B:(t + 1) * wl.B + 1]
        ix = torch.from_numpy(batch.indices[o[0]:o[-1]])
        W = torch.from_numpy(arena[toff[t]:toff[t + 1]].astype(np.float64))
        want = F.embedding_bag(ix, W, torch.from_numpy(o[:-1] - o[0]), mode="max").numpy()
        assert np.array_equal(ref[:, t * wl.D:(t + 1) * wl.D], want)


def test_max_of_quantised_rows_is_the_max_of_the_dequantised_table(oracle):
    wl = gen.workload("small_u8_d120")
    batch = gen.make_batches(wl, 1)[0]
    arena = gen.host_arena(wl)
    D = wl.D
    scale = arena[:, D:D + 4].copy().view(np.float32).astype(np.float64)
    bias = arena[:, D + 4:D + 8].copy().view(np.float32).astype(np.float64)
    deq = scale * arena[:, :D].astype(np.float64) + bias
    ref, bound = oracle.emb_bag(arena, wl.table_offsets(), batch.indices, batch.offsets, wl.B, "max")
    toff = wl.table_offsets()
    for t in range(wl.T):
        for b in range(0, wl.B, 7):
            seg = batch.indices[batch.offsets[t * wl.B + b]:batch.offsets[t * wl.B + b + 1]]
            want = deq[toff[t] + seg].max(axis=0) if len(seg) else np.zeros(D)
            assert np.allclose(ref[b, t * D:(t + 1) * D], want, rtol=1e-15, atol=0)
    assert np.all(bound >= np.abs(ref) - 1e-12)


# ------------------------------------------------------------------------------------------
# quantised rows with E4M3 8-bit floating-point codes (OCP 8-bit floating point, E4M3 variant)
# ------------------------------------------------------------------------------------------
def _one_row_lookup(oracle, codes, scale=1.0, bias=0.0):
    """Look up a single quantised row holding `codes` and return its elements."""
    D = len(codes)
    pad = (-(D + 8)) % 16
    row = np.zeros((1, D + pad + 8), dtype=np.uint8)
    row[0, :D] = codes
    row[0, D + pad:D + pad + 4] = np.array([scale], np.float32).view(np.uint8)
    row[0, D + pad + 4:] = np.array([bias], np.float32).view(np.uint8)
    ref, bound = oracle.emb_bag(row, np.array([0, 1], np.int64), np.array([0], np.int64),
                                np.array([0, 1], np.int64), 1, "sum", codes="fp8")
    return ref[0, :D], bound[0, :D]


def test_e4m3_values_typed_in(oracle):
    """Bit patterns and values from the format's definition: bias 7, 3 fraction bits, subnormals
    m * 2^-9, largest finite 448, no infinities."""
    cases = {0x00: 0.0, 0x01: 2.0 ** -9, 0x07: 7 * 2.0 ** -9, 0x08: 2.0 ** -6, 0x38: 1.0,
             0x3C: 1.5, 0x40: 2.0, 0x7E: 448.0, 0x77: 240.0, 0x78: 256.0, 0x81: -(2.0 ** -9),
             0xB8: -1.0, 0xFE: -448.0, 0x30: 0.5, 0x3F: 1.875}
    codes = np.array(sorted(cases), dtype=np.uint8)
    vals, bound = _one_row_lookup(oracle, codes)
    assert vals.tolist() == [cases[int(c)] for c in codes]
    assert bound.tolist() == [abs(cases[int(c)]) for c in codes]
    nan, _ = _one_row_lookup(oracle, np.array([0x7F, 0xFF], np.uint8))
    assert np.isnan(nan).all()


def test_e4m3_every_code_against_torch(oracle):
    """Second opinion on all 256 codes: torch's float8_e4m3fn, widened on the CPU."""
    import torch
    codes = np.arange(256, dtype=np.uint8)
    want = torch.from_numpy(codes.copy()).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    vals, _ = _one_row_lookup(oracle, codes)
    finite = ~np.isnan(want)
    assert finite.sum() == 254 and np.array_equal(vals[finite], want[finite])
    assert np.isnan(vals[~finite]).all()
    # scale and bias apply as for integer codes: element = scale * value + bias, bound from both terms
    vals, bound = _one_row_lookup(oracle, codes[finite], scale=0.25, bias=-3.0)
    assert np.array_equal(vals, 0.25 * want[finite] - 3.0)
    assert np.array_equal(bound, 0.25 * np.abs(want[finite]) + 3.0)


def test_e4m3_rows_brute_force(oracle):
    rng = np.random.default_rng(41)
    R, D, B = 9, 8, 4
    table, scale, bias = _quantised_table(rng, R, D)
    table[:, :D][(table[:, :D] & 0x7F) == 0x7F] = 0x3A         # no NaN codes
    toff = np.array([0, 5, 9], dtype=np.int64)
    lengths = np.array([3, 0, 2, 4, 1, 0, 5, 2])
    offsets = gen.lengths_to_offsets(lengths)
    idx = np.concatenate([rng.integers(0, 5, size=lengths[:4].sum()),
                          rng.integers(0, 4, size=lengths[4:].sum())]).astype(np.int64)

    def value(c):                                             # straight from the definition
        s, e, m = c >> 7, (c >> 3) & 15, c & 7
        v = Fraction(m, 8) * Fraction(1, 64) if e == 0 else (1 + Fraction(m, 8)) * Fraction(2) ** (e - 7)
        return -v if s else v

    for mode in ("sum", "mean", "max"):
        ref, bound = oracle.emb_bag(table, toff, idx, offsets, B, mode, codes="fp8")
        for t in range(2):
            for b in range(B):
                lo, hi = int(offsets[t * B + b]), int(offsets[t * B + b + 1])
                for d in range(D):
                    terms = []
                    for j in range(lo, hi):
                        r = int(toff[t]) + int(idx[j])
                        sc = Fraction(float(scale[r])) * value(int(table[r, d]))
                        terms.append((sc + Fraction(float(bias[r])), abs(sc) + abs(Fraction(float(bias[r])))))
                    if mode == "max":
                        a, m = max(terms, key=lambda x: x[0]) if terms else (Fraction(0), Fraction(0))
                    else:
                        a, m = sum(x[0] for x in terms), sum(x[1] for x in terms)
                        if mode == "mean" and terms:
                            a, m = a / len(terms), m / len(terms)
                    tol = 16 * 2.0 ** -53 * float(m) + 1e-300
                    assert abs(ref[b, t * D + d] - float(a)) <= tol
                    assert abs(bound[b, t * D + d] - float(m)) <= tol
