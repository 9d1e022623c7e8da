"""The entry point that allocates nothing (emb_bag_profile_hot_rows_noalloc) against the one that
takes a workspace (emb_bag_profile_hot_rows), through the C ABI: same ids, counts and numbers,
bit for bit, on two calls in a row that share the library's scratch array, the second with a
smaller input (so it must not see what the first left behind); sizes beyond the array are
refused."""
import numpy as np
import pytest
import torch

import paper_2410_22249_amd as emb
from inputgen import gen
from gpu_harness import DEV, to_dev

pytestmark = pytest.mark.gpu


def _both(indices, offsets, T, B, window, k):
    idx, off = to_dev(indices), to_dev(offsets)
    desc = emb.make_desc(T, B, 4, emb.EMB_F32, emb.EMB_SUM, len(indices), 0, 0)
    outs = []
    for noalloc in (False, True):
        ids = torch.full((T * k,), 99, dtype=torch.int64, device=DEV)
        counts = torch.full((T * k,), 99, dtype=torch.int32, device=DEV)
        num = torch.full((T,), 99, dtype=torch.int32, device=DEV)
        if noalloc:
            emb.emb_bag_profile_hot_rows_noalloc(desc, idx, off, window, k, ids, counts, num)
        else:
            ws = torch.full((emb.emb_bag_profile_hot_rows_workspace(T, window, k) // 8,), -1,
                            dtype=torch.int64, device=DEV)
            emb.emb_bag_profile_hot_rows(desc, idx, off, window, k, ids, counts, num, ws)
        torch.cuda.synchronize()
        outs.append((ids.cpu().numpy(), counts.cpu().numpy(), num.cpu().numpy()))
    return outs


def test_noalloc_equals_the_workspace_entry_point_on_two_calls_in_a_row():
    big = gen.workload("small_hot")                          # 5 tables, 36,621 lookups
    bb = gen.make_batches(big, 1)[0]
    small = gen.workload("tiny")                             # 3 tables, a handful of lookups
    sb = gen.make_batches(small, 1)[0]
    for wl, batch, window, k in ((big, bb, 1 << 14, 300), (small, sb, 64, 5), (big, bb, 200, 3)):
        ref, got = _both(batch.indices, batch.offsets, wl.T, wl.B, window, k)
        for r, g, what in zip(ref, got, ("ids", "counts", "num_hot")):
            assert np.array_equal(r, g), (wl.name, window, k, what)
        assert int(got[2].sum()) > 0


def test_noalloc_refuses_what_does_not_fit_its_scratch():
    wl = gen.workload("small_hot")
    batch = gen.make_batches(wl, 1)[0]
    idx, off = to_dev(batch.indices), to_dev(batch.offsets)
    desc = emb.make_desc(wl.T, wl.B, 4, emb.EMB_F32, emb.EMB_SUM, batch.num_lookups, 0, 0)
    k = 4
    ids = torch.zeros(wl.T * k, dtype=torch.int64, device=DEV)
    counts = torch.zeros(wl.T * k, dtype=torch.int32, device=DEV)
    # 5 tables * (2^19 + 4) words * 8 bytes = 20 MiB > 16 MiB
    assert emb.emb_bag_profile_hot_rows_workspace(wl.T, 1 << 18, k) > 16 << 20
    with pytest.raises(emb.EmbBagError) as ex:
        emb.emb_bag_profile_hot_rows_noalloc(desc, idx, off, 1 << 18, k, ids, counts, None)
    assert ex.value.status == -7
    # the largest window that fits: 5 * (2^18 + 4) * 8 bytes
    emb.emb_bag_profile_hot_rows_noalloc(desc, idx, off, 1 << 17, k, ids, counts, None)
    torch.cuda.synchronize()
    assert int(ids[0].item()) >= 0
