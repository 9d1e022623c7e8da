"""GPU parity for row-wise quantised rows with E4M3 8-bit floating-point codes (EMB_FP8ROW).  The
device turns the codes into fp32 with the hardware's conversion instruction; the first test pins
that conversion, code by code, to the oracle's reading of the format."""
import numpy as np
import pytest
import torch

import paper_2410_22249_amd as emb
from inputgen import gen
from gpu_harness import (DEV, arena_bytes, assert_close_to_oracle, device_arena, forward, to_dev,
                         tuning, upload_arena)

pytestmark = pytest.mark.gpu
FP8 = emb.EMB_FP8ROW


def _problem(name, **over):
    wl = gen.with_overrides(gen.workload(name), **over) if over else gen.workload(name)
    return wl, gen.make_batches(wl, 1)[0], gen.host_arena(wl)


def test_every_e4m3_code_is_converted_exactly(oracle):
    """254 rows, row r holding the r-th non-NaN code in all 24 positions, scale 1, bias 0, one
    lookup per bag: the output is the code's value, which fp32 represents exactly."""
    codes = np.array([c for c in range(256) if (c & 0x7F) != 0x7F], dtype=np.uint8)
    D = 24
    table = np.zeros((len(codes), D + 8), dtype=np.uint8)
    table[:, :D] = codes[:, None]
    table[:, D:D + 4] = np.array([1.0], np.float32).view(np.uint8)
    toff = np.array([0, len(codes)], np.int64)
    idx = np.arange(len(codes), dtype=np.int64)
    off = np.arange(len(codes) + 1, dtype=np.int64)
    ref, _ = oracle.emb_bag(table, toff, idx, off, len(codes), "sum", codes="fp8")
    for kw in (dict(stream=0), dict(stream=1), dict(stream=0, addressing=1)):
        with tuning(**kw):
            got = forward(upload_arena(table), toff, idx, off, len(codes), table_dtype=FP8).cpu().numpy()
        assert np.array_equal(got.astype(np.float64), ref), kw
    assert ref[codes.tolist().index(0x7E), 0] == 448.0 and ref[codes.tolist().index(0x01), 0] == 2.0 ** -9


@pytest.mark.parametrize("kind", [gen.KIND_NORMAL, gen.KIND_INT])
def test_device_fill_of_e4m3_rows_matches_host(kind):
    wl = gen.with_overrides(gen.workload("small_fp8_d120"), kind=kind)
    assert np.array_equal(arena_bytes(device_arena(wl)), gen.host_arena(wl).view(np.uint8))


@pytest.mark.parametrize("name", ["small_fp8_d120", "small_fp8_d504"])
@pytest.mark.parametrize("mode", ["sum", "mean", "max"])
def test_e4m3_rows_match_oracle(oracle, name, mode):
    wl, batch, arena = _problem(name)
    ref, bound, strict = oracle.emb_bag(arena, wl.table_offsets(), batch.indices, batch.offsets,
                                        wl.B, mode, codes="fp8", strict=True)
    dev = upload_arena(arena)
    for kw in (dict(), dict(addressing=1), dict(depth=8), dict(depth=2, xcd_remap=1), dict(stream=1),
               dict(stream=1, bags_per_group=5)):
        with tuning(**kw):
            got = forward(dev, wl.table_offsets(), batch.indices, batch.offsets, wl.B, mode,
                          table_dtype=FP8).cpu().numpy()
        assert_close_to_oracle(got, ref, bound, True, f"fp8/{name}/{mode}/{kw}", strict=strict)


def test_e4m3_rows_weights_short_bags_and_exact_integers(oracle):
    wl, batch, arena = _problem("small_fp8_d120", weighted=True)
    ref, bound = oracle.emb_bag(arena, wl.table_offsets(), batch.indices, batch.offsets, wl.B, "sum",
                                weights=batch.weights, codes="fp8")
    got = forward(upload_arena(arena), wl.table_offsets(), batch.indices, batch.offsets, wl.B,
                  weights=batch.weights, table_dtype=FP8).cpu().numpy()
    assert_close_to_oracle(got, ref, bound, True, "fp8 weighted")
    wl, batch, arena = _problem("small_fp8_d120", pooling=("uniform", 0, 3))
    ref, bound = oracle.emb_bag(arena, wl.table_offsets(), batch.indices, batch.offsets, wl.B, "mean",
                                codes="fp8")
    got = forward(upload_arena(arena), wl.table_offsets(), batch.indices, batch.offsets, wl.B, "mean",
                  table_dtype=FP8).cpu().numpy()
    assert_close_to_oracle(got, ref, bound, True, "fp8 short bags")
    # kind 1: every element is a multiple of 2^-9 below 3 in magnitude: sums are exact in any order
    wl, batch, arena = _problem("small_fp8_d504", kind=gen.KIND_INT)
    ref, _ = oracle.emb_bag(arena, wl.table_offsets(), batch.indices, batch.offsets, wl.B, "sum",
                            codes="fp8")
    for kw in (dict(stream=0), dict(stream=1)):
        with tuning(**kw):
            got = forward(upload_arena(arena), wl.table_offsets(), batch.indices, batch.offsets, wl.B,
                          table_dtype=FP8).cpu().numpy()
        assert np.array_equal(got.astype(np.float64), ref), kw


@pytest.mark.parametrize("D", [8, 24, 248, 1016])
def test_e4m3_row_widths(oracle, D):
    wl = gen.Workload(name="w", T=3, rows=(300, 17, 1), D=D, dtype="fp8row", B=29,
                      pooling=("uniform", 0, 70), dists=(("uniform",),) * 3, seed=0x5EED1100 + D)
    batch = gen.make_batches(wl, 1)[0]
    arena = gen.host_arena(wl)
    for mode in ("sum", "max"):
        ref, bound = oracle.emb_bag(arena, wl.table_offsets(), batch.indices, batch.offsets, wl.B,
                                    mode, codes="fp8")
        got = forward(upload_arena(arena), wl.table_offsets(), batch.indices, batch.offsets, wl.B,
                      mode, table_dtype=FP8).cpu().numpy()
        assert_close_to_oracle(got, ref, bound, True, f"fp8 widths/D{D}/{mode}")


def test_e4m3_rows_of_different_widths(oracle):
    from dataclasses import replace
    wl = replace(gen.mixed_workload("mixed_small"), dtype="fp8row", dims=(120, 8, 248, 1016, 56, 24, 504))
    batch = gen.make_batches(wl, 1)[0]
    tabs = gen.mixed_host_tables(wl)
    arena = torch.from_numpy(np.concatenate([t.reshape(-1) for t in tabs])).to(DEV)
    ref, bound = oracle.emb_bag_mixed(tabs, batch.indices, batch.offsets, wl.B, "mean", codes="fp8")
    out = torch.full((wl.B, int(sum(wl.dims))), float("nan"), dtype=torch.float32, device=DEV)
    desc = emb.make_mixed_desc(wl.dims, wl.B, FP8, emb.EMB_MEAN, batch.num_lookups, 0,
                               int(np.diff(wl.table_byte_offsets()).max()))
    emb.emb_bag_forward_mixed(desc, arena, to_dev(wl.table_byte_offsets()), to_dev(wl.out_offsets()),
                              to_dev(batch.indices), to_dev(batch.offsets), None, out)
    torch.cuda.synchronize()
    assert_close_to_oracle(out.cpu().numpy(), ref, bound, True, "fp8 mixed widths")
