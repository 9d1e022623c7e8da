"""Helpers shared by the GPU parity tests: upload a seeded problem, call the C-ABI forward through
the binding, and compare with the CPU oracle under the stated tolerances."""
from __future__ import annotations

from typing import Optional

import numpy as np
import torch

import paper_2410_22249_amd as emb
from inputgen import gen
from tuning_ctx import tuning  # noqa: F401  (re-exported for the GPU tests)

DEV = "cuda:0"

# Tolerances.  fp32 tables: |gpu - ref| <= 1e-5 * sum|terms| per output element.  fp16 tables
# (fp32 accumulation): within 1e-3 * |ref|, or within the fp32 bound when the sum cancels (the
# widening of half to fp32 is exact, so the fp32 bound is what the arithmetic supports).
F32_TOL = 1e-5
F16_REL = 1e-3


def to_dev(a: Optional[np.ndarray]):
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def upload_arena(arena: np.ndarray) -> torch.Tensor:
    """float32 / float16 arrays go up as they are; uint16 arrays hold bfloat16 bit patterns."""
    arena = np.ascontiguousarray(arena)
    if arena.dtype == np.uint16:
        return torch.from_numpy(arena.view(np.int16)).to(DEV).view(torch.bfloat16)
    return torch.from_numpy(arena).to(DEV)


TORCH_DTYPE = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16,
               "u8row": torch.uint8, "fp8row": torch.uint8}
EMB_DTYPE = {torch.float32: emb.EMB_F32, torch.float16: emb.EMB_F16, torch.bfloat16: emb.EMB_BF16,
             torch.uint8: emb.EMB_U8ROW}


def arena_dim(arena: torch.Tensor) -> int:
    """Logical embedding dimension: quantised (uint8) rows carry 8 bytes of scale and bias."""
    return arena.shape[1] - 8 if arena.dtype == torch.uint8 else arena.shape[1]


def arena_bytes(arena: torch.Tensor) -> np.ndarray:
    """Raw bytes of a device arena, for bit-for-bit comparisons with the host generator."""
    return arena.contiguous().view(torch.uint8).cpu().numpy()


def device_arena(wl: gen.Workload) -> torch.Tensor:
    """Allocate the arena on the device and fill it with the generator's kernel."""
    width = wl.D + 8 if wl.dtype in gen.QUANTISED else wl.D
    arena = torch.empty((wl.total_rows, width), dtype=TORCH_DTYPE[wl.dtype], device=DEV)
    gen.fill_arena_device(arena.data_ptr(), 0, wl.total_rows, wl.D, wl.dtype, wl.seed, wl.kind,
                          torch.cuda.current_stream().cuda_stream)
    return arena


def forward(arena: torch.Tensor, table_offsets: np.ndarray, indices, offsets, B: int,
            mode: str = "sum", weights=None, out_ld: int = 0, max_table_rows: Optional[int] = None,
            out: Optional[torch.Tensor] = None, fill: float = float("nan"),
            table_dtype: Optional[int] = None, hot_rows=None) -> torch.Tensor:
    """Run emb_bag_forward; numpy inputs are uploaded, torch inputs are used as they are.  The
    element type follows from the arena's dtype unless `table_dtype` names it (uint8 arenas hold
    integer codes by default, E4M3 codes with EMB_FP8ROW)."""
    T = len(table_offsets) - 1
    D = arena_dim(arena)
    toff_np = np.asarray(table_offsets, dtype=np.int64)
    if max_table_rows is None:
        max_table_rows = int(np.max(np.diff(toff_np))) if T else 0
    toff = to_dev(toff_np)
    idx = indices if isinstance(indices, torch.Tensor) else to_dev(np.asarray(indices, np.int64))
    off = offsets if isinstance(offsets, torch.Tensor) else to_dev(np.asarray(offsets, np.int64))
    w = weights if (weights is None or isinstance(weights, torch.Tensor)) else to_dev(
        np.asarray(weights, np.float32))
    nl = int(idx.numel()) if idx is not None else 0
    ld = out_ld if out_ld else T * D
    if out is None:
        out = torch.full((B, ld), fill, dtype=torch.float32, device=DEV)
    hot = None if hot_rows is None else to_dev(np.asarray(hot_rows, np.int64))
    desc = emb.make_desc(T, B, D, EMB_DTYPE[arena.dtype] if table_dtype is None else table_dtype,
                         emb.MODES[mode], nl, out_ld,
                         max_table_rows, hot_rows=hot)
    emb.emb_bag_forward(desc, arena, toff, idx if nl else None, off, w, out)
    torch.cuda.synchronize()
    return out


REL_FALLBACK_USED = 0   # elements that only the relative fp16 rule accepted, over the whole run


def assert_close_to_oracle(got: np.ndarray, ref: np.ndarray, bound: np.ndarray, f16: bool,
                           what: str = "", strict: Optional[np.ndarray] = None,
                           max_rel_fallback: int = 0) -> float:
    """Element-by-element check; returns max(err / bound) over elements with bound > 0.

    Every element type is held to |gpu - ref| <= 1e-5 * sum|terms| (accumulation is fp32 whatever
    the rows are).  The stated rule for fp16 tables, 1e-3 * |ref|, is kept as a fallback for at
    most `max_rel_fallback` elements (none by default) and the elements that needed it are
    counted in REL_FALLBACK_USED.  `strict`, where given (quantised rows), is the bound scale with
    an element taken as one term, |w * (scale * code + bias)|: the same tolerance must hold
    against it."""
    global REL_FALLBACK_USED
    got = got.astype(np.float64)
    err = np.abs(got - ref)
    ok = err <= F32_TOL * bound
    if f16:
        rel = ~ok & (err <= F16_REL * np.abs(ref))
        used = int(rel.sum())
        REL_FALLBACK_USED += used
        assert used <= max_rel_fallback, (f"{what}: {used} elements are within 1e-3 * |ref| but "
                                          f"not within 1e-5 * sum|terms|")
        ok |= rel
    if not ok.all():
        bad = np.argwhere(~ok)[0]
        raise AssertionError(f"{what}: {int((~ok).sum())} of {ok.size} elements out of tolerance; "
                             f"first at {tuple(bad)}: got {got[tuple(bad)]!r} ref {ref[tuple(bad)]!r} "
                             f"bound {bound[tuple(bad)]!r}")
    if strict is not None:
        worse = err > F32_TOL * strict
        assert not worse.any(), (f"{what}: {int(worse.sum())} elements exceed 1e-5 * sum|w * x| "
                                 f"(strict bound); worst ratio {float(np.max(err[worse] / strict[worse]))}")
    zero = bound == 0
    if zero.any():  # empty bags (and all-zero terms) must be exactly +0.0
        assert np.all(got[zero] == 0.0) and not np.signbit(got[zero]).any(), f"{what}: empty bag not +0"
    nz = bound > 0
    return float(np.max(err[nz] / bound[nz])) if nz.any() else 0.0
