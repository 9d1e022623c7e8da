"""Seeded synthetic inputs for the multi-table EmbeddingBag forward.

This module is the *input generator*: it serves both the HIP library's tests/bench and the
CPU oracle's tests, and holds none of the gather/pool arithmetic itself.  Everything is a pure
function of one 64-bit seed.

Workload shapes follow the paper's statement of the embedding stage (Sec. 3.1: per table a
batch of BS samples, each pooling "lookups per sample" rows of length ED) and its two
synthetic access patterns (Sec. 3.2: "random" = uniform on [0, R), "one item" = a single
repeated row).  The paper's production traces are not available; a Zipf law over a randomly
permuted row order stands in for their power-law hotness (Sec. 3.2).

Pieces
------
* `Workload`           - shape + distributions of one configuration (`workload(name)`).
* `table_values`       - procedural table values on the host (numpy), bit-identical to the
                         device fill kernel in `csrc/embgen.hip`.
* `fill_arena_device`  - run that fill kernel on a device buffer (ctypes, `libembgen.so`).
* `make_batches`       - CSR offsets + int64 indices (+ optional weights) for K batches.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libembgen.so")

# ----------------------------------------------------------------------------------------
# procedural table values
# ----------------------------------------------------------------------------------------
_K_ROW = np.uint64(0x9E3779B97F4A7C15)
_K_COL = np.uint64(0xD1B54A32D192ED03)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
_SCALE = np.float32(0.1) / np.float32(37837.2)  # sigma of the 4-field sum is 65536*sqrt(4/12)

KIND_NORMAL = 0
KIND_INT = 1


def _mix64(z: np.ndarray) -> np.ndarray:
    z = (z ^ (z >> np.uint64(30))) * _M1
    z = (z ^ (z >> np.uint64(27))) * _M2
    return z ^ (z >> np.uint64(31))


def table_values(seed: int, arena_rows: Sequence[int], D: int, dtype: str = "f32",
                 kind: int = KIND_NORMAL) -> np.ndarray:
    """Values of the given arena rows, shape [len(arena_rows), D], float32 or float16.

    dtype 'bf16' returns uint16 bit patterns (numpy has no bfloat16).
    kind 0: approximately N(0, 0.1^2) (sum of four 16-bit uniform fields, centred and scaled);
    kind 1: integers in [-8, 7] (sums of these are exact in fp32 in any order).
    """
    rows = np.asarray(arena_rows, dtype=np.uint64).reshape(-1, 1)
    if dtype in QUANTISED:
        return _quantised_rows(seed, rows, D, kind, fp8=dtype == "fp8row")
    cols = np.arange(D, dtype=np.uint64).reshape(1, -1)
    with np.errstate(over="ignore"):
        z = _mix64(np.uint64(seed & 0xFFFFFFFFFFFFFFFF) + rows * _K_ROW + cols * _K_COL)
    if kind == KIND_INT:
        v = ((z >> np.uint64(60)).astype(np.int64) - 8).astype(np.float32)
    elif kind == KIND_NORMAL:
        m = np.uint64(0xFFFF)
        s = ((z & m) + ((z >> np.uint64(16)) & m) + ((z >> np.uint64(32)) & m)
             + ((z >> np.uint64(48)) & m)).astype(np.int64) - 131070
        v = s.astype(np.float32) * _SCALE
    else:
        raise ValueError("kind must be 0 (normal) or 1 (int)")
    if dtype == "f16":
        return v.astype(np.float16)
    if dtype == "bf16":   # round to nearest even on the bit pattern; returned as uint16 bits
        u = v.view(np.uint32)
        return ((u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)).astype(np.uint16)
    if dtype == "f32":
        return v
    raise ValueError("dtype must be 'f32', 'f16' or 'bf16'")


_QSCALE = np.float32(3.5e-6)
_QSCALE_FP8 = np.float32(2.0e-6)
QUANTISED = ("u8row", "fp8row")   # D one-byte codes + fp32 scale + fp32 bias per row


def _quantised_rows(seed: int, rows: np.ndarray, D: int, kind: int, fp8: bool = False) -> np.ndarray:
    """Row-wise quantised rows, uint8 [n, D + 8]: D codes, fp32 scale, fp32 bias.
    code = bits 32..39 of the hash of (row, col); the hash of (row, col = D) picks the scale.
    Integer codes: kind 0: scale = (256 + a) * 3.5e-6 with a in [0, 255], bias = -128 * scale
    (elements roughly uniform in +-0.17, sigma about 0.1); kind 1: scale = 1, bias = -128
    (integers in [-128, 127]).
    E4M3 codes (fp8): the two NaN codes are moved to their neighbours (0x7F -> 0x7E, 0xFF -> 0xFE);
    kind 0: scale = (256 + a) * 2e-6, bias = -32 * scale (elements within +-0.46); kind 1: the
    top exponent bit is cleared (|value| < 2, a multiple of 2^-9), scale = 1, bias = -1, so sums
    of a few hundred elements are exact in fp32."""
    n = rows.shape[0]
    cols = np.arange(D + 1, dtype=np.uint64).reshape(1, -1)
    with np.errstate(over="ignore"):
        z = _mix64(np.uint64(seed & 0xFFFFFFFFFFFFFFFF) + rows * _K_ROW + cols * _K_COL)
    out = np.empty((n, D + 8), dtype=np.uint8)
    codes = ((z[:, :D] >> np.uint64(32)) & np.uint64(0xFF)).astype(np.uint8)
    if fp8:
        codes = np.where((codes & 0x7F) == 0x7F, codes & 0xFE, codes).astype(np.uint8)
        if kind == KIND_INT:
            codes &= np.uint8(0xBF)
    out[:, :D] = codes
    if kind == KIND_INT:
        scale = np.ones(n, dtype=np.float32)
    else:
        a = (z[:, D] & np.uint64(0xFF)).astype(np.int64)
        scale = (256 + a).astype(np.float32) * (_QSCALE_FP8 if fp8 else _QSCALE)
    if fp8:
        bias = (np.float32(-1.0 if kind == KIND_INT else -32.0) * scale).astype(np.float32)
    else:
        bias = (np.float32(-128.0) * scale).astype(np.float32)
    out[:, D:D + 4] = np.ascontiguousarray(scale).view(np.uint8).reshape(n, 4)
    out[:, D + 4:D + 8] = np.ascontiguousarray(bias).view(np.uint8).reshape(n, 4)
    return out


def table_values_range(seed: int, first_row: int, nrows: int, D: int, dtype: str = "f32",
                       kind: int = KIND_NORMAL, chunk_rows: int = 1 << 16) -> np.ndarray:
    """Rows [first_row, first_row + nrows) of the arena, generated in chunks."""
    if dtype in QUANTISED:
        out = np.empty((nrows, D + 8), dtype=np.uint8)
    else:
        out = np.empty((nrows, D), dtype={"f16": np.float16, "bf16": np.uint16}.get(dtype, np.float32))
    for r0 in range(0, nrows, chunk_rows):
        r1 = min(nrows, r0 + chunk_rows)
        out[r0:r1] = table_values(seed, np.arange(first_row + r0, first_row + r1, dtype=np.uint64),
                                  D, dtype, kind)
    return out


# ----------------------------------------------------------------------------------------
# device side (libembgen.so) - only used where a GPU is present
# ----------------------------------------------------------------------------------------
_lib = None


def load_lib() -> ctypes.CDLL:
    """Load libembgen.so (after torch, so that the HIP runtime torch ships is the one used)."""
    global _lib
    if _lib is None:
        import torch  # noqa: F401  (loads libamdhip64 first)
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is not built; run __graft_entry__.build() first")
        lib = ctypes.CDLL(LIB_PATH)
        lib.gen_fill_table.restype = ctypes.c_int
        lib.gen_fill_table.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64,
                                       ctypes.c_int32, ctypes.c_int32, ctypes.c_uint64,
                                       ctypes.c_int32, ctypes.c_void_p]
        lib.gen_copy_bytes.restype = ctypes.c_int
        lib.gen_copy_bytes.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64,
                                       ctypes.c_void_p]
        lib.gen_read_bytes.restype = ctypes.c_int
        lib.gen_read_bytes.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p,
                                       ctypes.c_void_p]
        lib.gen_alloc_arena.restype = ctypes.c_int
        lib.gen_alloc_arena.argtypes = [ctypes.POINTER(ctypes.c_void_p), ctypes.c_int64,
                                        ctypes.c_int32]
        lib.gen_free_arena.restype = ctypes.c_int
        lib.gen_free_arena.argtypes = [ctypes.c_void_p]
        lib.gen_scrub_cache.restype = ctypes.c_int
        lib.gen_scrub_cache.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p]
        _lib = lib
    return _lib


def fill_arena_device(dev_ptr: int, first_row: int, nrows: int, D: int, dtype: str, seed: int,
                      kind: int = KIND_NORMAL, stream: int = 0) -> None:
    """Fill arena rows [first_row, first_row+nrows) at device address `dev_ptr` (= address of
    row `first_row`) with `table_values`; asynchronous on `stream` (a hipStream_t as int)."""
    rc = load_lib().gen_fill_table(ctypes.c_void_p(dev_ptr), first_row, nrows, D,
                                   {"f32": 0, "f16": 1, "bf16": 2, "u8row": 3, "fp8row": 4}[dtype],
                                   ctypes.c_uint64(seed & 0xFFFFFFFFFFFFFFFF), kind,
                                   ctypes.c_void_p(stream))
    if rc != 0:
        raise RuntimeError(f"gen_fill_table failed with code {rc}")


class DeviceArena:
    """A table arena allocated straight from HIP, optionally physically contiguous.

    `tensor` is a torch view of the memory ([rows, D], through the CUDA array interface); the arena
    owns the memory and frees it in `close()` (call it only after the streams that used it have
    been synchronised).  If the contiguous request is refused the arena falls back to an ordinary
    allocation and says so in `kind`."""

    _TYPESTR = {"f32": "<f4", "f16": "<f2", "bf16": "<i2", "u8row": "|u1", "fp8row": "|u1"}

    def __init__(self, rows: int, D: int, dtype: str, contiguous: bool = True):
        import torch
        self.rows, self.D, self.dtype = int(rows), int(D), dtype
        width = self.D + 8 if dtype in QUANTISED else self.D    # elements per row in the view
        self.nbytes = self.rows * width * {"f32": 4, "u8row": 1, "fp8row": 1}.get(dtype, 2)
        lib = load_lib()
        p = ctypes.c_void_p()
        self.kind = "hip-contiguous" if contiguous else "hip-default"
        rc = lib.gen_alloc_arena(ctypes.byref(p), self.nbytes, 1 if contiguous else 0)
        if rc != 0 and contiguous:
            torch.cuda.synchronize()
            self.kind = "hip-default (contiguous refused)"
            rc = lib.gen_alloc_arena(ctypes.byref(p), self.nbytes, 0)
        if rc != 0 or not p.value:
            raise MemoryError(f"gen_alloc_arena({self.nbytes}) failed with hipError {rc}")
        self.ptr = int(p.value)
        self.__cuda_array_interface__ = {"shape": (self.rows, width), "typestr": self._TYPESTR[dtype],
                                         "data": (self.ptr, False), "version": 2, "strides": None}
        t = torch.as_tensor(self, device="cuda")
        self.tensor = t.view(torch.bfloat16) if dtype == "bf16" else t
        assert self.tensor.data_ptr() == self.ptr

    def data_ptr(self) -> int:
        return self.ptr

    def close(self) -> None:
        if getattr(self, "ptr", 0):
            self.tensor = None
            load_lib().gen_free_arena(ctypes.c_void_p(self.ptr))
            self.ptr = 0


def copy_bytes_device(dst_ptr: int, src_ptr: int, nbytes: int, stream: int = 0) -> None:
    rc = load_lib().gen_copy_bytes(ctypes.c_void_p(dst_ptr), ctypes.c_void_p(src_ptr), nbytes,
                                   ctypes.c_void_p(stream))
    if rc != 0:
        raise RuntimeError(f"gen_copy_bytes failed with code {rc}")


def read_bytes_device(src_ptr: int, nbytes: int, stream: int = 0) -> None:
    rc = load_lib().gen_read_bytes(ctypes.c_void_p(src_ptr), nbytes, None, ctypes.c_void_p(stream))
    if rc != 0:
        raise RuntimeError(f"gen_read_bytes failed with code {rc}")


def scrub_cache_device(buf_ptr: int, nbytes: int, stream: int = 0) -> None:
    rc = load_lib().gen_scrub_cache(ctypes.c_void_p(buf_ptr), nbytes, ctypes.c_void_p(stream))
    if rc != 0:
        raise RuntimeError(f"gen_scrub_cache failed with code {rc}")


# ----------------------------------------------------------------------------------------
# workloads
# ----------------------------------------------------------------------------------------
@dataclass(frozen=True)
class Workload:
    name: str
    T: int                      # number of tables
    rows: Tuple[int, ...]       # rows per table (len T)
    D: int                      # embedding dimension (uniform over tables)
    dtype: str                  # 'f32' | 'f16' | 'bf16' | 'u8row' | 'fp8row' (table storage; output is fp32)
    B: int                      # batch (bags per table)
    pooling: Tuple              # ('fixed', L) | ('uniform', lo, hi) inclusive
    dists: Tuple[Tuple, ...]    # per table: ('uniform',) | ('zipf', alpha) | ('one_item',)
    mode: str = "sum"           # 'sum' | 'mean' | 'max'
    weighted: bool = False
    seed: int = 0x5EED0000
    kind: int = KIND_NORMAL
    note: str = ""
    hot_head: int = 0           # Zipf tables only: ranks 1..hot_head sit in rows 0..hot_head-1 (the
                                # table after the offline hot-row relayout of paper Sec. 4.3)

    @property
    def elem_bytes(self) -> int:
        return {"f32": 4, "u8row": 1, "fp8row": 1}.get(self.dtype, 2)

    @property
    def row_bytes(self) -> int:
        if self.dtype in QUANTISED:   # D one-byte codes + fp32 scale + fp32 bias
            return self.D + 8
        return self.D * self.elem_bytes

    @property
    def total_rows(self) -> int:
        return int(sum(self.rows))

    @property
    def table_bytes(self) -> int:
        return self.total_rows * self.row_bytes

    @property
    def codes(self) -> str:
        """What the code bytes of quantised rows stand for: 'u8' integers or 'fp8' E4M3 numbers."""
        return "fp8" if self.dtype == "fp8row" else "u8"

    @property
    def num_bags(self) -> int:
        return self.T * self.B

    def table_offsets(self) -> np.ndarray:
        return np.concatenate([[0], np.cumsum(np.asarray(self.rows, dtype=np.int64))]).astype(np.int64)


# Zipf exponents whose expected unique-access % (R = 500,000 draws over 500,000 rows) equals the
# paper's table of unique access % per dataset (Sec. 3.2): high 4.05, med 20.50, low 46.21.
# Found by bisection on  U(alpha) = mean_k [1 - (1 - p_k)^R]  (see expected_unique_fraction).
PAPER_HOTNESS_ALPHA = {"paper_high": 1.3396, "paper_med": 1.0234, "paper_low": 0.6999}
PAPER_MIXES = {"paper_mix1": (100, 75, 50, 25), "paper_mix2": (62, 63, 63, 62),
               "paper_mix3": (25, 50, 75, 100)}


def expected_unique_fraction(R: int, alpha: float, n: int) -> float:
    """Expected fraction of the R rows touched by n independent Zipf(alpha) draws."""
    p = np.arange(1, R + 1, dtype=np.float64) ** (-float(alpha))
    p /= p.sum()
    return float(np.mean(-np.expm1(n * np.log1p(-p))))


@dataclass(frozen=True)
class MixedWorkload:
    """Tables of different widths (one element type).  Same batch machinery as `Workload`."""
    name: str
    T: int
    rows: Tuple[int, ...]
    dims: Tuple[int, ...]       # embedding dimension of each table
    dtype: str
    B: int
    pooling: Tuple
    dists: Tuple[Tuple, ...]
    mode: str = "sum"
    weighted: bool = False
    seed: int = 0x5EED0000
    kind: int = KIND_NORMAL

    @property
    def num_bags(self) -> int:
        return self.T * self.B

    @property
    def codes(self) -> str:
        """What the code bytes of quantised rows stand for: 'u8' integers or 'fp8' E4M3 numbers."""
        return "fp8" if self.dtype == "fp8row" else "u8"

    def row_bytes_of(self, t: int) -> int:
        d = self.dims[t]
        return d + 8 if self.dtype in QUANTISED else d * (4 if self.dtype == "f32" else 2)

    def table_byte_offsets(self) -> np.ndarray:
        sizes = [self.rows[t] * self.row_bytes_of(t) for t in range(self.T)]
        return np.concatenate([[0], np.cumsum(np.asarray(sizes, dtype=np.int64))]).astype(np.int64)

    def out_offsets(self) -> np.ndarray:
        return np.concatenate([[0], np.cumsum(np.asarray(self.dims, dtype=np.int64))]).astype(np.int64)

    def row_bases(self) -> np.ndarray:
        """First procedural row id of each table (rows are numbered across tables)."""
        return np.concatenate([[0], np.cumsum(np.asarray(self.rows, dtype=np.int64))]).astype(np.int64)

    @property
    def table_bytes(self) -> int:
        return int(self.table_byte_offsets()[-1])

    def gathered_bytes(self, batch: "Batch") -> int:
        per_table = np.diff(batch.offsets[::self.B])
        return int(sum(int(per_table[t]) * self.row_bytes_of(t) for t in range(self.T)))


def mixed_host_tables(wl: MixedWorkload) -> List[np.ndarray]:
    """Per-table host arrays with the same procedural values the device fill produces."""
    base = wl.row_bases()
    return [table_values_range(wl.seed, int(base[t]), wl.rows[t], wl.dims[t], wl.dtype, wl.kind)
            for t in range(wl.T)]


def mixed_fill_device(wl: MixedWorkload, arena_ptr: int, stream: int = 0) -> None:
    """Fill a device arena laid out by `table_byte_offsets` (one fill launch per table)."""
    base, boff = wl.row_bases(), wl.table_byte_offsets()
    for t in range(wl.T):
        fill_arena_device(arena_ptr + int(boff[t]), int(base[t]), wl.rows[t], wl.dims[t], wl.dtype,
                          wl.seed, wl.kind, stream)


def mixed_workload(name: str) -> MixedWorkload:
    if name == "mixed_small":
        return MixedWorkload(name=name, T=7, rows=(500, 33, 1000, 1, 257, 64, 90),
                             dims=(64, 4, 128, 256, 32, 96, 12), dtype="f32", B=53,
                             pooling=("uniform", 0, 120),
                             dists=(("uniform",), ("uniform",), ("zipf", 1.1), ("one_item",),
                                    ("uniform",), ("uniform",), ("uniform",)), seed=0x5EED0C01)
    if name == "mixed_cfg":   # 60 tables x 4 M rows, widths cycling 32 / 64 / 128 / 256 fp32 (115 GB)
        T = 60
        return MixedWorkload(name=name, T=T, rows=(4_000_000,) * T,
                             dims=tuple((32, 64, 128, 256)[t % 4] for t in range(T)), dtype="f32",
                             B=4096, pooling=("fixed", 80), dists=(("uniform",),) * T,
                             seed=0x5EED0C02)
    if name == "mixed_onehot":   # 26 tables x 1 M rows, widths cycling 16 / 32 / 64 / 128, one lookup per bag
        T = 26
        return MixedWorkload(name=name, T=T, rows=(1_000_000,) * T,
                             dims=tuple((16, 32, 64, 128)[t % 4] for t in range(T)), dtype="f32",
                             B=131072, pooling=("fixed", 1), dists=(("uniform",),) * T,
                             seed=0x5EED0C03)
    raise KeyError(name)


def _homog(name, T, R, D, dtype, B, pooling, dist, mode="sum", seed_off=0, **kw) -> Workload:
    return Workload(name=name, T=T, rows=(R,) * T, D=D, dtype=dtype, B=B, pooling=pooling,
                    dists=(dist,) * T, mode=mode, seed=0x5EED0000 + seed_off, **kw)


def workload(name: str) -> Workload:
    """The five benchmark configurations plus the paper's own shape and small test shapes."""
    if name == "cfg1":
        return _homog("cfg1", 8, 100_000, 64, "f32", 256, ("fixed", 20), ("uniform",), seed_off=1)
    if name == "cfg2":
        return _homog("cfg2", 26, 1_000_000, 64, "f32", 2048, ("uniform", 1, 40), ("uniform",),
                      seed_off=2)
    if name == "cfg3":
        return _homog("cfg3", 60, 4_000_000, 128, "f32", 4096, ("fixed", 80), ("uniform",),
                      seed_off=3)
    if name == "cfg4":
        return _homog("cfg4", 60, 4_000_000, 128, "f32", 4096, ("uniform", 40, 120),
                      ("zipf", 1.05), mode="mean", seed_off=4)
    if name == "cfg5":
        T = 100
        return Workload(name="cfg5", T=T, rows=(2_000_000,) * T, D=256, dtype="f16", B=8192,
                        pooling=("uniform", 1, 100),
                        dists=(("uniform",),) * (T // 2) + (("zipf", 1.2),) * (T - T // 2),
                        mode="sum", seed=0x5EED0005,
                        note="tables 0-49 uniform, tables 50-99 Zipf(1.2)")
    if name == "paper":  # Sec. 5 model: 250 tables x 500,000 x 128 fp32, BS 2048, pooling 150
        return _homog("paper", 250, 500_000, 128, "f32", 2048, ("fixed", 150), ("uniform",),
                      seed_off=6)
    if name == "paper_one_item":
        return _homog("paper_one_item", 250, 500_000, 128, "f32", 2048, ("fixed", 150),
                      ("one_item",), seed_off=7)
    if name in PAPER_HOTNESS_ALPHA:   # Zipf stand-ins for the paper's high / med / low hot traces
        return _homog(name, 250, 500_000, 128, "f32", 2048, ("fixed", 150),
                      ("zipf", PAPER_HOTNESS_ALPHA[name]), seed_off=8)
    if name in PAPER_MIXES:           # Sec. 5 table of heterogeneous mixtures (tables per hotness)
        hi, me, lo, rnd = PAPER_MIXES[name]
        dists = ((("zipf", PAPER_HOTNESS_ALPHA["paper_high"]),) * hi
                 + (("zipf", PAPER_HOTNESS_ALPHA["paper_med"]),) * me
                 + (("zipf", PAPER_HOTNESS_ALPHA["paper_low"]),) * lo + (("uniform",),) * rnd)
        T = len(dists)
        return Workload(name=name, T=T, rows=(500_000,) * T, D=128, dtype="f32", B=2048,
                        pooling=("fixed", 150), dists=dists, seed=0x5EED0009,
                        note="tables ordered high, med, low, random")
    # ---- small shapes for tests (the oracle finishes these in well under a second) ----
    if name == "tiny":
        return Workload(name="tiny", T=3, rows=(8, 5, 7), D=4, dtype="f32", B=4,
                        pooling=("uniform", 0, 5), dists=(("uniform",),) * 3, seed=0x5EED0010)
    if name == "small_f32_d64":   # 256-byte rows, ragged bags incl. empty, several chunks
        return Workload(name="small_f32_d64", T=5, rows=(1000, 37, 4096, 1, 513), D=64,
                        dtype="f32", B=67, pooling=("uniform", 0, 150),
                        dists=(("uniform",), ("uniform",), ("zipf", 1.05), ("one_item",),
                               ("uniform",)), seed=0x5EED0011)
    if name == "small_f32_d128":  # 512-byte rows
        return Workload(name="small_f32_d128", T=4, rows=(3000, 129, 2048, 77), D=128,
                        dtype="f32", B=131, pooling=("uniform", 0, 200),
                        dists=(("uniform",), ("zipf", 1.2), ("uniform",), ("uniform",)),
                        seed=0x5EED0012)
    if name == "small_u8_d120":    # 128-byte quantised rows
        return Workload(name="small_u8_d120", T=4, rows=(1200, 9, 2048, 77), D=120, dtype="u8row",
                        B=83, pooling=("uniform", 0, 140),
                        dists=(("uniform",), ("uniform",), ("zipf", 1.1), ("uniform",)),
                        seed=0x5EED0015)
    if name == "small_u8_d504":    # 512-byte quantised rows
        return Workload(name="small_u8_d504", T=3, rows=(900, 65, 400), D=504, dtype="u8row",
                        B=45, pooling=("uniform", 0, 130),
                        dists=(("uniform",), ("zipf", 1.2), ("uniform",)), seed=0x5EED0016)
    if name == "onehot":           # short bags: cfg2's tables, one lookup per bag, large batch
        return _homog("onehot", 26, 1_000_000, 64, "f32", 131072, ("fixed", 1), ("uniform",),
                      seed_off=0x18)
    if name == "short":            # cfg2's tables, 0..8 lookups per bag (a ninth of the bags empty)
        return _homog("short", 26, 1_000_000, 64, "f32", 32768, ("uniform", 0, 8), ("uniform",),
                      seed_off=0x19)
    if name == "hetero":           # cfg2's tables; 20 one-hot features, 6 multi-hot ones of 100
        specs = tuple(("fixed", 100) if t % 4 == 3 and t < 24 else ("fixed", 1) for t in range(26))
        return _homog("hetero", 26, 1_000_000, 64, "f32", 32768, ("per_table", specs), ("uniform",),
                      seed_off=0x1D)
    if name in ("cfg4_hot", "cfg5_hot", "paper_high_hot", "paper_med_hot"):
        # the same tables, bags and popularity ranks as the base workload, with each Zipf table
        # laid out hot rows first (8,192 rows of 512 bytes are one XCD's 4 MB of L2)
        return with_overrides(workload(name[:-4]), name=name, hot_head=8192)
    if name == "small_hot":        # small Zipf tables with a hot head, ragged bags, several chunks
        return Workload(name="small_hot", T=5, rows=(3000, 200, 4096, 64, 900), D=128,
                        dtype="f32", B=71, pooling=("uniform", 0, 200),
                        dists=(("zipf", 1.05), ("zipf", 1.2), ("uniform",), ("one_item",),
                               ("zipf", 0.8)), seed=0x5EED001E, hot_head=100)
    if name == "cfg3_max":         # cfg3 with max pooling
        return with_overrides(workload("cfg3"), name="cfg3_max", mode="max")
    if name == "cfg3_weighted":    # cfg3 with per-sample weights
        return with_overrides(workload("cfg3"), name="cfg3_weighted", weighted=True)
    if name == "small_fp8_d120":   # 128-byte rows of E4M3 codes
        return with_overrides(workload("small_u8_d120"), name="small_fp8_d120", dtype="fp8row",
                              seed=0x5EED001A)
    if name == "small_fp8_d504":   # 512-byte rows of E4M3 codes
        return with_overrides(workload("small_u8_d504"), name="small_fp8_d504", dtype="fp8row",
                              seed=0x5EED001B)
    if name == "cfg3_fp8":         # cfg3's shape with E4M3 rows (dim 120 -> 128-byte rows)
        return _homog("cfg3_fp8", 60, 4_000_000, 120, "fp8row", 4096, ("fixed", 80), ("uniform",),
                      seed_off=0x1C)
    if name == "cfg3_u8":          # cfg3's shape with quantised rows (dim 120 -> 128-byte rows)
        return _homog("cfg3_u8", 60, 4_000_000, 120, "u8row", 4096, ("fixed", 80), ("uniform",),
                      seed_off=0x17)
    if name == "small_bf16_d256":  # 512-byte bfloat16 rows
        return Workload(name="small_bf16_d256", T=3, rows=(1500, 33, 700), D=256,
                        dtype="bf16", B=61, pooling=("uniform", 0, 130),
                        dists=(("uniform",), ("zipf", 1.2), ("uniform",)), seed=0x5EED0014)
    if name == "small_f16_d256":  # 512-byte fp16 rows
        return Workload(name="small_f16_d256", T=4, rows=(2000, 65, 1024, 300), D=256,
                        dtype="f16", B=97, pooling=("uniform", 0, 130),
                        dists=(("uniform",), ("uniform",), ("zipf", 1.2), ("uniform",)),
                        seed=0x5EED0013)
    raise KeyError(f"unknown workload {name!r}")


def with_overrides(wl: Workload, **kw) -> Workload:
    from dataclasses import replace
    return replace(wl, **kw)


# ----------------------------------------------------------------------------------------
# lengths, offsets, indices, weights
# ----------------------------------------------------------------------------------------
_PURPOSE_LEN, _PURPOSE_IDX, _PURPOSE_PERM, _PURPOSE_W = 1, 2, 3, 4


def _rng(seed: int, purpose: int, batch_id: int = 0, table: int = 0) -> np.random.Generator:
    tag = (purpose << 56) | ((batch_id & 0xFFFFFF) << 32) | (table & 0xFFFFFFFF)
    key = np.array([seed & 0xFFFFFFFFFFFFFFFF, tag], dtype=np.uint64)
    return np.random.Generator(np.random.Philox(key=key))


def make_lengths(wl: Workload, batch_id: int = 0) -> np.ndarray:
    """Bag lengths in (t, b) order, int64 [T*B].  pooling is ("fixed", L), ("uniform", lo, hi)
    (inclusive), or ("per_table", (spec, spec, ...)) with one such spec per table, cycled."""
    n = wl.num_bags
    if wl.pooling[0] == "per_table":
        specs = wl.pooling[1]
        out = np.empty(n, dtype=np.int64)
        for t in range(wl.T):
            spec = specs[t % len(specs)]
            if spec[0] == "fixed":
                out[t * wl.B:(t + 1) * wl.B] = int(spec[1])
            elif spec[0] == "uniform":
                out[t * wl.B:(t + 1) * wl.B] = _rng(wl.seed, _PURPOSE_LEN, batch_id, t).integers(
                    int(spec[1]), int(spec[2]) + 1, size=wl.B, dtype=np.int64)
            else:
                raise ValueError(f"bad pooling spec {spec!r}")
        return out
    if wl.pooling[0] == "fixed":
        return np.full(n, int(wl.pooling[1]), dtype=np.int64)
    if wl.pooling[0] == "uniform":
        lo, hi = int(wl.pooling[1]), int(wl.pooling[2])
        return _rng(wl.seed, _PURPOSE_LEN, batch_id).integers(lo, hi + 1, size=n, dtype=np.int64)
    raise ValueError(f"bad pooling spec {wl.pooling!r}")


def lengths_to_offsets(lengths: np.ndarray) -> np.ndarray:
    """CSR offsets with the final total included: int64 [len+1], offsets[0] = 0."""
    off = np.zeros(len(lengths) + 1, dtype=np.int64)
    np.cumsum(lengths, out=off[1:])
    return off


_zipf_cdf_cache: Dict[Tuple[int, float], np.ndarray] = {}


def zipf_cdf(R: int, alpha: float) -> np.ndarray:
    """Cumulative distribution of P(k) ~ k^-alpha over ranks k = 1..R (fp64)."""
    key = (R, float(alpha))
    if key not in _zipf_cdf_cache:
        if len(_zipf_cdf_cache) > 4:
            _zipf_cdf_cache.clear()
        w = np.arange(1, R + 1, dtype=np.float64) ** (-float(alpha))
        c = np.cumsum(w)
        c /= c[-1]
        _zipf_cdf_cache[key] = c
    return _zipf_cdf_cache[key]


def zipf_ranks(rng: np.random.Generator, R: int, alpha: float, n: int) -> np.ndarray:
    """n independent 0-based ranks by inverse-CDF sampling."""
    u = rng.random(n)
    r = np.searchsorted(zipf_cdf(R, alpha), u, side="right")
    return np.minimum(r, R - 1).astype(np.int64)


def table_permutation(wl: Workload, t: int) -> np.ndarray:
    """Seeded bijection rank -> row for table t (fixed across batches).  With `hot_head` = K the K
    most popular ranks occupy rows 0..K-1 in order of popularity and the other ranks are scattered
    over the remaining rows: the layout a caller produces by profiling its lookups offline and
    moving the hot rows to the front."""
    R = wl.rows[t]
    K = min(int(getattr(wl, "hot_head", 0)), R)
    rng = _rng(wl.seed, _PURPOSE_PERM, 0, t)
    if K <= 0:
        return rng.permutation(R).astype(np.int64)
    return np.concatenate([np.arange(K, dtype=np.int64),
                           K + rng.permutation(R - K).astype(np.int64)])


def hot_rows(wl: Workload) -> np.ndarray:
    """What a caller passes as `hot_rows` for this workload, int64 [T]: the hot head of the Zipf
    tables, 0 (a streaming table) for uniform tables, the whole table for a one-item table."""
    out = np.zeros(wl.T, dtype=np.int64)
    for t, dist in enumerate(wl.dists):
        if dist[0] == "zipf":
            out[t] = min(int(wl.hot_head), wl.rows[t])
        elif dist[0] == "one_item":
            out[t] = wl.rows[t]
    return out


def one_item_row(wl: Workload, t: int) -> int:
    return int(_rng(wl.seed, _PURPOSE_PERM, 0, t).integers(0, wl.rows[t]))


@dataclass
class Batch:
    offsets: np.ndarray                  # int64 [T*B+1]
    indices: np.ndarray                  # int64 [NL], table-local row ids, bags in (t,b) order
    weights: Optional[np.ndarray] = None  # float32 [NL]

    @property
    def num_lookups(self) -> int:
        return int(self.offsets[-1])


def make_batches(wl: Workload, n_batches: int = 1, first_batch: int = 0) -> List[Batch]:
    """Generate `n_batches` independent batches (different lengths and indices, same tables).
    Tables are the outer loop so each Zipf permutation is built once."""
    ids = list(range(first_batch, first_batch + n_batches))
    offs = [lengths_to_offsets(make_lengths(wl, k)) for k in ids]
    idx = [np.empty(int(o[-1]), dtype=np.int64) for o in offs]
    for t in range(wl.T):
        R = wl.rows[t]
        dist = wl.dists[t]
        perm = table_permutation(wl, t) if dist[0] == "zipf" else None
        for k, o, ix in zip(ids, offs, idx):
            s, e = int(o[t * wl.B]), int(o[(t + 1) * wl.B])
            n = e - s
            rng = _rng(wl.seed, _PURPOSE_IDX, k, t)
            if dist[0] == "uniform":
                ix[s:e] = rng.integers(0, R, size=n, dtype=np.int64)
            elif dist[0] == "zipf":
                ix[s:e] = perm[zipf_ranks(rng, R, float(dist[1]), n)]
            elif dist[0] == "one_item":
                ix[s:e] = one_item_row(wl, t)
            else:
                raise ValueError(f"bad distribution {dist!r}")
    out = []
    for k, o, ix in zip(ids, offs, idx):
        w = None
        if wl.weighted:
            w = _rng(wl.seed, _PURPOSE_W, k).uniform(-1.0, 1.0, size=len(ix)).astype(np.float32)
        out.append(Batch(offsets=o, indices=ix, weights=w))
    return out


def host_arena(wl: Workload) -> np.ndarray:
    """The whole table arena on the host, [sum R_t, D] (only for shapes that fit in RAM)."""
    return table_values_range(wl.seed, 0, wl.total_rows, wl.D, wl.dtype, wl.kind)


def table_avg_len(wl, batch: "Batch") -> np.ndarray:
    """Average bag length of each table in a batch, float32 [T] (what a caller would pass as
    table_avg_len)."""
    per_table = np.diff(batch.offsets[::wl.B]).astype(np.float64)
    return (per_table / wl.B).astype(np.float32)


def compact_rows(wl: Workload, batch: Batch, bag_ids: Sequence[int]):
    """For a subset of bags, build a small self-contained problem (one 'table' holding only the
    rows those bags touch) so that a host-side checker can evaluate sampled bags of an arena
    that does not fit in host memory.  Returns (arena_small, indices_small, offsets_small,
    weights_small) where bag i of the small problem equals bag bag_ids[i] of the full one
    (weights_small is None for an unweighted batch)."""
    toff = wl.table_offsets()
    segs, lens, wsegs = [], [], []
    for g in bag_ids:
        t = int(g) // wl.B
        s, e = int(batch.offsets[g]), int(batch.offsets[g + 1])
        segs.append(batch.indices[s:e] + toff[t])
        lens.append(e - s)
        if batch.weights is not None:
            wsegs.append(batch.weights[s:e])
    arena_rows = np.concatenate(segs) if segs else np.zeros(0, dtype=np.int64)
    uniq, inv = np.unique(arena_rows, return_inverse=True)
    step = max(1, (1 << 24) // max(1, wl.D))      # rows per piece: bounded temporaries
    parts = [table_values(wl.seed, uniq[i:i + step], wl.D, wl.dtype, wl.kind)
             for i in range(0, max(len(uniq), 1), step)]
    small = np.concatenate(parts) if len(parts) > 1 else parts[0]
    if len(uniq) == 0:
        small = np.zeros((1, small.shape[1]), dtype=small.dtype)
    wsmall = None
    if batch.weights is not None:
        wsmall = np.concatenate(wsegs).astype(np.float32) if wsegs else np.zeros(0, np.float32)
    return small, inv.astype(np.int64), lengths_to_offsets(np.asarray(lens, dtype=np.int64)), wsmall
