"""Thin ctypes binding over libembbag.so: argument marshalling only.

Every step of the embedding-bag forward runs in the HIP kernels behind the C ABI declared in
`include/emb_bag.h`; torch is used here for device memory and streams only.  There is no CPU
fallback: if the shared library has not been built, importing fails with an error.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch  # imported before the library so that the HIP runtime torch ships is the one bound

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libembbag.so")

EMB_F32, EMB_F16, EMB_BF16, EMB_U8ROW, EMB_FP8ROW = 0, 1, 2, 3, 4
DTYPES = {"f32": EMB_F32, "f16": EMB_F16, "bf16": EMB_BF16, "u8row": EMB_U8ROW,
          "fp8row": EMB_FP8ROW}
EMB_SUM, EMB_MEAN, EMB_MAX = 0, 1, 2
MODES = {"sum": EMB_SUM, "mean": EMB_MEAN, "max": EMB_MAX}
EMB_OK = 0

EMB_HINT_DEFAULT, EMB_HINT_STREAMING = 0, 1

EMB_KERNEL_WAVE, EMB_KERNEL_STREAM = 0, 1
EXPORTS = ("emb_bag_forward", "emb_bag_forward_mixed", "emb_bag_plan_forward",
           "emb_bag_plan_forward_mixed", "emb_bag_validate", "emb_bag_profile_reuse",
           "emb_bag_profile_hot_rows", "emb_bag_profile_hot_rows_workspace",
           "emb_bag_profile_hot_rows_noalloc",
           "emb_bag_set_tuning", "emb_bag_get_tuning", "emb_bag_set_tuning_table",
           "emb_bag_tuning_defaults", "emb_bag_status_string", "emb_bag_version")


class emb_bag_tuning(ctypes.Structure):
    _fields_ = [(k, ctypes.c_int32) for k in (
        "depth", "addressing", "blocks_per_cu", "xcd_remap", "use_hints", "stream",
        "bags_per_group", "xcd_pieces", "per_table_launch", "fuse", "bags_per_wave", "hot_split",
        "station")] + [("reserved", ctypes.c_int32 * 3)]


class emb_bag_desc(ctypes.Structure):
    _fields_ = [("num_tables", ctypes.c_int32), ("dim", ctypes.c_int32),
                ("table_dtype", ctypes.c_int32), ("mode", ctypes.c_int32),
                ("batch", ctypes.c_int64), ("num_lookups", ctypes.c_int64),
                ("out_ld", ctypes.c_int64), ("max_table_rows", ctypes.c_int64),
                ("table_hints", ctypes.c_void_p),
                ("table_avg_len", ctypes.POINTER(ctypes.c_float)),
                ("hot_rows", ctypes.c_void_p), ("tuning", ctypes.POINTER(emb_bag_tuning))]


class emb_bag_mixed_desc(ctypes.Structure):
    _fields_ = [("num_tables", ctypes.c_int32), ("table_dtype", ctypes.c_int32),
                ("mode", ctypes.c_int32), ("reserved", ctypes.c_int32),
                ("batch", ctypes.c_int64), ("num_lookups", ctypes.c_int64),
                ("out_ld", ctypes.c_int64), ("max_table_bytes", ctypes.c_int64),
                ("dims", ctypes.POINTER(ctypes.c_int32)), ("table_hints", ctypes.c_void_p),
                ("table_avg_len", ctypes.POINTER(ctypes.c_float)),
                ("tuning", ctypes.POINTER(emb_bag_tuning))]


class emb_bag_plan(ctypes.Structure):
    _fields_ = [("kernel", ctypes.c_int32), ("lanes_per_row", ctypes.c_int32),
                ("depth", ctypes.c_int32), ("buffer_addressing", ctypes.c_int32),
                ("bags_per_group", ctypes.c_int32), ("xcd_pieces", ctypes.c_int32),
                ("listed", ctypes.c_int32), ("num_launches", ctypes.c_int32),
                ("grid_blocks", ctypes.c_int64), ("wavefronts", ctypes.c_int64),
                ("waves_per_table", ctypes.c_int64), ("waves_per_piece", ctypes.c_int64),
                ("blocks_per_piece", ctypes.c_int64), ("tables", ctypes.c_int64),
                ("fused", ctypes.c_int64), ("fused_grid_blocks", ctypes.c_int64),
                ("bags_per_wave", ctypes.c_int32), ("hot_split", ctypes.c_int32),
                ("station", ctypes.c_int32), ("reserved", ctypes.c_int32)]

    def as_dict(self) -> dict:
        return {name: int(getattr(self, name)) for name, _ in self._fields_}


class emb_bag_tuning_entry(ctypes.Structure):
    _fields_ = [("max_row_bytes", ctypes.c_int32), ("max_avg_len", ctypes.c_float),
                ("depth", ctypes.c_int32), ("bags_per_wave", ctypes.c_int32),
                ("stream", ctypes.c_int32), ("bags_per_group", ctypes.c_int32)]


class EmbBagError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {emb_bag_status_string(status)} (status {status})")


def _load(path: str = LIB_PATH) -> ctypes.CDLL:
    if not os.path.exists(path):
        raise ImportError(f"{path} is missing: build it with `python -c 'import "
                          f"__graft_entry__ as g; g.build()'` (there is no CPU fallback)")
    lib = ctypes.CDLL(path)
    P = ctypes.c_void_p
    lib.emb_bag_forward.restype = ctypes.c_int
    lib.emb_bag_forward.argtypes = [ctypes.POINTER(emb_bag_desc), P, P, P, P, P, P, P]
    lib.emb_bag_forward_mixed.restype = ctypes.c_int
    lib.emb_bag_forward_mixed.argtypes = [ctypes.POINTER(emb_bag_mixed_desc), P, P, P, P, P, P, P, P]
    lib.emb_bag_plan_forward.restype = ctypes.c_int
    lib.emb_bag_plan_forward.argtypes = [ctypes.POINTER(emb_bag_desc), ctypes.c_int,
                                         ctypes.c_int32, ctypes.POINTER(emb_bag_plan), P]
    lib.emb_bag_plan_forward_mixed.restype = ctypes.c_int
    lib.emb_bag_plan_forward_mixed.argtypes = [ctypes.POINTER(emb_bag_mixed_desc), ctypes.c_int,
                                               ctypes.c_int32, ctypes.POINTER(emb_bag_plan), P]
    lib.emb_bag_validate.restype = ctypes.c_int
    lib.emb_bag_validate.argtypes = [ctypes.POINTER(emb_bag_desc), P, P, P, P, P]
    lib.emb_bag_profile_reuse.restype = ctypes.c_int
    lib.emb_bag_profile_reuse.argtypes = [ctypes.POINTER(emb_bag_desc), P, P, ctypes.c_int32,
                                          ctypes.c_int32, P, P, P, P]
    lib.emb_bag_profile_hot_rows_workspace.restype = ctypes.c_int64
    lib.emb_bag_profile_hot_rows_workspace.argtypes = [ctypes.c_int32, ctypes.c_int64, ctypes.c_int64]
    lib.emb_bag_profile_hot_rows.restype = ctypes.c_int
    lib.emb_bag_profile_hot_rows.argtypes = [ctypes.POINTER(emb_bag_desc), P, P, ctypes.c_int64,
                                             ctypes.c_int64, P, P, P, P, ctypes.c_int64, P]
    lib.emb_bag_profile_hot_rows_noalloc.restype = ctypes.c_int
    lib.emb_bag_profile_hot_rows_noalloc.argtypes = [ctypes.POINTER(emb_bag_desc), P, P,
                                                     ctypes.c_int64, ctypes.c_int64, P, P, P, P]
    lib.emb_bag_set_tuning.restype = ctypes.c_int
    lib.emb_bag_set_tuning.argtypes = [ctypes.c_char_p, ctypes.c_int64]
    lib.emb_bag_set_tuning_table.restype = ctypes.c_int
    lib.emb_bag_set_tuning_table.argtypes = [ctypes.POINTER(emb_bag_tuning_entry), ctypes.c_int32]
    lib.emb_bag_tuning_defaults.restype = ctypes.c_int
    lib.emb_bag_tuning_defaults.argtypes = [ctypes.POINTER(emb_bag_tuning)]
    lib.emb_bag_get_tuning.restype = ctypes.c_int
    lib.emb_bag_get_tuning.argtypes = [ctypes.c_char_p, ctypes.POINTER(ctypes.c_int64)]
    lib.emb_bag_status_string.restype = ctypes.c_char_p
    lib.emb_bag_status_string.argtypes = [ctypes.c_int]
    lib.emb_bag_version.restype = ctypes.c_int
    lib.emb_bag_version.argtypes = []
    return lib


_lib = _load()


def lib() -> ctypes.CDLL:
    """The loaded C-ABI library (for callers that want the raw entry points)."""
    return _lib


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream_handle(stream) -> Optional[int]:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream or None
    if isinstance(stream, torch.cuda.Stream):
        return stream.cuda_stream or None
    return int(stream) or None


def make_desc(num_tables: int, batch: int, dim: int, table_dtype: int, mode: int,
              num_lookups: int, out_ld: int = 0, max_table_rows: int = 0,
              table_hints: Optional[torch.Tensor] = None, table_avg_len=None,
              hot_rows: Optional[torch.Tensor] = None, tuning=None) -> emb_bag_desc:
    """Fill the host descriptor.  `table_hints` (device uint8 [T]) and `hot_rows` (device int64
    [T]) are tensors, or None, that the caller keeps alive for as long as the descriptor is used;
    `table_avg_len` is a host sequence of T floats (or None), of which the descriptor keeps its
    own copy; `tuning` is a dict of tuning keys (the others at their defaults) that this
    descriptor is planned from instead of the process-wide keys, or None."""
    if table_hints is not None:
        if table_hints.dtype != torch.uint8 or table_hints.numel() != num_tables:
            raise ValueError("table_hints must be a uint8 tensor with one entry per table")
    if hot_rows is not None:
        if hot_rows.dtype != torch.int64 or hot_rows.numel() != num_tables:
            raise ValueError("hot_rows must be an int64 tensor with one entry per table")
    desc = emb_bag_desc(num_tables=num_tables, dim=dim, table_dtype=table_dtype, mode=mode,
                        batch=batch, num_lookups=num_lookups, out_ld=out_ld,
                        max_table_rows=max_table_rows, table_hints=_ptr(table_hints),
                        hot_rows=_ptr(hot_rows))
    _attach_avg_len(desc, table_avg_len, num_tables)
    _attach_tuning(desc, tuning)
    return desc


def emb_bag_tuning_defaults() -> emb_bag_tuning:
    """The tuning struct with the settings of a fresh process."""
    t = emb_bag_tuning()
    rc = _lib.emb_bag_tuning_defaults(ctypes.byref(t))
    if rc != EMB_OK:
        raise EmbBagError(rc, "emb_bag_tuning_defaults")
    return t


def _attach_tuning(desc, tuning) -> None:
    if tuning is None:
        return
    t = emb_bag_tuning_defaults()
    for k, v in tuning.items():
        if k not in dict(emb_bag_tuning._fields_) or k == "reserved":
            raise ValueError(f"unknown tuning key {k!r}")
        setattr(t, k, int(v))
    desc.tuning = ctypes.pointer(t)
    desc._tuning_keepalive = t


def _attach_avg_len(desc, table_avg_len, num_tables: int) -> None:
    if table_avg_len is None:
        return
    if len(table_avg_len) != num_tables:
        raise ValueError("table_avg_len must have one entry per table")
    arr = (ctypes.c_float * num_tables)(*[float(x) for x in table_avg_len])
    desc.table_avg_len = ctypes.cast(arr, ctypes.POINTER(ctypes.c_float))
    desc._avg_len_keepalive = arr


def emb_bag_forward(desc: emb_bag_desc, tables: torch.Tensor, table_offsets: torch.Tensor,
                    indices: torch.Tensor, offsets: torch.Tensor,
                    per_sample_weights: Optional[torch.Tensor], out: torch.Tensor,
                    stream=None) -> None:
    """Enqueue the pooled lookup (see `emb_bag_forward` in include/emb_bag.h).  All tensors are
    device tensors owned by the caller; `out` is written in place, asynchronously."""
    rc = _lib.emb_bag_forward(ctypes.byref(desc), _ptr(tables), _ptr(table_offsets),
                              _ptr(indices), _ptr(offsets), _ptr(per_sample_weights), _ptr(out),
                              _stream_handle(stream))
    if rc != EMB_OK:
        raise EmbBagError(rc, "emb_bag_forward")


def make_mixed_desc(dims, batch: int, table_dtype: int, mode: int, num_lookups: int,
                    out_ld: int = 0, max_table_bytes: int = 0,
                    table_hints: Optional[torch.Tensor] = None,
                    table_avg_len=None, tuning=None) -> emb_bag_mixed_desc:
    """Host descriptor for tables of different widths; `dims` is a sequence of the T widths and
    `table_avg_len` an optional sequence of T floats (the descriptor keeps its own host copies)."""
    arr = (ctypes.c_int32 * len(dims))(*[int(d) for d in dims])
    desc = emb_bag_mixed_desc(num_tables=len(dims), table_dtype=table_dtype, mode=mode, reserved=0,
                              batch=batch, num_lookups=num_lookups, out_ld=out_ld,
                              max_table_bytes=max_table_bytes,
                              dims=ctypes.cast(arr, ctypes.POINTER(ctypes.c_int32)),
                              table_hints=_ptr(table_hints))
    desc._dims_keepalive = arr
    _attach_avg_len(desc, table_avg_len, len(dims))
    _attach_tuning(desc, tuning)
    return desc


def emb_bag_forward_mixed(desc: emb_bag_mixed_desc, tables: torch.Tensor,
                          table_byte_offsets: torch.Tensor, out_offsets: torch.Tensor,
                          indices: torch.Tensor, offsets: torch.Tensor,
                          per_sample_weights: Optional[torch.Tensor], out: torch.Tensor,
                          stream=None) -> None:
    """Enqueue the pooled lookup over tables of different widths (see include/emb_bag.h)."""
    rc = _lib.emb_bag_forward_mixed(ctypes.byref(desc), _ptr(tables), _ptr(table_byte_offsets),
                                    _ptr(out_offsets), _ptr(indices), _ptr(offsets),
                                    _ptr(per_sample_weights), _ptr(out), _stream_handle(stream))
    if rc != EMB_OK:
        raise EmbBagError(rc, "emb_bag_forward_mixed")


def _plan(fn, where: str, desc, has_weights: bool, with_order: bool, *which):
    plan = emb_bag_plan()
    n = min(int(desc.num_tables), 1024)
    order = (ctypes.c_uint16 * max(n, 1))() if with_order else None
    rc = fn(ctypes.byref(desc), int(bool(has_weights)), *which, ctypes.byref(plan), order)
    if rc != EMB_OK:
        raise EmbBagError(rc, where)
    return (plan, list(order)[:int(plan.tables)]) if with_order else plan


def emb_bag_plan_forward(desc: emb_bag_desc, has_weights: bool = False, with_order: bool = False,
                         which: int = 0):
    """Launch number `which` of what emb_bag_forward would do for `desc` under the current tuning
    (host only, no GPU needed).  Returns the plan, or (plan, table order) with `with_order`."""
    return _plan(_lib.emb_bag_plan_forward, "emb_bag_plan_forward", desc, has_weights, with_order,
                 int(which))


def emb_bag_plan_forward_mixed(desc: emb_bag_mixed_desc, has_weights: bool = False,
                               with_order: bool = False, which: int = 0):
    """Launch number `which` of what emb_bag_forward_mixed would do for `desc` (host only, no GPU
    needed); plan.num_launches says how many there are."""
    return _plan(_lib.emb_bag_plan_forward_mixed, "emb_bag_plan_forward_mixed", desc, has_weights,
                 with_order, int(which))


def emb_bag_validate(desc: emb_bag_desc, table_offsets: torch.Tensor, indices: torch.Tensor,
                     offsets: torch.Tensor, num_bad: torch.Tensor, stream=None) -> None:
    """Enqueue the defect count into `num_bad` (device int64[1], zeroed by the caller)."""
    rc = _lib.emb_bag_validate(ctypes.byref(desc), _ptr(table_offsets), _ptr(indices),
                               _ptr(offsets), _ptr(num_bad), _stream_handle(stream))
    if rc != EMB_OK:
        raise EmbBagError(rc, "emb_bag_validate")


def emb_bag_profile_reuse(desc: emb_bag_desc, indices: torch.Tensor, offsets: torch.Tensor,
                          window: int, threshold_permille: int,
                          dup_count: Optional[torch.Tensor], window_used: Optional[torch.Tensor],
                          hints: Optional[torch.Tensor], stream=None) -> None:
    """Enqueue the per-table repeat count / hint derivation (device int32[T], int32[T], uint8[T])."""
    rc = _lib.emb_bag_profile_reuse(ctypes.byref(desc), _ptr(indices), _ptr(offsets), int(window),
                                    int(threshold_permille), _ptr(dup_count), _ptr(window_used),
                                    _ptr(hints), _stream_handle(stream))
    if rc != EMB_OK:
        raise EmbBagError(rc, "emb_bag_profile_reuse")


def emb_bag_profile_hot_rows_workspace(num_tables: int, window: int, k: int) -> int:
    """Bytes of workspace emb_bag_profile_hot_rows needs (raises for arguments out of range)."""
    n = int(_lib.emb_bag_profile_hot_rows_workspace(int(num_tables), int(window), int(k)))
    if n < 0:
        raise EmbBagError(n, "emb_bag_profile_hot_rows_workspace")
    return n


def emb_bag_profile_hot_rows(desc: emb_bag_desc, indices: torch.Tensor, offsets: torch.Tensor,
                             window: int, k: int, hot_ids: torch.Tensor, hot_counts: torch.Tensor,
                             num_hot: Optional[torch.Tensor], workspace: torch.Tensor,
                             stream=None) -> None:
    """Enqueue the per-table top-k row profile (device int64 [T*k], int32 [T*k], int32 [T]);
    `workspace` is a device tensor of at least emb_bag_profile_hot_rows_workspace(...) bytes."""
    rc = _lib.emb_bag_profile_hot_rows(ctypes.byref(desc), _ptr(indices), _ptr(offsets),
                                       int(window), int(k), _ptr(hot_ids), _ptr(hot_counts),
                                       _ptr(num_hot), _ptr(workspace),
                                       workspace.numel() * workspace.element_size(),
                                       _stream_handle(stream))
    if rc != EMB_OK:
        raise EmbBagError(rc, "emb_bag_profile_hot_rows")


def emb_bag_profile_hot_rows_noalloc(desc: emb_bag_desc, indices: torch.Tensor,
                                     offsets: torch.Tensor, window: int, k: int,
                                     hot_ids: torch.Tensor, hot_counts: torch.Tensor,
                                     num_hot: Optional[torch.Tensor], stream=None) -> None:
    """emb_bag_profile_hot_rows without a workspace (the library's own 16 MiB scratch array)."""
    rc = _lib.emb_bag_profile_hot_rows_noalloc(ctypes.byref(desc), _ptr(indices), _ptr(offsets),
                                               int(window), int(k), _ptr(hot_ids),
                                               _ptr(hot_counts), _ptr(num_hot),
                                               _stream_handle(stream))
    if rc != EMB_OK:
        raise EmbBagError(rc, "emb_bag_profile_hot_rows_noalloc")


def emb_bag_set_tuning(key: str, value: int) -> None:
    rc = _lib.emb_bag_set_tuning(key.encode(), int(value))
    if rc != EMB_OK:
        raise EmbBagError(rc, f"emb_bag_set_tuning({key!r}, {value})")


def emb_bag_set_tuning_table(entries) -> None:
    """Load a tuning table: a sequence of dicts with the fields of emb_bag_tuning_entry (missing
    fields mean "automatic"); an empty sequence clears it."""
    auto = {"depth": 0, "bags_per_wave": 0, "stream": -1, "bags_per_group": 0}
    arr = (emb_bag_tuning_entry * max(len(entries), 1))()
    for i, e in enumerate(entries):
        arr[i] = emb_bag_tuning_entry(int(e["max_row_bytes"]), float(e["max_avg_len"]),
                                      *[int(e.get(k, v)) for k, v in auto.items()])
    rc = _lib.emb_bag_set_tuning_table(arr, len(entries))
    if rc != EMB_OK:
        raise EmbBagError(rc, "emb_bag_set_tuning_table")


def emb_bag_get_tuning(key: str) -> int:
    v = ctypes.c_int64(0)
    rc = _lib.emb_bag_get_tuning(key.encode(), ctypes.byref(v))
    if rc != EMB_OK:
        raise EmbBagError(rc, f"emb_bag_get_tuning({key!r})")
    return int(v.value)


def emb_bag_status_string(status: int) -> str:
    return _lib.emb_bag_status_string(int(status)).decode()


def emb_bag_version() -> int:
    return int(_lib.emb_bag_version())
