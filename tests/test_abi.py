"""The C-ABI library loads and exports exactly what include/emb_bag.h declares; host-side
argument checks return their codes without touching a GPU."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "emb_bag.h")


def _declared_functions():
    src = open(HEADER).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(emb_bag_\w+)\s*\(", src)))


def test_header_functions_are_exported():
    import paper_2410_22249_amd as emb
    names = _declared_functions()
    assert set(names) == set(emb.EXPORTS)
    lib = ctypes.CDLL(emb.binding.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), f"{n} declared in emb_bag.h but not exported"


def test_status_codes_and_strings_match_header():
    import paper_2410_22249_amd as emb
    src = open(HEADER).read()
    codes = dict((k, int(v)) for k, v in re.findall(r"#define (EMB_(?:OK|ERR_\w+))\s+\(?(-?\d+)\)?", src))
    assert codes["EMB_OK"] == 0 and len(codes) == 10
    seen = set()
    for name, code in codes.items():
        s = emb.emb_bag_status_string(code)
        assert s and s != "unknown status", name
        seen.add(s)
    assert len(seen) == len(codes)
    assert emb.emb_bag_status_string(-999) == "unknown status"
    assert emb.emb_bag_version() >= 100


def test_desc_layout_matches_header():
    import paper_2410_22249_amd as emb
    assert ctypes.sizeof(emb.emb_bag_desc) == 4 * 4 + 4 * 8 + 4 * 8
    assert emb.emb_bag_desc.batch.offset == 16 and emb.emb_bag_desc.max_table_rows.offset == 40
    assert emb.emb_bag_desc.table_hints.offset == 48 and emb.emb_bag_desc.table_avg_len.offset == 56
    assert emb.emb_bag_desc.hot_rows.offset == 64 and emb.emb_bag_desc.tuning.offset == 72
    assert ctypes.sizeof(emb.emb_bag_tuning) == 64


def test_mixed_desc_layout_and_host_errors():
    import paper_2410_22249_amd as emb
    assert ctypes.sizeof(emb.emb_bag_mixed_desc) == 4 * 4 + 4 * 8 + 4 * 8
    assert emb.emb_bag_mixed_desc.dims.offset == 48 and emb.emb_bag_mixed_desc.table_avg_len.offset == 64
    assert emb.emb_bag_mixed_desc.tuning.offset == 72
    lib = emb.lib()
    fake = ctypes.c_void_p(0x1000)

    def call(desc, tables=fake, boff=fake, ooff=fake, idx=fake, off=fake, w=None, out=fake):
        return lib.emb_bag_forward_mixed(ctypes.byref(desc) if desc is not None else None, tables,
                                         boff, ooff, idx, off, w, out, None)

    ok = dict(batch=4, table_dtype=emb.EMB_F32, mode=emb.EMB_SUM, num_lookups=10)
    assert call(None) == -1
    assert call(emb.make_mixed_desc([64, 6], **ok)) == -2                   # 24-byte rows
    assert call(emb.make_mixed_desc([64, 512], **ok)) == -2                 # 2 KiB rows
    assert call(emb.make_mixed_desc([64, 0], **ok)) == -2
    assert call(emb.make_mixed_desc([64, 32], **{**ok, "table_dtype": 9})) == -3
    assert call(emb.make_mixed_desc([64, 32], **{**ok, "mode": 5})) == -4
    assert call(emb.make_mixed_desc([64, 32], **{**ok, "out_ld": 92})) == -2   # < 96
    assert call(emb.make_mixed_desc([64, 32], **{**ok, "batch": -1})) == -7
    assert call(emb.make_mixed_desc([64, 32], **{**ok, "mode": emb.EMB_MEAN}), w=fake) == -5
    assert call(emb.make_mixed_desc([64, 32], **ok), ooff=None) == -1
    assert call(emb.make_mixed_desc([64, 32], **ok), tables=ctypes.c_void_p(0x1004)) == -8
    assert call(emb.make_mixed_desc([120, 56], **{**ok, "table_dtype": emb.EMB_U8ROW}), out=None) == -1
    assert call(emb.make_mixed_desc([128], **{**ok, "table_dtype": emb.EMB_U8ROW})) == -2
    assert call(emb.make_mixed_desc([64, 32], **{**ok, "batch": 0}), tables=None, out=None) == 0


def test_generator_library_exports():
    from inputgen import gen
    lib = ctypes.CDLL(gen.LIB_PATH)
    for n in ("gen_fill_table", "gen_alloc_arena", "gen_free_arena", "gen_copy_bytes", "gen_read_bytes",
              "gen_scrub_cache"):
        assert hasattr(lib, n)


def test_host_side_argument_errors():
    """These return before any HIP call is made, so they run without a GPU."""
    import paper_2410_22249_amd as emb
    lib = emb.lib()
    fake = ctypes.c_void_p(0x1000)  # never dereferenced: every call below fails validation

    def fwd(desc, tables=fake, toff=fake, idx=fake, off=fake, w=None, out=fake):
        return lib.emb_bag_forward(ctypes.byref(desc) if desc is not None else None,
                                   tables, toff, idx, off, w, out, None)

    ok = dict(num_tables=2, batch=4, dim=64, table_dtype=emb.EMB_F32, mode=emb.EMB_SUM,
              num_lookups=10)
    assert fwd(None) == -1
    assert fwd(emb.make_desc(**{**ok, "table_dtype": 7})) == -3
    assert fwd(emb.make_desc(**{**ok, "mode": 3})) == -4
    assert fwd(emb.make_desc(**{**ok, "num_tables": 0})) == -2
    assert fwd(emb.make_desc(**{**ok, "dim": 0})) == -2
    assert fwd(emb.make_desc(**{**ok, "dim": 6})) == -2                       # 24-byte rows
    assert fwd(emb.make_desc(**{**ok, "dim": 4, "table_dtype": emb.EMB_F16})) == -2  # 8-byte rows
    assert fwd(emb.make_desc(**{**ok, "dim": 4, "table_dtype": emb.EMB_BF16})) == -2
    assert fwd(emb.make_desc(**{**ok, "dim": 32768})) == -2                   # row > 64 KiB
    assert fwd(emb.make_desc(**{**ok, "batch": -1})) == -7
    assert fwd(emb.make_desc(**{**ok, "num_lookups": -1})) == -7
    assert fwd(emb.make_desc(**{**ok, "out_ld": 100})) == -2                  # < T*D
    assert fwd(emb.make_desc(**{**ok, "out_ld": 130})) == -2                  # not a multiple of 4
    assert fwd(emb.make_desc(**{**ok, "mode": emb.EMB_MEAN}), w=fake) == -5
    assert fwd(emb.make_desc(**{**ok, "mode": emb.EMB_MAX}), w=fake) == -5
    assert fwd(emb.make_desc(**ok), tables=None) == -1
    assert fwd(emb.make_desc(**ok), out=None) == -1
    assert fwd(emb.make_desc(**ok), idx=None) == -1
    assert fwd(emb.make_desc(**ok), tables=ctypes.c_void_p(0x1008)) == -8
    assert fwd(emb.make_desc(**{**ok, "batch": 1 << 31})) == -7
    assert fwd(emb.make_desc(**{**ok, "batch": 0}), tables=None, out=None) == 0   # no-op
    assert lib.emb_bag_profile_reuse(None, fake, fake, 64, 20, fake, fake, fake, None) == -1
    assert lib.emb_bag_profile_reuse(ctypes.byref(emb.make_desc(**ok)), fake, None, 64, 20, fake,
                                     fake, fake, None) == -1
    assert lib.emb_bag_validate(None, fake, fake, fake, fake, None) == -1
    assert lib.emb_bag_validate(ctypes.byref(emb.make_desc(**ok)), fake, fake, fake, None, None) == -1


def test_tuning_keys():
    import paper_2410_22249_amd as emb
    for key, good, bad in (("depth", 8, 3), ("addressing", 1, 5), ("blocks_per_cu", 2, 9),
                           ("xcd_remap", 1, 2), ("use_hints", 0, 2),
                           ("stream", 0, 2), ("bags_per_group", 5, 64),
                           ("xcd_pieces", 4, 3), ("per_table_launch", 1, 2), ("fuse", 0, 2)):
        old = emb.emb_bag_get_tuning(key)
        emb.emb_bag_set_tuning(key, good)
        assert emb.emb_bag_get_tuning(key) == good
        with pytest.raises(emb.EmbBagError):
            emb.emb_bag_set_tuning(key, bad)
        assert emb.emb_bag_get_tuning(key) == good
        emb.emb_bag_set_tuning(key, old)
    with pytest.raises(emb.EmbBagError):
        emb.emb_bag_set_tuning("no_such_key", 1)
    with pytest.raises(emb.EmbBagError):
        emb.emb_bag_get_tuning("no_such_key")


def test_byte_accounting_matches_paper():
    """Sec. 3.1: 2048 x 150 x 128 x 4 B = 150 MiB per table, 37,500 MiB for 250 tables."""
    import json
    from paper_2410_22249_amd import metrics
    g = json.load(open(os.path.join(ROOT, "tests", "golden", "paper_constants.json")))
    per = g["bytes_per_table"]
    nl = per["batch"] * per["lookups_per_sample"]
    assert metrics.gathered_bytes(nl, per["dim"], per["elem_bytes"]) == per["bytes"] == per["mib"] << 20
    stage = g["bytes_whole_stage"]
    assert metrics.gathered_bytes(nl * stage["tables"], per["dim"], per["elem_bytes"]) == stage["mib"] << 20
    rb = g["row_bytes"]
    assert rb["dim"] * rb["elem_bytes"] == rb["bytes"]
    assert abs(rb["l2_set_aside_mb"] * 1e6 / rb["bytes"] - rb["vectors"]) / rb["vectors"] < 0.03
    li = g["load_instructions_per_table"]
    n = li["batch"] * li["lookups_per_sample"] * li["warps_per_sample"] * li["loads_per_lookup_per_warp"]
    assert abs(n / 1e6 - li["printed_millions"]) < 0.02
    # cfg3: 526.5 algorithmic bytes per lookup
    a = metrics.algorithmic_bytes(19_660_800, 60, 4096, 128, 4)
    assert abs(a / 19_660_800 - 526.5) < 0.1
