"""Structural guards: the header is plain C, the product path never touches the oracle, the oracle
never touches the product, and nothing committed depends on working files."""
import os
import re
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _py_files(*dirs):
    for d in dirs:
        for base, _, names in os.walk(os.path.join(ROOT, d)):
            for n in names:
                if n.endswith(".py"):
                    yield os.path.join(base, n)


def test_header_is_valid_c99(tmp_path):
    src = tmp_path / "use_header.c"
    src.write_text('#include "emb_bag.h"\n'
                   "int use(void) {\n"
                   "  emb_bag_desc d = {0};\n"
                   "  d.num_tables = 1; d.dim = 4; d.table_dtype = EMB_BF16; d.mode = EMB_MEAN;\n"
                   "  d.table_hints = 0; d.table_avg_len = 0;\n"
                   "  emb_bag_mixed_desc m = {0};\n"
                   "  m.num_tables = 2; m.dims = 0;\n"
                   "  (void)emb_bag_forward_mixed(&m, 0, 0, 0, 0, 0, 0, 0, 0);\n"
                   "  emb_bag_plan p;\n"
                   "  (void)emb_bag_plan_forward(&d, 0, 0, &p, 0);\n"
                   "  (void)emb_bag_plan_forward_mixed(&m, 0, 0, &p, 0);\n"
                   "  return emb_bag_forward(&d, 0, 0, 0, 0, 0, 0, 0) + emb_bag_version() +\n"
                   "         emb_bag_profile_reuse(&d, 0, 0, 64, -1, 0, 0, 0, 0) + EMB_HINT_STREAMING;\n"
                   "}\n")
    subprocess.run(["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-fsyntax-only",
                    "-I", os.path.join(ROOT, "include"), str(src)], check=True)


def test_binding_structs_match_the_header_as_the_c_compiler_lays_it_out(tmp_path):
    """sizeof and offsetof of every field, printed by a C program built from the header, against
    the ctypes mirror in the binding."""
    import ctypes
    import paper_2410_22249_amd as emb
    structs = {"emb_bag_desc": emb.emb_bag_desc, "emb_bag_mixed_desc": emb.emb_bag_mixed_desc,
               "emb_bag_plan": emb.emb_bag_plan, "emb_bag_tuning": emb.emb_bag_tuning,
               "emb_bag_tuning_entry": emb.emb_bag_tuning_entry}
    lines = ['#include <stdio.h>', '#include <stddef.h>', '#include "emb_bag.h"', "int main(void) {"]
    for cname, cls in structs.items():
        lines.append(f'  printf("{cname} %zu\\n", sizeof({cname}));')
        for field, _ in cls._fields_:
            lines.append(f'  printf("{cname}.{field} %zu\\n", offsetof({cname}, {field}));')
    lines += ["  return 0;", "}"]
    src, exe = tmp_path / "layout.c", tmp_path / "layout"
    src.write_text("\n".join(lines) + "\n")
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"),
                    "-o", str(exe), str(src)], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout
    seen = dict(line.split() for line in out.splitlines())
    for cname, cls in structs.items():
        assert int(seen[cname]) == ctypes.sizeof(cls), cname
        for field, _ in cls._fields_:
            assert int(seen[f"{cname}.{field}"]) == getattr(cls, field).offset, (cname, field)
    # every field of the header's structs is mirrored: same count of members
    hdr = open(os.path.join(ROOT, "include", "emb_bag.h")).read()
    for cname, cls in structs.items():
        body = hdr[hdr.index(f"typedef struct {cname} {{"):hdr.index(f"}} {cname};")]
        body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
        assert body.count(";") == len(cls._fields_), cname


def test_product_path_never_imports_the_oracle():
    pat = re.compile(r"^\s*(from|import)\s+oracle\b|emb_bag_oracle|reuse_oracle|hot_rows_oracle|liboracle", re.M)
    for f in _py_files("paper_2410_22249_amd", "inputgen"):
        assert not pat.search(open(f).read()), f"{f} refers to the oracle"
    for base, _, names in os.walk(os.path.join(ROOT, "paper_2410_22249_amd", "csrc")):
        for n in names:
            assert "oracle" not in open(os.path.join(base, n)).read().lower(), n
    hdr = open(os.path.join(ROOT, "include", "emb_bag.h")).read().lower()
    assert "oracle" not in hdr


def test_oracle_is_independent_of_the_product():
    pat = re.compile(r"paper_2410_22249_amd|libembbag|emb_bag\.h|inputgen", re.M)
    for name in os.listdir(os.path.join(ROOT, "oracle")):
        if name.endswith((".py", ".c", ".h")):
            assert not pat.search(open(os.path.join(ROOT, "oracle", name)).read()), name


def test_nothing_committed_uses_working_files():
    pat = re.compile(r"_work/|_work\b")
    for f in list(_py_files("paper_2410_22249_amd", "inputgen", "oracle", "tests")) + [
            os.path.join(ROOT, "bench.py"), os.path.join(ROOT, "__graft_entry__.py")]:
        if f.endswith("test_layout.py"):
            continue
        assert not pat.search(open(f).read()), f
