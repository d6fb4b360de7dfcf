"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol
the header declares, and validates arguments before touching the device."""
import ctypes
import os
import re

import pytest

import paper_2605_15508_amd as sts
from paper_2605_15508_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(sts.library_path()):
        from paper_2605_15508_amd.build import build

        build(force=True)
    return sts.load_library()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "sts.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sts_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert {"sts_select", "sts_sparse_attn", "sts_dense_attn"} <= set(names)
    for n in names:
        assert hasattr(lib, n), f"{n} declared in include/sts.h but not exported"
    assert sorted(binding.EXPORTS) == names


def test_version_and_strerror(lib):
    assert sts.sts_version() >= 100
    assert lib.sts_strerror(0) == b"ok"
    assert b"workspace" in lib.sts_strerror(-3)


def attn_params(**kw):
    base = dict(B=1, Tq=5, Hq=32, Hkv=8, d=128, N=4096, kv_stride_b=8 * 4096 * 128, kv_stride_h=4096 * 128,
                kv_stride_n=128, kmax=410, scale=0.088, out_dtype=0)
    base.update(kw)
    return binding.AttnParams(**base)


def test_attn_argument_validation(lib):
    ok = attn_params()
    assert lib.sts_attn_workspace_bytes(ctypes.byref(ok), 1) > 0
    for bad in (attn_params(d=96), attn_params(Tq=17), attn_params(Hq=30), attn_params(kv_stride_n=100),
                attn_params(Hq=512, Hkv=8)):
        assert lib.sts_attn_workspace_bytes(ctypes.byref(bad), 1) == 0
        assert lib.sts_sparse_attn(ctypes.byref(bad), None) < 0
    # valid shape but no workspace / no data: refused before any launch
    assert lib.sts_sparse_attn(ctypes.byref(ok), None) == -1


def test_attn_plan_groups_heads_by_head_map(lib):
    p = attn_params()
    s, u, nq = ctypes.c_int32(), ctypes.c_int32(), ctypes.c_int32()
    assert lib.sts_attn_plan(ctypes.byref(p), 1, ctypes.byref(s), ctypes.byref(u), ctypes.byref(nq)) == 0
    assert (u.value, nq.value) == (32, 1)            # no hint: one unit per query head
    hm = (ctypes.c_int32 * 32)(*[t // 2 for t in range(32)])
    p.head_map = ctypes.cast(hm, ctypes.c_void_p)
    assert lib.sts_attn_plan(ctypes.byref(p), 1, ctypes.byref(s), ctypes.byref(u), ctypes.byref(nq)) == 0
    assert (u.value, nq.value) == (16, 1)            # pairs share a gathered tile: 10 rows
    assert s.value >= 1
    hm2 = (ctypes.c_int32 * 32)(*[0] * 32)
    p.head_map = ctypes.cast(hm2, ctypes.c_void_p)
    assert lib.sts_attn_plan(ctypes.byref(p), 1, ctypes.byref(s), ctypes.byref(u), ctypes.byref(nq)) == 0
    assert (u.value, nq.value) == (8, 2)             # whole KV group: 20 rows -> 2 query tiles
    p.head_map = None
    assert lib.sts_attn_plan(ctypes.byref(p), 0, ctypes.byref(s), ctypes.byref(u), ctypes.byref(nq)) == 0
    assert (u.value, nq.value) == (8, 2)             # dense: one unit per KV head


def test_select_argument_validation(lib):
    hm = (ctypes.c_int32 * 4)(0, 1, 1, 0)
    p = binding.SelectParams(B=1, Hd=2, Tq=5, N=1000, Hq=4, k=10, head_map=ctypes.cast(hm, ctypes.c_void_p))
    assert lib.sts_select_workspace_bytes(ctypes.byref(p)) > 0
    assert lib.sts_select(ctypes.byref(p), None) == -1          # indices missing
    p.k = 0
    assert lib.sts_select_workspace_bytes(ctypes.byref(p)) == 0
    p.k = 10
    bad = (ctypes.c_int32 * 4)(0, 2, 1, 0)                      # draft head 2 does not exist
    p.head_map = ctypes.cast(bad, ctypes.c_void_p)
    p.indices = 256                                             # never dereferenced: map is checked first
    assert lib.sts_select(ctypes.byref(p), None) == -1


def test_per_head_budgets_are_validated(lib):
    hm = (ctypes.c_int32 * 4)(0, 1, 1, 0)
    p = binding.SelectParams(B=1, Hd=2, Tq=5, N=1000, Hq=4, k=10, head_map=ctypes.cast(hm, ctypes.c_void_p),
                             indices=256)
    for bad in ((0, 5), (5, 11), (-3, 2)):                      # below 1 or above the row pitch k
        kh = (ctypes.c_int32 * 2)(*bad)
        p.k_head = ctypes.cast(kh, ctypes.c_void_p)
        assert lib.sts_select(ctypes.byref(p), None) == -1
    kh = (ctypes.c_int32 * 2)(10, 1)                            # valid budgets: the next check (scores) fails
    p.k_head = ctypes.cast(kh, ctypes.c_void_p)
    assert lib.sts_select(ctypes.byref(p), None) == -1
    p.B = 0                                                     # empty batch: accepted, nothing enqueued
    assert lib.sts_select(ctypes.byref(p), None) == 0


def test_ctypes_structs_match_the_header(tmp_path):
    """The Python binding restates the parameter structs: compile the header as C11 and compare
    size and every field offset."""
    import subprocess

    structs = {"sts_select_params": binding.SelectParams, "sts_attn_params": binding.AttnParams,
               "sts_headmap_params": binding.HeadmapParams, "sts_union_params": binding.UnionParams}
    lines = ["#include <stdio.h>", "#include <stddef.h>", '#include "sts.h"', "int main(void) {"]
    for cname, cls in structs.items():
        lines.append(f'  printf("{cname} %zu\\n", sizeof({cname}));')
        for fname, _ in cls._fields_:
            lines.append(f'  printf("{cname}.{fname} %zu\\n", offsetof({cname}, {fname}));')
    lines += ["  return 0;", "}"]
    src = tmp_path / "layout.c"
    src.write_text("\n".join(lines))
    exe = tmp_path / "layout"
    subprocess.run(["gcc", "-std=c11", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe)],
                   check=True)
    got = dict(line.split() for line in subprocess.run([str(exe)], check=True, capture_output=True,
                                                       text=True).stdout.splitlines())
    for cname, cls in structs.items():
        assert int(got[cname]) == ctypes.sizeof(cls), cname
        for fname, _ in cls._fields_:
            assert int(got[f"{cname}.{fname}"]) == getattr(cls, fname).offset, f"{cname}.{fname}"
        # and no field of the header is missing from the binding
        text = re.sub(r"/\*.*?\*/", "", open(os.path.join(ROOT, "include", "sts.h")).read(), flags=re.S)
        body = re.search(r"typedef struct \{([^}]*)\} " + cname + ";", text).group(1)
        declared = re.findall(r"\b\*?([A-Za-z_][A-Za-z0-9_]*)\s*(?:,|;)", body)
        assert sorted(declared) == sorted(f for f, _ in cls._fields_), cname


def test_product_path_has_no_oracle_import():
    pkg = os.path.join(ROOT, "paper_2605_15508_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in text and "from oracle" not in text and "sts_oracle" not in text


def test_split_policy_is_a_function_of_the_shape_only(lib):
    """Deterministic results need a split count that depends on nothing but the shape."""
    def plan(**kw):
        p = attn_params(**kw)
        s, u, nq = ctypes.c_int32(), ctypes.c_int32(), ctypes.c_int32()
        assert lib.sts_attn_plan(ctypes.byref(p), kw.pop("_sparse", 1), ctypes.byref(s), ctypes.byref(u),
                                 ctypes.byref(nq)) == 0
        return s.value, u.value, nq.value
    # a short list is not split at all (its workgroup writes the result itself)
    assert plan(kmax=410)[0] == 1
    assert plan(kmax=512)[0] == 1
    # longer lists: at least two 32-key tiles per wave of the 4-wave workgroup
    s, u, _ = plan(kmax=3277)
    assert 1 < s <= (3277 // 32 + 1 + 7) // 8
    # block granularity counts tiles in tokens
    assert plan(kmax=52, page_size=8)[0] == plan(kmax=410)[0]
    big = plan(B=4, N=131072, kmax=13108, kv_stride_b=8 * 131072 * 128, kv_stride_h=131072 * 128)
    assert big[0] >= 1 and big == plan(B=4, N=131072, kmax=13108, kv_stride_b=8 * 131072 * 128,
                                       kv_stride_h=131072 * 128)


def test_page_and_tail_argument_validation(lib):
    assert lib.sts_attn_workspace_bytes(ctypes.byref(attn_params(page_size=8)), 1) > 0
    for bad in (attn_params(page_size=3), attn_params(page_size=64), attn_params(page_size=-1 * 0 + 5)):
        assert lib.sts_attn_workspace_bytes(ctypes.byref(bad), 1) == 0
    # a page table needs a pool size, a page stride and enough entries for N
    assert lib.sts_attn_workspace_bytes(ctypes.byref(attn_params(page_size=8, block_table=256, table_stride=512,
                                                                 num_pages=600, kv_stride_page=8 * 8 * 128)), 1) > 0
    for bad in (attn_params(page_size=8, block_table=256, table_stride=100, num_pages=600, kv_stride_page=8192),
                attn_params(page_size=8, block_table=256, table_stride=512, num_pages=0, kv_stride_page=8192),
                attn_params(page_size=8, block_table=256, table_stride=512, num_pages=600, kv_stride_page=0)):
        assert lib.sts_attn_workspace_bytes(ctypes.byref(bad), 1) == 0
    # k_new without v_new is refused
    assert lib.sts_attn_workspace_bytes(ctypes.byref(attn_params(k_new=256)), 1) == 0
    assert lib.sts_attn_workspace_bytes(ctypes.byref(attn_params(k_new=256, v_new=512)), 1) > 0


def test_headmap_argument_validation(lib):
    p = binding.HeadmapParams(S=2, R=4, Hd=3, Ht=5, N=100, k=10)
    assert lib.sts_headmap_workspace_bytes(ctypes.byref(p)) > 0
    assert lib.sts_head_map(ctypes.byref(p), None) == -1          # map missing
    p.k = 0
    assert lib.sts_headmap_workspace_bytes(ctypes.byref(p)) == 0
    sp = binding.SelectParams(B=1, Hd=2, Tq=5, N=1000, Hq=4, k=10, page_size=5000)
    assert lib.sts_select_workspace_bytes(ctypes.byref(sp)) == 0
