"""The built C-ABI library loads without a GPU and exports every function include/*.h declares."""
import ctypes
import os
import re

import paper_2503_08879_amd as sk

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    names = set()
    for header in sorted(os.listdir(os.path.join(ROOT, "include"))):
        assert header.endswith(".h")
        text = open(os.path.join(ROOT, "include", header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(sagekv_[a-z_0-9]+)\s*\(", text))
    return sorted(names)


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert "sagekv_select" in names and "sagekv_decode_attn" in names and len(names) == 20
    lib = ctypes.CDLL(sk.binding.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(sk.binding.EXPORTS) == names  # the binding wraps exactly the declared calls


def test_status_strings_and_host_side_checks():
    assert sk.binding.status_string(0) == "ok"
    assert "workspace" in sk.binding.status_string(3)
    good = sk.SelectDesc(32, 32, 8, 128, 0, 0, 131072, 8 * 131072 * 128, 131072 * 128, 128, 8 * 131072 * 128,
                         131072 * 128, 128, 4, 512, 3580, 4096)
    n = sk.sagekv_select_workspace_bytes(good)
    # config C3: a score row per KV head for the rows that have to be redone (128 MiB) + candidate records
    assert 32 * 8 * 131072 * 4 < n <= 0.35 * 2 ** 30
    dense = sk.SelectDesc(32, 32, 8, 128, 0, 0, 131072, 8 * 131072 * 128, 131072 * 128, 128, 8 * 131072 * 128,
                          131072 * 128, 128, 4, 512, 3580, 4096, sk.SELECT_DENSE)
    assert sk.sagekv_select_workspace_bytes(dense) > 32 * 8 * 4 * 131072 * 4  # the one-sweep dense path keeps fp32 logits
    bad = sk.SelectDesc(32, 32, 8, 128, 0, 0, 131072, 8 * 131072 * 128, 131072 * 128, 128, 8 * 131072 * 128,
                        131072 * 128, 128, 4, 512, 131072, 4096)
    assert sk.sagekv_select_workspace_bytes(bad) == 0
    # null pointers are rejected on the host, before any launch (safe without a GPU)
    code = sk.binding.lib().sagekv_select(ctypes.byref(good), None, None, None, None, None, None, None, None, 0, None)
    assert code == 1
    dd = sk.decode_desc(1, 32, 8, 128, 0, 4, 3580, 512, 4096)  # few rows: split rows need scratch
    assert sk.sagekv_decode_workspace_bytes(dd) > 0
    assert sk.binding.lib().sagekv_decode_attn(ctypes.byref(dd), None, None, None, 10, None, None, 0, None) == 1
    dd.compact_capacity = 100
    assert sk.sagekv_decode_workspace_bytes(dd) == 0


def test_paper_budget_matches_the_printed_splits_and_the_oracle(ref):
    """Host-only call: the two splits the paper prints (App. A.2), the oracle's rule over a grid,
    and the error cases."""
    path = os.path.join(ROOT, "tests", "golden", "paper_budget.txt")
    rows = [list(map(int, l.split())) for l in open(path) if l.strip() and not l.startswith("#")]
    assert len(rows) == 2
    for B, G, sink, k, recent in rows:
        assert sk.sagekv_paper_budget(B, G) == (sink, k, recent)
    for G in (1, 2, 3, 4, 5, 7, 8, 16):
        for B in (4 * G, 4 * G + 1, 100, 1000, 1024, 4096, 8192, 10000, 1 << 20):
            if B < 4 * G:
                continue
            s, k, r = sk.sagekv_paper_budget(B, G)
            assert (s, k, r) == ref.paper_budget(B, G)
            assert s + G * k + r == B and k >= 1 and k & (k - 1) == 0 and r >= 0
    i32 = ctypes.c_int32
    a, b, c = i32(-7), i32(-7), i32(-7)
    L = sk.binding.lib()
    assert L.sagekv_paper_budget(8192, 0, ctypes.byref(a), ctypes.byref(b), ctypes.byref(c)) == 1
    assert L.sagekv_paper_budget(27, 7, ctypes.byref(a), ctypes.byref(b), ctypes.byref(c)) == 1
    assert L.sagekv_paper_budget(8192, 4, None, ctypes.byref(b), ctypes.byref(c)) == 1
    assert (a.value, b.value, c.value) == (-7, -7, -7)


def test_header_is_plain_c_and_a_c_program_links(tmp_path):
    """The boundary is usable from C: the header compiles as strict C99, and a C program that calls the
    host-only entry points links against the library and runs without a GPU.  The struct sizes seen by
    C are those the ctypes binding marshals."""
    import subprocess

    src = tmp_path / "abi.c"
    src.write_text(r'''
#include <stdio.h>
#include "sagekv.h"
int main(void) {
  sagekv_select_desc d = {0};
  d.n_problems = 32; d.n_q_heads = 32; d.n_kv_heads = 8; d.head_dim = 128; d.dtype = SAGEKV_BF16;
  d.head_mode = SAGEKV_HEADS_GROUP_SUM; d.L = 131072;
  d.k_stride_problem = d.v_stride_problem = 8LL * 131072 * 128;
  d.k_stride_head = d.v_stride_head = 131072LL * 128; d.k_stride_token = d.v_stride_token = 128;
  d.n_sink = 4; d.n_recent = 512; d.k = 3580; d.compact_capacity = 4096;
  sagekv_decode_desc dd = {32, 32, 8, 128, SAGEKV_BF16, SAGEKV_HEADS_GROUP_SUM, 4, 3580, 512, 4096, 0};
  printf("%zu %zu %zu %zu %zu %s\n", sizeof(sagekv_select_desc), sizeof(sagekv_decode_desc), sizeof(sagekv_paged_kv),
         sagekv_select_workspace_bytes(&d), sagekv_decode_workspace_bytes(&dd), sagekv_status_string(SAGEKV_ERR_WORKSPACE));
  return sagekv_select(&d, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0) == SAGEKV_ERR_INVALID_ARG ? 0 : 1;
}
''')
    inc = os.path.join(ROOT, "include")
    libdir = os.path.dirname(sk.binding.LIB_PATH)
    exe = tmp_path / "abi"
    subprocess.check_call(["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-I", inc, str(src), "-o", str(exe),
                           "-L", libdir, "-lsagekv", f"-Wl,-rpath,{libdir}"])
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split(maxsplit=5)
    assert [int(x) for x in out[:3]] == [ctypes.sizeof(sk.SelectDesc), ctypes.sizeof(sk.DecodeDesc), ctypes.sizeof(sk.PagedKV)]
    assert int(out[3]) == sk.sagekv_select_workspace_bytes(sk.SelectDesc(
        32, 32, 8, 128, 0, 0, 131072, 8 * 131072 * 128, 131072 * 128, 128, 8 * 131072 * 128, 131072 * 128, 128,
        4, 512, 3580, 4096, 0))
    assert int(out[4]) == 0 and "workspace" in out[5]
