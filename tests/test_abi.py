"""The built C-ABI library loads without a GPU and exports every function include/sagekv.h declares."""
import ctypes
import os
import re

import paper_2503_08879_amd as sk

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "sagekv.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sagekv_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert "sagekv_select" in names and "sagekv_decode_attn" in names and len(names) == 14
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
    assert n > 32 * 8 * 4 * 131072 * 4  # at least the fp32 logits
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
