"""The C-ABI library loads on a machine without a GPU and exports every symbol that
include/ratsparse.h declares; the binding declares the same set."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "ratsparse.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b([a-z_0-9]+)\s*\(", text)) - {"defined"})


def test_library_exports_every_declared_symbol():
    from paper_2605_28640_amd import binding
    names = _declared()
    assert {"rat_scan", "quest_page_meta", "quest_select_decode", "moba_select_prefill",
            "snapkv_compress", "sparse_attn_decode", "sparse_attn_prefill"} <= set(names)
    lib = ctypes.CDLL(binding.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), n
    assert set(names) == set(binding.SIGNATURES), set(names) ^ set(binding.SIGNATURES)


def test_status_strings_and_host_side_validation():
    from paper_2605_28640_amd import binding
    lib = binding.load()
    assert lib.ratsparse_status_string(0) == b"ok"
    assert b"gfx950" in lib.ratsparse_version()
    bad = binding.make_shape(1, 3, 2, 128, 64, 16, binding.RS_BF16)  # Hq not a multiple of Hkv
    assert lib.rat_scan_workspace_bytes(ctypes.byref(bad), 64) == 0
    s = binding.make_shape(1, 2, 2, 96, 64, 16, binding.RS_BF16)  # unsupported head dim
    assert lib.quest_page_meta(ctypes.byref(s), 16, 16, 0, 16, None) == 2
    s = binding.make_shape(1, 2, 2, 128, 64, 16, binding.RS_BF16)
    assert lib.quest_page_meta(ctypes.byref(s), None, None, 0, 16, None) == 1  # null pointers
    assert lib.quest_page_meta(ctypes.byref(s), 16, 16, 0, 65, None) == 1  # past the capacity
    assert lib.rat_scan_workspace_bytes(ctypes.byref(s), 4096) > binding.RS_WS_CTRL_BYTES
