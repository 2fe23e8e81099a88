"""CPU-only checks of the C-ABI library: it loads, exports every symbol include/gr.h declares, and its
host-side size queries and argument validation behave (no kernel is launched)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def gr():
    import paper_2512_11529_amd as gr
    if not os.path.exists(gr.LIB_PATH):
        from paper_2512_11529_amd import build
        build.build_lib()
    gr.load_library()
    return gr


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "gr.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(gr_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(gr):
    names = _declared_functions()
    assert {"gr_beam_attn", "gr_item_mask_build", "gr_beam_select", "gr_status_string"} <= set(names)
    lib = ctypes.CDLL(gr.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), f"{n} declared in gr.h but not exported"


def test_status_strings(gr):
    for s in range(0, -6, -1):
        assert gr.gr_status_string(s).startswith("GR_")
    assert "unknown" in gr.gr_status_string(-99)


def test_size_queries(gr):
    lib = gr.load_library()
    assert lib.gr_item_mask_bytes(10_000_000, 3, 8192) > 8192 * 8192 // 8 + 3 * 4 * 10_000_000
    assert lib.gr_item_mask_bytes(10, 2, 8) == 0 and lib.gr_item_mask_bytes(0, 3, 8) == 0
    assert lib.gr_item_mask_bytes(10, 3, 40000) == 0
    assert lib.gr_beam_select_workspace_bytes(32, 256, 8192, 3) >= 2 * 32 * 256 * 4
    assert gr.attn_workspace_bytes(32, 256, 32, 8, 128, 4096, total_L=32 * 4096) == 0   # uniform batch, enough units: nothing
    assert gr.attn_workspace_bytes(32, 256, 32, 8, 128, 4096, total_L=32 * 4096 - 5) == 256  # ragged: the dispatch order of 32 requests
    assert gr.attn_workspace_bytes(1, 256, 32, 8, 128, 4096) > 0              # one request cannot fill the chip: split L


def test_null_and_range_arguments_are_rejected_on_the_host(gr):
    lib = gr.load_library()
    assert lib.gr_beam_attn(None, None, 0, None) == -1
    assert lib.gr_beam_select(None, None, 0, None) == -1
    assert lib.gr_item_mask_build(None, 10, 3, 8, None, 0, None, 0, None) == -1
    assert lib.gr_beam_reorder(1, 4, 3, 2, 64, 1, None, None, None, None) == -1      # null pointers
    assert lib.gr_beam_reorder(1, 4, 3, 2, 64, 4, None, None, None, None) == -1      # u > ND
    p = gr._SelectParams()
    p.B, p.W, p.V, p.depth, p.step = 1, 4, 8, 3, 5
    assert lib.gr_beam_select(ctypes.byref(p), None, 0, None) == -1
    a = gr._AttnParams()
    a.B, a.W, a.Hq, a.Hkv, a.d, a.ND, a.u = 1, 4, 8, 3, 64, 3, 1      # Hq % Hkv != 0
    assert lib.gr_beam_attn(ctypes.byref(a), None, 0, None) == -1


def test_product_package_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2512_11529_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".h", ".cpp")):
                src = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in src.lower().replace("the oracle", ""), f"{f} mentions the oracle"
