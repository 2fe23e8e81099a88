"""GPU: gr_beam_select_noalloc (static device scratch inside the library, no allocation) gives exactly what
gr_beam_select gives with a caller workspace - two calls in a row through the raw C ABI, the second one smaller,
plus the size limit."""
import ctypes

import numpy as np
import pytest

import gr_synth
from gpu_util import to_dev

pytestmark = pytest.mark.gpu


class SelectParams(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("W", ctypes.c_int32), ("V", ctypes.c_int32), ("depth", ctypes.c_int32),
                ("step", ctypes.c_int32), ("flags", ctypes.c_int32),
                ("mask", ctypes.c_void_p), ("logits", ctypes.c_void_p), ("scores_in", ctypes.c_void_p),
                ("prefix_in", ctypes.c_void_p), ("range_in", ctypes.c_void_p), ("parent_out", ctypes.c_void_p),
                ("token_out", ctypes.c_void_p), ("scores_out", ctypes.c_void_p), ("prefix_out", ctypes.c_void_p),
                ("range_out", ctypes.c_void_p), ("item_index_out", ctypes.c_void_p)]


def _outputs(torch, B, W, depth, dev):
    return dict(parent=torch.full((B, W), -7, dtype=torch.int32, device=dev), token=torch.full((B, W), -7, dtype=torch.int32, device=dev),
                scores=torch.full((B, W), 7.0, dtype=torch.float32, device=dev), prefix=torch.full((B, W, depth), -7, dtype=torch.int32, device=dev),
                range=torch.full((B, W, 2), -7, dtype=torch.int32, device=dev), item_index=torch.full((B, W), -7, dtype=torch.int32, device=dev))


def _params(mask, logits, sc, pf, rg, step, out):
    B, W, V = logits.shape
    p = SelectParams()
    p.B, p.W, p.V, p.depth, p.step, p.flags = B, W, V, pf.shape[2], step, 0
    p.mask = mask.data_ptr() if mask is not None else None
    p.logits, p.scores_in, p.prefix_in, p.range_in = logits.data_ptr(), sc.data_ptr(), pf.data_ptr(), rg.data_ptr()
    p.parent_out, p.token_out, p.scores_out = out["parent"].data_ptr(), out["token"].data_ptr(), out["scores"].data_ptr()
    p.prefix_out, p.range_out, p.item_index_out = out["prefix"].data_ptr(), out["range"].data_ptr(), out["item_index"].data_ptr()
    return p


def test_noalloc_matches_workspace_entry_point_on_two_calls_in_a_row():
    import torch
    import paper_2512_11529_amd as gr
    lib = ctypes.CDLL(gr.LIB_PATH)
    lib.gr_beam_select.restype = ctypes.c_int32
    lib.gr_beam_select.argtypes = [ctypes.POINTER(SelectParams), ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    lib.gr_beam_select_noalloc.restype = ctypes.c_int32
    lib.gr_beam_select_noalloc.argtypes = [ctypes.POINTER(SelectParams), ctypes.c_void_p]
    lib.gr_beam_select_workspace_bytes.restype = ctypes.c_size_t
    lib.gr_beam_select_workspace_bytes.argtypes = [ctypes.c_int32] * 4
    lib.gr_beam_select_noalloc_max_workspace_bytes.restype = ctypes.c_size_t
    dev = torch.device("cuda:0")
    gr.load_library()
    limit = lib.gr_beam_select_noalloc_max_workspace_bytes()
    assert limit == 16 << 20

    # first a masked level-1 step at a size that spans streamed and gathered rows, then a smaller unconstrained one
    cases = []
    cfg = gr_synth.get_config(2)                     # B=8 W=128 V=8192, 1 M items
    items = gr_synth.make_item_table(cfg)
    mask = gr.gr_item_mask_build(to_dev(items), cfg.V)
    sc0, pf0, rg0 = gr_synth.initial_beam_state(cfg.B, cfg.W, cfg.ND)
    st0 = gr.gr_beam_select(mask, to_dev(gr_synth.make_logits(cfg, 0)), to_dev(sc0), to_dev(pf0), to_dev(rg0), 0)
    cases.append((mask, to_dev(gr_synth.make_logits(cfg, 1)), st0["scores"], st0["prefix"], st0["range"], 1))
    rng = np.random.default_rng(77)
    B2, W2, V2 = 3, 24, 1000
    sc2 = np.sort(-3.0 * rng.random((B2, W2)).astype(np.float32), axis=1)[:, ::-1].copy()
    cases.append((None, to_dev((2.0 * rng.standard_normal((B2, W2, V2))).astype(np.float32)), to_dev(sc2),
                  to_dev(np.full((B2, W2, 3), -1, np.int32)), to_dev(np.zeros((B2, W2, 2), np.int32)), 0))
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    for m, logits, sc, pf, rg, step in cases:
        B, W, V = logits.shape
        need = lib.gr_beam_select_workspace_bytes(B, W, V, 3)
        assert need <= limit
        ws = torch.empty(need, dtype=torch.uint8, device=dev)
        want, got = _outputs(torch, B, W, 3, dev), _outputs(torch, B, W, 3, dev)
        assert lib.gr_beam_select(ctypes.byref(_params(m, logits, sc, pf, rg, step, want)), ctypes.c_void_p(ws.data_ptr()), need, stream) == 0
        torch.cuda.synchronize()
        # the caching allocator's count of allocations made so far (frees by Python's garbage collector do not touch it)
        before = torch.cuda.memory_stats()["allocation.all.allocated"]
        assert lib.gr_beam_select_noalloc(ctypes.byref(_params(m, logits, sc, pf, rg, step, got)), stream) == 0
        torch.cuda.synchronize()
        assert torch.cuda.memory_stats()["allocation.all.allocated"] == before
        for k in want:
            assert torch.equal(got[k], want[k]), f"B={B} W={W} V={V}: {k} differs between the two entry points"
        assert bool((got["parent"] >= 0).all())

    # a shape whose workspace exceeds the static array is refused before anything runs
    Bx, Wx, Vx = 64, 512, 8192
    assert lib.gr_beam_select_workspace_bytes(Bx, Wx, Vx, 3) > limit
    p = SelectParams()
    p.B, p.W, p.V, p.depth, p.step = Bx, Wx, Vx, 3, 0
    assert lib.gr_beam_select_noalloc(ctypes.byref(p), stream) == -3
