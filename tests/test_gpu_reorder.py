"""GPU parity: gr_beam_reorder (in-place unshared-cache update, Section 5.1) against the oracle's gather
into a fresh buffer.  Byte-exact: the call only moves data.  Token slots >= u must stay untouched."""
import numpy as np
import pytest

import gr_synth
from gpu_util import bf16_to_dev, to_dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gr():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_2512_11529_amd as gr
    gr.load_library()
    return gr


def _parents(rng, B, W, kind):
    if kind == "identity":
        return np.tile(np.arange(W, dtype=np.int32), (B, 1))
    if kind == "reverse":
        return np.tile(np.arange(W - 1, -1, -1, dtype=np.int32), (B, 1))
    if kind == "one":                      # every survivor extends the same beam
        return np.full((B, W), W // 2, dtype=np.int32)
    if kind == "shift_up":                 # the pattern a naive top-down in-place copy gets wrong
        return np.tile(np.maximum(np.arange(W, dtype=np.int32) - 1, 0), (B, 1))
    if kind == "shift_down":               # ... and a naive bottom-up copy
        return np.tile(np.minimum(np.arange(W, dtype=np.int32) + 1, W - 1), (B, 1))
    p = rng.integers(0, W, size=(B, W)).astype(np.int32)
    if kind == "random_dead":
        p[rng.random((B, W)) < 0.2] = -1
    return p


def _run(gr, oracle_lib, B, W, ND, Hkv, d, u, kind, seed=0):
    import torch
    rng = np.random.default_rng(seed)
    k = rng.integers(0, 65536, size=(B, W, ND, Hkv, d)).astype(np.uint16)
    v = rng.integers(0, 65536, size=(B, W, ND, Hkv, d)).astype(np.uint16)
    parent = _parents(rng, B, W, kind)
    dk, dv = bf16_to_dev(k), bf16_to_dev(v)
    gr.gr_beam_reorder(to_dev(parent), dk, dv, u)
    torch.cuda.synchronize()
    got_k = dk.view(torch.int16).cpu().numpy().view(np.uint16)
    got_v = dv.view(torch.int16).cpu().numpy().view(np.uint16)
    want_k = oracle_lib.unshared_reorder(k.copy(), parent)
    want_v = oracle_lib.unshared_reorder(v.copy(), parent)
    np.testing.assert_array_equal(got_k[:, :, :u], want_k[:, :, :u], err_msg=f"K {kind}")
    np.testing.assert_array_equal(got_v[:, :, :u], want_v[:, :, :u], err_msg=f"V {kind}")
    np.testing.assert_array_equal(got_k[:, :, u:], k[:, :, u:], err_msg=f"K slots >= u touched ({kind})")
    np.testing.assert_array_equal(got_v[:, :, u:], v[:, :, u:], err_msg=f"V slots >= u touched ({kind})")


@pytest.mark.parametrize("kind", ["identity", "reverse", "one", "shift_up", "shift_down", "random", "random_dead"])
def test_permutation_patterns(gr, oracle_lib, kind):
    _run(gr, oracle_lib, 3, 37, 3, 2, 64, 2, kind)            # ragged: 37 beams, partial last slice


@pytest.mark.parametrize("B,W,ND,Hkv,d,u", [
    (1, 16, 3, 8, 64, 3),          # tiny config geometry
    (8, 128, 3, 8, 128, 1),        # one pass of 128 beams
    (4, 256, 3, 8, 128, 3),        # benchmark geometry (fewer requests): two passes
    (2, 512, 3, 8, 128, 2),        # four passes
    (1, 2048, 2, 1, 8, 2),         # the widest supported beam, narrowest row (16 bytes per token)
    (2, 5, 4, 3, 24, 4),           # odd sizes: Hkv*d*2 = 144 bytes per token
])
def test_shapes(gr, oracle_lib, B, W, ND, Hkv, d, u):
    _run(gr, oracle_lib, B, W, ND, Hkv, d, u, "random_dead", seed=B * 1000 + W)


def test_u_zero_is_a_no_op_and_bad_shapes_are_rejected(gr, oracle_lib):
    import torch
    k = torch.zeros((1, 4, 3, 2, 8), dtype=torch.bfloat16, device="cuda:0")
    v = torch.ones_like(k)
    parent = torch.tensor([[3, 2, 1, 0]], dtype=torch.int32, device="cuda:0")
    gr.gr_beam_reorder(parent, k, v, 0)
    torch.cuda.synchronize()
    assert float(v.float().min()) == 1.0
    wide = torch.zeros((1, 2049, 1, 1, 8), dtype=torch.bfloat16, device="cuda:0")
    with pytest.raises(gr.GrError):
        gr.gr_beam_reorder(torch.zeros((1, 2049), dtype=torch.int32, device="cuda:0"), wide, wide.clone(), 1)


def test_decode_loop_is_self_consistent(gr, oracle_lib):
    """Three decode steps with select -> reorder -> append -> attention on the GPU equal the same loop
    on the oracle: the reorder is what makes each beam attend to its own ancestors' tokens."""
    import torch
    from gpu_util import run_attn, run_select
    cfg = gr_synth.get_config(1)
    B, W, ND, Hq, Hkv, d, V = cfg.B, cfg.W, cfg.ND, cfg.Hq, cfg.Hkv, cfg.d, cfg.V
    items = gr_synth.make_item_table(cfg)
    mask = gr.gr_item_mask_build(to_dev(items), V)
    sc, pf, rg = gr_synth.initial_beam_state(B, W, ND)
    scale = float(np.float32(1 / np.sqrt(d)))
    k_host = np.zeros((B, W, ND, Hkv, d), dtype=np.uint16)
    v_host = np.zeros_like(k_host)
    k_dev, v_dev = bf16_to_dev(k_host), bf16_to_dev(v_host)
    for s in range(ND):
        a = gr_synth.make_attention_inputs(cfg, s)
        # this step's new token for every beam goes to slot s of its (already reordered) cache
        k_host[:, :, s] = a["k_unshared"][:, :, s]
        v_host[:, :, s] = a["v_unshared"][:, :, s]
        k_dev[:, :, s] = bf16_to_dev(a["k_unshared"][:, :, s])
        v_dev[:, :, s] = bf16_to_dev(a["v_unshared"][:, :, s])
        a_gpu = dict(a, k_unshared=k_dev.view(torch.int16).cpu().numpy().view(np.uint16),
                     v_unshared=v_dev.view(torch.int16).cpu().numpy().view(np.uint16))
        out, _ = run_attn(gr, a_gpu, scale, want_lse=False)
        ref, _ = oracle_lib.attn_unified(a["q"], a["k_shared"], a["v_shared"], a["cu_seqlens"], k_host, v_host, s + 1, scale, None)
        assert np.abs(out.reshape(-1, d) - ref).max() <= 2e-2
        logits = gr_synth.make_logits(cfg, s)
        got = run_select(gr, mask, logits, sc, pf, rg, s)
        want = oracle_lib.beam_select(items, logits, sc, pf, s)
        np.testing.assert_array_equal(got["parent"], want["parent"])
        gr.gr_beam_reorder(to_dev(got["parent"]), k_dev, v_dev, s + 1)
        oracle_lib.unshared_reorder(k_host, want["parent"])
        oracle_lib.unshared_reorder(v_host, want["parent"])
        sc, pf, rg = want["scores"], want["prefix"], want["range"]
    torch.cuda.synchronize()
    np.testing.assert_array_equal(k_dev.view(torch.int16).cpu().numpy().view(np.uint16), k_host)
