"""GPU: the unshared cache followed through a slot table instead of being moved (Section 5.1's hand-over of the
per-beam cache between decode steps, with no cache bytes moved).

The oracle side keeps a LOGICAL cache per beam, reordered by the plain gather definition (oracle unshared_reorder)
and extended by each beam's new token; the GPU side keeps the rows where they were written and updates the table with
gr_beam_slot_update.  After every step gr_beam_attn_slots must give the oracle's attention over the logical cache
(max-abs <= 2e-2) and, bit for bit on live beams, what gr_beam_attn gives on a cache moved by gr_beam_reorder."""
import numpy as np
import pytest

import gr_synth
from gpu_util import bf16_to_dev, rand_attn_case, to_dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gr():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_2512_11529_amd as gr
    gr.load_library()
    return gr


def _random_parents(rng, B, W, live, n_dead):
    """Parents drawn from the live beams of the previous generation (repeats allowed, unsorted); the last n_dead
    slots of every request are dead (-1)."""
    parent = np.full((B, W), -1, dtype=np.int32)
    for b in range(B):
        cand = np.flatnonzero(live[b])
        parent[b, :W - n_dead] = rng.choice(cand, size=W - n_dead, replace=True)
    return parent


def test_slot_update_is_the_gather_of_the_parents_rows(gr):
    import torch
    rng = np.random.default_rng(7)
    B, W, ND = 3, 70, 3
    live = np.ones((B, W), dtype=bool)
    want = (np.arange(W)[:, None] * ND + np.arange(ND)[None, :]).astype(np.int32)[None].repeat(B, 0)   # identity
    slot = None
    for u in range(1, ND + 1):
        parent = _random_parents(rng, B, W, live, n_dead=u * 3)
        got = gr.gr_beam_slot_update(to_dev(parent), slot, u, ND)
        torch.cuda.synchronize()
        new = (np.arange(W)[:, None] * ND + np.arange(ND)[None, :]).astype(np.int32)[None].repeat(B, 0)
        for b in range(B):
            for j in range(W):
                if parent[b, j] >= 0:
                    new[b, j, :u] = want[b, parent[b, j], :u]
        np.testing.assert_array_equal(got.cpu().numpy(), new, err_msg=f"u={u}")
        want, slot, live = new, got, parent >= 0
    # u = 0: nothing is shared yet, every beam owns its rows
    got0 = gr.gr_beam_slot_update(to_dev(parent), slot, 0, ND)
    ident = (np.arange(W)[:, None] * ND + np.arange(ND)[None, :]).astype(np.int32)[None].repeat(B, 0)
    np.testing.assert_array_equal(got0.cpu().numpy(), ident)


@pytest.mark.parametrize("B,W,Hq,Hkv,d,lens", [
    (2, 20, 8, 2, 128, (130, 64)),        # g = 4: eight beams per wave
    (1, 40, 4, 4, 64, (100,)),            # g = 1, d = 64: 32 beams x 3 own tokens per wave, three mini-tiles
    (1, 30, 6, 2, 64, (70,)),             # g = 3: beams straddle wave boundaries
    (2, 70, 8, 2, 128, (0, 300)),         # several row blocks; one request with no prompt at all
])
def test_attention_through_slots_over_three_steps(gr, oracle_lib, B, W, Hq, Hkv, d, lens):
    import torch
    ND = 3
    rng = np.random.default_rng(B * 1000 + W)
    scale = float(np.float32(1 / np.sqrt(d)))
    a = rand_attn_case(B * 31 + W, B, W, Hq, Hkv, d, ND, ND, lens)
    cu = a["cu_seqlens"]
    max_L, total_L = int(np.diff(cu).max()), int(cu[-1])
    ks, vs, d_cu = bf16_to_dev(a["k_shared"]), bf16_to_dev(a["v_shared"]), to_dev(cu)
    # physical rows: beam j writes the K/V of its token t to row (j, t), once
    phys_k, phys_v = a["k_unshared"], a["v_unshared"]
    d_pk, d_pv = bf16_to_dev(phys_k), bf16_to_dev(phys_v)
    # the moved copy (the paper's procedure) and the oracle's logical cache start with token 0 in place
    d_ck, d_cv = d_pk.clone(), d_pv.clone()
    log_k, log_v = phys_k.copy(), phys_v.copy()
    slot = None
    live = np.ones((B, W), dtype=bool)
    for s in range(ND):
        u = s + 1
        if s > 0:
            parent = _random_parents(rng, B, W, live, n_dead=2 * s)
            d_parent = to_dev(parent)
            slot = gr.gr_beam_slot_update(d_parent, slot, s, ND)
            gr.gr_beam_reorder(d_parent, d_ck, d_cv, s)
            d_ck[:, :, s] = d_pk[:, :, s]                  # every beam's new token goes to its own row
            d_cv[:, :, s] = d_pv[:, :, s]
            oracle_lib.unshared_reorder(log_k, parent)
            oracle_lib.unshared_reorder(log_v, parent)
            log_k[:, :, s:] = phys_k[:, :, s:]
            log_v[:, :, s:] = phys_v[:, :, s:]
            live = parent >= 0
        q = gr_synth.f32_to_bf16_bits(rng.standard_normal((B, W, Hq, d), dtype=np.float32))
        d_q = bf16_to_dev(q)
        if slot is None:
            slot = gr.gr_beam_slot_update(to_dev(np.zeros((B, W), dtype=np.int32)), None, 0, ND)      # the identity table
        out_s, _ = gr.gr_beam_attn_slots(d_q, ks, vs, d_cu, d_pk, d_pv, slot, u, scale, max_L, total_L)
        out_c, _ = gr.gr_beam_attn(d_q, ks, vs, d_cu, d_ck, d_cv, u, scale, max_L, total_L)
        torch.cuda.synchronize()
        ref, _ = oracle_lib.attn_unified(q, a["k_shared"], a["v_shared"], cu, log_k, log_v, u, scale)
        ref = ref.reshape(B, W, Hq, d)
        got = out_s.float().cpu().numpy()
        err = np.abs(got[live] - ref[live]).max()
        assert err <= 2e-2, f"step {s}: slots vs oracle max-abs {err}"
        assert torch.equal(out_s[to_dev(live)], out_c[to_dev(live)]), f"step {s}: slots and moved cache differ"


def test_entries_outside_the_block_read_the_beams_own_row(gr):
    import torch
    B, W, Hq, Hkv, d, ND = 1, 12, 4, 2, 128, 3
    a = rand_attn_case(99, B, W, Hq, Hkv, d, ND, 2, (90,))
    cu = a["cu_seqlens"]
    args = (bf16_to_dev(a["q"]), bf16_to_dev(a["k_shared"]), bf16_to_dev(a["v_shared"]), to_dev(cu),
            bf16_to_dev(a["k_unshared"]), bf16_to_dev(a["v_unshared"]))
    ident = (np.arange(W)[:, None] * ND + np.arange(ND)[None, :]).astype(np.int32)[None]
    bad = ident.copy()
    bad[0, 3, 0] = -5
    bad[0, 7, 1] = W * ND
    bad[0, 9, 0] = 2 ** 30
    scale = float(np.float32(1 / np.sqrt(d)))
    want, _ = gr.gr_beam_attn(*args, 2, scale, 90, 90)
    got_i, _ = gr.gr_beam_attn_slots(*args, to_dev(ident), 2, scale, 90, 90)
    got_b, _ = gr.gr_beam_attn_slots(*args, to_dev(bad), 2, scale, 90, 90)
    torch.cuda.synchronize()
    assert torch.equal(got_i, want) and torch.equal(got_b, want)


def test_argument_errors(gr):
    import ctypes
    import torch
    lib = gr.load_library()                                  # GR_ERR_INVALID_ARG = -1
    t = torch.zeros(64, dtype=torch.int32, device="cuda:0")
    p = ctypes.c_void_p(t.data_ptr())
    assert lib.gr_beam_slot_update(2, 4, 3, 1, p, p, p, None) == -1          # slot_in aliases slot_out
    assert lib.gr_beam_slot_update(2, 4, 3, 4, p, None, p, None) == -1       # u > ND
    assert lib.gr_beam_slot_update(2, 4, 3, 1, None, None, p, None) == -1    # parent missing
    assert lib.gr_beam_attn_slots(None, p, None, 0, None) == -1
    torch.cuda.synchronize()


def test_slot_cycle_as_a_graph_replays_to_the_eager_result(gr):
    """Attention through the table, then the table's update, captured once and replayed with eager work in between."""
    import torch
    B, W, Hq, Hkv, d, ND = 2, 24, 8, 2, 128, 3
    rng = np.random.default_rng(5)
    a = rand_attn_case(17, B, W, Hq, Hkv, d, ND, ND, (200, 77))
    cu = a["cu_seqlens"]
    scale = float(np.float32(1 / np.sqrt(d)))
    q, ks, vs, d_cu = bf16_to_dev(a["q"]), bf16_to_dev(a["k_shared"]), bf16_to_dev(a["v_shared"]), to_dev(cu)
    pk, pv = bf16_to_dev(a["k_unshared"]), bf16_to_dev(a["v_unshared"])
    live = np.ones((B, W), dtype=bool)
    parents = []
    for s in range(1, ND):
        parents.append(_random_parents(rng, B, W, live, n_dead=s))
        live = parents[-1] >= 0
    d_par = [to_dev(p) for p in parents]
    zero_parent = to_dev(np.zeros((B, W), dtype=np.int32))
    slots = [torch.empty((B, W, ND), dtype=torch.int32, device="cuda:0") for _ in range(2)]
    outs = [torch.empty((B, W, Hq, d), dtype=torch.bfloat16, device="cuda:0") for _ in range(ND)]
    ws = torch.empty(max(gr.attn_workspace_bytes(B, W, Hq, Hkv, d, 200), 256), dtype=torch.uint8, device="cuda:0")

    def cycle():
        gr.gr_beam_slot_update(zero_parent, None, 0, ND, out=slots[0])
        for s in range(ND):
            gr.gr_beam_attn_slots(q, ks, vs, d_cu, pk, pv, slots[s & 1], s + 1, scale, 200, 277, out=outs[s], workspace=ws)
            if s + 1 < ND:
                gr.gr_beam_slot_update(d_par[s], slots[s & 1], s + 1, ND, out=slots[(s + 1) & 1])

    cycle()
    torch.cuda.synchronize()
    want = [o.clone() for o in outs]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        cycle()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        cycle()
    for rep in range(3):
        for o in outs:
            o.zero_()
        for t in slots:
            t.fill_(-7)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for s in range(ND):
            assert torch.equal(outs[s], want[s]), f"replay {rep}, step {s}"
