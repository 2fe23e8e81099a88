"""GPU: one decode step (attention -> item step -> cache reorder) captured as a HIP graph replays to
the oracle's results (attention within 2e-2, beams and the reordered cache bit-exact) and to the eager
step's, on every replay.  The entry points only enqueue kernels on the caller's stream (no allocation,
no synchronisation, no memset nodes), which is what makes the step capturable as a whole."""
import numpy as np
import pytest

import gr_synth
from gpu_util import bf16_to_dev, to_dev

pytestmark = pytest.mark.gpu


def test_step_graph_replays_match_oracle_and_eager(oracle_lib):
    import torch
    import paper_2512_11529_amd as gr
    gr.load_library()
    cfg = gr_synth.get_config(1)
    B, W, ND, Hq, Hkv, d, V = cfg.B, cfg.W, cfg.ND, cfg.Hq, cfg.Hkv, cfg.d, cfg.V
    dev = torch.device("cuda:0")
    items = gr_synth.make_item_table(cfg)
    mask = gr.gr_item_mask_build(to_dev(items), V)
    a = gr_synth.make_attention_inputs(cfg, 1)
    cu = a["cu_seqlens"]
    q, ks, vs = bf16_to_dev(a["q"]), bf16_to_dev(a["k_shared"]), bf16_to_dev(a["v_shared"])
    ku0, vu0 = bf16_to_dev(a["k_unshared"]), bf16_to_dev(a["v_unshared"])
    ku, vu = ku0.clone(), vu0.clone()
    d_cu = to_dev(cu)
    scale = float(np.float32(1 / np.sqrt(d)))
    max_L, total_L = int(np.diff(cu).max()), int(cu[-1])
    out = torch.empty_like(q)
    ws_attn = torch.empty(max(gr.attn_workspace_bytes(B, W, Hq, Hkv, d, max_L), 256), dtype=torch.uint8, device=dev)
    ws_sel = torch.empty(gr.select_workspace_bytes(B, W, V, ND), dtype=torch.uint8, device=dev)
    sc, pf, rg = gr_synth.initial_beam_state(B, W, ND)
    # a level-1 state to select from: run level 0 eagerly first
    logits0, logits1 = to_dev(gr_synth.make_logits(cfg, 0)), to_dev(gr_synth.make_logits(cfg, 1))
    st0 = gr.gr_beam_select(mask, logits0, to_dev(sc), to_dev(pf), to_dev(rg), 0)
    sel = {k: torch.empty_like(v) for k, v in st0.items()}

    def step():
        gr.gr_beam_attn(q, ks, vs, d_cu, ku, vu, 2, scale, max_L, total_L, out=out, workspace=ws_attn)
        gr.gr_beam_select(mask, logits1, st0["scores"], st0["prefix"], st0["range"], 1, out=sel, workspace=ws_sel)
        gr.gr_beam_reorder(sel["parent"], ku, vu, 2)

    step()
    torch.cuda.synchronize()
    want = dict(out=out.clone(), ku=ku.clone(), vu=vu.clone(), **{k: v.clone() for k, v in sel.items()})

    # what the oracle says the step must produce
    ref_out, _ = oracle_lib.attn_unified(a["q"], a["k_shared"], a["v_shared"], cu, a["k_unshared"], a["v_unshared"], 2, scale)
    ref_out = ref_out.reshape(B, W, Hq, d)
    st0_host = {k: v.cpu().numpy() for k, v in st0.items()}
    ref_sel = oracle_lib.beam_select(items, gr_synth.make_logits(cfg, 1), st0_host["scores"], st0_host["prefix"], 1)
    ref_ku = oracle_lib.unshared_reorder(a["k_unshared"].copy(), ref_sel["parent"])
    ref_vu = oracle_lib.unshared_reorder(a["v_unshared"].copy(), ref_sel["parent"])

    def check_against_oracle(got, what):
        err = np.abs(got["out"].float().cpu().numpy() - ref_out).max()
        assert err <= 2e-2, f"{what}: attention max-abs {err}"
        for k in ("parent", "token", "prefix", "range", "item_index"):
            np.testing.assert_array_equal(got[k].cpu().numpy(), ref_sel[k], err_msg=f"{what}: {k}")
        np.testing.assert_allclose(got["scores"].cpu().numpy(), ref_sel["scores"], rtol=1e-5, atol=0, err_msg=f"{what}: scores")
        for name, ref in (("ku", ref_ku), ("vu", ref_vu)):
            bits = got[name].view(torch.int16).cpu().numpy().view(np.uint16)
            np.testing.assert_array_equal(bits[:, :, :2], ref[:, :, :2], err_msg=f"{what}: reordered {name}")

    check_against_oracle(want, "eager step")

    def reset():
        ku.copy_(ku0); vu.copy_(vu0); out.zero_()
        for v in sel.values():
            v.zero_()

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        reset(); step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    reset()
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step()
    for rep in range(3):
        reset()                                  # eager work and a synchronisation between replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        got = dict(out=out, ku=ku, vu=vu, **sel)
        check_against_oracle(got, f"replay {rep}")
        for k in want:
            assert torch.equal(got[k], want[k]), f"replay {rep}: {k} differs from the eager step"


def test_two_batches_on_two_streams_match_oracle(oracle_lib):
    """Two independent batches, one stream each (equal priority), enqueued alternately so that their kernels
    overlap on the GPU; each batch owns its inputs, outputs and workspaces.  Both must come out as the oracle says:
    batch A runs the level-1 step (u = 2), batch B the level-2 step (u = 3) of the same request."""
    import torch
    import paper_2512_11529_amd as gr
    gr.load_library()
    cfg = gr_synth.get_config(1)
    B, W, ND, Hq, Hkv, d, V = cfg.B, cfg.W, cfg.ND, cfg.Hq, cfg.Hkv, cfg.d, cfg.V
    dev = torch.device("cuda:0")
    items = gr_synth.make_item_table(cfg)
    mask = gr.gr_item_mask_build(to_dev(items), V)
    scale = float(np.float32(1 / np.sqrt(d)))
    sc, pf, rg = gr_synth.initial_beam_state(B, W, ND)
    logits = [gr_synth.make_logits(cfg, s) for s in range(ND)]
    # beam states entering levels 1 and 2 (from the oracle: the batches' inputs do not depend on the code under test)
    states = [dict(scores=sc, prefix=pf, range=rg)]
    for s in range(2):
        r = oracle_lib.beam_select(items, logits[s], states[s]["scores"], states[s]["prefix"], s)
        states.append(dict(scores=r["scores"], prefix=r["prefix"], range=r["range"]))
    torch.cuda.synchronize()

    batches = []
    for level in (1, 2):
        a = gr_synth.make_attention_inputs(cfg, level)
        cu = a["cu_seqlens"]
        max_L, total_L = int(np.diff(cu).max()), int(cu[-1])
        st = states[level]
        bt = dict(level=level, a=a, u=level + 1, max_L=max_L, total_L=total_L, stream=torch.cuda.Stream(),
                  q=bf16_to_dev(a["q"]), ks=bf16_to_dev(a["k_shared"]), vs=bf16_to_dev(a["v_shared"]), cu=to_dev(cu),
                  ku0=bf16_to_dev(a["k_unshared"]), vu0=bf16_to_dev(a["v_unshared"]),
                  logits=to_dev(logits[level]), sc=to_dev(st["scores"]), pf=to_dev(st["prefix"]), rg=to_dev(st["range"]),
                  ws_attn=torch.empty(max(gr.attn_workspace_bytes(B, W, Hq, Hkv, d, max_L), 256), dtype=torch.uint8, device=dev),
                  ws_sel=torch.empty(gr.select_workspace_bytes(B, W, V, ND), dtype=torch.uint8, device=dev))
        bt["ku"], bt["vu"] = bt["ku0"].clone(), bt["vu0"].clone()
        bt["out"] = torch.empty_like(bt["q"])
        bt["sel"] = dict(parent=torch.empty((B, W), dtype=torch.int32, device=dev), token=torch.empty((B, W), dtype=torch.int32, device=dev),
                         scores=torch.empty((B, W), dtype=torch.float32, device=dev), prefix=torch.empty((B, W, ND), dtype=torch.int32, device=dev),
                         range=torch.empty((B, W, 2), dtype=torch.int32, device=dev), item_index=torch.empty((B, W), dtype=torch.int32, device=dev))
        batches.append(bt)
    torch.cuda.synchronize()

    def enqueue(bt):
        s = bt["stream"]
        with torch.cuda.stream(s):
            bt["ku"].copy_(bt["ku0"]); bt["vu"].copy_(bt["vu0"])
        gr.gr_beam_attn(bt["q"], bt["ks"], bt["vs"], bt["cu"], bt["ku"], bt["vu"], bt["u"], scale, bt["max_L"], bt["total_L"],
                        out=bt["out"], workspace=bt["ws_attn"], stream=s)
        gr.gr_beam_select(mask, bt["logits"], bt["sc"], bt["pf"], bt["rg"], bt["level"], out=bt["sel"], workspace=bt["ws_sel"], stream=s)
        gr.gr_beam_reorder(bt["sel"]["parent"], bt["ku"], bt["vu"], bt["u"], stream=s)

    for _ in range(8):                     # alternate, no synchronisation in between: the two streams run concurrently
        for bt in batches:
            enqueue(bt)
    torch.cuda.synchronize()

    for bt in batches:
        a, level, u = bt["a"], bt["level"], bt["u"]
        ref_out, _ = oracle_lib.attn_unified(a["q"], a["k_shared"], a["v_shared"], a["cu_seqlens"], a["k_unshared"], a["v_unshared"], u, scale)
        err = np.abs(bt["out"].float().cpu().numpy() - ref_out.reshape(B, W, Hq, d)).max()
        assert err <= 2e-2, f"level {level}: attention max-abs {err}"
        st = states[level]
        ref = oracle_lib.beam_select(items, logits[level], st["scores"], st["prefix"], level)
        for k in ("parent", "token", "prefix", "range", "item_index"):
            np.testing.assert_array_equal(bt["sel"][k].cpu().numpy(), ref[k], err_msg=f"level {level}: {k}")
        np.testing.assert_allclose(bt["sel"]["scores"].cpu().numpy(), ref["scores"], rtol=1e-5, atol=0)
        for name, src in (("ku", a["k_unshared"]), ("vu", a["v_unshared"])):
            want = oracle_lib.unshared_reorder(src.copy(), ref["parent"])
            bits = bt[name].view(torch.int16).cpu().numpy().view(np.uint16)
            np.testing.assert_array_equal(bits[:, :, :u], want[:, :, :u], err_msg=f"level {level}: reordered {name}")
