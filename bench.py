#!/usr/bin/env python3
"""Benchmark of the generative-recommendation decode hot path on one MI355X.

A step = one decode step over the whole batch: gr_beam_attn (u = s+1 own tokens per beam) followed
by gr_beam_select at trie level s, for s cycling 0,1,2.  Inputs are synthetic (gr_synth), resident
in HBM before the timed region; the beam state fed to level s is the real state produced by levels
0..s-1.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 3] [--no-cpu-baseline]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0


def _stored_traffic(config_id):
    """HBM bytes per attention launch measured with rocprofv3 --pmc (FETCH_SIZE + WRITE_SIZE, scaled by a plain
    copy of known size); the figures and the commands that produced them are in profiles/attn_hbm_traffic.txt."""
    path = os.path.join(ROOT, "profiles", "attn_hbm_traffic.txt")
    try:
        for line in open(path):
            parts = line.split()
            if len(parts) >= 3 and parts[0] == "traffic_bytes_per_launch" and parts[1] == f"config{config_id}":
                return float(parts[2])
    except OSError:
        pass
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=60)
    ap.add_argument("--warmup", type=int, default=12)
    ap.add_argument("--config", type=int, default=3, help="workload id 1..5 (3 and 5 are the W=256 headline shapes)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-requests", type=int, default=0, help="requests timed on the CPU oracle (0 = auto)")
    ap.add_argument("--flags", type=int, default=0, help="GR_SELECT_* flags for the item step")
    ap.add_argument("--no-mask", action="store_true", help="unconstrained item step (mask = NULL)")
    ap.add_argument("--prewarm-ms", type=float, default=60.0,
                    help="untimed: run the step loop for this long before the W warm-up steps, so that the GPU's clock "
                         "management has settled (the first ~25 ms of sustained work after idle run ~20%% slower)")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the untimed extras reported beside the headline (cache reorder timing, whole-step HIP graph replay)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (known HBM traffic) so that rocprofv3 FETCH_SIZE / WRITE_SIZE "
                         "readings of the same run can be scaled")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; requests are independent and would shard across GPUs with no exchange, "
              "so --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import gr_synth
    import paper_2512_11529_amd as gr

    if not os.path.exists(gr.LIB_PATH):
        import __graft_entry__
        __graft_entry__.build()
    gr.load_library()          # raises if the HIP library is missing: there is no fallback path
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    cfg = gr_synth.get_config(args.config)
    B, W, V, ND, Hq, Hkv, d = cfg.B, cfg.W, cfg.V, cfg.ND, cfg.Hq, cfg.Hkv, cfg.d
    scale = float(np.float32(1.0 / np.sqrt(d)))

    def bf(a):
        return torch.from_numpy(a.view(np.int16)).to(dev).view(torch.bfloat16)

    # ---------------- inputs: generated on the host, uploaded once
    t_gen = time.time()
    items = gr_synth.make_item_table(cfg)
    cu = gr_synth.make_prompt_lengths(cfg)
    lens = np.diff(cu).astype(np.int64)
    max_L, total_L = int(lens.max()), int(cu[-1])
    kv_host = gr_synth.generate.make_kv_shared(cfg, cu)
    k_sh, v_sh = bf(kv_host[0]), bf(kv_host[1])
    d_cu = torch.from_numpy(cu).to(dev)
    attn_in, logits_host, logits = [], [], []
    for s in range(ND):
        a = gr_synth.make_attention_inputs(cfg, s, kv_shared=kv_host)
        attn_in.append(dict(q=bf(a["q"]), ku=bf(a["k_unshared"]), vu=bf(a["v_unshared"]), u=a["u"], host=a))
        lg = gr_synth.make_logits(cfg, s)
        logits_host.append(lg)
        logits.append(torch.from_numpy(lg).to(dev))
    mask = None if args.no_mask else gr.gr_item_mask_build(torch.from_numpy(items).to(dev), V)
    t_gen = time.time() - t_gen

    # ---------------- fixed buffers (nothing is allocated inside the timed region)
    out = torch.empty((B, W, Hq, d), dtype=torch.bfloat16, device=dev)
    ws_attn_bytes = gr.attn_workspace_bytes(B, W, Hq, Hkv, d, max_L)
    ws_attn = torch.empty(max(ws_attn_bytes, 256), dtype=torch.uint8, device=dev)
    ws_sel = torch.empty(gr.select_workspace_bytes(B, W, V, ND), dtype=torch.uint8, device=dev)
    sc0, pf0, rg0 = gr_synth.initial_beam_state(B, W, ND)
    state = [dict(scores=torch.from_numpy(sc0).to(dev), prefix=torch.from_numpy(pf0).to(dev), range=torch.from_numpy(rg0).to(dev))]
    mk = lambda: dict(parent=torch.empty((B, W), dtype=torch.int32, device=dev), token=torch.empty((B, W), dtype=torch.int32, device=dev),
                      scores=torch.empty((B, W), dtype=torch.float32, device=dev), prefix=torch.empty((B, W, ND), dtype=torch.int32, device=dev),
                      range=torch.empty((B, W, 2), dtype=torch.int32, device=dev), item_index=torch.empty((B, W), dtype=torch.int32, device=dev))
    sel_out = [mk() for _ in range(ND)]

    def attn(s):
        a = attn_in[s]
        gr.gr_beam_attn(a["q"], k_sh, v_sh, d_cu, a["ku"], a["vu"], a["u"], scale, max_L, total_L, out=out, workspace=ws_attn)

    def select(s):
        st = state[s]
        gr.gr_beam_select(mask, logits[s], st["scores"], st["prefix"], st["range"], s, flags=args.flags, out=sel_out[s], workspace=ws_sel)

    # real beam chain once: the state entering level s is what levels 0..s-1 selected
    for s in range(ND):
        select(s)
        state.append(dict(scores=sel_out[s]["scores"], prefix=sel_out[s]["prefix"], range=sel_out[s]["range"]))
    torch.cuda.synchronize()
    live_rows = [int((state[s]["scores"] > float("-inf")).sum().item()) for s in range(ND)]

    if args.calibrate_copy:
        src = torch.zeros(1 << 28, dtype=torch.float32, device=dev)      # 1 GiB
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ---------------- warm-up, then K timed steps
    prewarm_steps = 0
    t_pre = time.perf_counter()
    while (time.perf_counter() - t_pre) * 1e3 < args.prewarm_ms:
        for s in range(ND):
            attn(s); select(s)
        torch.cuda.synchronize()
        prewarm_steps += ND
    for i in range(args.warmup):
        attn(i % ND); select(i % ND)
    torch.cuda.synchronize()
    K = args.steps
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(K)]
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    e0.record()
    for i in range(K):
        s = i % ND
        ev[i][0].record()
        attn(s)
        ev[i][1].record()
        select(s)
        ev[i][2].record()
    e1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    total_ms = e0.elapsed_time(e1)
    attn_ms = [ev[i][0].elapsed_time(ev[i][1]) for i in range(K)]
    sel_ms = [ev[i][1].elapsed_time(ev[i][2]) for i in range(K)]
    ms_per_step = total_ms / K
    steps_per_s = 1000.0 / ms_per_step

    # ---------------- roofline of the dominant kernel (attention, bf16 MFMA)
    # algorithmic FLOPs per launch = 4 * W * Hq * d * sum_b (L_b + u)   (QK^T and PV, 2 flops per MAC)
    flops = [4.0 * W * Hq * d * float((lens + (s + 1)).sum()) for s in range(ND)]
    attn_flops_avg = float(np.mean([flops[i % ND] for i in range(K)]))
    attn_ms_avg = float(np.mean(attn_ms))
    attn_tflops = attn_flops_avg / (attn_ms_avg * 1e-3) / 1e12
    roofline = dict(bound="mfma", kernel="k_beam_attn", achieved=round(attn_tflops, 2), peak=PEAK_BF16_TFLOPS, unit="TFLOP/s",
                    frac=round(attn_tflops / PEAK_BF16_TFLOPS, 4), traffic=_stored_traffic(cfg.config_id),
                    avg_launch_ms=round(attn_ms_avg, 4), flops_per_launch=attn_flops_avg)
    # item step: algorithmic bytes of a dense pass = live rows * (4V logits + V/8 mask bits)
    sel_by_level = {}
    for s in range(ND):
        ms = [sel_ms[i] for i in range(K) if i % ND == s]
        if ms:
            dense_bytes = live_rows[s] * (4.0 * V + V / 8.0)
            sel_by_level[f"level{s}"] = dict(ms=round(float(np.mean(ms)), 4), live_rows=live_rows[s],
                                             dense_GBps=round(dense_bytes / (float(np.mean(ms)) * 1e-3) / 1e9, 1))

    # ---------------- extras, outside the headline's timed region
    reorder, graph = None, None
    if not args.no_extras:
        # (1) in-place move of the surviving beams' decode cache (gr_beam_reorder) with the parents each level selected
        ku_w, vu_w = attn_in[ND - 1]["ku"].clone(), attn_in[ND - 1]["vu"].clone()
        reorder = {}
        for s in range(ND):
            par = sel_out[s]["parent"]
            for _ in range(2):
                gr.gr_beam_reorder(par, ku_w, vu_w, s + 1)
            r0, r1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            reps = 10
            r0.record()
            for _ in range(reps):
                gr.gr_beam_reorder(par, ku_w, vu_w, s + 1)
            r1.record()
            torch.cuda.synchronize()
            ms = r0.elapsed_time(r1) / reps
            moved = 2.0 * 2.0 * B * W * (s + 1) * Hkv * d * 2          # K and V, read + write
            reorder[f"u{s + 1}"] = dict(ms=round(ms, 4), GBps=round(moved / (ms * 1e-3) / 1e9, 1))
        del ku_w, vu_w
        # (2) the ND-level cycle (attention + item step per level) captured once as a HIP graph and replayed
        try:
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                for s in range(ND):
                    attn(s); select(s)
            torch.cuda.current_stream().wait_stream(side)
            torch.cuda.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                for s in range(ND):
                    attn(s); select(s)
            ref = {k: sel_out[ND - 1][k].clone() for k in ("parent", "token", "scores")}
            t_pre = time.perf_counter()
            while (time.perf_counter() - t_pre) * 1e3 < max(args.prewarm_ms, 1.0):
                g.replay()
                torch.cuda.synchronize()
            cycles = max(1, K // ND)
            g0, g1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            g0.record()
            for _ in range(cycles):
                g.replay()
            g1.record()
            torch.cuda.synchronize()
            gms = g0.elapsed_time(g1) / (cycles * ND)
            same = all(bool(torch.equal(ref[k], sel_out[ND - 1][k])) for k in ref)
            graph = dict(ms_per_step=round(gms, 4), steps_per_s=round(1000.0 / gms, 3), cycles=cycles, replay_matches_eager=same)
        except Exception as e:          # the headline above stands on its own
            graph = dict(error=f"{type(e).__name__}: {e}"[:300])

    # ---------------- CPU oracle on a bounded sample of the same workload
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        oracle.build()
        nb = args.cpu_sample_requests or max(1, min(B, {1: 1, 2: 8, 3: 8, 4: 1, 5: 8}.get(cfg.config_id, 1)))
        t_cpu = time.perf_counter()
        sc, pf, _ = gr_synth.initial_beam_state(nb, W, ND)
        n_steps_cpu = 1 if cfg.config_id == 4 else ND      # the long-prompt shape: one step is already ~20 s
        for s in range(n_steps_cpu):
            a = attn_in[s]["host"]
            bb, ww, hh = np.meshgrid(np.arange(nb), np.arange(W), np.arange(Hq), indexing="ij")
            tri = np.stack([bb.ravel(), ww.ravel(), hh.ravel()], axis=1).astype(np.int32)
            oracle.attn_unified(a["q"], a["k_shared"], a["v_shared"], a["cu_seqlens"], a["k_unshared"], a["v_unshared"], a["u"], scale, tri)
            r = oracle.beam_select(None if args.no_mask else items, np.ascontiguousarray(logits_host[s][:nb]), sc, pf, s)
            sc, pf = r["scores"], r["prefix"]
        t_cpu = time.perf_counter() - t_cpu
        cpu_steps_per_s = (n_steps_cpu * nb / B) / t_cpu
        cpu = dict(value=round(cpu_steps_per_s, 6), unit="steps/s", cores=oracle.num_threads(), kind="oracle",
                   sample=f"requests 0..{nb - 1} of {B}, {n_steps_cpu} decode step(s), all beams and heads; "
                          f"{t_cpu:.1f} s; scaled by {nb}/{B} (requests are independent)",
                   seconds=round(t_cpu, 2))

    line = dict(
        metric="beam decode steps/s (attn+mask+top-W)", value=round(steps_per_s, 3), unit="steps/s", n_gpus=1, steps=K,
        warmup=args.warmup, ms_per_step=round(ms_per_step, 4), higher_is_better=True, scaling="weak", vs_baseline=None,
        dtype="bf16", data="synthetic",
        config=dict(workload=f"config{cfg.config_id}:{cfg.name}", B=B, W=W, V=V, L=(cfg.L_min if cfg.L_min == cfg.L_max else f"U[{cfg.L_min},{cfg.L_max}]"),
                    total_L=total_L, Hq=Hq, Hkv=Hkv, d=d, decode_steps=ND, n_items=cfg.n_items, mask=(not args.no_mask), flags=args.flags,
                    step_definition="one gr_beam_attn + one gr_beam_select over the whole batch; levels cycle 0,1,2"),
        request_steps_per_s=round(steps_per_s * B, 1),
        roofline=roofline, cpu_baseline=cpu,
        attn=dict(ms_by_u={f"u{s + 1}": round(float(np.mean([attn_ms[i] for i in range(K) if i % ND == s] or [0])), 4) for s in range(ND)},
                  tflops=round(attn_tflops, 2)),
        select=sel_by_level, reorder=reorder, graph=graph, prewarm=dict(ms=args.prewarm_ms, steps=prewarm_steps), wall_s=round(wall, 3), input_gen_s=round(t_gen, 1))
    print(json.dumps(line))


if __name__ == "__main__":
    main()
