#!/usr/bin/env python3
"""Benchmark of the generative-recommendation decode hot path on one MI355X.

A step = one decode step over the whole batch: gr_beam_attn (u = s+1 own tokens per beam) followed
by gr_beam_select at trie level s, for s cycling 0,1,2.  Inputs are synthetic (gr_synth), resident
in HBM before the timed region; the beam state fed to level s is the real state produced by levels
0..s-1.  Prints ONE JSON line: the headline (steps/s), `roofline` (attention, bf16 MFMA), `roofline_select`
(item step on its dense paths, HBM), `cpu_baseline` (the oracle on the host cores), and extras measured
outside the headline's timed region (cache reorder, whole-step HIP graph, two batches on two streams,
measured machine peaks).

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 3] [--no-cpu-baseline]
    python bench.py --sweep-attn-plan        # the (B, L, W) x (row tile, L segments) table the launch rule is fitted to
    python bench.py --issue-test             # how much VALU work hides behind MFMAs on this chip (attention roofline discussion)
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


def _elapsed(torch, fn, reps):
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / reps


def measured_peaks(torch, gr, dev):
    """What this GPU sustains: a plain streaming read of 1 GiB and back-to-back bf16 MFMAs on N(0,1) operands."""
    sink = torch.zeros(4, dtype=torch.float32, device=dev)
    src = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
    src.view(torch.float32).normal_()
    for _ in range(20):
        gr.gr_diag_stream_read(src, sink)
    ms = _elapsed(torch, lambda: gr.gr_diag_stream_read(src, sink), 20)
    read_gbs = src.numel() / (ms * 1e-3) / 1e9
    del src
    ops = torch.randn(8192, dtype=torch.float32, device=dev).to(torch.bfloat16)          # 16 KiB of bf16 N(0,1)
    wgs, iters = 256 * 4, 4096
    flops = 0.0
    for _ in range(10):
        flops = gr.gr_diag_mfma_loop(ops, wgs, iters, sink)
    ms = _elapsed(torch, lambda: gr.gr_diag_mfma_loop(ops, wgs, iters, sink), 10)
    return dict(hbm_read_GBps=round(read_gbs, 1), bf16_mfma_TFLOPs=round(flops / (ms * 1e-3) / 1e12, 1),
                how="plain 16-byte-load read of 1 GiB; 1024 workgroups x 8 waves of back-to-back 32x32x16 bf16 MFMAs on N(0,1) operands, both after the clock has settled")


def summarize_trace(path):
    """Mean kernel duration per decode level over the last 60 steps of a rocprofv3 kernel-trace CSV of this benchmark
    (run with --no-extras: the trace then ends with the timed steps, each = k_beam_attn, k_rows, k_select)."""
    import collections
    import csv
    rows = [r for r in csv.DictReader(open(path)) if any(k in r["Kernel_Name"] for k in ("k_rows", "k_select", "k_beam_attn"))]
    rows.sort(key=lambda r: int(r["Start_Timestamp"]))
    seq = [("k_rows" if "k_rows" in r["Kernel_Name"] else "k_select" if "k_select" in r["Kernel_Name"] else "k_beam_attn",
            int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) for r in rows][-180:]
    acc = collections.defaultdict(list)
    for i in range(0, len(seq) - 2, 3):
        trio = seq[i:i + 3]
        if [t[0] for t in trio] != ["k_beam_attn", "k_rows", "k_select"]:
            raise SystemExit(f"unexpected kernel order at {i}: {trio}")
        for name, dur in trio:
            acc[((i // 3) % 3, name)].append(dur)
    for name in ("k_beam_attn", "k_rows", "k_select"):
        print(f"{name:12s} " + "   ".join(f"level{lvl} {sum(acc[(lvl, name)]) / max(len(acc[(lvl, name)]), 1) / 1e3:7.1f} us" for lvl in range(3)))


def issue_test(torch, gr, dev, sigma=0.01):
    """How much vector work hides behind matrix instructions on one SIMD: time per slot of { MFMA, n FMA, m exp } per wave,
    for two and four waves per SIMD (nanoseconds per slot and SIMD; the MFMA-only row is the matrix pipe's own rate)."""
    sink = torch.zeros(4, dtype=torch.float32, device=dev)
    ops = (torch.randn(8192, dtype=torch.float32, device=dev) * sigma).to(torch.bfloat16)
    iters = 2048
    combos = [(1, 0, 0), (1, 2, 0), (1, 4, 0), (1, 8, 0), (1, 12, 0), (1, 0, 1), (1, 2, 1), (1, 3, 1), (1, 4, 1), (1, 4, 2),
              (0, 4, 0), (0, 12, 0), (0, 0, 1), (0, 0, 4), (0, 4, 1)]
    print(f"operands N(0, {sigma}^2) bf16")
    print("mfma n_fma n_exp | ns per slot and SIMD: 2 waves/SIMD  4 waves/SIMD")
    for mf, nv, nx in combos:
        cells = []
        for wgs in (256, 512):
            run = lambda: gr.gr_diag_issue_loop(ops, wgs, iters, nv, nx, mf, sink)
            for _ in range(3):
                run()
            ms = _elapsed(torch, run, 5)
            slots = wgs * 8 / 1024 * iters * 4
            cells.append(f"{ms * 1e6 / slots:6.1f}")
        print(f"{mf:4d} {nv:5d} {nx:5d} | {cells[0]}  {cells[1]}", flush=True)
    # the MFMA's first operand from LDS (one conflict-free ds_read_b128 per wave and read), as in the attention loop
    print("with the MFMA's A operand read from LDS every k-th slot (0 = from registers); two waves per SIMD")
    print("n_fma n_exp | every 0   every 2   every 1")
    rounds = 680
    for nv, nx, evs in ((0, 0, (0, 2, 1)), (3, 1, (0, 2, 1)), (5, 0, (0, None, 1)), (0, 2, (0, None, 1))):
        cells = []
        for ev in evs:
            if ev is None:
                cells.append("     -")
                continue
            run = lambda: gr.gr_diag_issue_loop_lds(ops, 256, rounds, nv, nx, ev, sink)
            for _ in range(3):
                run()
            ms = _elapsed(torch, run, 5)
            cells.append(f"{ms * 1e6 / (256 * 8 / 1024 * rounds * 12):6.1f}")
        print(f"{nv:5d} {nx:5d} | " + "    ".join(cells), flush=True)


def sweep_attn_plan(torch, gr, dev):
    """Attention time (u = 2) for every row tile and L split the kernel has, on the shapes the launch rule was fitted to.
    gr_diag_attn_plan(rows, segments) overrides the rule; the workspace is sized by the binding for whichever plan is in force."""
    import numpy as np
    import gr_synth
    shapes = [(8, 2048, 128), (4, 16384, 512), (1, 4096, 256), (2, 8192, 256), (16, 1024, 256), (4, 2048, 512), (64, 512, 128), (32, 4096, 256)]
    Hq, Hkv, d, ND = 32, 8, 128, 3
    scale = float(np.float32(1 / np.sqrt(d)))
    print("B, L, W | rule us | " + " ".join(f"{r}x{n}" for r in (128, 256) for n in (1, 2, 4, 8, 16)))
    for B, L, W in shapes:
        q = torch.randn((B, W, Hq, d), device=dev).to(torch.bfloat16)
        ks = torch.randn((B * L, Hkv, d), device=dev).to(torch.bfloat16)
        vs = torch.randn((B * L, Hkv, d), device=dev).to(torch.bfloat16)
        ku = torch.randn((B, W, ND, Hkv, d), device=dev).to(torch.bfloat16)
        vu = torch.randn((B, W, ND, Hkv, d), device=dev).to(torch.bfloat16)
        cu = torch.arange(0, (B + 1) * L, L, dtype=torch.int32, device=dev)
        out = torch.empty_like(q)

        def run():
            gr.gr_beam_attn(q, ks, vs, cu, ku, vu, 2, scale, L, B * L, out=out)

        def timed():
            for _ in range(5):
                run()
            return _elapsed(torch, run, 10) * 1e3
        gr.gr_diag_attn_plan(0, 0)
        t_pre = time.perf_counter()
        while time.perf_counter() - t_pre < 0.06:        # let the clock settle under this shape's load before the first column
            run()
            torch.cuda.synchronize()
        cells = [f"{timed():.0f}"]
        for rows in (128, 256):
            for nseg in (1, 2, 4, 8, 16):
                gr.gr_diag_attn_plan(rows, nseg)
                try:
                    cells.append(f"{timed():.0f}")
                except gr.GrError:
                    cells.append("-")
        gr.gr_diag_attn_plan(0, 0)
        print(f"{B}, {L}, {W} | " + " | ".join([cells[0], " ".join(cells[1:])]), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=60)
    ap.add_argument("--warmup", type=int, default=12)
    ap.add_argument("--config", type=int, default=3, help="workload id 1..5 (3 and 5 are the W=256 headline shapes)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-requests", type=int, default=0, help="requests timed on the CPU oracle (0 = auto)")
    ap.add_argument("--flags", type=int, default=0, help="GR_SELECT_* flags for the item step of the headline")
    ap.add_argument("--no-mask", action="store_true", help="unconstrained item step (mask = NULL) in the headline")
    ap.add_argument("--prewarm-ms", type=float, default=60.0,
                    help="untimed: run the step loop for this long before the W warm-up steps, so that the GPU's clock "
                         "management has settled (the first ~25 ms of sustained work after idle run ~20%% slower)")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip everything measured outside the headline's timed region (dense-path item step, cache reorder, "
                         "HIP graph, two streams, measured peaks)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (known HBM traffic) so that rocprofv3 FETCH_SIZE / WRITE_SIZE "
                         "readings of the same run can be scaled")
    ap.add_argument("--layers", type=int, default=4, help="attention calls per decode step in the per-layer extra leg")
    ap.add_argument("--sweep-attn-plan", action="store_true", help="print the launch-plan sweep table and exit")
    ap.add_argument("--issue-test", action="store_true", help="print the MFMA / VALU issue test table and exit")
    ap.add_argument("--issue-sigma", type=float, default=0.01, help="standard deviation of the issue test's MFMA operands")
    ap.add_argument("--summarize-trace", metavar="CSV", help="per-level kernel means from a rocprofv3 kernel-trace CSV of this benchmark "
                                                              "(made with --kernel-trace --output-format csv ... --no-extras), then exit; needs no GPU")
    args = ap.parse_args()
    if args.summarize_trace:
        summarize_trace(args.summarize_trace)
        return
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
    if args.sweep_attn_plan:
        sweep_attn_plan(torch, gr, dev)
        return
    if args.issue_test:
        issue_test(torch, gr, dev, args.issue_sigma)
        return
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
    mask_blob = gr.gr_item_mask_build(torch.from_numpy(items).to(dev), V)
    mask = None if args.no_mask else mask_blob
    t_gen = time.time() - t_gen

    # ---------------- fixed buffers (nothing is allocated inside the timed region)
    def make_buffers():
        mk = lambda: dict(parent=torch.empty((B, W), dtype=torch.int32, device=dev), token=torch.empty((B, W), dtype=torch.int32, device=dev),
                          scores=torch.empty((B, W), dtype=torch.float32, device=dev), prefix=torch.empty((B, W, ND), dtype=torch.int32, device=dev),
                          range=torch.empty((B, W, 2), dtype=torch.int32, device=dev), item_index=torch.empty((B, W), dtype=torch.int32, device=dev))
        return dict(out=torch.empty((B, W, Hq, d), dtype=torch.bfloat16, device=dev),
                    ws_attn=torch.empty(max(gr.attn_workspace_bytes(B, W, Hq, Hkv, d, max_L), 256), dtype=torch.uint8, device=dev),
                    ws_sel=torch.empty(gr.select_workspace_bytes(B, W, V, ND), dtype=torch.uint8, device=dev),
                    sel_out=[mk() for _ in range(ND)])
    buf = make_buffers()
    sc0, pf0, rg0 = gr_synth.initial_beam_state(B, W, ND)
    state = [dict(scores=torch.from_numpy(sc0).to(dev), prefix=torch.from_numpy(pf0).to(dev), range=torch.from_numpy(rg0).to(dev))]

    def attn(s, bufs=buf, stream=None):
        a = attn_in[s]
        gr.gr_beam_attn(a["q"], k_sh, v_sh, d_cu, a["ku"], a["vu"], a["u"], scale, max_L, total_L, out=bufs["out"], workspace=bufs["ws_attn"], stream=stream)

    def select(s, bufs=buf, stream=None, m="headline", flags=None):
        st = state[s]
        gr.gr_beam_select(mask if m == "headline" else m, logits[s], st["scores"], st["prefix"], st["range"], s,
                          flags=args.flags if flags is None else flags, out=bufs["sel_out"][s], workspace=bufs["ws_sel"], stream=stream)

    # real beam chain once (with the mask, whatever the headline uses): the state entering level s is what levels 0..s-1 selected
    for s in range(ND):
        select(s, m=mask_blob, flags=0)
        state.append(dict(scores=buf["sel_out"][s]["scores"].clone(), prefix=buf["sel_out"][s]["prefix"].clone(), range=buf["sel_out"][s]["range"].clone()))
    torch.cuda.synchronize()
    live_rows = [int((state[s]["scores"] > float("-inf")).sum().item()) for s in range(ND)]

    if args.calibrate_copy:
        src = torch.zeros(1 << 28, dtype=torch.float32, device=dev)      # 1 GiB
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ---------------- the first launches after idle (reported, not part of the headline)
    time.sleep(0.2)
    cold_ms = _elapsed(torch, lambda: attn(ND - 1), 20)

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
    sel_by_level = {}
    for s in range(ND):
        ms = [sel_ms[i] for i in range(K) if i % ND == s]
        if ms:
            sel_by_level[f"level{s}"] = dict(ms=round(float(np.mean(ms)), 4), live_rows=live_rows[s])

    # ---------------- extras, outside the headline's timed region
    roofline_select, reorder, graph, streams, peaks, prefill, layers, fp8kv = None, None, None, None, None, None, None, None
    if not args.no_extras:
        # (0) the item step on its dense paths: every live row streamed in full (GR_SELECT_FORCE_DENSE, and mask = NULL),
        # on the levels where all B*W rows are live.  Algorithmic bytes = live rows x (4V logits + V/8 mask bits); the time
        # is the whole gr_beam_select call (rows kernel + selection kernel).  An attention launch runs (untimed) before
        # every timed call, as in the headline loop: the logits are not in any cache and the clock is in its loaded state.
        legs = {}
        worst = None
        for name, m, fl, mask_bytes in (("forced_dense", mask_blob, gr.GR_SELECT_FORCE_DENSE, V / 8.0), ("no_mask", None, 0, 0.0)):
            for s in range(ND):
                if live_rows[s] != B * W:
                    continue
                reps = 12
                e = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(reps)]
                for r in range(reps):
                    attn(s)
                    e[r][0].record()
                    select(s, m=m, flags=fl)
                    e[r][1].record()
                torch.cuda.synchronize()
                ms = float(np.mean([e[r][0].elapsed_time(e[r][1]) for r in range(2, reps)]))
                nbytes = live_rows[s] * (4.0 * V + mask_bytes)
                gbs = nbytes / (ms * 1e-3) / 1e9
                legs[f"{name}_level{s}"] = dict(ms=round(ms, 4), bytes=nbytes, GBps=round(gbs, 1), frac=round(gbs / PEAK_HBM_GBS, 4))
                if worst is None or gbs < worst[1]:
                    worst = (f"{name}_level{s}", gbs, ms, nbytes)
        if worst:
            roofline_select = dict(bound="hbm", kernel="k_rows + k_select (whole gr_beam_select call)", achieved=round(worst[1], 1), peak=PEAK_HBM_GBS,
                                   unit="GB/s", frac=round(worst[1] / PEAK_HBM_GBS, 4), leg=worst[0], legs=legs,
                                   note="dense paths only (every live row streamed); achieved/frac = the slowest leg; the default path gathers "
                                        "rows with few valid children and is reported as time in `select`")
        # (1) in-place move of the surviving beams' decode cache (gr_beam_reorder) with the parents each level selected
        ku_w, vu_w = attn_in[ND - 1]["ku"].clone(), attn_in[ND - 1]["vu"].clone()
        reorder = dict(note="GBps counts bytes read + written; the 67-200 MB working set partly lives in the 256 MB Infinity Cache, "
                            "so this is a cache-inclusive rate, not an HBM rate")
        for s in range(ND):
            par = buf["sel_out"][s]["parent"]
            for _ in range(2):
                gr.gr_beam_reorder(par, ku_w, vu_w, s + 1)
            ms = _elapsed(torch, lambda: gr.gr_beam_reorder(par, ku_w, vu_w, s + 1), 10)
            moved = 2.0 * 2.0 * B * W * (s + 1) * Hkv * d * 2          # K and V, read + write
            reorder[f"u{s + 1}"] = dict(ms=round(ms, 4), GBps_cache_inclusive=round(moved / (ms * 1e-3) / 1e9, 1))
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
            ref = {k: buf["sel_out"][ND - 1][k].clone() for k in ("parent", "token", "scores")}
            t_pre = time.perf_counter()
            while (time.perf_counter() - t_pre) * 1e3 < max(args.prewarm_ms, 1.0):
                g.replay()
                torch.cuda.synchronize()
            cycles = max(1, K // ND)
            gms = _elapsed(torch, g.replay, cycles) / ND
            same = all(bool(torch.equal(ref[k], buf["sel_out"][ND - 1][k])) for k in ref)
            graph = dict(ms_per_step=round(gms, 4), steps_per_s=round(1000.0 / gms, 3), cycles=cycles, replay_matches_eager=same)
            # the same cycle with the cache move between the item step and the next attention (attn -> select -> reorder)
            ku_g = [attn_in[s]["ku"].clone() for s in range(ND)]
            vu_g = [attn_in[s]["vu"].clone() for s in range(ND)]

            def full_cycle():
                for s in range(ND):
                    a = attn_in[s]
                    gr.gr_beam_attn(a["q"], k_sh, v_sh, d_cu, ku_g[s], vu_g[s], a["u"], scale, max_L, total_L, out=buf["out"], workspace=buf["ws_attn"])
                    select(s)
                    gr.gr_beam_reorder(buf["sel_out"][s]["parent"], ku_g[s], vu_g[s], s + 1)
            for _ in range(3):
                full_cycle()
            torch.cuda.synchronize()
            eager2 = _elapsed(torch, full_cycle, cycles) / ND
            g2 = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g2):
                full_cycle()
            for _ in range(3):
                g2.replay()
            torch.cuda.synchronize()
            gms2 = _elapsed(torch, g2.replay, cycles) / ND
            graph["with_reorder"] = dict(graph_ms_per_step=round(gms2, 4), graph_steps_per_s=round(1000.0 / gms2, 3),
                                         eager_ms_per_step=round(eager2, 4), eager_steps_per_s=round(1000.0 / eager2, 3))
            # and with a slot table that follows the beams instead of moving their rows (attn_slots -> select -> slot update)
            slots = [torch.empty((B, W, ND), dtype=torch.int32, device=dev) for _ in range(2)]
            ident_parent = torch.zeros((B, W), dtype=torch.int32, device=dev)

            def slot_cycle():
                gr.gr_beam_slot_update(ident_parent, None, 0, ND, out=slots[0])
                for s in range(ND):
                    a = attn_in[s]
                    gr.gr_beam_attn_slots(a["q"], k_sh, v_sh, d_cu, ku_g[s], vu_g[s], slots[s & 1], a["u"], scale, max_L, total_L,
                                          out=buf["out"], workspace=buf["ws_attn"])
                    select(s)
                    gr.gr_beam_slot_update(buf["sel_out"][s]["parent"], slots[s & 1], s + 1, ND, out=slots[(s + 1) & 1])
            for _ in range(3):
                slot_cycle()
            torch.cuda.synchronize()
            g3 = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g3):
                slot_cycle()
            for _ in range(3):
                g3.replay()
            torch.cuda.synchronize()
            gms3 = _elapsed(torch, g3.replay, cycles) / ND
            graph["with_slots"] = dict(graph_ms_per_step=round(gms3, 4), graph_steps_per_s=round(1000.0 / gms3, 3),
                                       note="no cache bytes move: gr_beam_attn_slots reads each beam's rows through the table "
                                            "that gr_beam_slot_update maintains")
            del ku_g, vu_g
        except Exception as e:          # the headline above stands on its own
            graph = dict(error=f"{type(e).__name__}: {e}"[:300])
        # (3) two independent batches on two streams of equal priority (one stream per batch): aggregate rate
        try:
            buf2 = make_buffers()
            s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
            for st_ in (s1, s2):
                st_.wait_stream(torch.cuda.current_stream())
            cycles = max(1, K // ND)

            def both(n):
                for _ in range(n):
                    for s in range(ND):
                        attn(s, buf, s1); select(s, buf, s1)
                        attn(s, buf2, s2); select(s, buf2, s2)
            both(2)
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            both(cycles)
            torch.cuda.synchronize()
            dt = time.perf_counter() - t1
            agree = all(bool(torch.equal(buf["sel_out"][ND - 1][k], buf2["sel_out"][ND - 1][k])) for k in ("parent", "token", "scores"))
            streams = dict(batches=2, aggregate_steps_per_s=round(2 * cycles * ND / dt, 3), single_stream_steps_per_s=round(steps_per_s, 3),
                           both_batches_agree=agree)
            del buf2
        except Exception as e:
            streams = dict(error=f"{type(e).__name__}: {e}"[:300])
        # (4) the prefill that would have produced the shared cache: causal attention over the same packed prompts
        try:
            qp = torch.randn((total_L, Hq, d), device=dev).to(torch.bfloat16)
            op = torch.empty_like(qp)
            run_p = lambda: gr.gr_prefill_attn(qp, k_sh, v_sh, d_cu, scale, max_L, total_L, out=op)
            for _ in range(3):
                run_p()
            ms = _elapsed(torch, run_p, 5)
            pf_flops = 4.0 * Hq * d * float((lens * (lens + 1) // 2).sum())
            prefill = dict(ms=round(ms, 4), TFLOPs=round(pf_flops / (ms * 1e-3) / 1e12, 1), frac=round(pf_flops / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4),
                           flops=pf_flops, note="causal: 4*Hq*d*sum_b L_b(L_b+1)/2 flops; q is N(0,1) bf16 [total_L,Hq,d]")
            del qp, op
        except Exception as e:
            prefill = dict(error=f"{type(e).__name__}: {e}"[:300])
        # (4b) the same attention over a prompt cache stored as FP8 E4M3 codes (one scale per tensor)
        try:
            def to_fp8(t):
                scale = float(t.float().abs().max().item()) / 448.0
                codes = torch.empty(t.shape, dtype=torch.uint8, device=dev)
                step_rows = 1 << 16
                for r0 in range(0, t.shape[0], step_rows):      # in slices: the fp32 intermediate of the whole cache is large
                    codes[r0:r0 + step_rows] = (t[r0:r0 + step_rows].float() / scale).to(torch.float8_e4m3fn).view(torch.uint8)
                return codes, scale
            k8, k_scale = to_fp8(k_sh)
            v8, v_scale = to_fp8(v_sh)
            a3 = attn_in[ND - 1]
            run8 = lambda: gr.gr_beam_attn_fp8kv(a3["q"], k8, v8, k_scale, v_scale, d_cu, a3["ku"], a3["vu"], a3["u"], scale, max_L, total_L,
                                                 out=buf["out"], workspace=buf["ws_attn"])
            for _ in range(5):
                run8()
            ms = _elapsed(torch, run8, 10)
            fp8kv = dict(ms=round(ms, 4), TFLOPs=round(flops[ND - 1] / (ms * 1e-3) / 1e12, 1), bf16_cache_ms=round(float(np.mean([attn_ms[i] for i in range(K) if i % ND == ND - 1] or [0])), 4),
                         note="u = 3 launch; codes widened to bf16 on the way into LDS, bf16 MFMA as before; the cache is half the bytes")
            del k8, v8
        except Exception as e:
            fp8kv = dict(error=f"{type(e).__name__}: {e}"[:300])
        # (5) a per-layer loop: n_layers attention calls (each layer its own K/V and Q) + one item step per decode step,
        # the three levels captured as one graph.  Layer count is a stand-in (no model geometry is given); what it shows
        # is that the step scales by the attention time per layer with nothing added between the calls.
        try:
            n_layers = args.layers
            lay = [dict(q=torch.randn_like(attn_in[0]["q"].float()).to(torch.bfloat16), ks=torch.randn_like(k_sh.float()).to(torch.bfloat16),
                        vs=torch.randn_like(v_sh.float()).to(torch.bfloat16)) for _ in range(n_layers)]

            def layered_cycle():
                for s in range(ND):
                    a = attn_in[s]
                    for l in lay:
                        gr.gr_beam_attn(l["q"], l["ks"], l["vs"], d_cu, a["ku"], a["vu"], a["u"], scale, max_L, total_L, out=buf["out"], workspace=buf["ws_attn"])
                    select(s)
            layered_cycle()
            torch.cuda.synchronize()
            g3 = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g3):
                layered_cycle()
            for _ in range(2):
                g3.replay()
            torch.cuda.synchronize()
            cyc = max(1, K // (ND * n_layers))
            lms = _elapsed(torch, g3.replay, cyc) / ND
            layers = dict(n_layers=n_layers, graph_ms_per_step=round(lms, 4), steps_per_s=round(1000.0 / lms, 3),
                          ms_per_layer=round((lms - float(np.mean(sel_ms))) / n_layers, 4), note="N(0,1) Q/K/V per layer; one item step per decode step")
            del lay
        except Exception as e:
            layers = dict(error=f"{type(e).__name__}: {e}"[:300])
        # (6) what the machine sustains, next to the datasheet peaks
        try:
            peaks = measured_peaks(torch, gr, dev)
            roofline["peak_measured"] = peaks["bf16_mfma_TFLOPs"]
            roofline["frac_of_measured"] = round(attn_tflops / peaks["bf16_mfma_TFLOPs"], 4)
            if roofline_select:
                roofline_select["peak_measured"] = peaks["hbm_read_GBps"]
                roofline_select["frac_of_measured"] = round(roofline_select["achieved"] / peaks["hbm_read_GBps"], 4)
        except Exception as e:
            peaks = dict(error=f"{type(e).__name__}: {e}"[:300])

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
        roofline=roofline, roofline_select=roofline_select, cpu_baseline=cpu,
        attn=dict(ms_by_u={f"u{s + 1}": round(float(np.mean([attn_ms[i] for i in range(K) if i % ND == s] or [0])), 4) for s in range(ND)},
                  tflops=round(attn_tflops, 2), ms_first20_after_idle=round(cold_ms, 4)),
        select=sel_by_level, reorder=reorder, graph=graph, two_streams=streams, prefill=prefill, fp8kv=fp8kv, layers=layers, peaks_measured=peaks,
        prewarm=dict(ms=args.prewarm_ms, steps=prewarm_steps), wall_s=round(wall, 3), input_gen_s=round(t_gen, 1))
    print(json.dumps(line))


if __name__ == "__main__":
    main()
