"""GPU parity: gr_prefill_attn (causal attention over packed prompts, paper Sections 2.2.1 / 5.1) against the
oracle's row-by-row definition.  Tolerances as for the decode attention: bf16 output, max-abs <= 2e-2 on
unit-variance inputs; LSE within 2e-3."""
import numpy as np
import pytest

import gr_synth
from gpu_util import bf16_to_dev, to_dev

pytestmark = pytest.mark.gpu


def _case(seed, lens, Hq, Hkv, d):
    rng = np.random.default_rng(seed)
    cu = np.zeros(len(lens) + 1, dtype=np.int32)
    cu[1:] = np.cumsum(lens)
    T = max(int(cu[-1]), 1)
    bf = lambda *s: gr_synth.f32_to_bf16_bits(rng.standard_normal(s, dtype=np.float32))
    return dict(q=bf(T, Hq, d), k=bf(T, Hkv, d), v=bf(T, Hkv, d), cu=cu)


def _run(gr, c, scale, want_lse=True):
    import torch
    T, Hq, d = c["q"].shape
    lens = np.diff(c["cu"])
    lse = torch.full((T, Hq), 7.0, dtype=torch.float32, device="cuda:0") if want_lse else None
    out = torch.full((T, Hq, d), 7.0, dtype=torch.bfloat16, device="cuda:0")
    gr.gr_prefill_attn(bf16_to_dev(c["q"]), bf16_to_dev(c["k"]), bf16_to_dev(c["v"]), to_dev(c["cu"]), scale,
                       int(lens.max()) if len(lens) else 0, int(c["cu"][-1]), out=out, lse_out=lse)
    torch.cuda.synchronize()
    return out.float().cpu().numpy(), (lse.cpu().numpy() if want_lse else None)


@pytest.mark.parametrize("lens,Hq,Hkv,d", [
    ((5, 19, 1, 33), 4, 2, 64),            # shorter than a tile, a one-token request
    ((70,), 8, 8, 64),                     # g = 1: 256 tokens per row block, ragged second tile
    ((130, 64, 257), 32, 8, 128),          # the benchmark's head geometry; several row blocks, block-aligned and ragged ends
    ((300,), 8, 2, 128),
    ((100, 37, 0, 129), 16, 2, 64),        # g = 8 and an empty request in the middle
    ((64, 128, 192), 4, 1, 128),           # tile-aligned lengths
])
def test_prefill_matches_oracle(oracle_lib, lens, Hq, Hkv, d):
    import paper_2512_11529_amd as gr
    gr.load_library()
    c = _case(hash((lens, Hq, Hkv, d)) % 1000, lens, Hq, Hkv, d)
    scale = float(np.float32(1 / np.sqrt(d)))
    out, lse = _run(gr, c, scale)
    ref, ref_lse = oracle_lib.prefill_attn_causal(c["q"], c["k"], c["v"], c["cu"], scale)
    T = int(c["cu"][-1])
    ref = ref.reshape(T, Hq, d)
    ref_lse = ref_lse.reshape(T, Hq)
    err = np.abs(out[:T] - ref).max()
    assert err <= 2e-2, f"max-abs {err}"
    np.testing.assert_allclose(lse[:T], ref_lse, rtol=0, atol=2e-3)


def test_prefill_long_prompt_sampled_rows(oracle_lib):
    """L = 4096 at the benchmark's head geometry: 16 row blocks per KV head, up to 64 tiles per block.  Rows checked:
    the first and last token of every 64-token block (diagonal tiles, block edges) and a seeded sample, every head."""
    import paper_2512_11529_amd as gr
    gr.load_library()
    L, Hq, Hkv, d = 4096, 32, 8, 128
    c = _case(77, (L,), Hq, Hkv, d)
    scale = float(np.float32(1 / np.sqrt(d)))
    out, lse = _run(gr, c, scale)
    rng = np.random.default_rng(5)
    toks = sorted(set([0, 1, 2, L - 1] + [64 * k for k in range(L // 64)] + [64 * k + 63 for k in range(L // 64)] + list(rng.integers(0, L, 120))))
    tri = np.array([(0, i, h) for i in toks for h in range(Hq)], dtype=np.int32)
    ref, ref_lse = oracle_lib.prefill_attn_causal(c["q"], c["k"], c["v"], c["cu"], scale, tri)
    got = out[tri[:, 1], tri[:, 2]]
    err = np.abs(got - ref).max()
    assert err <= 2e-2, f"max-abs {err}"
    np.testing.assert_allclose(lse[tri[:, 1], tri[:, 2]], ref_lse, rtol=0, atol=2e-3)


def test_prefill_ragged_batch_touches_only_its_rows(oracle_lib):
    """Rows past total_L in the output buffer stay untouched; every row below is written."""
    import torch
    import paper_2512_11529_amd as gr
    gr.load_library()
    c = _case(9, (40, 200, 3), 8, 2, 64)
    T = int(c["cu"][-1])
    pad = 5
    q = torch.cat([bf16_to_dev(c["q"]), torch.zeros((pad, 8, 64), dtype=torch.bfloat16, device="cuda:0")])
    k = torch.cat([bf16_to_dev(c["k"]), torch.zeros((pad, 2, 64), dtype=torch.bfloat16, device="cuda:0")])
    v = k.clone(); v[:T] = bf16_to_dev(c["v"])
    out = torch.full_like(q, 7.0)
    gr.gr_prefill_attn(q, k, v, to_dev(c["cu"]), 0.125, 200, T, out=out)
    torch.cuda.synchronize()
    assert (out[T:] == 7.0).all()
    ref, _ = oracle_lib.prefill_attn_causal(c["q"], c["k"], c["v"], c["cu"], 0.125)
    assert np.abs(out[:T].float().cpu().numpy() - ref.reshape(T, 8, 64)).max() <= 2e-2


def test_prefill_rejects_bad_arguments():
    import torch
    import paper_2512_11529_amd as gr
    gr.load_library()
    dev = torch.device("cuda:0")
    q = torch.zeros((8, 4, 64), dtype=torch.bfloat16, device=dev)
    kv = torch.zeros((8, 2, 64), dtype=torch.bfloat16, device=dev)
    cu = torch.tensor([0, 8], dtype=torch.int32, device=dev)
    for scale in (0.0, -1.0, float("nan"), float("inf")):
        with pytest.raises(gr.GrError) as e:
            gr.gr_prefill_attn(q, kv, kv, cu, scale, 8, 8)
        assert e.value.status == -1
    q32 = torch.zeros((8, 4, 32), dtype=torch.bfloat16, device=dev)
    kv32 = torch.zeros((8, 2, 32), dtype=torch.bfloat16, device=dev)
    with pytest.raises(gr.GrError) as e:
        gr.gr_prefill_attn(q32, kv32, kv32, cu, 0.1, 8, 8)
    assert e.value.status == -2
    with pytest.raises(gr.GrError) as e:                 # total_L larger than B * max_L
        gr.gr_prefill_attn(q, kv, kv, cu, 0.1, 4, 8)
    assert e.value.status == -1
    out, _ = gr.gr_prefill_attn(q, kv, kv, torch.tensor([0, 0], dtype=torch.int32, device=dev), 0.1, 0, 0)     # empty batch: nothing to do
    torch.cuda.synchronize()


def test_prefill_ragged_long_batch_sampled_rows(oracle_lib):
    """Eight prompts of 512..8192 tokens (the length mix of the high-concurrency workload) at the benchmark's head
    geometry: the grid is sized by the longest prompt, so most row blocks of the short requests leave at once and the
    rest are dispatched heaviest first.  Rows checked per request: first, last, the last row of the first block, the
    rows on both sides of every 1024th token, and a seeded sample; every head."""
    import paper_2512_11529_amd as gr
    gr.load_library()
    Hq, Hkv, d = 32, 8, 128
    rng = np.random.default_rng(12)
    lens = tuple(int(x) for x in rng.integers(512, 8193, size=8))
    c = _case(78, lens, Hq, Hkv, d)
    scale = float(np.float32(1 / np.sqrt(d)))
    out, lse = _run(gr, c, scale)
    tri = []
    for b, L in enumerate(lens):
        toks = {0, L - 1, 63, 64} | {t for k in range(1024, L, 1024) for t in (k - 1, k)} | set(int(x) for x in rng.integers(0, L, 12))
        tri += [(b, i, h) for i in sorted(toks) for h in range(Hq)]
    tri = np.array(tri, dtype=np.int32)
    ref, ref_lse = oracle_lib.prefill_attn_causal(c["q"], c["k"], c["v"], c["cu"], scale, tri)
    rows = c["cu"][tri[:, 0]] + tri[:, 1]
    err = np.abs(out[rows, tri[:, 2]] - ref).max()
    assert err <= 2e-2, f"max-abs {err}"
    np.testing.assert_allclose(lse[rows, tri[:, 2]], ref_lse, rtol=0, atol=2e-3)
    assert np.isfinite(out[:int(c["cu"][-1])]).all()
