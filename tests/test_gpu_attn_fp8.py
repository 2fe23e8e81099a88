"""GPU parity: gr_beam_attn_fp8kv (shared-prefix beam attention over a prompt cache stored as FP8 E4M3 codes with one
scale per tensor; paper Section 5.1's separated cache with its shared half at one byte per element) against the
oracle's unified-cache attention on the widened values (code * scale as fp32).  Quantisation is part of the INPUT
here, so the bar is the one of the bf16 path: max-abs <= 2e-2 on bf16 outputs, LSE within 2e-3."""
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


def _quantise(bits):
    x = gr_synth.bf16_bits_to_f32(bits)
    scale = np.float32(max(float(np.abs(x).max()), 1e-6) / 448.0)
    codes = gr_synth.f32_to_e4m3_bits(x / scale)
    return codes, scale


def _check(gr, oracle_lib, a, sm_scale, triples=None):
    import torch
    B, W, Hq, d = a["q"].shape
    k8, ks = _quantise(a["k_shared"])
    v8, vs = _quantise(a["v_shared"])
    cu = a["cu_seqlens"]
    lse = torch.empty((B, W, Hq), dtype=torch.float32, device="cuda:0")
    out, _ = gr.gr_beam_attn_fp8kv(bf16_to_dev(a["q"]), to_dev(k8), to_dev(v8), float(ks), float(vs), to_dev(cu),
                                   bf16_to_dev(a["k_unshared"]), bf16_to_dev(a["v_unshared"]), a["u"], sm_scale,
                                   int(np.diff(cu).max()) if len(cu) > 1 else 0, int(cu[-1]), lse_out=lse)
    torch.cuda.synchronize()
    out, lse = out.float().cpu().numpy(), lse.cpu().numpy()
    kf = (gr_synth.e4m3_bits_to_f32(k8) * ks).astype(np.float32)
    vf = (gr_synth.e4m3_bits_to_f32(v8) * vs).astype(np.float32)
    ref, ref_lse = oracle_lib.attn_unified_f32kv(a["q"], kf, vf, cu, a["k_unshared"], a["v_unshared"], a["u"], sm_scale, triples)
    if triples is None:
        got, got_lse = out.reshape(-1, d), lse.reshape(-1)
    else:
        got, got_lse = out[triples[:, 0], triples[:, 1], triples[:, 2]], lse[triples[:, 0], triples[:, 1], triples[:, 2]]
    err = np.abs(got - ref).max()
    assert err <= 2e-2, f"max-abs {err}"
    fin = np.isfinite(ref_lse)
    np.testing.assert_allclose(got_lse[fin], ref_lse[fin], rtol=0, atol=2e-3)


@pytest.mark.parametrize("B,W,Hq,Hkv,d,u,lens", [
    (2, 5, 8, 2, 128, 2, (7, 150)),
    (3, 24, 4, 4, 64, 1, (64, 1, 130)),
    (1, 70, 8, 2, 128, 3, (333,)),
    (2, 16, 16, 4, 128, 3, (0, 200)),           # a request with no prompt: only its own tokens
    (1, 40, 4, 4, 64, 0, (257,)),               # no own tokens: the prompt loop alone (scales still applied)
    (2, 96, 32, 8, 128, 3, (100, 1500)),        # enough rows for the L split
])
def test_fp8kv_matches_oracle(gr, oracle_lib, B, W, Hq, Hkv, d, u, lens):
    a = rand_attn_case(300 + B + W + d, B, W, Hq, Hkv, d, 3, u, lens)
    _check(gr, oracle_lib, a, float(np.float32(1 / np.sqrt(d))))


@pytest.mark.parametrize("d", [64, 128])
@pytest.mark.parametrize("rows,segments", [(128, 1), (256, 1), (128, 3), (256, 2)])
def test_fp8kv_every_launch_plan(gr, oracle_lib, d, rows, segments):
    B, W, Hq, Hkv = 2, 160, 8, 2
    a = rand_attn_case(400 + d + rows + segments, B, W, Hq, Hkv, d, 3, 2, (333, 1100))
    rng = np.random.default_rng(6)
    n = 200
    tri = np.stack([rng.integers(0, B, n), rng.integers(0, W, n), rng.integers(0, Hq, n)], axis=1).astype(np.int32)
    tri[:4] = [[0, 0, 0], [1, W - 1, Hq - 1], [0, 63, 7], [1, 64, 0]]
    gr.gr_diag_attn_plan(rows, segments)
    try:
        _check(gr, oracle_lib, a, float(np.float32(1 / np.sqrt(d))), tri)
    finally:
        gr.gr_diag_attn_plan(0, 0)


def test_fp8kv_every_code_is_widened_exactly(gr, oracle_lib):
    """All 254 finite codes appear in K and V (one dominant key per query picks single V rows, so a wrong code -> value
    map or a wrong byte order inside the 8-byte pieces shows up at full magnitude)."""
    import torch
    B, W, Hq, Hkv, d, L = 1, 8, 2, 1, 64, 128
    a = rand_attn_case(9, B, W, Hq, Hkv, d, 3, 0, (L,))
    codes = np.array([c for c in range(256) if (c & 0x7F) != 0x7F], dtype=np.uint8)
    rng = np.random.default_rng(2)
    k8 = rng.choice(codes, size=(L, Hkv, d)).astype(np.uint8)
    v8 = np.resize(codes, (L, Hkv, d)).astype(np.uint8)
    ks, vs = np.float32(2.0 ** -9), np.float32(2.0 ** -6)
    cu = a["cu_seqlens"]
    out, _ = gr.gr_beam_attn_fp8kv(bf16_to_dev(a["q"]), to_dev(k8), to_dev(v8), float(ks), float(vs), to_dev(cu),
                                   bf16_to_dev(a["k_unshared"]), bf16_to_dev(a["v_unshared"]), 0, 1.0, L, L)
    torch.cuda.synchronize()
    kf = (gr_synth.e4m3_bits_to_f32(k8) * ks).astype(np.float32)
    vf = (gr_synth.e4m3_bits_to_f32(v8) * vs).astype(np.float32)
    ref, _ = oracle_lib.attn_unified_f32kv(a["q"], kf, vf, cu, a["k_unshared"], a["v_unshared"], 0, 1.0)
    err = np.abs(out.float().cpu().numpy().reshape(-1, d) - ref).max()
    assert err <= 2e-2, f"max-abs {err}"


def test_fp8kv_rejects_bad_scales(gr):
    a = rand_attn_case(1, 1, 2, 2, 2, 64, 3, 1, (5,))
    k8, _ = _quantise(a["k_shared"])
    for ks, vs in ((0.0, 1.0), (1.0, -1.0), (float("nan"), 1.0), (1.0, float("inf"))):
        with pytest.raises(gr.GrError) as e:
            gr.gr_beam_attn_fp8kv(bf16_to_dev(a["q"]), to_dev(k8), to_dev(k8), ks, vs, to_dev(a["cu_seqlens"]),
                                  bf16_to_dev(a["k_unshared"]), bf16_to_dev(a["v_unshared"]), 1, 1.0, 5, 5)
        assert e.value.status == -1
