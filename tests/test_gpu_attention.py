"""GPU parity: gr_beam_attn against the CPU oracle's unified-cache attention (Sections 5.1-5.2).

Bar: max-abs error <= 2e-2 on bf16 outputs (bf16 in, fp32 accumulate), plus a tighter bound derived
from the arithmetic: the output is a convex combination of bf16 values whose weights carry a bf16
rounding (2^-9 relative) and the result is rounded to bf16 once more, so |err| <= 2^-7 * max|V| with
a wide margin.
"""
import numpy as np
import pytest

import gr_synth
from gpu_util import rand_attn_case, run_attn

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gr():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_2512_11529_amd as gr
    gr.load_library()
    return gr


def _check(gr, oracle_lib, a, scale, triples=None):
    out, lse = run_attn(gr, a, scale)
    B, W, Hq, d = a["q"].shape
    ref, ref_lse = oracle_lib.attn_unified(a["q"], a["k_shared"], a["v_shared"], a["cu_seqlens"], a["k_unshared"],
                                           a["v_unshared"], a["u"], scale, triples)
    if triples is None:
        got, got_lse = out.reshape(-1, d), lse.reshape(-1)
    else:
        got = out[triples[:, 0], triples[:, 1], triples[:, 2]]
        got_lse = lse[triples[:, 0], triples[:, 1], triples[:, 2]]
    err = np.abs(got - ref).max()
    vmax = float(np.abs(gr_synth.bf16_bits_to_f32(a["v_shared"])).max()) if a["v_shared"].size else 1.0
    vmax = max(vmax, float(np.abs(gr_synth.bf16_bits_to_f32(a["v_unshared"])).max()))
    assert err <= 2e-2, f"max-abs {err}"
    assert err <= 2.0 ** -7 * vmax, f"max-abs {err} vs derived bound {2.0 ** -7 * vmax}"
    fin = np.isfinite(ref_lse)
    np.testing.assert_allclose(got_lse[fin], ref_lse[fin], rtol=0, atol=2e-3)
    return err


def test_tiny_config_all_steps(gr, oracle_lib):
    cfg = gr_synth.get_config(1)
    for step in range(cfg.ND):
        a = gr_synth.make_attention_inputs(cfg, step)
        _check(gr, oracle_lib, a, float(np.float32(1 / np.sqrt(cfg.d))))


@pytest.mark.parametrize("B,W,Hq,Hkv,d,u,lens", [
    (2, 5, 8, 2, 128, 2, (70, 333)),          # ragged tails, GQA g=4, W*g = 20 rows (partial row block)
    (3, 24, 4, 4, 64, 1, (1, 64, 129)),       # g=1, d=64, one-token prompt, exact tile, tile+1
    (1, 70, 8, 2, 128, 3, (517,)),            # 280 rows: two row blocks
    (2, 16, 16, 4, 128, 3, (0, 200)),         # an empty prompt: only the beam's own tokens
    (1, 3, 2, 1, 64, 2, (1000,)),             # g=2
    (2, 96, 32, 8, 128, 3, (2048, 1500)),     # the benchmark head geometry; long enough to split L
    (1, 40, 4, 4, 64, 3, (100,)),             # g=1: 32 beams x 3 own tokens per wave = three unshared mini-tiles
    (2, 20, 4, 2, 128, 3, (64, 10)),          # g=2: 16 beams x 3 = 48 own-token rows, two mini-tiles
    (1, 30, 6, 2, 64, 2, (130,)),             # g=3: beams straddle wave boundaries (32 is not a multiple of g)
    (1, 300, 8, 2, 128, 3, (0,)),             # no prompt at all, several row blocks: own tokens only
    (1, 200, 4, 2, 64, 2, (300,)),            # d=64 with more than 128 rows per KV head: the 8-wave d=64 kernel
    (1, 8, 8, 2, 128, 1, (1500,)),            # 32 rows per KV head, long prompt: 4-wave kernel with L split in five
])
def test_random_shapes(gr, oracle_lib, B, W, Hq, Hkv, d, u, lens):
    a = rand_attn_case(B * 100 + W, B, W, Hq, Hkv, d, 3, u, lens)
    _check(gr, oracle_lib, a, float(np.float32(1 / np.sqrt(d))))


def test_structured_inputs_give_order_one_outputs(gr, oracle_lib):
    # one dominant key per query makes the output a single V row (magnitude ~1), so layout or
    # indexing mistakes cannot hide under small averaged values
    B, W, Hq, Hkv, d = 2, 9, 8, 2, 128
    a = rand_attn_case(5, B, W, Hq, Hkv, d, 3, 3, (150, 97))
    rng = np.random.default_rng(0)
    q = gr_synth.bf16_bits_to_f32(a["q"])
    for b in range(B):
        lo, hi = a["cu_seqlens"][b], a["cu_seqlens"][b + 1]
        for hk in range(Hkv):
            j = int(rng.integers(lo, hi))
            a["k_shared"][j, hk] = gr_synth.f32_to_bf16_bits(8.0 * q[b, int(rng.integers(W)), hk * (Hq // Hkv)])
    for b in range(B):
        for w in range(0, W, 2):
            a["k_unshared"][b, w, 1, 0] = gr_synth.f32_to_bf16_bits(8.0 * q[b, w, 1])
    _check(gr, oracle_lib, a, 1.0)


def test_scores_rising_along_the_prompt_raise_the_reference_on_every_tile(gr, oracle_lib):
    # keys proportional to one query with a factor that grows with the position: that query's scores climb by ~15 bits per
    # 64-token tile (the lazily raised reference maximum and the O / row-sum rescale run on every tile), the last key
    # dominates, and for the opposite sign the first tile holds the maximum and everything later underflows
    B, W, Hq, Hkv, d, L = 1, 4, 4, 1, 64, 1000
    for sign in (1.0, -1.0):
        a = rand_attn_case(17, B, W, Hq, Hkv, d, 3, 2, (L,))
        q0 = gr_synth.bf16_bits_to_f32(a["q"])[0, 0, 0]
        ramp = (np.arange(L, dtype=np.float32) / 50.0)[:, None]
        a["k_shared"][:, 0] = gr_synth.f32_to_bf16_bits(sign * ramp * q0[None, :])
        _check(gr, oracle_lib, a, 0.125)


def test_wide_beam_sampled_rows(gr, oracle_lib):
    # W = 2048 beams (8192 query rows per KV head, 32 row blocks): sampled outputs against the oracle
    B, W, Hq, Hkv, d = 1, 2048, 8, 2, 64
    a = rand_attn_case(31, B, W, Hq, Hkv, d, 3, 3, (200,))
    rng = np.random.default_rng(3)
    tri = np.stack([np.zeros(300, np.int64), rng.integers(0, W, 300), rng.integers(0, Hq, 300)], axis=1).astype(np.int32)
    tri[:4] = [[0, 0, 0], [0, W - 1, Hq - 1], [0, 255, 3], [0, 256, 4]]
    _check(gr, oracle_lib, a, float(np.float32(1 / np.sqrt(d))), tri)


def test_separated_cache_is_w_independent_of_other_beams(gr, oracle_lib):
    # changing one beam's own tokens must not change any other beam's output
    a = rand_attn_case(9, 1, 6, 4, 2, 64, 3, 2, (90,))
    out0, _ = run_attn(gr, a, 0.125)
    a2 = dict(a); a2["k_unshared"] = a["k_unshared"].copy(); a2["k_unshared"][0, 2] ^= 0x8000
    out1, _ = run_attn(gr, a2, 0.125)
    keep = [w for w in range(6) if w != 2]
    np.testing.assert_array_equal(out0[0, keep], out1[0, keep])
    assert not np.array_equal(out0[0, 2], out1[0, 2])


def test_argument_errors(gr):
    import torch
    from gpu_util import bf16_to_dev, to_dev
    a = rand_attn_case(1, 1, 2, 2, 2, 32, 3, 1, (5,))     # d = 32 unsupported
    with pytest.raises(gr.GrError) as e:
        run_attn(gr, a, 1.0)
    assert e.value.status == -2
    a = rand_attn_case(1, 1, 2, 2, 2, 64, 3, 1, (5,))
    a["u"] = 4
    with pytest.raises(gr.GrError) as e:
        run_attn(gr, a, 1.0)
    assert e.value.status == -1
    # a tensor that does not start on a 16-byte boundary is refused (the kernels move 16-byte pieces)
    a = rand_attn_case(2, 1, 2, 2, 2, 64, 3, 1, (5,))
    q = bf16_to_dev(a["q"])
    shifted = torch.empty(q.numel() + 8, dtype=torch.bfloat16, device=q.device)[1:1 + q.numel()].view(q.shape)
    shifted.copy_(q)
    assert shifted.data_ptr() % 16 == 2
    with pytest.raises(gr.GrError) as e:
        gr.gr_beam_attn(shifted, bf16_to_dev(a["k_shared"]), bf16_to_dev(a["v_shared"]), to_dev(a["cu_seqlens"]),
                        bf16_to_dev(a["k_unshared"]), bf16_to_dev(a["v_unshared"]), 1, 1.0, 5, 5)
    assert e.value.status == -1


@pytest.mark.parametrize("d", [64, 128])
@pytest.mark.parametrize("rows,segments", [(128, 1), (256, 1), (128, 3), (256, 2), (256, 16)])
def test_every_launch_plan_matches_oracle(gr, oracle_lib, d, rows, segments):
    """Both workgroup sizes and the L-split path of both head sizes, forced through the plan override (the built-in rule
    picks only one of them per shape): ragged batch, 640 query rows per KV head, a prompt that ends inside a tile."""
    B, W, Hq, Hkv = 2, 160, 8, 2
    a = rand_attn_case(50 + d + rows + segments, B, W, Hq, Hkv, d, 3, 2, (333, 1100))
    rng = np.random.default_rng(4)
    n = 240
    tri = np.stack([rng.integers(0, B, n), rng.integers(0, W, n), rng.integers(0, Hq, n)], axis=1).astype(np.int32)
    tri[:6] = [[0, 0, 0], [1, W - 1, Hq - 1], [0, 31, 3], [1, 32, 4], [0, 63, 7], [1, 64, 0]]
    gr.gr_diag_attn_plan(rows, segments)
    try:
        _check(gr, oracle_lib, a, float(np.float32(1 / np.sqrt(d))), tri)
    finally:
        gr.gr_diag_attn_plan(0, 0)
