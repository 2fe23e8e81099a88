"""Pins for the oracle's attention (paper Sections 5.1-5.2).  CPU only.

The oracle is the unified-cache definition.  It is pinned here against (a) torch's library attention
on the concatenated per-beam sequence, (b) an independently written staged computation (shared
stage, unshared stage, online-softmax merge - the decomposition Section 5.2 describes) and
(c) closed forms / invariants.
"""
import json
import os

import numpy as np
import pytest
import torch

import gr_synth
from gr_synth import bf16_bits_to_f32, f32_to_bf16_bits


def _rand_case(seed, B=2, W=5, Hq=8, Hkv=2, d=32, ND=3, u=2, lens=(7, 19)):
    rng = np.random.default_rng(seed)
    cu = np.zeros(B + 1, dtype=np.int32)
    cu[1:] = np.cumsum(lens)
    bf = lambda *s: f32_to_bf16_bits(rng.standard_normal(s, dtype=np.float32))
    return dict(q=bf(B, W, Hq, d), k_shared=bf(int(cu[-1]), Hkv, d), v_shared=bf(int(cu[-1]), Hkv, d),
                cu_seqlens=cu, k_unshared=bf(B, W, ND, Hkv, d), v_unshared=bf(B, W, ND, Hkv, d), u=u)


def _run(oracle_lib, c, scale, triples=None):
    return oracle_lib.attn_unified(c["q"], c["k_shared"], c["v_shared"], c["cu_seqlens"], c["k_unshared"],
                                   c["v_unshared"], c["u"], scale, triples)


@pytest.mark.parametrize("u", [0, 1, 3])
def test_matches_torch_sdpa_on_concatenated_sequence(oracle_lib, u):
    c = _rand_case(1, u=u)
    B, W, Hq, d = c["q"].shape
    Hkv = c["k_shared"].shape[1]
    g = Hq // Hkv
    scale = 0.375
    out, lse = _run(oracle_lib, c, scale)
    out = out.reshape(B, W, Hq, d)
    q = torch.from_numpy(bf16_bits_to_f32(c["q"]).astype(np.float64))
    ks = torch.from_numpy(bf16_bits_to_f32(c["k_shared"]).astype(np.float64))
    vs = torch.from_numpy(bf16_bits_to_f32(c["v_shared"]).astype(np.float64))
    ku = torch.from_numpy(bf16_bits_to_f32(c["k_unshared"]).astype(np.float64))
    vu = torch.from_numpy(bf16_bits_to_f32(c["v_unshared"]).astype(np.float64))
    for b in range(B):
        lo, hi = int(c["cu_seqlens"][b]), int(c["cu_seqlens"][b + 1])
        for w in range(W):
            k = torch.cat([ks[lo:hi], ku[b, w, :u]], 0).repeat_interleave(g, dim=1)   # [n, Hq, d]
            v = torch.cat([vs[lo:hi], vu[b, w, :u]], 0).repeat_interleave(g, dim=1)
            ref = torch.nn.functional.scaled_dot_product_attention(
                q[b, w][None, :, None, :], k.permute(1, 0, 2)[None], v.permute(1, 0, 2)[None], scale=scale)
            np.testing.assert_allclose(out[b, w], ref[0, :, 0, :].numpy(), rtol=0, atol=1e-12)


def _staged(c, scale, b, w, hq):
    """Shared stage, unshared stage and online-softmax merge, written independently in numpy fp64."""
    Hq, d = c["q"].shape[2:]
    Hkv = c["k_shared"].shape[1]
    hk = hq // (Hq // Hkv)
    lo, hi = int(c["cu_seqlens"][b]), int(c["cu_seqlens"][b + 1])
    q = bf16_bits_to_f32(c["q"][b, w, hq]).astype(np.float64)

    def stage(K, V):
        if K.shape[0] == 0:
            return -np.inf, 0.0, np.zeros(d)
        s = scale * (K.astype(np.float64) @ q)
        m = s.max()
        p = np.exp(s - m)
        return m, p.sum(), p @ V.astype(np.float64)

    m1, l1, o1 = stage(bf16_bits_to_f32(c["k_shared"][lo:hi, hk]), bf16_bits_to_f32(c["v_shared"][lo:hi, hk]))
    m2, l2, o2 = stage(bf16_bits_to_f32(c["k_unshared"][b, w, :c["u"], hk]), bf16_bits_to_f32(c["v_unshared"][b, w, :c["u"], hk]))
    m = max(m1, m2)
    a1 = np.exp(m1 - m) if l1 > 0 else 0.0
    a2 = np.exp(m2 - m) if l2 > 0 else 0.0
    l = l1 * a1 + l2 * a2
    return (o1 * a1 + o2 * a2) / l, m + np.log(l)


def test_separated_cache_equals_unified_cache(oracle_lib):
    c = _rand_case(2, u=3, lens=(33, 5))
    B, W, Hq, d = c["q"].shape
    scale = float(np.float32(1.0 / np.sqrt(d)))
    out, lse = _run(oracle_lib, c, scale)
    out = out.reshape(B, W, Hq, d)
    lse = lse.reshape(B, W, Hq)
    for b in range(B):
        for w in range(W):
            for hq in range(Hq):
                o, l = _staged(c, scale, b, w, hq)
                np.testing.assert_allclose(out[b, w, hq], o, rtol=0, atol=1e-12)
                assert abs(lse[b, w, hq] - l) < 1e-12


def test_triples_subset_matches_full(oracle_lib):
    c = _rand_case(3)
    B, W, Hq, d = c["q"].shape
    full, lse_full = _run(oracle_lib, c, 0.25)
    tri = np.array([[1, 4, 7], [0, 0, 0], [1, 2, 3]], dtype=np.int32)
    sub, lse = _run(oracle_lib, c, 0.25, tri)
    for i, (b, w, h) in enumerate(tri):
        np.testing.assert_array_equal(sub[i], full.reshape(B, W, Hq, d)[b, w, h])
        assert lse[i] == lse_full.reshape(B, W, Hq)[b, w, h]


def test_closed_forms(oracle_lib):
    gold = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "closed_forms.json")))
    # equal keys => mean of the value rows (prompt rows and the beam's own rows alike)
    vals = np.array(gold["attention_equal_keys"]["values"], dtype=np.float32)       # 4 rows, d=2
    d = 2
    q = f32_to_bf16_bits(np.array([[[[0.5, -1.5]]]], dtype=np.float32))             # B=W=Hq=1
    k_sh = f32_to_bf16_bits(np.tile(np.array([[[0.25, 2.0]]], dtype=np.float32), (3, 1, 1)))
    v_sh = f32_to_bf16_bits(vals[:3].reshape(3, 1, d))
    k_un = f32_to_bf16_bits(np.tile(np.array([0.25, 2.0], dtype=np.float32), (1, 1, 2, 1, 1)))
    v_un = f32_to_bf16_bits(np.stack([vals[3], np.array([99.0, 99.0], dtype=np.float32)]).reshape(1, 1, 2, 1, d))
    cu = np.array([0, 3], dtype=np.int32)
    out, lse = oracle_lib.attn_unified(q, k_sh, v_sh, cu, k_un, v_un, 1, 0.75)      # only 1 own token valid
    np.testing.assert_allclose(out[0], gold["attention_equal_keys"]["mean"], atol=1e-14)
    s = 0.75 * (0.5 * 0.25 - 1.5 * 2.0)
    assert abs(lse[0] - (s + np.log(4.0))) < 1e-13

    c = _rand_case(4, u=2)
    B, W, Hq, dd = c["q"].shape
    # all value rows equal to one vector => that vector
    vec = f32_to_bf16_bits(np.linspace(-1, 1, dd, dtype=np.float32))
    c2 = dict(c); c2["v_shared"] = np.broadcast_to(vec, c["v_shared"].shape).copy()
    c2["v_unshared"] = np.broadcast_to(vec, c["v_unshared"].shape).copy()
    out, _ = _run(oracle_lib, c2, 0.3125)
    np.testing.assert_allclose(out, np.broadcast_to(bf16_bits_to_f32(vec), out.shape), atol=1e-13)
    # one key aligned with the query and scaled up dominates => its value row (here a decode-token row)
    c3 = dict(c); c3["k_unshared"] = c["k_unshared"].copy()
    b, w, hq = 1, 3, 5
    hk = hq // (Hq // c["k_shared"].shape[1])
    c3["k_unshared"][b, w, 1, hk] = f32_to_bf16_bits(64.0 * bf16_bits_to_f32(c["q"][b, w, hq]))
    out, _ = _run(oracle_lib, c3, 1.0, np.array([[b, w, hq]], dtype=np.int32))
    np.testing.assert_allclose(out[0], bf16_bits_to_f32(c["v_unshared"][b, w, 1, hk]), atol=1e-9)


def test_invariants(oracle_lib):
    c = _rand_case(5, u=2, lens=(11, 6))
    B, W, Hq, d = c["q"].shape
    out, lse = _run(oracle_lib, c, 0.25)
    # permuting the prompt rows of a request (K and V together) changes nothing
    perm = np.concatenate([np.random.default_rng(0).permutation(11), 11 + np.random.default_rng(1).permutation(6)])
    c2 = dict(c); c2["k_shared"] = c["k_shared"][perm].copy(); c2["v_shared"] = c["v_shared"][perm].copy()
    out2, lse2 = _run(oracle_lib, c2, 0.25)
    np.testing.assert_allclose(out2, out, atol=1e-13)
    np.testing.assert_allclose(lse2, lse, atol=1e-13)
    # slots beyond u are ignored
    c3 = dict(c); c3["k_unshared"] = c["k_unshared"].copy(); c3["k_unshared"][:, :, 2] = 0x7F80  # +inf bits
    out3, _ = _run(oracle_lib, c3, 0.25)
    np.testing.assert_array_equal(out3, out)
    # beams with identical queries and identical own tokens give identical outputs
    c4 = {k: (v.copy() if isinstance(v, np.ndarray) else v) for k, v in c.items()}
    c4["q"][:, 1] = c4["q"][:, 0]; c4["k_unshared"][:, 1] = c4["k_unshared"][:, 0]; c4["v_unshared"][:, 1] = c4["v_unshared"][:, 0]
    out4, _ = _run(oracle_lib, c4, 0.25)
    out4 = out4.reshape(B, W, Hq, d)
    np.testing.assert_array_equal(out4[:, 0], out4[:, 1])
    # GQA: query head h reads KV head h // g - changing another KV head leaves it unchanged
    c5 = dict(c); c5["k_shared"] = c["k_shared"].copy(); c5["k_shared"][:, 1] = 0
    out5, _ = _run(oracle_lib, c5, 0.25)
    g = Hq // c["k_shared"].shape[1]
    np.testing.assert_array_equal(out5.reshape(B, W, Hq, d)[:, :, :g], out.reshape(B, W, Hq, d)[:, :, :g])
    assert not np.array_equal(out5.reshape(B, W, Hq, d)[:, :, g:], out.reshape(B, W, Hq, d)[:, :, g:])


# ---- the variant that takes the prompt K/V as fp32 values (narrow storage formats widened by the caller) -------------
def test_f32kv_variant_equals_the_bf16_routine_on_bf16_values(oracle_lib):
    """bf16 values are fp32 values: on them the two routines must agree to the last bit of their fp64 arithmetic."""
    c = _rand_case(21, u=2)
    ref, ref_lse = _run(oracle_lib, c, 0.375)
    got, got_lse = oracle_lib.attn_unified_f32kv(c["q"], bf16_bits_to_f32(c["k_shared"]), bf16_bits_to_f32(c["v_shared"]), c["cu_seqlens"],
                                                 c["k_unshared"], c["v_unshared"], c["u"], 0.375)
    np.testing.assert_array_equal(got, ref)
    np.testing.assert_array_equal(got_lse, ref_lse)


def test_f32kv_variant_matches_torch_sdpa_with_scaled_fp8_values(oracle_lib):
    """FP8 codes times per-tensor scales as the prompt cache, bf16 own tokens: torch's library attention in fp64 on the
    concatenated sequence; and linearity in the V scale (doubling it doubles the prompt's share of the output)."""
    c = _rand_case(22, B=2, W=3, Hq=4, Hkv=2, d=16, u=1, lens=(9, 14))
    k_scale, v_scale = np.float32(0.4375), np.float32(1.75)
    k8 = gr_synth.e4m3_bits_to_f32(gr_synth.f32_to_e4m3_bits(bf16_bits_to_f32(c["k_shared"]) / k_scale)) * k_scale
    v8 = gr_synth.e4m3_bits_to_f32(gr_synth.f32_to_e4m3_bits(bf16_bits_to_f32(c["v_shared"]) / v_scale)) * v_scale
    scale = 0.25
    out, lse = oracle_lib.attn_unified_f32kv(c["q"], k8, v8, c["cu_seqlens"], c["k_unshared"], c["v_unshared"], c["u"], scale)
    B, W, Hq, d = c["q"].shape
    g = Hq // 2
    out = out.reshape(B, W, Hq, d)
    q = torch.from_numpy(bf16_bits_to_f32(c["q"]).astype(np.float64))
    ku = torch.from_numpy(bf16_bits_to_f32(c["k_unshared"]).astype(np.float64))
    vu = torch.from_numpy(bf16_bits_to_f32(c["v_unshared"]).astype(np.float64))
    ks, vs = torch.from_numpy(k8.astype(np.float64)), torch.from_numpy(v8.astype(np.float64))
    for b in range(B):
        lo, hi = int(c["cu_seqlens"][b]), int(c["cu_seqlens"][b + 1])
        for w in range(W):
            k = torch.cat([ks[lo:hi], ku[b, w, :1]], 0).repeat_interleave(g, dim=1)
            v = torch.cat([vs[lo:hi], vu[b, w, :1]], 0).repeat_interleave(g, dim=1)
            ref = torch.nn.functional.scaled_dot_product_attention(q[b, w][None, :, None, :], k.permute(1, 0, 2)[None], v.permute(1, 0, 2)[None], scale=scale)
            np.testing.assert_allclose(out[b, w], ref[0, :, 0, :].numpy(), rtol=0, atol=1e-12)
    # with no own tokens the output is linear in the prompt V values
    o1, _ = oracle_lib.attn_unified_f32kv(c["q"], k8, v8, c["cu_seqlens"], c["k_unshared"], c["v_unshared"], 0, scale)
    o2, _ = oracle_lib.attn_unified_f32kv(c["q"], k8, (2 * v8).astype(np.float32), c["cu_seqlens"], c["k_unshared"], c["v_unshared"], 0, scale)
    np.testing.assert_allclose(o2, 2 * o1, rtol=1e-15, atol=0)


def test_e4m3_helpers_match_torch(oracle_lib):
    """The FP8 E4M3 encode / decode used to build such inputs, against torch's float8_e4m3fn."""
    codes = np.arange(256, dtype=np.uint8)
    mine = gr_synth.e4m3_bits_to_f32(codes)
    ref = torch.from_numpy(codes).view(torch.float8_e4m3fn).float().numpy()
    ok = ~np.isnan(ref)
    np.testing.assert_array_equal(mine[ok], ref[ok])
    assert np.isnan(mine[~ok]).all() and (~ok).sum() == 2
    rng = np.random.default_rng(0)
    x = (rng.standard_normal(100000) * rng.choice([1e-3, 0.1, 1, 10, 100], 100000)).astype(np.float32)
    x = x[np.abs(x) <= 448]
    np.testing.assert_array_equal(gr_synth.f32_to_e4m3_bits(x), torch.from_numpy(x).to(torch.float8_e4m3fn).view(torch.uint8).numpy())
    np.testing.assert_array_equal(gr_synth.f32_to_e4m3_bits(np.array([1e9, -1e9], dtype=np.float32)), [0x7E, 0xFE])      # saturates
