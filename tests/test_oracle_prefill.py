"""Pins for the oracle's causal prompt attention (paper Sections 2.2.1 and 5.1: the prefill that fills the
shared cache).  CPU only.

The oracle states the definition row by row.  It is pinned against
  (a) torch's library attention with its own causal masking (is_causal=True) on each request and head;
  (b) the decode-side oracle routine, already pinned elsewhere: the LAST token of a prompt sees every key, so its
      row equals unified attention of one beam with no own tokens over the same prompt;
  (c) closed forms: token 0 returns v_0 exactly; with all keys equal, token i returns the mean of v_0..v_i and
      lse = s + log(i + 1);
  (d) causality as an invariant: changing K/V (or Q) rows after position i leaves row i unchanged, and changing
      row i's own key changes it;
  (e) packing: a request computed alone equals the same request inside a packed batch.
Each pin is also run against planted mistakes (a strict j < i limit, keys of the neighbouring request, a wrong KV
head) and must reject them.
"""
import numpy as np
import pytest
import torch

from gr_synth import bf16_bits_to_f32, f32_to_bf16_bits


def _case(seed, lens=(5, 19, 1, 33), Hq=4, Hkv=2, d=16):
    rng = np.random.default_rng(seed)
    cu = np.zeros(len(lens) + 1, dtype=np.int32)
    cu[1:] = np.cumsum(lens)
    bf = lambda *s: f32_to_bf16_bits(rng.standard_normal(s, dtype=np.float32))
    T = int(cu[-1])
    return dict(q=bf(T, Hq, d), k=bf(T, Hkv, d), v=bf(T, Hkv, d), cu=cu)


def _all(fn, c, scale):
    out, lse = fn(c["q"], c["k"], c["v"], c["cu"], scale)
    rows = [(b, i, h) for b in range(len(c["cu"]) - 1) for i in range(int(c["cu"][b + 1] - c["cu"][b])) for h in range(c["q"].shape[1])]
    return {r: (out[n], lse[n]) for n, r in enumerate(rows)}


# ---- pins, written against any fn(q, k, v, cu, scale, triples=None) -> (out, lse) ---------------------------
def pin_torch_causal(fn, seed=3):
    c = _case(seed)
    scale = 0.3125
    got = _all(fn, c, scale)
    Hq, d = c["q"].shape[1:]
    g = Hq // c["k"].shape[1]
    q = torch.from_numpy(bf16_bits_to_f32(c["q"]).astype(np.float64))
    k = torch.from_numpy(bf16_bits_to_f32(c["k"]).astype(np.float64)).repeat_interleave(g, dim=1)
    v = torch.from_numpy(bf16_bits_to_f32(c["v"]).astype(np.float64)).repeat_interleave(g, dim=1)
    for b in range(len(c["cu"]) - 1):
        lo, hi = int(c["cu"][b]), int(c["cu"][b + 1])
        ref = torch.nn.functional.scaled_dot_product_attention(q[lo:hi].permute(1, 0, 2)[None], k[lo:hi].permute(1, 0, 2)[None],
                                                               v[lo:hi].permute(1, 0, 2)[None], is_causal=True, scale=scale)[0]
        for i in range(hi - lo):
            for h in range(Hq):
                np.testing.assert_allclose(got[(b, i, h)][0], ref[h, i].numpy(), rtol=0, atol=1e-12, err_msg=f"b={b} i={i} h={h}")


def pin_last_token_equals_decode_oracle(fn, attn_unified, seed=4):
    c = _case(seed)
    scale = 0.25
    got = _all(fn, c, scale)
    T, Hq, d = c["q"].shape
    Hkv = c["k"].shape[1]
    B = len(c["cu"]) - 1
    # one beam per request whose query is the prompt's last token; no own tokens (u = 0)
    q_last = np.stack([c["q"][int(c["cu"][b + 1]) - 1] for b in range(B)])[:, None]        # [B, 1, Hq, d]
    empty = np.zeros((B, 1, 1, Hkv, d), dtype=np.uint16)
    ref, ref_lse = attn_unified(q_last, c["k"], c["v"], c["cu"], empty, empty, 0, scale)
    ref = ref.reshape(B, Hq, d)
    ref_lse = ref_lse.reshape(B, Hq)
    for b in range(B):
        i = int(c["cu"][b + 1] - c["cu"][b]) - 1
        for h in range(Hq):
            np.testing.assert_allclose(got[(b, i, h)][0], ref[b, h], rtol=0, atol=1e-13)
            np.testing.assert_allclose(got[(b, i, h)][1], ref_lse[b, h], rtol=0, atol=1e-12)


def pin_closed_forms(fn, seed=5):
    c = _case(seed, lens=(9, 4))
    scale = 0.5
    # every key of a request equal to one vector: uniform weights over the visible prefix
    for b in range(2):
        lo, hi = int(c["cu"][b]), int(c["cu"][b + 1])
        c["k"][lo:hi] = c["k"][lo]
    got = _all(fn, c, scale)
    Hq = c["q"].shape[1]
    g = Hq // c["k"].shape[1]
    vf = bf16_bits_to_f32(c["v"]).astype(np.float64)
    qf = bf16_bits_to_f32(c["q"]).astype(np.float64)
    kf = bf16_bits_to_f32(c["k"]).astype(np.float64)
    for b in range(2):
        lo, hi = int(c["cu"][b]), int(c["cu"][b + 1])
        for i in range(hi - lo):
            for h in range(Hq):
                out, lse = got[(b, i, h)]
                np.testing.assert_allclose(out, vf[lo:lo + i + 1, h // g].mean(axis=0), rtol=0, atol=1e-13)
                s = scale * float(qf[lo + i, h] @ kf[lo, h // g])
                np.testing.assert_allclose(lse, s + np.log(i + 1), rtol=0, atol=1e-12)
    # token 0 sees only itself: its value row comes back bit for bit
    c2 = _case(seed + 1)
    got2 = _all(fn, c2, scale)
    v2 = bf16_bits_to_f32(c2["v"]).astype(np.float64)
    for b in range(len(c2["cu"]) - 1):
        for h in range(Hq):
            np.testing.assert_array_equal(got2[(b, 0, h)][0], v2[int(c2["cu"][b]), h // g])


def pin_causality(fn, seed=6):
    c = _case(seed, lens=(12, 7))
    scale = 0.4375
    base = _all(fn, c, scale)
    i0 = 5
    lo = int(c["cu"][0])
    rng = np.random.default_rng(99)
    later = dict(c, k=c["k"].copy(), v=c["v"].copy(), q=c["q"].copy())
    for name in ("k", "v", "q"):
        later[name][lo + i0 + 1:int(c["cu"][1])] = f32_to_bf16_bits(rng.standard_normal(later[name][lo + i0 + 1:int(c["cu"][1])].shape).astype(np.float32))
    got = _all(fn, later, scale)
    Hq = c["q"].shape[1]
    for i in range(i0 + 1):
        for h in range(Hq):
            np.testing.assert_array_equal(got[(0, i, h)][0], base[(0, i, h)][0])
    for i in range(7):                                   # the other request is untouched
        for h in range(Hq):
            np.testing.assert_array_equal(got[(1, i, h)][0], base[(1, i, h)][0])
    own = dict(c, k=c["k"].copy())
    own["k"][lo + i0] = f32_to_bf16_bits(rng.standard_normal(own["k"][lo + i0].shape).astype(np.float32))
    got = _all(fn, own, scale)
    assert all(not np.array_equal(got[(0, i0, h)][0], base[(0, i0, h)][0]) for h in range(Hq)), "a token must see its own key"


def pin_packing(fn, seed=7):
    c = _case(seed)
    scale = 0.34375
    packed = _all(fn, c, scale)
    for b in range(len(c["cu"]) - 1):
        lo, hi = int(c["cu"][b]), int(c["cu"][b + 1])
        alone = dict(q=np.ascontiguousarray(c["q"][lo:hi]), k=np.ascontiguousarray(c["k"][lo:hi]), v=np.ascontiguousarray(c["v"][lo:hi]),
                     cu=np.array([0, hi - lo], dtype=np.int32))
        solo = _all(fn, alone, scale)
        for (bb, i, h), (o, l) in solo.items():
            np.testing.assert_array_equal(packed[(b, i, h)][0], o)
            assert packed[(b, i, h)][1] == l


def test_prefill_oracle_matches_torch_causal_attention(oracle_lib):
    pin_torch_causal(oracle_lib.prefill_attn_causal)


def test_prefill_oracle_last_token_equals_decode_oracle(oracle_lib):
    pin_last_token_equals_decode_oracle(oracle_lib.prefill_attn_causal, oracle_lib.attn_unified)


def test_prefill_oracle_closed_forms(oracle_lib):
    pin_closed_forms(oracle_lib.prefill_attn_causal)


def test_prefill_oracle_is_causal_and_sees_itself(oracle_lib):
    pin_causality(oracle_lib.prefill_attn_causal)


def test_prefill_oracle_packing(oracle_lib):
    pin_packing(oracle_lib.prefill_attn_causal)


def test_prefill_oracle_rejects_bad_rows(oracle_lib):
    c = _case(1)
    for bad in ([[0, 5, 0]], [[4, 0, 0]], [[0, 0, 4]], [[0, -1, 0]]):      # request 0 has 5 tokens, 4 requests, 4 heads
        with pytest.raises(RuntimeError):
            oracle_lib.prefill_attn_causal(c["q"], c["k"], c["v"], c["cu"], 0.3, np.array(bad, dtype=np.int32))


def test_prefill_pins_reject_planted_mistakes(oracle_lib):
    """Mutants built on the oracle in numpy fp64: each must fail at least the pin aimed at it, and every mutant must
    fail the library comparison."""
    def make(limit, kv_head, row_shift):
        def fn(q, k, v, cu, scale, triples=None):
            qf, kf, vf = (bf16_bits_to_f32(x).astype(np.float64) for x in (q, k, v))
            Hq, d = q.shape[1:]
            g = Hq // k.shape[1]
            outs, lses = [], []
            for b in range(len(cu) - 1):
                lo, hi = int(cu[b]), int(cu[b + 1])
                for i in range(hi - lo):
                    for h in range(Hq):
                        n = max(limit(i), 1)
                        start = max(lo + row_shift, 0)
                        s = scale * (kf[start:start + n, kv_head(h, g)] @ qf[lo + i, h])
                        p = np.exp(s - s.max())
                        outs.append(p @ vf[start:start + n, kv_head(h, g)] / p.sum())
                        lses.append(s.max() + np.log(p.sum()))
            return np.array(outs), np.array(lses)
        return fn

    good = make(lambda i: i + 1, lambda h, g: h // g, 0)
    pin_torch_causal(good); pin_closed_forms(good); pin_causality(good); pin_packing(good)          # the harness itself is sound
    strict = make(lambda i: i, lambda h, g: h // g, 0)               # a token does not see itself
    full = make(lambda i: 10 ** 6, lambda h, g: h // g, 0)           # no causal limit (numpy slicing clips at the array end)
    head = make(lambda i: i + 1, lambda h, g: h % 2, 0)              # wrong query-head -> KV-head map
    shifted = make(lambda i: i + 1, lambda h, g: h // g, -1)         # keys start one row early: leaks the previous request
    for name, m in (("strict", strict), ("full", full), ("head", head), ("shifted", shifted)):
        with pytest.raises(AssertionError):
            pin_torch_causal(m)
    with pytest.raises(AssertionError):
        pin_causality(strict)
    with pytest.raises(AssertionError):
        pin_causality(full)
    with pytest.raises(AssertionError):
        pin_closed_forms(head)
    with pytest.raises(AssertionError):
        pin_packing(shifted)
