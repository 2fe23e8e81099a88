"""GPU parity: gr_item_mask_build and gr_beam_select against the CPU oracle (Sections 6.1-6.3).

Beam indices, tokens, prefixes, table ranges and item indices must be bit-exact; scores within 1e-5
relative.  Every call goes through the C ABI via the thin binding.
"""
import itertools

import numpy as np
import pytest

import gr_synth
from gpu_util import assert_select_equal, dev, run_select, to_dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gr():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_2512_11529_amd as gr
    gr.load_library()
    return gr


def _random_table(rng, V, n):
    keys = np.sort(rng.choice(V ** 3, size=n, replace=False)).astype(np.int64)
    return np.stack([keys // (V * V), (keys // V) % V, keys % V], axis=1).astype(np.int32)


def _parse_blob(blob, V):
    b = blob.cpu().numpy()
    hdr = b[:256].view(np.int64)
    i32 = b[:16].view(np.int32)
    assert i32[1] == V and i32[2] == 3
    words = int(i32[3])
    n_items, n_pairs = int(hdr[2]), int(hdr[3])
    off = {k: int(hdr[4 + i]) for i, k in enumerate(["l0", "l1", "off1", "pair_off", "pair_t2", "pair_row", "t3", "total"])}
    take = lambda o, n, dt: b[o:o + n * np.dtype(dt).itemsize].view(dt)
    return dict(words=words, n_items=n_items, n_pairs=n_pairs,
                l0=take(off["l0"], words, np.uint32), l1=take(off["l1"], V * words, np.uint32).reshape(V, words),
                off1=take(off["off1"], V + 1, np.int32), pair_off=take(off["pair_off"], V + 1, np.int32),
                pair_t2=take(off["pair_t2"], n_pairs, np.int32), pair_row=take(off["pair_row"], n_pairs + 1, np.int32),
                t3=take(off["t3"], n_items, np.int32))


@pytest.mark.parametrize("V,n", [(5, 40), (37, 3000), (64, 1), (256, 2000), (100, 50000)])
def test_mask_blob_matches_bruteforce(gr, oracle_lib, V, n):
    rng = np.random.default_rng(V + n)
    items = _random_table(rng, V, n)
    m = _parse_blob(gr.gr_item_mask_build(to_dev(items), V), V)
    bit = lambda words, v: (int(words[v >> 5]) >> (v & 31)) & 1
    a0 = oracle_lib.mask_row(items, V, np.zeros(0, np.int32))
    assert [bit(m["l0"], v) for v in range(V)] == [int(a == 0) for a in a0]
    t1s = np.unique(items[:, 0])
    for t1 in list(t1s[:5]) + list(t1s[-3:]) + [int(x) for x in rng.choice(V, 3)]:
        a1 = oracle_lib.mask_row(items, V, np.array([t1], np.int32))
        assert [bit(m["l1"][t1], v) for v in range(V)] == [int(a == 0) for a in a1]
    first = items[:, 0]
    np.testing.assert_array_equal(m["off1"], np.searchsorted(first, np.arange(V + 1), side="left"))
    pairs, pair_first = np.unique(items[:, :2], axis=0, return_index=True)
    assert m["n_pairs"] == len(pairs) and m["n_items"] == n
    np.testing.assert_array_equal(m["pair_t2"], pairs[:, 1])
    np.testing.assert_array_equal(m["pair_row"], np.append(pair_first, n))
    np.testing.assert_array_equal(m["pair_off"], np.searchsorted(pairs[:, 0], np.arange(V + 1), side="left"))
    np.testing.assert_array_equal(m["t3"], items[:, 2])
    assert sum(bin(int(w)).count("1") for w in m["l1"].ravel()) == len(pairs)


def test_mask_build_rejects_bad_tables(gr):
    good = np.array([[0, 1, 2], [0, 1, 3], [2, 0, 0]], dtype=np.int32)
    gr.gr_item_mask_build(to_dev(good), 4)
    for bad in (good[[0, 2, 1]], good[[0, 0, 1]]):
        with pytest.raises(gr.GrError) as e:
            gr.gr_item_mask_build(to_dev(bad), 4)
        assert e.value.status == -4
    with pytest.raises(gr.GrError) as e:
        gr.gr_item_mask_build(to_dev(good), 3)
    assert e.value.status == -4
    neg = good.copy(); neg[0, 0] = -1
    with pytest.raises(gr.GrError):
        gr.gr_item_mask_build(to_dev(neg), 4)


def _three_steps(gr, oracle_lib, items, logits_fn, B, W, V, flags=0, chain="oracle"):
    mask = gr.gr_item_mask_build(to_dev(items), V) if items is not None else None
    sc, pf, rg = gr_synth.initial_beam_state(B, W, 3)
    for step in range(3):
        logits = logits_fn(step)
        want = oracle_lib.beam_select(items, logits, sc, pf, step)
        got = run_select(gr, mask, logits, sc, pf, rg, step, flags)
        assert_select_equal(got, want, f"step {step}")
        sc, pf, rg = want["scores"], want["prefix"], want["range"]
    return want


def test_tiny_config_all_steps(gr, oracle_lib):
    cfg = gr_synth.get_config(1)
    items = gr_synth.make_item_table(cfg)
    want = _three_steps(gr, oracle_lib, items, lambda s: gr_synth.make_logits(cfg, s), cfg.B, cfg.W, cfg.V)
    np.testing.assert_array_equal(items[want["item_index"][0]], want["prefix"][0])


@pytest.mark.parametrize("flags", [0, 1])
@pytest.mark.parametrize("B,W,V,n", [(3, 7, 37, 3000), (2, 24, 200, 20000), (1, 130, 1000, 200000), (4, 33, 8192, 300000),
                                      (2, 5, 4, 30)])
def test_random_shapes_masked(gr, oracle_lib, B, W, V, n, flags):
    rng = np.random.default_rng(B * 1000 + W)
    items = _random_table(rng, V, n)
    _three_steps(gr, oracle_lib, items, lambda s: (2.5 * rng.standard_normal((B, W, V))).astype(np.float32), B, W, V, flags)


@pytest.mark.parametrize("B,W,V", [(2, 16, 256), (1, 100, 999), (3, 64, 8192), (1, 1, 5), (2, 9, 20000), (1, 300, 4096)])
def test_unconstrained_all_beams_live(gr, oracle_lib, B, W, V):
    rng = np.random.default_rng(V)
    logits = (2.0 * rng.standard_normal((B, W, V))).astype(np.float32)
    sc = (-3.0 * rng.random((B, W))).astype(np.float32)
    pf = np.full((B, W, 3), -1, np.int32)
    rg = np.zeros((B, W, 2), np.int32)
    want = oracle_lib.beam_select(None, logits, sc, pf, 0)
    got = run_select(gr, None, logits, sc, pf, rg, 0)
    assert_select_equal(got, want)


def test_maximum_sizes(gr, oracle_lib):
    """The documented limits: W = 2048 beams (more live rows than the selection kernel keeps keys for in
    registers, more survivors than the counting sort takes) and V = 32768 (the widest mask row)."""
    rng = np.random.default_rng(77)
    B, W, V = 1, 2048, 1024
    logits = (2.0 * rng.standard_normal((B, W, V))).astype(np.float32)
    sc = (-3.0 * rng.random((B, W))).astype(np.float32)
    pf = np.full((B, W, 3), -1, np.int32)
    rg = np.zeros((B, W, 2), np.int32)
    assert_select_equal(run_select(gr, None, logits, sc, pf, rg, 0), oracle_lib.beam_select(None, logits, sc, pf, 0))
    items = _random_table(rng, 4096, 400000)
    _three_steps(gr, oracle_lib, items, lambda s: (2.5 * rng.standard_normal((1, 600, 4096))).astype(np.float32), 1, 600, 4096)
    items = _random_table(rng, 32768, 100000)
    _three_steps(gr, oracle_lib, items, lambda s: (2.5 * rng.standard_normal((2, 8, 32768))).astype(np.float32), 2, 8, 32768)
    _three_steps(gr, oracle_lib, items, lambda s: (2.5 * rng.standard_normal((2, 8, 32768))).astype(np.float32), 2, 8, 32768, flags=1)


def test_ties_resolved_by_lowest_flat_index(gr, oracle_lib):
    rng = np.random.default_rng(11)
    B, W, V = 2, 12, 300
    # half-integer logits and equal input scores: thousands of exactly equal candidates
    logits = (np.round(rng.standard_normal((B, W, V)) * 2) / 2).astype(np.float32)
    logits[:, 1] = logits[:, 0]
    sc = np.zeros((B, W), np.float32)
    pf = np.full((B, W, 3), -1, np.int32)
    rg = np.zeros((B, W, 2), np.int32)
    assert_select_equal(run_select(gr, None, logits, sc, pf, rg, 0), oracle_lib.beam_select(None, logits, sc, pf, 0))
    # all candidates equal: the first W flat indices win
    logits[:] = 0.25
    got = run_select(gr, None, logits, sc, pf, rg, 0)
    assert_select_equal(got, oracle_lib.beam_select(None, logits, sc, pf, 0))
    np.testing.assert_array_equal(got["parent"][0], np.zeros(W)); np.testing.assert_array_equal(got["token"][0], np.arange(W))


@pytest.mark.parametrize("W,V,levels", [(64, 1024, 1), (40, 8192, 3), (256, 2048, 7)])
def test_massive_ties_take_the_exact_fallback(gr, oracle_lib, W, V, levels):
    # tens of thousands of exactly equal candidates: the survivors cannot fit in LDS, so the exact
    # radix select over all candidates must produce the same beams
    rng = np.random.default_rng(W + V)
    logits = rng.integers(0, levels, size=(2, W, V)).astype(np.float32)
    sc = np.zeros((2, W), np.float32)
    sc[1] = -np.round(rng.random(W) * 2)
    pf = np.full((2, W, 3), -1, np.int32)
    rg = np.zeros((2, W, 2), np.int32)
    assert_select_equal(run_select(gr, None, logits, sc, pf, rg, 0), oracle_lib.beam_select(None, logits, sc, pf, 0))


def test_dead_beams_and_fewer_candidates_than_slots(gr, oracle_lib):
    items = np.array([[0, 0, 0], [0, 0, 1], [2, 1, 1]], dtype=np.int32)
    rng = np.random.default_rng(3)
    B, W, V = 2, 5, 3
    _three_steps(gr, oracle_lib, items, lambda s: rng.standard_normal((B, W, V)).astype(np.float32), B, W, V)
    # every beam dead
    mask = gr.gr_item_mask_build(to_dev(items), V)
    sc = np.full((B, W), -np.inf, np.float32)
    pf = np.full((B, W, 3), -1, np.int32); rg = np.zeros((B, W, 2), np.int32)
    logits = rng.standard_normal((B, W, V)).astype(np.float32)
    assert_select_equal(run_select(gr, mask, logits, sc, pf, rg, 0), oracle_lib.beam_select(items, logits, sc, pf, 0))


def test_argument_errors_are_reported_not_crashes(gr):
    import torch
    B, W, V = 1, 4, 8
    logits = torch.zeros((B, W, V), device=dev())
    sc = torch.zeros((B, W), device=dev())
    pf = torch.full((B, W, 3), -1, dtype=torch.int32, device=dev())
    rg = torch.zeros((B, W, 2), dtype=torch.int32, device=dev())
    with pytest.raises(gr.GrError) as e:
        gr.gr_beam_select(None, logits, sc, pf, rg, 3)
    assert e.value.status == -1
    with pytest.raises(gr.GrError) as e:
        gr.gr_beam_select(None, logits, sc, pf, rg, 0, out=dict(prefix=pf))
    assert e.value.status == -1
    with pytest.raises(gr.GrError) as e:
        gr.gr_beam_select(None, logits, sc, pf, rg, 0, workspace=torch.empty(256, dtype=torch.uint8, device=dev())[:16])
    assert e.value.status in (-1, -3)
