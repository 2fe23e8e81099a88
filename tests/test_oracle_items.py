"""Pins for the oracle's item step (paper Sections 2.2.1, 6.1, 6.2).  CPU only.

Mask: brute-force membership.  Masked log-softmax: closed forms and torch.log_softmax.
Selection: numpy lexsort on tiny inputs, the paper's min-heap early-termination walk as a second
implementation, invariants, and brute-force enumeration of every item's total score.
"""
import itertools
import json
import os

import numpy as np
import pytest
import torch

import gr_synth


def _random_table(rng, V, depth, n):
    allrows = np.array(list(itertools.product(range(V), repeat=depth)), dtype=np.int32)
    pick = np.sort(rng.choice(len(allrows), size=n, replace=False))
    return allrows[pick]


def _f32(x):
    return np.asarray(x, dtype=np.float32)


# ------------------------------------------------------------------ mask (Section 6.1)
@pytest.mark.parametrize("V,depth,n", [(5, 3, 17), (8, 3, 60), (16, 2, 40), (3, 3, 27)])
def test_mask_rows_equal_bruteforce_membership(oracle_lib, V, depth, n):
    rng = np.random.default_rng(V * 100 + n)
    items = _random_table(rng, V, depth, n)
    assert oracle_lib.check_table(items, V) == 0
    rows = {tuple(r) for r in items.tolist()}
    for plen in range(depth):
        for prefix in itertools.product(range(V), repeat=plen):
            a = oracle_lib.mask_row(items, V, np.array(prefix, dtype=np.int32))
            for v in range(V):
                want = any(r[:plen + 1] == prefix + (v,) for r in rows)
                assert (a[v] == 0.0) == want and (a[v] == 0.0 or a[v] == -np.inf)
    # counting invariants
    a0 = oracle_lib.mask_row(items, V, np.zeros(0, dtype=np.int32))
    assert int((a0 == 0).sum()) == len(np.unique(items[:, 0]))


def test_check_table_rejects_bad_tables(oracle_lib):
    good = np.array([[0, 1, 2], [0, 1, 3], [2, 0, 0]], dtype=np.int32)
    assert oracle_lib.check_table(good, 4) == 0
    assert oracle_lib.check_table(good[[0, 2, 1]], 4) == 3          # unsorted
    assert oracle_lib.check_table(good[[0, 0, 1]], 4) == 2          # duplicate
    assert oracle_lib.check_table(good, 3) == 2                     # token 3 out of range for V=3
    bad = good.copy(); bad[0, 0] = -1
    assert oracle_lib.check_table(bad, 4) == 1


# ------------------------------------------------------------------ masked log-softmax (Sections 6.1, 6.2)
def test_logprob_closed_forms(oracle_lib):
    gold = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "closed_forms.json")))
    V, depth = 4, 3
    for case in gold["uniform_logprob"]["cases"]:
        n = case["n_valid"]
        items = np.array([[t, 0, 0] for t in range(n)], dtype=np.int32)
        logits = np.full((1, 1, V), 1.25, dtype=np.float32)
        logits[0, 0, n:] = 50.0                                      # invalid tokens must not matter
        r = oracle_lib.beam_select(items, logits, _f32([[0.0]]), np.full((1, 1, depth), -1, np.int32), 0)
        assert r["token"][0, 0] == 0 and r["parent"][0, 0] == 0
        assert abs(float(r["scores"][0, 0]) - case["logprob"]) < 1e-7
    two = gold["two_token_softmax"]
    items = np.array([[0, 0, 0], [1, 0, 0]], dtype=np.int32)
    logits = np.zeros((1, 2, V), dtype=np.float32)
    logits[0, :, :2] = _f32(two["logits"])
    logits[0, :, 2:] = 9.0
    scores_in = _f32([[-1.5, -2.5]])
    r = oracle_lib.beam_select(items, logits, scores_in, np.full((1, 2, depth), -1, np.int32), 0)
    want = sorted([(-1.5 + two["logprobs"][0], 0, 0), (-1.5 + two["logprobs"][1], 0, 1),
                   (-2.5 + two["logprobs"][0], 1, 0), (-2.5 + two["logprobs"][1], 1, 1)], reverse=True)[:2]
    for j in range(2):
        assert abs(float(r["scores"][0, j]) - want[j][0]) < 1e-6
        assert (int(r["parent"][0, j]), int(r["token"][0, j])) == want[j][1:]


def test_all_valid_equals_torch_log_softmax_and_probabilities_sum_to_one(oracle_lib):
    rng = np.random.default_rng(7)
    B, W, V = 2, 6, 37
    logits = _f32(3.0 * rng.standard_normal((B, W, V)))
    scores_in = _f32(-rng.random((B, W)) * 4)
    # W' = W*V output slots so every candidate is returned
    big_scores = np.full((B, W * V), -np.inf, np.float32); big_scores[:, :W] = scores_in
    big_logits = np.zeros((B, W * V, V), np.float32); big_logits[:, :W] = logits
    r = oracle_lib.beam_select(None, big_logits, big_scores, np.full((B, W * V, 3), -1, np.int32), 0)
    lp = torch.log_softmax(torch.from_numpy(logits.astype(np.float64)), dim=-1).numpy()
    for b in range(B):
        got = np.full((W, V), np.nan)
        got[r["parent"][b], r["token"][b]] = r["scores"][b]
        assert not np.isnan(got).any()
        np.testing.assert_allclose(got, scores_in[b][:, None] + lp[b], rtol=0, atol=2e-6)
        np.testing.assert_allclose(np.exp(got.astype(np.float64) - scores_in[b][:, None]).sum(-1), 1.0, atol=1e-5)
        assert (np.diff(r["scores"][b]) <= 0).all()


def test_masked_probabilities_renormalise_over_valid_tokens(oracle_lib):
    rng = np.random.default_rng(8)
    V, depth = 8, 3
    items = _random_table(rng, V, depth, 90)
    W = 64
    logits = _f32(2.0 * rng.standard_normal((1, W, V)))
    sc, pf, _ = gr_synth.initial_beam_state(1, W, depth)
    r0 = oracle_lib.beam_select(items, logits, sc, pf, 0)
    n_live = int((r0["scores"][0] > -np.inf).sum())
    assert n_live == len(np.unique(items[:, 0]))
    np.testing.assert_allclose(np.exp(r0["scores"][0, :n_live].astype(np.float64)).sum(), 1.0, atol=1e-6)
    # a prefix with a single valid child: log-prob 0, score carried over to within an ulp
    items1 = np.array([[0, 3, 1], [1, 2, 2], [1, 2, 5]], dtype=np.int32)
    pf = np.full((1, 2, depth), -1, np.int32); pf[0, 0, 0] = 0; pf[0, 1, 0] = 1
    r = oracle_lib.beam_select(items1, logits[:, :2], _f32([[-3.25, -0.5]]), pf, 1)
    assert list(r["token"][0]) == [2, 3] and list(r["parent"][0]) == [1, 0]
    assert abs(float(r["scores"][0, 1]) + 3.25) <= 4e-7 and abs(float(r["scores"][0, 0]) + 0.5) <= 1e-7
    np.testing.assert_array_equal(r["range"][0], [[1, 3], [0, 1]])


# ------------------------------------------------------------------ selection (Section 6.2)
def _numpy_candidates(logits, scores_in, valid):
    """Independent statement of the candidate scores, used only to order them with lexsort."""
    W, V = logits.shape
    cand = np.full((W, V), -np.inf, dtype=np.float32)
    for w in range(W):
        if not scores_in[w] > -np.inf or not valid[w].any():
            continue
        x = logits[w]
        m = x[valid[w]].max()
        S = np.exp(x[valid[w]].astype(np.float64) - np.float64(m)).sum()
        lse = np.float32(np.float64(m) + np.log(S))
        bias = np.float32(scores_in[w] - lse)
        cand[w, valid[w]] = (bias + x[valid[w]]).astype(np.float32)
    return cand


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_selection_equals_lexsort_and_heap_walk(oracle_lib, seed):
    rng = np.random.default_rng(seed)
    V, depth, W, B = 11, 3, 7, 3
    items = _random_table(rng, V, depth, 200)
    sc, pf, _ = gr_synth.initial_beam_state(B, W, depth)
    for step in range(depth):
        # coarse logits => many exact ties, so the tie-break rule is exercised
        logits = _f32(np.round(2.0 * rng.standard_normal((B, W, V)) * 2) / 2)
        r = oracle_lib.beam_select(items, logits, sc, pf, step)
        h = oracle_lib.beam_select_heap(items, logits, sc, pf, step)
        for k in r:
            np.testing.assert_array_equal(r[k], h[k], err_msg=k)
        rows = {tuple(x) for x in items.tolist()}
        for b in range(B):
            valid = np.zeros((W, V), bool)
            for w in range(W):
                if sc[b, w] > -np.inf:
                    pre = tuple(pf[b, w, :step])
                    valid[w] = [any(t[:step + 1] == pre + (v,) for t in rows) for v in range(V)]
            cand = _numpy_candidates(logits[b], sc[b], valid).ravel()
            order = np.lexsort((np.arange(W * V), -cand.astype(np.float64)))[:W]
            n_fin = int(np.isfinite(cand[order]).sum())
            np.testing.assert_array_equal(r["parent"][b, :n_fin], order[:n_fin] // V)
            np.testing.assert_array_equal(r["token"][b, :n_fin], order[:n_fin] % V)
            np.testing.assert_array_equal(r["scores"][b, :n_fin], cand[order[:n_fin]])
            assert (r["parent"][b, n_fin:] == -1).all() and (r["token"][b, n_fin:] == -1).all()
            assert (r["scores"][b, n_fin:] == -np.inf).all()
            assert h["visited"][b] <= valid.sum()
        sc, pf = r["scores"], r["prefix"]


def test_early_termination_visits_fewer_leaves(oracle_lib):
    cfg = gr_synth.get_config(1)
    items = gr_synth.make_item_table(cfg)
    sc, pf, _ = gr_synth.initial_beam_state(cfg.B, cfg.W, cfg.ND)
    total_visited = total_valid = 0
    for step in range(cfg.ND):
        logits = gr_synth.make_logits(cfg, step)
        r = oracle_lib.beam_select(items, logits, sc, pf, step)
        h = oracle_lib.beam_select_heap(items, logits, sc, pf, step)
        for k in r:
            np.testing.assert_array_equal(r[k], h[k], err_msg=k)
        for w in range(cfg.W):
            if sc[0, w] > -np.inf:
                total_valid += int((oracle_lib.mask_row(items, cfg.V, pf[0, w, :step]) == 0).sum())
        total_visited += int(h["visited"][0])
        sc, pf = r["scores"], r["prefix"]
    assert total_visited < total_valid


def test_ties_go_to_the_lowest_flat_index(oracle_lib):
    W, V = 4, 6
    logits = np.zeros((1, W, V), np.float32)
    scores_in = np.zeros((1, W), np.float32)
    r = oracle_lib.beam_select(None, logits, scores_in, np.full((1, W, 3), -1, np.int32), 0)
    np.testing.assert_array_equal(r["parent"][0], [0, 0, 0, 0])
    np.testing.assert_array_equal(r["token"][0], [0, 1, 2, 3])
    # a strictly better candidate late in flat order still comes first
    logits[0, 3, 5] = 1.0
    r = oracle_lib.beam_select(None, logits, scores_in, np.full((1, W, 3), -1, np.int32), 0)
    assert (r["parent"][0, 0], r["token"][0, 0]) == (3, 5)
    np.testing.assert_array_equal(r["parent"][0, 1:], [0, 0, 0])
    np.testing.assert_array_equal(r["token"][0, 1:], [0, 1, 2])


def test_dead_beams_and_short_candidate_lists(oracle_lib):
    items = np.array([[0, 0, 0], [0, 0, 1], [2, 1, 1]], dtype=np.int32)
    W, V, depth = 5, 3, 3
    rng = np.random.default_rng(3)
    logits = _f32(rng.standard_normal((1, W, V)))
    sc, pf, _ = gr_synth.initial_beam_state(1, W, depth)
    r = oracle_lib.beam_select(items, logits, sc, pf, 0)
    assert sorted(r["token"][0, :2].tolist()) == [0, 2] and (r["token"][0, 2:] == -1).all()
    assert (r["scores"][0, 2:] == -np.inf).all() and (r["range"][0, 2:] == 0).all() and (r["prefix"][0, 2:] == -1).all()
    # dead beams (-inf) never parent anything, even with huge logits
    logits2 = logits.copy(); logits2[0, 2:] = 100.0
    r1 = oracle_lib.beam_select(items, logits2, r["scores"], r["prefix"], 1)
    assert set(r1["parent"][0, :2].tolist()) == {0, 1} and (r1["parent"][0, 2:] == -1).all()


def _run_beam_search(oracle_lib, items, V, depth, W, tables):
    """Three steps with logits that depend only on the beam's prefix."""
    sc, pf, _ = gr_synth.initial_beam_state(1, W, depth)
    for step in range(depth):
        logits = np.zeros((1, W, V), np.float32)
        for w in range(W):
            if sc[0, w] > -np.inf:
                logits[0, w] = tables[step][tuple(pf[0, w, :step])]
        r = oracle_lib.beam_select(items, logits, sc, pf, step)
        sc, pf = r["scores"], r["prefix"]
    return r


@pytest.mark.parametrize("seed", [0, 1])
def test_beam_search_equals_bruteforce_enumeration_of_item_scores(oracle_lib, seed):
    """W at least the number of valid prefixes at every level => nothing is pruned, so the final
    list is every item ordered by its total log-probability (each level renormalised over the valid
    children of the prefix)."""
    rng = np.random.default_rng(100 + seed)
    V, depth, n = 6, 3, 40
    items = _random_table(rng, V, depth, n)
    tables = [{p: _f32(2.0 * rng.standard_normal(V)) for p in itertools.product(range(V), repeat=k)} for k in range(depth)]
    W = 48
    r = _run_beam_search(oracle_lib, items, V, depth, W, tables)
    rows = [tuple(x) for x in items.tolist()]
    total = []
    for it in rows:
        s = 0.0
        for k in range(depth):
            pre = it[:k]
            children = sorted({x[k] for x in rows if x[:k] == pre})
            x = tables[k][pre].astype(np.float64)
            s += x[it[k]] - np.log(np.exp(x[children]).sum())
        total.append(s)
    order = sorted(range(n), key=lambda i: -total[i])
    got_items = [tuple(x) for x in r["prefix"][0, :n].tolist()]
    got_scores = r["scores"][0, :n].astype(np.float64)
    np.testing.assert_allclose(got_scores, [total[i] for i in order], atol=5e-6)
    for j, i in enumerate(order):
        # positions whose neighbours are clearly separated must hold exactly that item
        lo = total[order[j - 1]] - total[i] if j > 0 else 1.0
        hi = total[i] - total[order[j + 1]] if j + 1 < n else 1.0
        if lo > 1e-4 and hi > 1e-4:
            assert got_items[j] == rows[i]
    assert sorted(got_items) == sorted(rows)
    np.testing.assert_array_equal(items[r["item_index"][0, :n]], r["prefix"][0, :n])
    assert (r["scores"][0, n:] == -np.inf).all() and (r["item_index"][0, n:] == -1).all()


def test_invariants_on_tiny_config(oracle_lib):
    cfg = gr_synth.get_config(1)
    items = gr_synth.make_item_table(cfg)
    rows = {tuple(x) for x in items.tolist()}
    prefixes = [{r[:k + 1] for r in rows} for k in range(cfg.ND)]
    sc, pf, _ = gr_synth.initial_beam_state(cfg.B, cfg.W, cfg.ND)
    for step in range(cfg.ND):
        r = oracle_lib.beam_select(items, gr_synth.make_logits(cfg, step), sc, pf, step)
        s = r["scores"][0]
        assert (np.diff(s) <= 0).all() and np.isfinite(s).all()
        pairs = list(zip(r["parent"][0].tolist(), r["token"][0].tolist()))
        assert len(set(pairs)) == cfg.W
        for j in range(cfg.W):
            assert sc[0, r["parent"][0, j]] > -np.inf
            assert tuple(r["prefix"][0, j, :step + 1]) in prefixes[step]
            lo, hi = r["range"][0, j]
            assert hi > lo and all(tuple(items[i, :step + 1]) == tuple(r["prefix"][0, j, :step + 1]) for i in (lo, hi - 1))
            assert (lo == 0 or tuple(items[lo - 1, :step + 1]) != tuple(r["prefix"][0, j, :step + 1]))
            assert (hi == len(items) or tuple(items[hi, :step + 1]) != tuple(r["prefix"][0, j, :step + 1]))
        sc, pf = r["scores"], r["prefix"]
    np.testing.assert_array_equal(items[r["item_index"][0]], r["prefix"][0])
