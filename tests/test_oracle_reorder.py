"""Pins for the oracle's unshared-cache reorder (paper Section 5.1).  CPU only.

The gather-into-a-fresh-buffer statement (oracle.unshared_reorder) is pinned by
  * the paper's own in-place procedure (direction indices, upward writes walking down, then the remaining
    writes walking up) as a second, independently written routine: equal results on seeded parent arrays of
    the kind beam order produces (live rows first, parents non-decreasing);
  * algebra that holds for any correct reorder and restates no gather: the identity parent changes nothing,
    a permutation followed by its inverse restores the cache, two reorders in a row equal one reorder by the
    composed parent array, and a cache whose row r is filled with the value r turns into the parent array;
  * the hazard the paper warns about: a strictly downward (or upward) in-place copy loop gets the shift
    patterns wrong, the two-sweep procedure does not.
Every pin is also run against a reorder with an off-by-one planted in its parent lookup and must reject it.
"""
import numpy as np
import pytest


def _cache(rng, B, W, row_shape=(3, 2, 4)):
    return rng.integers(0, 60000, size=(B, W) + row_shape).astype(np.uint16)


def _sorted_parents(rng, B, W, n_dead=0):
    """Parent arrays as beam order gives them: live rows first with non-decreasing parents, dead rows last."""
    p = np.sort(rng.integers(0, W, size=(B, W)), axis=1).astype(np.int32)
    if n_dead:
        p[:, W - n_dead:] = -1
    return p


# ---- the pins, written against any callable reorder(kv, parent) -> kv -------------------------------------
def pin_identity(reorder, rng):
    B, W = 2, 9
    kv = _cache(rng, B, W)
    ident = np.tile(np.arange(W, dtype=np.int32), (B, 1))
    np.testing.assert_array_equal(reorder(kv.copy(), ident), kv)


def pin_permutation_then_inverse(reorder, rng):
    B, W = 3, 17
    kv = _cache(rng, B, W)
    p = np.stack([rng.permutation(W) for _ in range(B)]).astype(np.int32)
    inv = np.argsort(p, axis=1).astype(np.int32)
    np.testing.assert_array_equal(reorder(reorder(kv.copy(), p), inv), kv)


def pin_composition(reorder, rng):
    B, W = 2, 13
    kv = _cache(rng, B, W)
    p = rng.integers(0, W, size=(B, W)).astype(np.int32)
    q = rng.integers(0, W, size=(B, W)).astype(np.int32)
    pq = np.take_along_axis(p, q, axis=1)                  # slot j of the second generation descends from p[q[j]]
    np.testing.assert_array_equal(reorder(reorder(kv.copy(), p), q), reorder(kv.copy(), pq))


def pin_row_labels(reorder, rng):
    B, W = 2, 11
    kv = np.empty((B, W, 2, 1, 4), dtype=np.uint16)
    kv[:] = np.arange(W, dtype=np.uint16)[None, :, None, None, None] + 1      # row r holds r + 1 everywhere
    p = rng.integers(0, W, size=(B, W)).astype(np.int32)
    p[0, 3] = -1
    p[1, W - 1] = -1
    got = reorder(kv.copy(), p)
    assert (got == got[:, :, :1, :1, :1]).all()
    np.testing.assert_array_equal(got[:, :, 0, 0, 0].astype(np.int32) - 1, p)  # dead rows come out as 0 -> -1


def pin_two_sweeps(reorder, two_sweeps, rng):
    for W, n_dead in ((1, 0), (2, 0), (7, 0), (16, 3), (64, 0), (64, 9), (257, 1)):
        B = 3
        kv = _cache(rng, B, W)
        p = _sorted_parents(rng, B, W, n_dead)
        want, direction = two_sweeps(kv.copy(), p)
        np.testing.assert_array_equal(reorder(kv.copy(), p), want, err_msg=f"W={W} dead={n_dead}")
        live = p >= 0
        j = np.tile(np.arange(W), (B, 1))
        np.testing.assert_array_equal(direction, np.where(live, np.sign(p - j), 0))


PINS = [pin_identity, pin_permutation_then_inverse, pin_composition, pin_row_labels]


@pytest.mark.parametrize("pin", PINS, ids=lambda f: f.__name__)
def test_reorder_pin(oracle_lib, pin):
    pin(oracle_lib.unshared_reorder, np.random.default_rng(11))


def test_reorder_equals_the_papers_two_sweep_procedure(oracle_lib):
    pin_two_sweeps(oracle_lib.unshared_reorder, oracle_lib.unshared_reorder_two_sweeps, np.random.default_rng(12))


def test_two_sweep_procedure_satisfies_the_algebra_on_sorted_parents(oracle_lib):
    """The second routine on its own: identity, row labels and composition, restricted to sorted parents."""
    rng = np.random.default_rng(13)
    two = lambda kv, p: oracle_lib.unshared_reorder_two_sweeps(kv, p)[0]
    pin_identity(two, rng)
    B, W = 2, 12
    kv = np.empty((B, W, 1, 1, 8), dtype=np.uint16)
    kv[:] = np.arange(W, dtype=np.uint16)[None, :, None, None, None] + 1
    p = _sorted_parents(rng, B, W, n_dead=2)
    got = two(kv.copy(), p)
    np.testing.assert_array_equal(got[:, :, 0, 0, 0].astype(np.int32) - 1, p)
    q = _sorted_parents(rng, B, W)
    p2 = _sorted_parents(rng, B, W)
    kv = _cache(rng, B, W)
    np.testing.assert_array_equal(two(two(kv.copy(), p2), q), two(kv.copy(), np.take_along_axis(p2, q, axis=1)))


def test_two_sweep_procedure_rejects_unsorted_parents(oracle_lib):
    kv = _cache(np.random.default_rng(0), 1, 4)
    for bad in ([2, 1, 3, 3], [0, -1, 2, 3], [0, 1, 2, 4]):
        before = kv.copy()
        with pytest.raises(ValueError):
            oracle_lib.unshared_reorder_two_sweeps(kv, np.array([bad], dtype=np.int32))
        np.testing.assert_array_equal(kv, before)


def test_naive_sweeps_hit_the_write_before_read_hazard(oracle_lib):
    """Section 5.1: a strictly downward or strictly upward in-place copy overwrites entries before they are read."""
    rng = np.random.default_rng(14)
    W = 8
    kv = _cache(rng, 1, W)

    def naive(order, p):
        a = kv.copy()
        for j in order:
            a[0, j] = a[0, p[0, j]]
        return a

    shift_down = np.array([[0, 0, 1, 2, 3, 4, 5, 6]], dtype=np.int32)      # every block moves one row down
    shift_up = np.array([[1, 2, 3, 4, 5, 6, 7, 7]], dtype=np.int32)        # every block moves one row up
    mixed = np.array([[1, 2, 2, 2, 3, 4, 5, 6]], dtype=np.int32)           # both directions in one array
    for p in (shift_down, shift_up, mixed):
        want = oracle_lib.unshared_reorder(kv.copy(), p)
        got, _ = oracle_lib.unshared_reorder_two_sweeps(kv.copy(), p)
        np.testing.assert_array_equal(got, want)
    assert not np.array_equal(naive(range(W), shift_down), oracle_lib.unshared_reorder(kv.copy(), shift_down))
    assert not np.array_equal(naive(range(W - 1, -1, -1), shift_up), oracle_lib.unshared_reorder(kv.copy(), shift_up))
    assert not np.array_equal(naive(range(W), mixed), oracle_lib.unshared_reorder(kv.copy(), mixed))
    assert not np.array_equal(naive(range(W - 1, -1, -1), mixed), oracle_lib.unshared_reorder(kv.copy(), mixed))


def test_pins_reject_an_off_by_one_gather(oracle_lib):
    """A mistake planted in the parent lookup (row parent+1 instead of row parent) must fail every pin."""
    def mutant(kv, parent):
        W = parent.shape[1]
        return oracle_lib.unshared_reorder(kv, np.where(parent >= 0, (parent + 1) % W, parent).astype(np.int32))

    for pin in PINS:
        with pytest.raises(AssertionError):
            pin(mutant, np.random.default_rng(11))
    with pytest.raises(AssertionError):
        pin_two_sweeps(mutant, oracle_lib.unshared_reorder_two_sweeps, np.random.default_rng(12))
