"""Pins for the oracle's reading of the shuffle the paper inserts into the sorting
of the pairs (Sec. 3, footnote to the sorting step; Sec. 5, data augmentation):
pairs of equal cost are visited in a seeded pseudo-random order.  The hash values
themselves are arbitrary; what is pinned is that the tie-break is a bijection,
that the result equals the (already pinned) index-order procedure run on the
pair list rearranged by that bijection, and the behaviour the paper asks of it
(variation between seeds, none where costs differ).  (CPU only.)
"""
import numpy as np
import pytest

from paper_2103_15076_amd import meshgen


def test_tie_break_is_a_bijection_and_seed_zero_is_the_identity(oracle):
    for i in (0, 1, 2, 12345, 2 ** 31 - 1, 2 ** 32 - 1):
        assert oracle.tie_break(0, i) == i
    for seed in (1, 0xDEADBEEF, 0x1234_5678_9ABC_DEF0):
        vals = np.array([oracle.tie_break(seed, i) for i in range(1 << 16)], np.uint64)
        assert np.unique(vals).size == vals.size
        assert 0 <= vals.min() and vals.max() < 2 ** 32
        # not the identity, and not monotone: neighbours land far apart
        assert (np.diff(vals.astype(np.int64)) < 0).mean() > 0.3
    a = [oracle.tie_break(7, i) for i in range(64)]
    b = [oracle.tie_break(8, i) for i in range(64)]
    assert np.argsort(a).tolist() != np.argsort(b).tolist()


@pytest.mark.parametrize("seed", range(1, 25))
@pytest.mark.parametrize("absorb", [False, True])
def test_shuffled_selection_is_the_index_order_procedure_on_the_rearranged_list(oracle, seed, absorb):
    """Lines 3-11 with the shuffle == the same lines without it on the pair list
    sorted by tie_break(seed, index): the default procedure breaks ties by list
    position, so rearranging the list is all the shuffle may do."""
    rng = np.random.default_rng(seed)
    n = int(rng.integers(4, 40))
    pairs = set()
    while len(pairs) < min(3 * n, n * (n - 1) // 2):
        a, b = rng.integers(0, n, 2)
        if a != b:
            pairs.add((min(a, b), max(a, b)))
    E = np.array(sorted(pairs), np.int32)
    key = rng.integers(0, 4, E.shape[0]).astype(np.uint32)   # few distinct keys: ties everywhere
    n_remove = int(rng.integers(0, n))
    s = 0x9000_0000_0000_0000 + 7919 * seed
    sel, via, removed = oracle.select_shuffled(E, key, n, n_remove, s, absorb)
    perm = np.argsort(np.array([oracle.tie_break(s, i) for i in range(E.shape[0])], np.uint64), kind="stable")
    if absorb:
        sel_p, via_p, removed_p = oracle.select_absorb(E[perm], key[perm], n, n_remove)
        via_back = np.where(via_p >= 0, perm[np.maximum(via_p, 0)], -1)
        assert np.array_equal(via, via_back)
    else:
        sel_p, removed_p = oracle.select(E[perm], key[perm], n, n_remove)
        assert np.all(via == -1)
    back = np.zeros_like(sel)
    back[perm] = sel_p
    assert np.array_equal(sel, back) and removed == removed_p


def test_distinct_costs_leave_no_room_for_the_shuffle(oracle):
    """With no two keys equal the order of the pairs is fixed by the costs alone:
    any seed gives the result of the procedure without shuffle."""
    rng = np.random.default_rng(1)
    V, F = meshgen.icosphere(3, seed=None)
    E = oracle.edges(F)
    key = rng.permutation(E.shape[0]).astype(np.uint32) * np.uint32(3) + np.uint32(5)
    for n_remove in (10, 200, 642):
        ref, n_ref = oracle.select(E, key, V.shape[0], n_remove)
        ref_a, via_a, na = oracle.select_absorb(E, key, V.shape[0], n_remove)
        for seed in (1, 99, 0xABCDEF0123):
            sel, via, n = oracle.select_shuffled(E, key, V.shape[0], n_remove, seed)
            assert np.array_equal(sel, ref) and n == n_ref
            sel, via, n = oracle.select_shuffled(E, key, V.shape[0], n_remove, seed, absorb=True)
            assert np.array_equal(sel, ref_a) and np.array_equal(via, via_a) and n == na


def test_flat_regions_vary_with_the_seed_and_only_with_the_seed(oracle):
    """A flat lattice: every cost is +0, so the shuffle decides everything; the
    budget is still met exactly and the run is reproducible."""
    V, F = meshgen.flat_grid(25, 20, spacing=0.25)
    target = V.shape[0] // 3
    base = oracle.decimate(V, F, target)
    runs = {s: oracle.decimate(V, F, target, shuffle_seed=s) for s in (1, 2, 3, 0xFFFF_FFFF_FFFF_FFFF)}
    again = oracle.decimate(V, F, target, shuffle_seed=2)
    assert np.array_equal(runs[2]["cluster_id"], again["cluster_id"]) and np.array_equal(runs[2]["verts"], again["verts"])
    ids = [base["cluster_id"]] + [r["cluster_id"] for r in runs.values()]
    for i in range(len(ids)):
        for j in range(i + 1, len(ids)):
            assert not np.array_equal(ids[i], ids[j])
    for r in runs.values():
        assert r["status"] == 0 and r["verts"].shape[0] == target
        assert np.abs(r["verts"][:, 2]).max() == 0.0  # still in the plane
        assert np.array_equal(np.unique(r["cluster_id"]), np.arange(target))
