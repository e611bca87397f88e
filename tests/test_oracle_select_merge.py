"""Pins for Stage I pruning, the SetA/SetB split, Eq. 3-10 and the merge."""
import itertools

import numpy as np
import pytest

from oracle import tokencarve_oracle as orc
from tests.helpers_cpu import best_subset_by_sum


def test_topk_equals_best_subset_by_enumeration(rng):
    for n, k in ((10, 4), (14, 7), (16, 5)):
        E = rng.standard_normal(n)
        order = orc.select_topk(E, k)
        assert set(order.tolist()) == best_subset_by_sum(E, k)
        assert np.all(np.diff(E[order]) <= 0)


def test_topk_ties_go_to_lower_index_and_is_permutation_equivariant(rng):
    E = np.array([0.5, 0.9, 0.5, 0.9, 0.1, 0.5])
    np.testing.assert_array_equal(orc.select_topk(E, 5), [1, 3, 0, 2, 5])
    E = rng.standard_normal(30)
    perm = rng.permutation(30)
    assert set(perm[orc.select_topk(E[perm], 11)]) == set(orc.select_topk(E, 11))


def test_split_is_top_half_and_bottom_half(rng):
    order = orc.select_topk(rng.standard_normal(40), 17)
    A, B = orc.split_sets(order)
    assert len(A) == 8 and len(B) == 9
    np.testing.assert_array_equal(np.concatenate([A, B]), order)


def test_similarity_is_cosine_and_equals_normalised_gram(rng):
    Zm = rng.standard_normal((12, 20))
    A, B = np.array([0, 3, 5]), np.array([1, 2, 7, 9])
    sim = orc.similarity(Zm, A, B)
    assert sim.shape == (4, 3)
    G = Zm @ Zm.T
    for j, b in enumerate(B):
        for i, a in enumerate(A):
            assert abs(sim[j, i] - G[b, a] / np.sqrt(G[b, b] * G[a, a])) < 1e-13
    assert np.all(np.abs(sim) <= 1 + 1e-13)
    np.testing.assert_allclose(np.diag(orc.similarity(Zm, A, A)), 1.0, rtol=1e-13)
    np.testing.assert_allclose(orc.similarity(3.0 * Zm, A, B), sim, rtol=1e-12)   # scale free


def _brute_force_merge(X, Zm, order, k_final):
    """Every Set-B token points at its most similar Set-A token; the merged set maximises the
    summed similarity over all subsets of the required size (enumeration)."""
    A, B = orc.split_sets(order)
    m = len(order) - k_final
    cos = lambda u, v: float(u @ v / (np.linalg.norm(u) * np.linalg.norm(v)))
    best, val = {}, {}
    for b in B:
        sims = [(cos(Zm[b], Zm[a]), -a) for a in A]
        top = max(sims)
        best[b], val[b] = -top[1], top[0]
    choice = max(itertools.combinations(sorted(B), m), key=lambda c: sum(val[b] for b in c))
    groups = {a: [a] for a in A}
    for b in choice:
        groups[best[b]].append(b)
    for b in B:
        if b not in choice:
            groups[b] = [b]
    kept = sorted(groups)
    return kept, np.stack([X[groups[a]].mean(axis=0) for a in kept]), set(choice)


@pytest.mark.parametrize("seed", range(6))
def test_merge_matches_brute_force_assignment(seed):
    g = np.random.default_rng(100 + seed)
    n, kp, kf = 14, 9, 6
    X, Zm = g.standard_normal((n, 5)), g.standard_normal((n, 7))
    order = orc.select_topk(g.standard_normal(n), kp)
    out = orc.merge(X, Zm, order, kf)
    kept, rows, chosen = _brute_force_merge(X, Zm, order, kf)
    np.testing.assert_array_equal(out["kept_idx"], kept)
    np.testing.assert_allclose(out["X_out"], rows, rtol=1e-13, atol=1e-14)
    assert {int(out["set_b"][j]) for j in out["merged"]} == chosen


def test_merge_conserves_mass_and_counts(rng):
    n, kp, kf = 40, 24, 15
    X, Zm = rng.standard_normal((n, 6)), rng.standard_normal((n, 9))
    order = orc.select_topk(rng.standard_normal(n), kp)
    out = orc.merge(X, Zm, order, kf)
    dst, kept = out["merge_dst"], out["kept_idx"]
    assert len(kept) == kf and np.all(np.diff(kept) > 0)
    assert (dst >= 0).sum() == kp and (dst == -1).sum() == n - kp
    sizes = np.array([(dst == a).sum() for a in kept])
    assert sizes.sum() == kp
    np.testing.assert_allclose((out["X_out"] * sizes[:, None]).sum(axis=0), X[order].sum(axis=0), rtol=1e-12)
    A, B = orc.split_sets(order)
    assert set(A) <= set(kept)                       # Set A always survives
    assert all(dst[b] in set(A) or dst[b] == b for b in B)
    assert sum(dst[b] != b for b in B) == kp - kf


def test_merge_degenerate_cases(rng):
    n = 20
    X, Zm = rng.standard_normal((n, 4)), rng.standard_normal((n, 6))
    order = orc.select_topk(rng.standard_normal(n), 10)
    # nothing merged: a pure gather of the survivors in position order
    out = orc.merge(X, Zm, order, 10)
    np.testing.assert_array_equal(out["kept_idx"], np.sort(order))
    np.testing.assert_array_equal(out["X_out"], X[np.sort(order)])
    # all of Set B merged: exactly Set A is left
    out = orc.merge(X, Zm, order, 5)
    np.testing.assert_array_equal(out["kept_idx"], np.sort(order[:5]))
    # an exact duplicate of a Set-A token has similarity 1 and leaves that token unchanged
    A, B = orc.split_sets(order)
    Z2, X2 = Zm.copy(), X.copy()
    Z2[B[0]], X2[B[0]] = Zm[A[2]], X[A[2]]
    out = orc.merge(X2, Z2, order, 9)
    assert out["merge_dst"][B[0]] == A[2]
    row = list(out["kept_idx"]).index(A[2])
    np.testing.assert_allclose(out["X_out"][row], X[A[2]], rtol=1e-14)
    with pytest.raises(ValueError):
        orc.merge(X, Zm, order, 4)                   # would need more merges than |SetB|


def test_merge_tie_rules():
    # two Set-A tokens identical: the argmax tie goes to the lower original index;
    # two Set-B tokens identical: the top-m tie goes to the lower original index.
    Zm = np.array([[1.0, 0.0], [1.0, 0.0], [0.9, 0.1], [0.9, 0.1], [0.0, 1.0]])
    X = np.arange(10.0).reshape(5, 2)
    order = np.array([1, 0, 3, 2])                   # A = {1, 0}, B = {3, 2}
    out = orc.merge(X, Zm, order, 3)
    assert out["merge_dst"][2] == 0 and out["merge_dst"][3] == 3
    np.testing.assert_array_equal(out["kept_idx"], [0, 1, 3])
    np.testing.assert_allclose(out["X_out"][0], (X[0] + X[2]) / 2)


def test_whole_path_on_tiny_workload_shapes():
    from workloads import CONFIGS, make_image
    w = CONFIGS["tiny"]
    im = make_image(w, 0)
    out = orc.compress(im["Q"], im["K"], im["V"], im["X"][w.n_sys:w.n_sys + w.n_vis], w.n_sys, w.n_vis,
                       w.k_prune, w.k_final, lam=w.lam, dtype=w.dtype)
    assert out["X_out"].shape == (12, 256) and len(out["order"]) == 16
    assert len(out["merged"]) == 4
    # lambda = 0 / 1 reduce the ranking to the ICS / attention-score ranking
    for lam, key in ((0.0, "C"), (1.0, "S")):
        o = orc.compress(im["Q"], im["K"], im["V"], im["X"][w.n_sys:w.n_sys + w.n_vis], w.n_sys, w.n_vis,
                         w.k_prune, w.k_final, lam=lam, dtype=w.dtype)
        np.testing.assert_array_equal(o["order"], np.argsort(-o[key], kind="stable")[:16])
