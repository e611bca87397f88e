"""(1) The stored tiny-configuration fixture is reproduced by the oracle.  (2) Plausible mistakes
planted in the oracle (on the CPU) are caught by the pins: each mutant must fail at least one pin."""
import json
import os

import numpy as np
import pytest

from oracle import tokencarve_oracle as orc
from tests import test_oracle_attention as t_attn
from tests import test_oracle_ipgs as t_ipgs
from tests import test_oracle_select_merge as t_sel
from workloads import CONFIGS, make_image

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "tiny_oracle.json")


def test_tiny_fixture_is_reproduced():
    doc = json.load(open(GOLDEN))
    w = CONFIGS["tiny"]
    im = make_image(w, 0)
    out = orc.compress(im["Q"], im["K"], im["V"], im["X"][w.n_sys:w.n_sys + w.n_vis], w.n_sys, w.n_vis,
                       w.k_prune, w.k_final, lam=w.lam, dtype=w.dtype)
    np.testing.assert_allclose(out["sigma"][:12], doc["sigma"], rtol=1e-9)
    np.testing.assert_allclose(out["C"], doc["C"], rtol=1e-9)
    np.testing.assert_allclose(out["S"], doc["S"], rtol=1e-9)
    np.testing.assert_allclose(out["E"], doc["E"], rtol=1e-8, atol=1e-12)
    assert out["order"].tolist() == doc["order"]
    assert out["kept_idx"].tolist() == doc["kept_idx"]
    assert out["merge_dst"].tolist() == doc["merge_dst"]
    np.testing.assert_allclose(out["X_out"][0][:8], doc["X_out_row0_first8"], rtol=1e-7)
    # planted rank of the hidden states does not survive attention with i.i.d. Q, K, V, but the
    # spectrum must still be non-increasing and positive
    assert np.all(np.diff(doc["sigma"]) <= 0) and doc["sigma"][-1] > 0


def _rng():
    return np.random.default_rng(20250310)


def _mutant_attn(kind):
    real = orc.attn_output

    def f(Q, K, V, n_sys, n_vis, causal=True, scale=None, n_prompt_q=0):
        Z, S = real(Q, K, V, n_sys, n_vis, causal, scale, n_prompt_q)
        if kind == "prompt_rows_divided_by_visual_count":
            return Z, S * (n_vis + n_prompt_q) / n_vis
        if kind == "prompt_rows_ignored":
            return real(Q, K, V, n_sys, n_vis, causal, scale, 0)
        if kind == "prompt_rows_taken_before_the_visual_block":
            if n_prompt_q == 0 or n_sys < n_prompt_q:
                return Z, S
            _, S_shift = real(Q, K, V, n_sys - n_prompt_q, n_vis + n_prompt_q, causal, scale, 0)
            return Z, S_shift[n_prompt_q:]
        if kind == "score_not_averaged_over_heads":
            return Z, S * np.asarray(Q).shape[0]
        if kind == "score_of_rows_instead_of_columns":
            return Z, np.full_like(S, S.mean())
        if kind == "strict_causal_mask":          # key p itself hidden from query p
            H, L, dh = np.asarray(Q).shape
            Q2 = np.asarray(Q, dtype=np.float64)
            K2 = np.asarray(K, dtype=np.float64).copy()
            V2 = np.asarray(V, dtype=np.float64)
            if not causal:
                return Z, S
            Zs = np.zeros_like(Z)
            for h in range(H):
                for q in range(n_vis):
                    p = n_sys + q
                    lg = (K2[h, :p] @ Q2[h, p]) * (scale or 1 / np.sqrt(dh)) if p > 0 else np.zeros(1)
                    a = np.exp(lg - lg.max())
                    a /= a.sum()
                    Zs[q, h * dh:(h + 1) * dh] = a @ V2[h, :max(p, 1)]
            return Zs, S
        raise ValueError(kind)
    return f


@pytest.mark.parametrize("kind", ["score_not_averaged_over_heads", "score_of_rows_instead_of_columns",
                                  "strict_causal_mask"])
def test_attention_mutants_are_caught(monkeypatch, kind):
    monkeypatch.setattr(orc, "attn_output", _mutant_attn(kind))
    pins = [t_attn.test_uniform_attention_closed_form_causal, t_attn.test_attention_score_mass_balance,
            t_attn.test_matches_scalar_loops_including_attention_score]
    failed = 0
    for pin in pins:
        try:
            pin(_rng())
        except AssertionError:
            failed += 1
    assert failed >= 1, "mutant %s slipped through the attention pins" % kind


@pytest.mark.parametrize("kind", ["prompt_rows_divided_by_visual_count", "prompt_rows_ignored",
                                  "prompt_rows_taken_before_the_visual_block"])
def test_prompt_row_mutants_are_caught(monkeypatch, kind):
    monkeypatch.setattr(orc, "attn_output", _mutant_attn(kind))
    pins = [t_attn.test_prompt_rows_uniform_attention_closed_form,
            t_attn.test_prompt_rows_match_scalar_loops_and_reduce_to_eq_3_7,
            t_attn.test_prompt_rows_are_a_weighted_mix_of_two_visual_style_means]
    failed = 0
    for pin in pins:
        try:
            pin(_rng())
        except AssertionError:
            failed += 1
    assert failed >= 2, "mutant %s slipped through the prompt-row pins" % kind


def _mutant_ics(kind):
    def f(O, sv_rtol=0.0):
        U, s, Vt = np.linalg.svd(np.asarray(O, dtype=np.float64), full_matrices=False)
        if kind == "sigma_dropped":
            C = np.abs(U).sum(axis=1)
        elif kind == "right_vectors_used":
            C = (np.abs(Vt.T[:U.shape[0]]) * s).sum(axis=1)
        elif kind == "squared_terms":
            C = np.sqrt(((U * s) ** 2).sum(axis=1))
        elif kind == "sign_kept":
            C = np.abs((U * s).sum(axis=1))
        else:
            raise ValueError(kind)
        return C, s, U
    return f


@pytest.mark.parametrize("kind", ["sigma_dropped", "right_vectors_used", "squared_terms", "sign_kept"])
def test_score_mutants_are_caught(monkeypatch, kind):
    monkeypatch.setattr(orc, "ics", _mutant_ics(kind))
    pins = [t_ipgs.test_rank_one_score_closed_form, t_ipgs.test_orthogonal_rows_score_is_row_norm,
            t_ipgs.test_score_bounds_between_l2_and_sqrt_rank_l2, t_ipgs.test_independent_one_sided_jacobi_agrees,
            t_ipgs.test_score_symmetries]
    failed = 0
    for pin in pins:
        try:
            pin(_rng())
        except AssertionError:
            failed += 1
    assert failed >= 1, "mutant %s slipped through the score pins" % kind


def test_selection_and_merge_mutants_are_caught(monkeypatch):
    # ascending instead of descending sort
    monkeypatch.setattr(orc, "select_topk", lambda E, k: np.argsort(np.asarray(E), kind="stable")[:k].astype(np.int64))
    with pytest.raises(AssertionError):
        t_sel.test_topk_equals_best_subset_by_enumeration(_rng())
    monkeypatch.undo()
    # ties to the higher index
    monkeypatch.setattr(orc, "select_topk",
                        lambda E, k: (len(E) - 1 - np.argsort(-np.asarray(E)[::-1], kind="stable"))[:k].astype(np.int64))
    with pytest.raises(AssertionError):
        t_sel.test_topk_ties_go_to_lower_index_and_is_permutation_equivariant(_rng())
    monkeypatch.undo()
    # un-normalised similarity (dot product instead of cosine)
    monkeypatch.setattr(orc, "similarity", lambda m, a, b: np.asarray(m)[b] @ np.asarray(m)[a].T)
    with pytest.raises(AssertionError):
        t_sel.test_similarity_is_cosine_and_equals_normalised_gram(_rng())
    monkeypatch.undo()
    # transposed similarity operand (SetA rows against SetB columns)
    real_sim = orc.similarity
    monkeypatch.setattr(orc, "similarity", lambda m, a, b: real_sim(m, b, a).T[:len(b), :len(a)] * 0 + real_sim(m, a, b)[::-1])
    caught = 0
    for seed in range(6):
        try:
            t_sel.test_merge_matches_brute_force_assignment(seed)
        except AssertionError:
            caught += 1
    assert caught >= 1
