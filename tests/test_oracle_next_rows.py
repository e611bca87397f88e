"""Pins for the oracle functions beyond the compression path: information quantity (matrix rank),
sequence re-assembly with original position ids, rotary tables, KV-cache share."""
import os

import numpy as np
import pytest

from oracle import tokencarve_oracle as orc
from tests.helpers_cpu import rank_by_elimination
from workloads.generate import planted_lowrank

HERE = os.path.dirname(os.path.abspath(__file__))


def test_rank_of_an_exactly_low_rank_matrix():
    rng = np.random.default_rng(1)
    for n, d, r in ((40, 96, 7), (64, 64, 64), (30, 200, 1), (50, 20, 12)):
        A = rng.standard_normal((n, r)) @ rng.standard_normal((r, d))
        rank, sigma = orc.info_rank(A, rtol=1e-10)
        assert rank == min(r, n, d)
        assert sigma.shape == (min(n, d),) and np.all(np.diff(sigma) <= 1e-9 * sigma[0])


def test_rank_matches_gaussian_elimination_on_small_matrices():
    rng = np.random.default_rng(2)
    for trial in range(20):
        n, d = rng.integers(2, 9, size=2)
        r = int(rng.integers(0, min(n, d) + 1))
        A = rng.integers(-3, 4, size=(n, r)).astype(float) @ rng.integers(-3, 4, size=(r, d)).astype(float)
        assert orc.info_rank(A, rtol=1e-9)[0] == rank_by_elimination(A)


def test_rank_threshold_separates_planted_signal_from_noise():
    rng = np.random.default_rng(3)
    s = np.linspace(10.0, 1.0, 8)
    A = planted_lowrank(rng, 64, 256, s, 0.01)     # noise singular values about 0.01 (sqrt(64) + sqrt(256)) = 0.24
    assert orc.info_rank(A, rtol=0.05)[0] == 8     # threshold 0.5: between the signal (>= 1) and the noise
    assert orc.info_rank(A, rtol=1e-9)[0] == 64    # noise makes it full rank
    assert orc.info_rank(A)[0] == 64               # default threshold 256 * 2^-23


def test_rank_of_kept_rows_and_invariances():
    rng = np.random.default_rng(4)
    A = rng.standard_normal((32, 5)) @ rng.standard_normal((5, 48))
    rows = rng.permutation(32)[:12]
    r1, s1 = orc.info_rank(A, rows, rtol=1e-10)
    r2, s2 = orc.info_rank(A, rows[::-1], rtol=1e-10)      # row order does not matter
    r3, s3 = orc.info_rank(3.0 * A, rows, rtol=1e-10)      # nor does scale
    assert r1 == r2 == r3 == 5
    np.testing.assert_allclose(s1, s2, rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(3.0 * s1, s3, rtol=1e-10, atol=1e-12)
    assert orc.info_rank(A, rows[:3], rtol=1e-10)[0] == 3  # fewer rows than the rank
    assert orc.info_rank(A, rows[:0])[0] == 0
    assert orc.info_rank(np.zeros((4, 6)))[0] == 0
    # sum of squared singular values = squared Frobenius norm of the kept rows
    assert abs((s1 ** 2).sum() - (A[rows] ** 2).sum()) < 1e-9 * (A[rows] ** 2).sum()


def test_rank_curve_is_monotone_and_normalised():
    rng = np.random.default_rng(5)
    A = planted_lowrank(rng, 96, 128, 20.0 * np.arange(1, 25) ** -0.8, 0.01)
    order = rng.permutation(96)
    counts = [96, 64, 48, 32, 24, 16, 8, 4]
    ranks = [orc.info_rank(A, order[:k], rtol=0.02)[0] for k in counts]
    assert all(a >= b for a, b in zip(ranks, ranks[1:]))   # dropping rows never raises the rank
    assert all(r <= k for r, k in zip(ranks, counts))
    curve = orc.visual_token_information(ranks)
    assert curve.max() == 1.0 and curve.min() == 0.0


def test_assembled_sequence_keeps_text_rows_and_original_positions():
    rng = np.random.default_rng(6)
    n_sys, n_vis, n_prompt, D, kf = 4, 16, 5, 8, 6
    L = n_sys + n_vis + n_prompt
    H = rng.standard_normal((L, D))
    kept = np.sort(rng.permutation(n_vis)[:kf])
    X_out = rng.standard_normal((kf, D))
    H_new, pos = orc.assemble_sequence(H, X_out, kept, n_sys, n_vis)
    assert H_new.shape == (L - n_vis + kf, D) and pos.shape == (L - n_vis + kf,)
    np.testing.assert_array_equal(H_new[:n_sys], H[:n_sys])
    np.testing.assert_array_equal(H_new[n_sys:n_sys + kf], X_out)
    np.testing.assert_array_equal(H_new[n_sys + kf:], H[n_sys + n_vis:])
    assert np.all(np.diff(pos) > 0)
    np.testing.assert_array_equal(pos[:n_sys], np.arange(n_sys))
    np.testing.assert_array_equal(pos[n_sys:n_sys + kf], n_sys + kept)
    np.testing.assert_array_equal(pos[n_sys + kf:], np.arange(n_sys + n_vis, L))
    # keeping every visual token gives the original sequence back
    H_all, pos_all = orc.assemble_sequence(H, H[n_sys:n_sys + n_vis], np.arange(n_vis), n_sys, n_vis)
    np.testing.assert_array_equal(H_all, H)
    np.testing.assert_array_equal(pos_all, np.arange(L))


def test_rotary_tables_closed_forms_and_relative_position_property():
    d = 16
    pos = np.array([0, 1, 7, 40, 611])
    cos, sin = orc.rope_tables(pos, d, base=10000.0)
    assert cos.shape == (5, d // 2)
    np.testing.assert_allclose(cos[0], 1.0)
    np.testing.assert_allclose(sin[0], 0.0)
    np.testing.assert_allclose(cos ** 2 + sin ** 2, 1.0, rtol=1e-14)
    np.testing.assert_allclose(cos[:, 0], np.cos(pos), rtol=1e-14)          # theta_0 = 1
    np.testing.assert_allclose(sin[2, 4], np.sin(7 * 10000.0 ** -0.5), rtol=1e-14)  # i = d/4: theta = base^-1/2
    # <R(p) q, R(p') k> depends on p - p' only: the reason kept tokens must keep their position ids
    rng = np.random.default_rng(7)
    q, k = rng.standard_normal((1, d)), rng.standard_normal((1, d))

    def score(p, pp):
        cq, sq = orc.rope_tables([p], d)
        ck, sk = orc.rope_tables([pp], d)
        return float((orc.apply_rope(q, cq, sq) @ orc.apply_rope(k, ck, sk).T)[0, 0])

    assert abs(score(40, 33) - score(611, 604)) < 1e-10
    assert abs(score(40, 33) - score(40, 32)) > 1e-3
    # a rotation keeps the norm
    c, s = orc.rope_tables([123], d)
    assert abs(np.linalg.norm(orc.apply_rope(q, c, s)) - np.linalg.norm(q)) < 1e-12


def test_kv_cache_share_reproduces_the_papers_table():
    rows = [l.split() for l in open(os.path.join(HERE, "golden", "kv_cache_table.txt")) if l.strip() and not l.startswith("#")]
    table = {int(a): float(b) for a, b in rows}
    # 36 system tokens + a TextVQA prompt: the three compressed columns are reproduced to the printed
    # digit by a text length of about 80 tokens (sample average), with 2 of 32 layers uncompressed
    for kept, pct in table.items():
        got = 100.0 * orc.kv_cache_fraction(80, 576, kept, 32, 2)
        assert abs(got - pct) < 0.15, (kept, got, pct)
    # a plausible mistake (compressing the first layers too) misses the table by many points
    assert abs(100.0 * orc.kv_cache_fraction(80, 576, 64, 32, 0) - table[64]) > 4.0
    assert orc.kv_cache_fraction(80, 576, 576, 32, 2) == 1.0


# ---------------------------------------------------------------------------------------------
# planted mistakes: each plausible wrong version of these functions must fail at least one pin
# ---------------------------------------------------------------------------------------------
def _pins():
    return [test_rank_of_an_exactly_low_rank_matrix, test_rank_matches_gaussian_elimination_on_small_matrices,
            test_rank_threshold_separates_planted_signal_from_noise, test_rank_of_kept_rows_and_invariances,
            test_rank_curve_is_monotone_and_normalised, test_assembled_sequence_keeps_text_rows_and_original_positions,
            test_rotary_tables_closed_forms_and_relative_position_property, test_kv_cache_share_reproduces_the_papers_table]


def _caught(monkeypatch, name, mutant):
    monkeypatch.setattr(orc, name, mutant)
    failed = 0
    for pin in _pins():
        try:
            pin()
        except AssertionError:
            failed += 1
    return failed


def test_planted_mistakes_in_rank_sequence_and_cache_functions_are_caught(monkeypatch):
    real_rank, real_asm, real_rope, real_kv = orc.info_rank, orc.assemble_sequence, orc.rope_tables, orc.kv_cache_fraction

    def rank_absolute_threshold(O, rows=None, rtol=None):            # threshold not relative to sigma_max
        r, s = real_rank(O, rows, rtol)
        t = rtol if rtol is not None else 1e-7
        return int((s > t).sum()), s

    def rank_ignores_rows(O, rows=None, rtol=None):                  # always the whole matrix
        return real_rank(O, None, rtol)

    def rank_counts_squared(O, rows=None, rtol=None):                # eigenvalues of the Gram matrix compared instead of sigma
        r, s = real_rank(O, rows, rtol)
        t = rtol if rtol is not None else 1e-7
        return (int((s ** 2 > t * s[0] ** 2).sum()) if s.size and s[0] > 0 else 0), s

    def asm_compacted_positions(H, X_out, kept_idx, n_sys, n_vis):   # positions renumbered 0..L'-1
        Hn, pos = real_asm(H, X_out, kept_idx, n_sys, n_vis)
        return Hn, np.arange(len(pos))

    def asm_prompt_before_visual(H, X_out, kept_idx, n_sys, n_vis):
        Hn, pos = real_asm(H, X_out, kept_idx, n_sys, n_vis)
        k = len(kept_idx)
        return np.concatenate([Hn[:n_sys], Hn[n_sys + k:], Hn[n_sys:n_sys + k]]), pos

    def rope_wrong_exponent(pos_ids, head_dim, base=10000.0):        # theta_i = base^(-i/d) instead of base^(-2i/d)
        i = np.arange(head_dim // 2, dtype=np.float64)
        ang = np.asarray(pos_ids, dtype=np.float64)[:, None] * (base ** (-i / head_dim))[None, :]
        return np.cos(ang), np.sin(ang)

    def rope_swapped(pos_ids, head_dim, base=10000.0):
        c, s = real_rope(pos_ids, head_dim, base)
        return s, c

    def kv_all_layers_short(n_text, n_vis, n_kept, n_layers, n_layers_before):
        return real_kv(n_text, n_vis, n_kept, n_layers, 0)

    def kv_visual_only(n_text, n_vis, n_kept, n_layers, n_layers_before):   # text tokens forgotten
        return real_kv(0, n_vis, n_kept, n_layers, n_layers_before)

    for name, mutant in [("info_rank", rank_absolute_threshold), ("info_rank", rank_ignores_rows),
                         ("info_rank", rank_counts_squared), ("assemble_sequence", asm_compacted_positions),
                         ("assemble_sequence", asm_prompt_before_visual), ("rope_tables", rope_wrong_exponent),
                         ("rope_tables", rope_swapped), ("kv_cache_fraction", kv_all_layers_short),
                         ("kv_cache_fraction", kv_visual_only)]:
        assert _caught(monkeypatch, name, mutant) >= 1, "mutant %s survives every pin" % mutant.__name__
        monkeypatch.undo()
    assert _caught(monkeypatch, "info_rank", real_rank) == 0         # and the real functions pass them all
