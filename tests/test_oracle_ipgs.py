"""Pins for the oracle's SVD / information contribution score / combined score
(Section 3.3.1, Eq. 3-5, 3-6, 3-8)."""
import numpy as np
import pytest

from oracle import tokencarve_oracle as orc
from tests.helpers_cpu import hestenes_svd
from workloads import CONFIGS, make_image
from workloads.generate import planted_lowrank


def test_squared_singular_values_sum_to_frobenius_norm(rng):
    O = rng.standard_normal((40, 96))
    _, s, _ = orc.ics(O)
    assert abs((s ** 2).sum() - (O ** 2).sum()) <= 1e-12 * (O ** 2).sum()


def test_row_energy_identity_from_row_expansion(rng):
    # Eq. 3-5: Z(x) = sum_i u_xi sigma_i v_i^T with orthonormal v_i  =>  sum_i (u_xi sigma_i)^2 = |Z(x)|^2
    O = rng.standard_normal((30, 50))
    _, s, U = orc.ics(O)
    np.testing.assert_allclose(((U * s) ** 2).sum(axis=1), (O ** 2).sum(axis=1), rtol=1e-12)
    np.testing.assert_allclose(U.T @ U, np.eye(30), atol=1e-12)


def test_exact_rank_recovery_on_planted_lowrank():
    g = np.random.Generator(np.random.Philox(7))
    s_true = np.linspace(10.0, 1.0, 8)
    O = planted_lowrank(g, 64, 256, s_true, noise=0.0)
    _, s, _ = orc.ics(O)
    np.testing.assert_allclose(s[:8], s_true, rtol=1e-10)
    assert np.all(s[8:] <= 1e-12 * s[0])
    assert int((s > 1e-9 * s[0]).sum()) == 8


def test_planted_spectrum_survives_noise_within_weyl_bound():
    g = np.random.Generator(np.random.Philox(8))
    s_true = np.linspace(10.0, 1.0, 8)
    clean = planted_lowrank(g, 64, 256, s_true, noise=0.0)
    noise = 0.01 * g.standard_normal((64, 256))
    _, s, _ = orc.ics(clean + noise)
    bound = np.linalg.norm(noise, 2)
    assert np.all(np.abs(s[:8] - s_true) <= bound * (1 + 1e-12))
    assert np.all(s[8:] <= bound * (1 + 1e-12))
    assert s[7] > 3 * s[8]                       # visible gap at the planted rank


def test_orthogonal_rows_score_is_row_norm(rng):
    # mutually orthogonal rows with distinct norms: U is a permutation, C(x) = |O_x|
    Qm, _ = np.linalg.qr(rng.standard_normal((20, 12)))
    norms = np.linspace(5.0, 0.5, 12)
    O = (Qm * norms).T                           # 12 rows in R^20
    C, s, _ = orc.ics(O)
    np.testing.assert_allclose(C, norms, rtol=1e-12)
    np.testing.assert_allclose(s, norms, rtol=1e-12)


def test_rank_one_score_closed_form(rng):
    a, b = rng.standard_normal(15), rng.standard_normal(33)
    C, _, _ = orc.ics(np.outer(a, b))
    np.testing.assert_allclose(C, np.abs(a) * np.linalg.norm(b), rtol=1e-10, atol=1e-12)


def test_score_bounds_between_l2_and_sqrt_rank_l2(rng):
    O = rng.standard_normal((25, 40))
    C, _, _ = orc.ics(O)
    row = np.linalg.norm(O, axis=1)
    assert np.all(C >= row * (1 - 1e-12))
    assert np.all(C <= np.sqrt(25) * row * (1 + 1e-12))


def test_score_symmetries(rng):
    O = rng.standard_normal((18, 30))
    C, _, _ = orc.ics(O)
    np.testing.assert_allclose(orc.ics(-2.5 * O)[0], 2.5 * C, rtol=1e-11)
    W, _ = np.linalg.qr(rng.standard_normal((30, 30)))
    np.testing.assert_allclose(orc.ics(O @ W)[0], C, rtol=1e-10)      # right-orthogonal invariance
    perm = rng.permutation(18)
    np.testing.assert_allclose(orc.ics(O[perm])[0], C[perm], rtol=1e-10)
    dup = np.vstack([O, O[3:4]])
    Cd = orc.ics(dup)[0]
    assert abs(Cd[3] - Cd[-1]) <= 1e-10 * Cd[3]


def test_score_is_not_the_transposed_or_unweighted_variant(rng):
    # guards against using V instead of U, or dropping sigma: both break the closed forms above
    a, b = np.abs(rng.standard_normal(6)) + 0.1, rng.standard_normal(9)
    C, _, _ = orc.ics(np.outer(a, b))
    assert C.shape == (6,)
    assert np.argmax(C) == np.argmax(a)
    assert not np.allclose(C, np.abs(a) / np.linalg.norm(a))          # would be the sigma-free version


def test_independent_one_sided_jacobi_agrees(rng):
    # LAPACK SVD (oracle) vs Hestenes rotations written here: same sigma, same C.
    g = np.random.Generator(np.random.Philox(11))
    O = planted_lowrank(g, 24, 40, np.linspace(6, 1, 5), noise=0.05)
    C, s, _ = orc.ics(O)
    Uh, sh = hestenes_svd(O)
    np.testing.assert_allclose(sh, s, rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose((np.abs(Uh) * sh).sum(axis=1), C, rtol=1e-8)


def test_independent_route_on_tiny_workload():
    w = CONFIGS["tiny"]
    im = make_image(w, 0)
    Z, _ = orc.attn_output(im["Q"], im["K"], im["V"], w.n_sys, w.n_vis)
    O = orc.to_storage(Z, w.dtype)
    C, s, _ = orc.ics(O)
    Uh, sh = hestenes_svd(O)
    np.testing.assert_allclose(sh, s, rtol=1e-9, atol=1e-12)
    np.testing.assert_allclose((np.abs(Uh) * sh).sum(axis=1), C, rtol=1e-7)
    # Gram route: eigenvalues of O O^T are sigma^2 (what the GPU path exploits)
    lam = np.linalg.eigvalsh(O @ O.T)[::-1]
    np.testing.assert_allclose(np.sqrt(np.maximum(lam, 0)), s, rtol=1e-6, atol=1e-9 * s[0])


def test_sv_rtol_drops_small_terms(rng):
    O = planted_lowrank(np.random.Generator(np.random.Philox(5)), 16, 32, np.array([8.0, 4.0, 2.0]), 1e-6)
    C_all, s, U = orc.ics(O)
    C_cut, _, _ = orc.ics(O, sv_rtol=1e-3)
    np.testing.assert_allclose(C_cut, (np.abs(U[:, :3]) * s[:3]).sum(axis=1), rtol=1e-12)
    assert np.all(C_cut <= C_all)


def test_minmax_and_combined_score(rng):
    C = rng.uniform(50, 300, 40)
    S = rng.uniform(1e-5, 1e-2, 40)
    for lam in (0.0, 0.3, 1.0):
        E = orc.combined_score(C, S, lam, orc.NORM_MINMAX)
        assert E.min() >= 0.0 and E.max() <= 1.0
    np.testing.assert_array_equal(np.argsort(-orc.combined_score(C, S, 0.0), kind="stable"),
                                  np.argsort(-C, kind="stable"))
    np.testing.assert_array_equal(np.argsort(-orc.combined_score(C, S, 1.0), kind="stable"),
                                  np.argsort(-S, kind="stable"))
    # literal Eq. 3-8
    np.testing.assert_allclose(orc.combined_score(C, S, 0.25, orc.NORM_NONE), 0.75 * C + 0.25 * S)
    # token that is best in both gets exactly 1; constant vectors map to zeros
    C2, S2 = C.copy(), S.copy()
    C2[5], S2[5] = 1e3, 1.0
    assert orc.combined_score(C2, S2, 0.5)[5] == 1.0
    np.testing.assert_array_equal(orc.minmax(np.full(4, 2.0)), np.zeros(4))


@pytest.mark.parametrize("seed", [0, 1])
def test_gram_rounding_floor_is_reported_and_small_for_tiny(seed):
    w = CONFIGS["tiny"]
    im = make_image(w, seed)
    Z, _ = orc.attn_output(im["Q"], im["K"], im["V"], w.n_sys, w.n_vis)
    O = orc.to_storage(Z, w.dtype)
    assert orc.gram_precision_floor(O, np.float64) < 1e-6
    assert orc.min_relative_gap(orc.ics(O)[1]) > 0


def test_min_relative_gap_closed_form():
    # gaps 3, 0.5 (and 6.5 down to the negligible value): relative to sigma_1 = 10 the smallest is 0.05;
    # values below floor * sigma_1 do not count
    s = np.array([10.0, 7.0, 6.5, 1e-9])
    assert orc.min_relative_gap(s) == pytest.approx(0.05, rel=1e-12)
    assert orc.min_relative_gap(s, floor=1e-12) == pytest.approx(0.05, rel=1e-12)          # 6.5 - 1e-9 is not smaller
    assert orc.min_relative_gap(np.array([10.0, 7.0, 6.5, 6.4]), floor=0.69) == pytest.approx(0.3, rel=1e-12)  # only 10 and 7 lie above 6.9
    assert orc.min_relative_gap(np.array([4.0, 4.0, 1.0])) == 0.0                           # a repeated value
    assert orc.min_relative_gap(np.array([5.0])) == np.inf
    # scaling the spectrum does not change a relative gap
    assert orc.min_relative_gap(1e6 * s) == pytest.approx(orc.min_relative_gap(s), rel=1e-12)


def test_gram_precision_floor_closed_form():
    # Orthogonal rows: G is diagonal, C(x) = ||O_x|| = sqrt(G_xx), so rounding G to float32 changes C(x) by
    # sqrt(fl32(G_xx)) / sqrt(G_xx) - 1 and nothing else.  Row 0 = 3 (1, 2^-13): G_00 = 9 (1 + 2^-26) rounds to 9
    # in float32 (half a unit in the last place of 9 is 2^-21 > 9 * 2^-26), row 1 has G_11 = 4 exactly.  Every
    # entry of O itself is a float32 number: rounding O instead of G would report 0.
    O = np.zeros((2, 4))
    O[0, 0], O[0, 1] = 3.0, 3.0 * 2.0 ** -13
    O[1, 2] = 2.0
    expect = 1.0 - 1.0 / np.sqrt(1.0 + 2.0 ** -26)     # relative, not absolute (which would be three times that)
    assert orc.gram_precision_floor(O, np.float32) == pytest.approx(expect, rel=1e-6)
    assert orc.gram_precision_floor(O, np.float64) < 1e-15
    # the largest change over the tokens is reported: swapping the rows changes nothing
    assert orc.gram_precision_floor(O[::-1].copy(), np.float32) == pytest.approx(expect, rel=1e-6)
