"""Pins for the oracle's attention step (Eq. 3-1, 3-2, 3-7): closed forms, a library
special case and a scalar-loop evaluation."""
import numpy as np
import torch

from oracle import tokencarve_oracle as orc
from tests.helpers_cpu import softmax_attention_loops


def _rand(rng, H, L, dh):
    return (rng.standard_normal((H, L, dh)) for _ in range(3))


def test_uniform_attention_closed_form_causal(rng):
    # Q = 0 makes every allowed key equally likely: Z_q is the running mean of V and
    # S(x) = (1/N) sum_{q >= x} 1/(L_s+q+1).
    H, L, dh, Ls, N = 3, 21, 8, 4, 12
    _, K, V = _rand(rng, H, L, dh)
    Z, S = orc.attn_output(np.zeros((H, L, dh)), K, V, Ls, N, causal=True)
    for q in range(N):
        expect = np.concatenate([V[h, :Ls + q + 1].mean(axis=0) for h in range(H)])
        np.testing.assert_allclose(Z[q], expect, rtol=1e-13, atol=1e-13)
    S_expect = np.array([sum(1.0 / (Ls + q + 1) for q in range(x, N)) / N for x in range(N)])
    np.testing.assert_allclose(S, S_expect, rtol=1e-13)


def test_uniform_attention_closed_form_full(rng):
    H, L, dh, Ls, N = 2, 17, 4, 3, 9
    _, K, V = _rand(rng, H, L, dh)
    Z, S = orc.attn_output(np.zeros((H, L, dh)), K, V, Ls, N, causal=False)
    expect = np.concatenate([V[h].mean(axis=0) for h in range(H)])
    np.testing.assert_allclose(Z, np.tile(expect, (N, 1)), rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(S, np.full(N, 1.0 / L), rtol=1e-13)


def test_one_hot_attention_picks_one_value_row(rng):
    # a huge logit on key `tgt` makes the softmax one-hot: Z_q = V[tgt]; S counts the hits.
    H, L, dh, Ls, N = 2, 16, 8, 2, 10
    Q, K, V = _rand(rng, H, L, dh)
    tgt = Ls + 1                                  # visible to every visual query q >= 1
    K = np.zeros_like(K)
    K[:, tgt, 0] = 1.0
    Q = np.zeros_like(Q)
    Q[:, :, 0] = 1e4
    Z, S = orc.attn_output(Q, K, V, Ls, N, causal=True)
    for q in range(1, N):
        np.testing.assert_allclose(Z[q], np.concatenate([V[h, tgt] for h in range(H)]), rtol=1e-12)
    assert abs(S[1] - (N - 1) / N) < 1e-12       # queries 1..N-1 put all mass on visual token 1
    assert np.all(S[2:] < 1e-12)


def test_rows_of_softmax_sum_to_one_via_constant_values(rng):
    H, L, dh, Ls, N = 2, 20, 4, 5, 11
    Q, K, _ = _rand(rng, H, L, dh)
    Z, _ = orc.attn_output(Q, K, np.ones((H, L, dh)), Ls, N, causal=True)
    np.testing.assert_allclose(Z, 1.0, rtol=1e-13)


def test_matches_torch_sdpa_float64(rng):
    # the library's scaled-dot-product attention is the textbook special case of Eq. 3-1/3-2
    H, L, dh, Ls, N = 4, 40, 16, 6, 25
    Q, K, V = _rand(rng, H, L, dh)
    for causal in (True, False):
        Z, _ = orc.attn_output(Q, K, V, Ls, N, causal=causal)
        tq, tk, tv = (torch.from_numpy(np.ascontiguousarray(a)) for a in (Q, K, V))
        ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=causal)
        ref = ref[:, Ls:Ls + N].permute(1, 0, 2).reshape(N, H * dh).numpy()
        np.testing.assert_allclose(Z, ref, rtol=1e-11, atol=1e-12)


def test_matches_scalar_loops_including_attention_score(rng):
    H, L, dh, Ls, N = 2, 13, 4, 3, 7
    Q, K, V = _rand(rng, H, L, dh)
    for causal in (True, False):
        Z, S = orc.attn_output(Q, K, V, Ls, N, causal=causal, scale=0.37)
        Zl, Sl = softmax_attention_loops(Q, K, V, Ls, N, causal, 0.37)
        np.testing.assert_allclose(Z, Zl, rtol=1e-12, atol=1e-13)
        np.testing.assert_allclose(S, Sl, rtol=1e-12)


# ---- text-guided variant of Eq. 3-7: the first P prompt rows join the visual query rows ----
def test_prompt_rows_uniform_attention_closed_form(rng):
    # Q = 0, causal: a query at position p spreads 1/(p+1) over keys 0..p; every prompt row sees every
    # visual key, so S(x) = [sum_{q >= x} 1/(L_s+q+1) + sum_{t < P} 1/(L_s+N+t+1)] / (N + P).
    H, L, dh, Ls, N, P = 2, 30, 4, 8, 11, 6
    _, K, V = _rand(rng, H, L, dh)
    Z, S = orc.attn_output(np.zeros((H, L, dh)), K, V, Ls, N, causal=True, n_prompt_q=P)
    tail = sum(1.0 / (Ls + N + t + 1) for t in range(P))
    S_expect = np.array([(sum(1.0 / (Ls + q + 1) for q in range(x, N)) + tail) / (N + P) for x in range(N)])
    np.testing.assert_allclose(S, S_expect, rtol=1e-13)
    Z0, _ = orc.attn_output(np.zeros((H, L, dh)), K, V, Ls, N, causal=True)
    np.testing.assert_array_equal(Z, Z0)              # the attention output does not depend on P


def test_prompt_rows_match_scalar_loops_and_reduce_to_eq_3_7(rng):
    H, L, dh, Ls, N = 2, 18, 4, 5, 7
    Q, K, V = _rand(rng, H, L, dh)
    for causal in (True, False):
        for P in (0, 1, 5, L - Ls - N):
            Z, S = orc.attn_output(Q, K, V, Ls, N, causal=causal, scale=0.41, n_prompt_q=P)
            Zl, Sl = softmax_attention_loops(Q, K, V, Ls, N, causal, 0.41, P)
            np.testing.assert_allclose(Z, Zl, rtol=1e-12, atol=1e-13)
            np.testing.assert_allclose(S, Sl, rtol=1e-12)
        Z, S = orc.attn_output(Q, K, V, Ls, N, causal=causal, scale=0.41, n_prompt_q=0)
        Z0, S0 = orc.attn_output(Q, K, V, Ls, N, causal=causal, scale=0.41)
        np.testing.assert_array_equal(S, S0)
        np.testing.assert_array_equal(Z, Z0)


def test_prompt_rows_are_a_weighted_mix_of_two_visual_style_means(rng):
    # the mean over N + P rows is the row-count-weighted mean of the visual-row mean (Eq. 3-7) and of the
    # mean over the P prompt rows alone, which is Eq. 3-7 of a sequence whose "visual" queries are the
    # prompt rows: computed here from the full softmax of torch's attention with a one-hot value matrix
    H, L, dh, Ls, N, P = 3, 28, 8, 8, 10, 7
    Q, K, V = _rand(rng, H, L, dh)
    _, S = orc.attn_output(Q, K, V, Ls, N, causal=True, n_prompt_q=P)
    _, S_vis = orc.attn_output(Q, K, V, Ls, N, causal=True)
    tq, tk = (torch.from_numpy(np.ascontiguousarray(a)) for a in (Q, K))
    eye = torch.eye(L, dtype=torch.float64).expand(H, L, L)      # values = identity: the output IS the matrix A
    A = torch.nn.functional.scaled_dot_product_attention(tq, tk, eye, is_causal=True).numpy()
    S_prompt = A[:, Ls + N:Ls + N + P, Ls:Ls + N].mean(axis=(0, 1))
    np.testing.assert_allclose(S, (N * S_vis + P * S_prompt) / (N + P), rtol=1e-12)


def test_prompt_rows_out_of_range_is_an_error(rng):
    import pytest
    H, L, dh, Ls, N = 1, 10, 4, 2, 5
    Q, K, V = _rand(rng, H, L, dh)
    with pytest.raises(ValueError):
        orc.attn_output(Q, K, V, Ls, N, n_prompt_q=L - Ls - N + 1)
    with pytest.raises(ValueError):
        orc.attn_output(Q, K, V, Ls, N, n_prompt_q=-1)


def test_attention_score_mass_balance(rng):
    # full (non-causal) softmax: the visual columns of each row hold 1 - (mass on text keys);
    # with no text tokens at all the scores sum to exactly 1.
    H, L, dh = 3, 12, 4
    Q, K, V = _rand(rng, H, L, dh)
    _, S = orc.attn_output(Q, K, V, 0, L, causal=False)
    assert abs(S.sum() - 1.0) < 1e-13
    _, S = orc.attn_output(Q, K, V, 0, L, causal=True)
    assert abs(S.sum() - 1.0) < 1e-13


def test_storage_rounding_matches_torch():
    x = np.random.default_rng(1).standard_normal(20000) * np.logspace(-20, 20, 20000)
    x = np.concatenate([x, [0.0, 1.0, 1.00390625, 1.001953125, 1.005859375, -3.0e38]])
    mine = orc.to_storage(x, "bf16")
    ref = torch.from_numpy(x).to(torch.bfloat16).to(torch.float64).numpy()
    np.testing.assert_array_equal(mine, ref)
    np.testing.assert_array_equal(orc.to_storage(x, "f32"), x.astype(np.float32).astype(np.float64))


def test_half_precision_storage_rounding_closed_forms():
    """IEEE half: 11 significant bits, ties to even, largest finite value 65504, subnormals down to 2^-24."""
    x = np.array([1.0 + 2.0 ** -11, 1.0 + 3 * 2.0 ** -11, 1.0 + 2.0 ** -10, -(2.0 + 2.0 ** -10), 65504.0, 65519.9,
                  2.0 ** -24, 0.6 * 2.0 ** -24, 2.0 ** -14 * (1 + 2.0 ** -10), 0.1])
    got = orc.to_storage(x, "f16")
    expect = np.array([1.0, 1.0 + 2.0 ** -9, 1.0 + 2.0 ** -10, -2.0, 65504.0, 65504.0,
                       2.0 ** -24, 2.0 ** -24, 2.0 ** -14 * (1 + 2.0 ** -10), 0.0999755859375])
    np.testing.assert_array_equal(got, expect)
    from workloads.generate import round_to_storage
    rng = np.random.default_rng(3)
    y = rng.standard_normal(1000) * 10.0 ** rng.integers(-6, 4, 1000)
    np.testing.assert_array_equal(round_to_storage(y, "f16").astype(np.float64), orc.to_storage(y, "f16"))
    # idempotent, monotone, within half a unit in the last place
    r = orc.to_storage(y, "f16")
    np.testing.assert_array_equal(orc.to_storage(r, "f16"), r)
    big = np.abs(y) >= 2.0 ** -14
    assert np.all(np.abs(r - y)[big] <= 2.0 ** -11 * np.abs(y)[big])
