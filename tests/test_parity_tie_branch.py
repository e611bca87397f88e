"""The merge check of the GPU parity suite accepts a result that differs from the oracle only where the
oracle's own margin is inside the 1e-4 tie band, and only if that result is itself a valid choice.  The
validator is exercised here on the CPU with hand-made 'library outputs' (no GPU, no library call)."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from oracle import tokencarve_oracle as orc   # noqa: E402
from tests import parity                       # noqa: E402


class _P:
    k_prune, k_final = 6, 5


def _case():
    # Set A = tokens 0,1,2 ; Set B = 3,4,5.  Token 3 is (almost) equally similar to 0 and 1: a tie at 5e-5.
    n, d = 6, 8
    Z = np.zeros((n, d))
    Z[0, 0] = 1.0
    Z[1, 1] = 1.0
    Z[2, 2] = 1.0
    Z[3, 0], Z[3, 1] = 1.0, 1.0 - 1e-4          # cos with 0: 0.7071..., with 1: 5e-5 * 0.707 less
    Z[4, 2], Z[4, 3] = 1.0, 2.0
    Z[5, 4] = 1.0
    X = np.arange(n * 4, dtype=np.float64).reshape(n, 4)
    order = np.arange(n)
    ref = orc.merge(X, Z, order, _P.k_final, out_dtype="f32")
    sim = orc.similarity(Z, ref["set_a"], ref["set_b"])
    assert (np.sort(sim[0])[-1] - np.sort(sim[0])[-2]) < 1e-4
    return X, Z, order, ref, sim


def test_the_other_side_of_a_tie_is_accepted_and_checked():
    X, Z, order, ref, sim = _case()
    assert ref["merge_dst"][3] == 0                      # the oracle sends 3 to 0
    dst = ref["merge_dst"].copy()
    dst[3] = 1                                           # a library that rounds the other way sends it to 1
    kept, X_out = orc.average_rows(X, dst, "f32")
    parity.check_merge_choice(_P, ref, sim, order, kept, dst, X, X_out, "f32", 0)


def test_a_choice_outside_the_tie_band_is_rejected():
    X, Z, order, ref, sim = _case()
    dst = ref["merge_dst"].copy()
    dst[3] = 2                                           # similarity 0 with token 2: not a tie
    kept, X_out = orc.average_rows(X, dst, "f32")
    with pytest.raises(AssertionError):
        parity.check_merge_choice(_P, ref, sim, order, kept, dst, X, X_out, "f32", 0)


def test_wrong_rows_for_a_valid_choice_are_rejected():
    X, Z, order, ref, sim = _case()
    dst = ref["merge_dst"].copy()
    dst[3] = 1
    kept, X_out = orc.average_rows(X, dst, "f32")
    bad = X_out.copy()
    bad[1, 0] += 1.0                                     # the averaged row of token 1 is off
    with pytest.raises(AssertionError):
        parity.check_merge_choice(_P, ref, sim, order, kept, dst, X, bad, "f32", 0)
    # merging a different token than the cut allows is rejected too
    dst2 = ref["merge_dst"].copy()
    dst2[3] = 3
    dst2[5] = 0
    kept2, X2 = orc.average_rows(X, dst2, "f32")
    with pytest.raises(AssertionError):
        parity.check_merge_choice(_P, ref, sim, order, kept2, dst2, X, X2, "f32", 0)
