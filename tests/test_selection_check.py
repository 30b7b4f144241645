"""The near-tie rule of the GPU parity tests, tested on the CPU with planted mistakes: on a token whose
top-(k+1) normalised logits hold a near-tie several selections are valid, and check_selection must accept
exactly those."""
import numpy as np
import pytest

from tests.gpu_util import check_selection


def _case():
    z = np.array([[5.0, 3.0, 3.0 + 2e-7, 1.0, -2.0],       # experts 1 and 2 tie for second place
                  [4.0, 1.0, 0.5, -1.0, 3.0]])             # no tie: 0 then 4
    ref = np.array([[0, 2], [0, 4]])
    return z, ref


def test_valid_choices_on_a_tie_token_pass():
    z, ref = _case()
    for pick in ([0, 2], [0, 1]):
        tie, merged = check_selection(z, ref, np.array([pick, [0, 4]]), 2)
        assert tie.tolist() == [True, False]
        assert merged.tolist() == [pick, [0, 4]]


@pytest.mark.parametrize("bad, msg", [
    ([[0, 3], [0, 4]], "below the k-th largest"),       # arbitrary wrong expert on the tie token
    ([[2, 0], [0, 4]], "descending"),                   # right experts, wrong slot order
    ([[0, 0], [0, 4]], "repeated"),
    ([[0, 7], [0, 4]], "out of range"),
    ([[0, 2], [4, 0]], "outside near-ties"),            # a token without a tie must match bit for bit
])
def test_planted_mistakes_fail(bad, msg):
    z, ref = _case()
    with pytest.raises(AssertionError, match=msg):
        check_selection(z, ref, np.array(bad), 2)


def test_gates_are_checked_on_every_token():
    z, ref = _case()
    scores = np.maximum(z, 0.0) / np.linalg.norm(z, axis=1, keepdims=True)
    good = np.take_along_axis(scores, ref, axis=1)
    check_selection(z, ref, ref, 2, scores=scores, got_gate=good, tol=1e-6)
    wrong = good.copy()
    wrong[0, 1] *= 1.5                                   # the tie token's second gate
    with pytest.raises(AssertionError, match="gates differ"):
        check_selection(z, ref, ref, 2, scores=scores, got_gate=wrong, tol=1e-6)
