"""The comparison rules of the GPU parity tests, checked on the CPU against the oracle alone: the free-running
protocol's score band (a token may end in a different state on the two sides only if its score is within 2e-3 of
the score at one of eq. 10's two cuts)."""
import numpy as np
import pytest

from oracle import arkv_oracle as O
from helpers import TOL, score_band_check


def _case(seed, n=400, n_o=90, b=250):
    r = np.random.default_rng(seed)
    S = r.random(n) ** 4 + 1e-3
    pos = r.permutation(n)
    state = np.where(r.random(n) < 0.2, O.STATE_Q, O.STATE_O).astype(np.int8)
    return S, pos, state, n_o, b


def test_identical_choices_pass():
    S, pos, state, n_o, b = _case(0)
    new = O.tailor_assign(S, pos, state, n_o, b)
    assert score_band_check(S, pos, new, new.copy(), n_o, b) is True


@pytest.mark.parametrize("seed", range(5))
def test_rounding_sized_noise_stays_inside_the_band(seed):
    """Scores perturbed by 1e-6 relative (what fp32 accumulation does): whatever the perturbed ranking changes
    lies next to a cut."""
    S, pos, state, n_o, b = _case(seed)
    # plant near-ties on both cuts so that the perturbation does flip some tokens
    order = np.argsort(-S)
    for cut in (n_o, b):
        S[order[cut - 2:cut + 2]] = S[order[cut]] * (1 + np.array([2e-7, 1e-7, 0.0, -1e-7]))
    ref = O.tailor_assign(S, pos, state, n_o, b)
    r = np.random.default_rng(100 + seed)
    flipped = 0
    for _ in range(20):
        got = O.tailor_assign(S * (1 + 1e-6 * r.standard_normal(len(S))), pos, state, n_o, b)
        flipped += not score_band_check(S, pos, ref, got, n_o, b)
    assert flipped > 0


def test_a_token_far_from_both_cuts_fails():
    S, pos, state, n_o, b = _case(1)
    ref = O.tailor_assign(S, pos, state, n_o, b)
    order = np.argsort(-S)
    got = ref.copy()
    j = order[5]                                   # a top token, far above both cuts
    assert abs(S[j] - S[order[n_o]]) / S[order[n_o]] > 10 * TOL
    got[j] = O.STATE_E
    with pytest.raises(AssertionError):
        score_band_check(S, pos, ref, got, n_o, b)
    got = ref.copy()
    j = order[-1]                                  # the lowest-ranked token, kept by mistake
    got[j] = O.STATE_Q
    with pytest.raises(AssertionError):
        score_band_check(S, pos, ref, got, n_o, b)


def test_gross_score_errors_fail():
    """Scores off by 5 % re-rank tokens well outside the band."""
    S, pos, state, n_o, b = _case(2, n=4000, n_o=900, b=2500)
    ref = O.tailor_assign(S, pos, state, n_o, b)
    r = np.random.default_rng(7)
    got = O.tailor_assign(S * (1 + 0.05 * r.standard_normal(len(S))), pos, state, n_o, b)
    with pytest.raises(AssertionError):
        score_band_check(S, pos, ref, got, n_o, b)
