"""Closed-form speed models (Thm 3.1, Thm 3.2 and corollaries, Thm 3.6, App. A.2) against simulations
of the propose/verify process they describe.  CPU only."""
import numpy as np
import pytest

from paper_2502_01662_amd import speedup as S


def _simulate(alpha, gamma_q, gamma_p, c, cycles, rng, alternate):
    """Renewal simulation: each cycle drafts gamma_q tokens (the first is free when the previous cycle,
    gamma_p drafts long, accepted everything and ``alternate`` is on), the verifier runs once, drafts are
    accepted independently with probability alpha up to the first rejection; a rejection appends the
    resampled token, full acceptance appends nothing more.  Returns tokens per unit of time."""
    acc_q = rng.random((cycles, gamma_q)) < alpha
    first_rej = np.where(acc_q.all(axis=1), gamma_q, np.argmin(acc_q, axis=1))
    tokens = np.where(first_rej < gamma_q, first_rej + 1, gamma_q)
    cached = (rng.random((cycles, gamma_p)) < alpha).all(axis=1) if alternate else np.zeros(cycles, bool)
    time = 1.0 + c * (gamma_q - cached.astype(np.float64))
    return tokens.sum() / time.sum()


@pytest.mark.parametrize("alpha,gamma", [(0.0, 3), (0.3, 1), (0.55, 4), (0.8, 6), (0.95, 8), (1.0, 5)])
def test_expected_tokens_matches_simulation(alpha, gamma):
    rng = np.random.default_rng(5)
    rate = _simulate(alpha, gamma, 1, 0.0, 400_000, rng, alternate=False)      # c = 0: time = cycles
    assert rate == pytest.approx(S.expected_tokens(alpha, gamma), rel=5e-3)


@pytest.mark.parametrize("alpha,gamma,c", [(0.5, 2, 0.1), (0.7, 4, 0.3), (0.9, 6, 0.05), (0.6, 3, 1.0)])
def test_naive_speedup_matches_simulation(alpha, gamma, c):
    rng = np.random.default_rng(6)
    rate = _simulate(alpha, gamma, 1, c, 400_000, rng, alternate=False)
    assert rate * (1.0 + c) == pytest.approx(S.naive_cos_speedup(alpha, gamma, c), rel=5e-3)


@pytest.mark.parametrize("alpha,gq,gp,c", [(0.5, 2, 2, 0.2), (0.8, 4, 2, 0.5), (0.9, 3, 5, 1.0), (0.65, 1, 1, 0.4)])
def test_alternate_speedup_matches_simulation(alpha, gq, gp, c):
    rng = np.random.default_rng(7)
    rate = _simulate(alpha, gq, gp, c, 400_000, rng, alternate=True)
    assert rate * (1.0 + c) == pytest.approx(S.alternate_proposal_speedup(alpha, gq, gp, c), rel=5e-3)


def test_alternate_proposal_never_slower_at_length_one():
    # Cor. 3.7: gamma_q = gamma_p = 1 never loses to plain collaboration; equality only at c = 0 or alpha = 0
    for alpha in np.linspace(0.0, 1.0, 21):
        for c in (0.0, 0.05, 0.5, 1.0, 3.0):
            s = S.alternate_proposal_speedup(alpha, 1, 1, c)
            assert s >= 1.0 - 1e-12
            if c > 0 and alpha > 0:
                assert s > 1.0
    # and it is never below Naive-CoS at the same lengths
    for alpha in (0.2, 0.6, 0.9):
        for g in (1, 3, 6):
            assert S.alternate_proposal_speedup(alpha, g, g, 0.3) >= S.naive_cos_speedup(alpha, g, 0.3)


def test_ensemble_bounds_and_corollaries():
    assert S.ensemble_alpha_lower_bound(0.3) == 0.3
    assert S.ensemble_alpha_lower_bound(0.3, may_swap_roles=True) == 0.7          # Cor. 3.3
    for lam in np.linspace(0.0, 1.0, 11):
        assert S.ensemble_alpha_lower_bound(lam, may_swap_roles=True) >= 0.5
    # Cor. 3.4: alpha >= lam > c/(1+c) makes gamma = 2 a strict win
    for c in (0.05, 0.3, 1.0):
        lam = c / (1.0 + c) + 1e-3
        assert S.speeds_up_for_some_gamma(lam, c)
        assert S.naive_cos_speedup(lam, 2, c) > 1.0
        assert not S.speeds_up_for_some_gamma(c / (1.0 + c) - 1e-3, c)
        assert S.naive_cos_speedup(c / (1.0 + c) - 1e-3, 2, c) < 1.0


def test_best_gamma_is_the_grid_maximum_and_grows_with_alpha():
    last = 0
    for alpha in (0.3, 0.6, 0.8, 0.9, 0.97):
        g, s = S.best_gamma(alpha, c=0.1, gamma_max=24)
        assert s == max(S.naive_cos_speedup(alpha, k, 0.1) for k in range(1, 25))
        assert g >= last
        last = g
    g, s = S.best_gamma(0.8, c=0.1, gamma_max=24, alternate=True)
    assert s == max(S.alternate_proposal_speedup(0.8, k, k, 0.1) for k in range(1, 25))


def test_mean_acceptance_and_argument_checks():
    assert S.mean_acceptance([[0.5, 1.0], [0.0, 0.5]]) == 0.5
    with pytest.raises(ValueError):
        S.mean_acceptance([])
    with pytest.raises(ValueError):
        S.expected_tokens(1.2, 3)
    with pytest.raises(ValueError):
        S.expected_tokens(0.5, 0)
    with pytest.raises(ValueError):
        S.naive_cos_speedup(0.5, 2, -1.0)
