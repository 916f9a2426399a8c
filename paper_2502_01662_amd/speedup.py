"""Closed-form speed models of collaborative speculation, for choosing the proposal length.

Host-side arithmetic only (no GPU, no model): the formulas of Sec. 3.2 (Thm 3.1, Thm 3.2 and its
corollaries), Sec. 3.3 (Thm 3.6) and App. A.2, fed by an acceptance rate ``alpha`` — for instance the
mean of the per-position rates ``alpha[B][gamma]`` that ``cos_verify`` can return (Eq. 7).

Cost model of the paper: one call of the verifier costs 1, one call of the proposer costs ``c``;
plain collaborative decoding pays ``1 + c`` per token.  Verification itself is taken to be free.
"""
from __future__ import annotations

from typing import Iterable, Optional, Tuple


def _check_alpha(alpha: float) -> float:
    alpha = float(alpha)
    if not 0.0 <= alpha <= 1.0:
        raise ValueError(f"acceptance rate must lie in [0, 1], got {alpha}")
    return alpha


def expected_tokens(alpha: float, gamma: int) -> float:
    """App. A.2: expected number of tokens one propose/verify cycle appends when the bonus token is
    not appended: ``(1 - alpha^gamma) / (1 - alpha)`` (``gamma`` in the limit alpha -> 1)."""
    alpha = _check_alpha(alpha)
    if gamma < 1:
        raise ValueError("gamma must be at least 1")
    if alpha == 1.0:
        return float(gamma)
    return (1.0 - alpha ** gamma) / (1.0 - alpha)


def naive_cos_speedup(alpha: float, gamma: int, c: float) -> float:
    """Thm 3.1: expected speed-up of Naive-CoS over plain collaborative decoding."""
    if c < 0:
        raise ValueError("cost coefficient must be non-negative")
    return expected_tokens(alpha, gamma) * (1.0 + c) / (1.0 + c * gamma)


def alternate_proposal_speedup(alpha: float, gamma_q: int, gamma_p: int, c: float) -> float:
    """Thm 3.6: expected speed-up of one cycle of the alternate proposal framework in which the
    proposer drafts ``gamma_q`` tokens and the previous cycle (the other model's) drafted ``gamma_p``:
    with probability ``alpha^gamma_p`` the first draft is the cached bonus token and costs nothing."""
    alpha = _check_alpha(alpha)
    if c < 0:
        raise ValueError("cost coefficient must be non-negative")
    if gamma_p < 1:
        raise ValueError("gamma_p must be at least 1")
    return expected_tokens(alpha, gamma_q) * (1.0 + c) / (1.0 + c * gamma_q - (alpha ** gamma_p) * c)


def ensemble_alpha_lower_bound(lam: float, may_swap_roles: bool = False) -> float:
    """Thm 3.2: for r = lam*q + (1-lam)*p with q the proposer, alpha >= lam; if either model may
    propose (Cor. 3.3) the bound is max(lam, 1 - lam) >= 1/2."""
    lam = float(lam)
    if not 0.0 <= lam <= 1.0:
        raise ValueError("lambda must lie in [0, 1]")
    return max(lam, 1.0 - lam) if may_swap_roles else lam


def speeds_up_for_some_gamma(lam: float, c: float) -> bool:
    """Cor. 3.4: lam > c / (1 + c) guarantees a proposal length that beats plain ensembling."""
    return lam > c / (1.0 + c)


def best_gamma(alpha: float, c: float, gamma_max: int = 16, alternate: bool = False) -> Tuple[int, float]:
    """The proposal length in 1..gamma_max with the largest modelled speed-up, and that speed-up.
    ``alternate`` uses Thm 3.6 with both models drafting the same length."""
    best: Optional[Tuple[int, float]] = None
    for g in range(1, gamma_max + 1):
        s = alternate_proposal_speedup(alpha, g, g, c) if alternate else naive_cos_speedup(alpha, g, c)
        if best is None or s > best[1]:
            best = (g, s)
    assert best is not None
    return best


def mean_acceptance(alpha_rows: Iterable[Iterable[float]]) -> float:
    """Average of per-position acceptance rates (Eq. 7), e.g. of the ``alpha`` output of ``cos_verify``
    moved to the host; the single ``alpha`` the theorems take."""
    total, count = 0.0, 0
    for row in alpha_rows:
        for a in row:
            total += float(a)
            count += 1
    if count == 0:
        raise ValueError("no acceptance rates given")
    return total / count
