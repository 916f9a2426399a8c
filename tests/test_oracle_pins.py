"""Pins of the float64 CPU oracle against what the paper and mathematics fix.

No implementation exists to compare against, and the paper prints no worked
numeric example of a verification step, so every pin here is one of: an
independent library routine (scipy), a hand-derived closed form (also stored
under tests/golden/), an identity the paper proves (App. A.1 output law,
Eq. (7), Thm 3.2, App. A.2), a special case that reduces to textbook
speculative sampling (Sec. 3.2, lambda = 0), or brute force on tiny inputs.
"""
import math
import os
from fractions import Fraction

import numpy as np
import pytest
from scipy import special, stats

from oracle import cos_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rng(seed):
    return np.random.default_rng(seed)


def _bf16_bits(x32: np.ndarray) -> np.ndarray:
    """float32 values that are exactly representable in bf16 -> their 16-bit patterns."""
    bits = x32.astype(np.float32).view(np.uint32)
    assert np.all((bits & 0xFFFF) == 0)
    return (bits >> 16).astype(np.uint16)


def _round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even to bf16, returned as float32 values."""
    bits = x.astype(np.float32).view(np.uint32).astype(np.uint64)
    rounded = (bits + 0x7FFF + ((bits >> 16) & 1)) & 0xFFFF0000
    return rounded.astype(np.uint32).view(np.float32)


def _read_golden(name):
    """Golden files: '#' comments, then 'key: v v v' lines of decimals or fractions a/b."""
    out = {}
    with open(os.path.join(GOLDEN, name)) as fh:
        for line in fh:
            line = line.split("#")[0].strip()
            if not line:
                continue
            key, vals = line.split(":")
            out[key.strip()] = np.array([float(Fraction(v)) for v in vals.split()])
    return out


# --------------------------------------------------------------------------
# storage formats
# --------------------------------------------------------------------------

def test_f16_widening_every_bit_pattern_against_numpy():
    """IEEE binary16 -> float64 is exact: all 65536 patterns against numpy's float16 (NaNs as NaNs)."""
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    got = O.row_to_f64(bits, O.DTYPE_F16)
    want = bits.view(np.float16).astype(np.float64)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], want[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(want[~nan]))          # -0.0 keeps its sign
    known = np.array([0x3C00, 0xC000, 0x7BFF, 0x0001, 0x0400, 0x3555, 0xFC00], dtype=np.uint16)
    assert np.array_equal(O.row_to_f64(known, O.DTYPE_F16),
                          np.array([1.0, -2.0, 65504.0, 2.0 ** -24, 2.0 ** -14, 0.333251953125, -np.inf]))


def test_f16_logits_through_the_whole_step_equal_their_float32_copies():
    """binary16 -> float32 is exact, so the same values stored as float32 must give the same result."""
    rng = _rng(17)
    n, B, gamma, V = 2, 50, 3, 64
    h = (rng.standard_normal((n, B, gamma + 1, V)) * 2).astype(np.float16)
    drafts = rng.integers(0, V, (B, gamma)).astype(np.int32)
    proposer = rng.integers(0, n, B).astype(np.int32)
    ua, ur = rng.random((B, gamma)), rng.random(B)
    for mode, w in ((O.ENSEMBLE, [0.3, 0.7]), (O.CONTRASTIVE, [0.5, 0.1])):
        a = O.verify(h.view(np.uint16), O.DTYPE_F16, drafts, proposer, mode, w, ua, ur, all_positions=True)
        b = O.verify(h.astype(np.float32), O.DTYPE_F32, drafts, proposer, mode, w, ua, ur, all_positions=True)
        assert a.status == 0 and b.status == 0
        assert np.array_equal(a.out_tokens, b.out_tokens) and np.array_equal(a.r_at_draft, b.r_at_draft)
        assert np.array_equal(a.cdf_hi, b.cdf_hi)
    assert O.verify(h.view(np.uint16), 3, drafts, proposer, O.ENSEMBLE, [0.3, 0.7], ua, ur).status == -3


def test_bf16_widening_known_patterns():
    bits = np.array([0x3F80, 0xC000, 0x0000, 0x8000, 0x7F80, 0xFF80, 0x3DCD, 0x4049], dtype=np.uint16)
    want = np.array([1.0, -2.0, 0.0, -0.0, np.inf, -np.inf, 0.10009765625, 3.140625])
    got = O.row_to_f64(bits, O.DTYPE_BF16)
    assert np.array_equal(got, want)
    assert np.signbit(got[3])


def test_f32_widening_is_exact():
    x = _rng(1).standard_normal(1000).astype(np.float32)
    assert np.array_equal(O.row_to_f64(x, O.DTYPE_F32), x.astype(np.float64))


# --------------------------------------------------------------------------
# softmax (Sec. 3.2)
# --------------------------------------------------------------------------

@pytest.mark.parametrize("V,scale", [(1, 1.0), (8, 1.0), (1000, 3.0), (32000, 2.5), (128256, 3.0)])
def test_softmax_matches_library_routine(V, scale):
    l = _rng(V).standard_normal(V) * scale
    s = O.softmax(l)
    assert np.allclose(s, special.softmax(l), rtol=1e-13, atol=0)
    assert abs(s.sum() - 1.0) < 1e-12


def test_softmax_closed_form_and_shift_invariance():
    g = _read_golden("softmax_hand.txt")
    s = O.softmax(g["logits"])
    assert np.allclose(s, g["softmax"], rtol=1e-15, atol=0)
    # softmax(log p) = p and softmax(l + c) = softmax(l)
    p = np.array([0.5, 0.25, 0.125, 0.125])
    assert np.allclose(O.softmax(np.log(p)), p, rtol=1e-15)
    assert np.allclose(O.softmax(np.log(p) + 700.0), p, rtol=1e-12)
    assert np.allclose(O.softmax(np.log(p) - 700.0), p, rtol=1e-12)


def test_softmax_minus_inf_logit_has_probability_zero():
    s = O.softmax(np.array([0.0, -np.inf, math.log(3.0)]))
    assert np.allclose(s, [0.25, 0.0, 0.75], rtol=1e-15)


# --------------------------------------------------------------------------
# weighted ensemble (Eq. 4; n-model coefficients of Sec. 4.1 / Alg. 2)
# --------------------------------------------------------------------------

def test_ensemble_hand_example():
    g = _read_golden("ensemble_eq4_hand.txt")
    s = np.stack([O.softmax(np.log(g["p0"])), O.softmax(np.log(g["p1"]))])
    r = O.combine_ensemble(s, g["w"])
    assert np.allclose(r, g["r"], rtol=1e-15)


def test_ensemble_properties():
    rng = _rng(7)
    n, V = 4, 500
    s = np.stack([O.softmax(rng.standard_normal(V) * 3) for _ in range(n)])
    w = np.array([0.1, 0.2, 0.3, 0.4])
    r = O.combine_ensemble(s, w)
    assert abs(r.sum() - 1.0) < 1e-12
    assert np.allclose(r, (w[:, None] * s).sum(0), rtol=1e-14)        # Eq. (4) retyped with numpy
    for m in range(n):                                                 # one-hot weights pick one model
        e = np.zeros(n)
        e[m] = 1.0
        assert np.array_equal(O.combine_ensemble(s, e), s[m])
    # a transposed operand or swapped weights would change this asymmetric case
    r2 = O.combine_ensemble(s[::-1].copy(), w)
    assert not np.allclose(r, r2)


@pytest.mark.parametrize("n", [2, 3, 4])
def test_thm_3_2_acceptance_rate_lower_bound(n):
    """Thm 3.2: with the proposer's weight lambda, alpha = sum min(q, r) >= lambda."""
    rng = _rng(100 + n)
    for trial in range(20):
        V = 64
        s = np.stack([O.softmax(rng.standard_normal(V) * 4) for _ in range(n)])
        w = rng.dirichlet(np.ones(n))
        r = O.combine_ensemble(s, w)
        for pi in range(n):
            alpha = np.minimum(s[pi], r).sum()
            assert alpha >= w[pi] - 1e-12
    # equality iff the distributions do not overlap
    s = np.array([[0.5, 0.5, 0.0, 0.0], [0.0, 0.0, 0.25, 0.75]])
    r = O.combine_ensemble(s, np.array([0.3, 0.7]))
    assert abs(np.minimum(s[0], r).sum() - 0.3) < 1e-15


# --------------------------------------------------------------------------
# contrastive combine (Eq. 5) + plausibility mask
# --------------------------------------------------------------------------

def test_contrastive_alpha0_is_eq5():
    rng = _rng(11)
    V = 777
    lp, lq = rng.standard_normal(V) * 3, rng.standard_normal(V) * 2
    for mu in (0.0, 0.1, 0.5, 1.0):
        r, count = O.combine_contrastive(lp, lq, mu, 0.0)
        assert count == V
        assert np.allclose(r, special.softmax(lp - mu * lq), rtol=1e-12)
    r, _ = O.combine_contrastive(lp, lq, 0.0, 0.0)       # mu = 0: the expert alone
    assert np.allclose(r, O.softmax(lp), rtol=1e-13)
    # expert and amateur are not interchangeable
    r_swapped, _ = O.combine_contrastive(lq, lp, 0.5, 0.0)
    r_ok, _ = O.combine_contrastive(lp, lq, 0.5, 0.0)
    assert not np.allclose(r_ok, r_swapped)


def test_contrastive_mask_hand_example():
    g = _read_golden("contrastive_eq5_mask_hand.txt")
    r, count = O.combine_contrastive(np.log(g["p_expert_unnorm"]), np.log(g["p_amateur_unnorm"]),
                                     float(g["mu"][0]), float(g["alpha_cd"][0]))
    assert count == int(g["mask_size"][0])
    assert np.allclose(r, g["r"], rtol=1e-14, atol=0)


def test_contrastive_mask_properties():
    rng = _rng(12)
    V = 2000
    lp, lq = rng.standard_normal(V) * 3, rng.standard_normal(V) * 2
    p = special.softmax(lp)
    for alpha_cd in (0.5, 0.1, 0.01, 1.0):
        r, count = O.combine_contrastive(lp, lq, 0.5, alpha_cd)
        mask = p >= alpha_cd * p.max() * (1 - 1e-12)
        assert count == mask.sum()
        assert np.all(r[~mask] == 0.0)
        assert r[np.argmax(lp)] > 0.0                    # the expert's argmax is always plausible
        assert abs(r.sum() - 1.0) < 1e-12
        c = lp - 0.5 * lq
        want = np.where(mask, np.exp(c - c[mask].max()), 0.0)
        assert np.allclose(r, want / want.sum(), rtol=1e-12)
    # threshold exactly on a token: '>=' keeps it (bf16-exact difference of ln(alpha) impossible in
    # general, so use alpha_cd = 1: only ties with the maximum survive)
    lp2 = np.array([1.0, 3.0, 3.0, 2.0])
    r, count = O.combine_contrastive(lp2, np.zeros(4), 0.5, 1.0)
    assert count == 2 and np.allclose(r, [0, 0.5, 0.5, 0])


# --------------------------------------------------------------------------
# acceptance test (Eq. 2 / Eq. 6)
# --------------------------------------------------------------------------

def test_accept_rule_and_conventions():
    assert O.accept(0.49, 0.1, 0.2) == (True, 0.5)
    assert O.accept(0.5, 0.1, 0.2) == (False, 0.5)       # strict '<'
    assert O.accept(0.999999999, 0.3, 0.2)[0]            # ratio >= 1: always accepted
    assert O.accept(0.0, 0.0, 0.2) == (False, 0.0)       # r(d) = 0: never accepted, even at u = 0
    assert O.accept(0.0, 0.0, 0.0) == (False, 0.0)
    acc, ratio = O.accept(0.9, 0.1, 0.0)
    assert acc and math.isinf(ratio)
    # r and q are not interchangeable
    assert O.accept(0.6, 0.2, 0.1)[0] and not O.accept(0.6, 0.1, 0.2)[0]


# --------------------------------------------------------------------------
# residual (Sec. 3.2, App. A.1) and Eq. (7)
# --------------------------------------------------------------------------

def test_residual_mass_identities():
    rng = _rng(21)
    for trial in range(10):
        V = 300
        q = O.softmax(rng.standard_normal(V) * 3)
        p = O.softmax(rng.standard_normal(V) * 3)
        r = O.combine_ensemble(np.stack([q, p]), np.array([0.4, 0.6]))
        f, F = O.sample_weights(r, q, residual=True)
        assert np.all(f >= 0)
        assert abs((f / F).sum() - 1.0) < 1e-12                          # norm(.) sums to 1
        assert abs(F - (1.0 - np.minimum(q, r).sum())) < 1e-12           # App. A.1
        assert abs(F - 0.5 * np.abs(r - q).sum()) < 1e-12                # Eq. (7)
        assert np.all(f[r <= q] == 0.0)
        assert np.allclose(f[r > q], (r - q)[r > q], rtol=0, atol=0)
        fb, Fb = O.sample_weights(r, q, residual=False)                  # bonus: f = r
        assert np.array_equal(fb, r) and abs(Fb - 1.0) < 1e-12
    # sign: max(0, r - q), not max(0, q - r)
    f, F = O.sample_weights(np.array([0.7, 0.3]), np.array([0.2, 0.8]), residual=True)
    assert np.allclose(f, [0.5, 0.0]) and abs(F - 0.5) < 1e-15


# --------------------------------------------------------------------------
# inverse CDF
# --------------------------------------------------------------------------

def test_inverse_cdf_brute_force():
    rng = _rng(31)
    for V in (1, 2, 5, 8):
        for trial in range(20):
            f = rng.random(V) * (rng.random(V) < 0.7)
            if f.sum() == 0:
                f[rng.integers(V)] = 0.3
            F = float(np.sum(f))
            cum = np.cumsum(f) / F
            pos = np.nonzero(f)[0]
            edges = np.concatenate([[0.0], cum[pos]])
            us = [0.0, np.nextafter(1.0, 0.0)]
            for e in edges[:-1]:
                us += [e + 1e-9, max(e - 1e-9, 0.0)]
            us += list(rng.random(30))
            for u in us:
                tok, clamped, lo, hi = O.inverse_cdf(f, F, u)
                want = int(pos[np.searchsorted(cum[pos], u, side="right")]) if u < cum[pos][-1] else int(pos[-1])
                assert tok == want, (f, u, tok, want)
                assert f[tok] > 0
                assert lo <= u + 1e-12 and (u < hi + 1e-12)
                assert abs((hi - lo) - f[tok] / F) < 1e-12
            assert O.inverse_cdf(f, F, 0.0)[0] == pos[0]                  # u = 0: first token with mass
            assert O.inverse_cdf(f, F, np.nextafter(1.0, 0.0))[0] == pos[-1]  # u -> 1-: last one


def test_inverse_cdf_tail_clamp():
    f = np.array([0.25, 0.0, 0.5, 0.0])
    tok, clamped, lo, hi = O.inverse_cdf(f, 0.75, 1.0)    # t == F: no prefix exceeds it
    assert (tok, clamped) == (2, True)
    tok, clamped, _, _ = O.inverse_cdf(f, 0.75, 0.5)
    assert (tok, clamped) == (2, False)


# --------------------------------------------------------------------------
# whole step: helpers
# --------------------------------------------------------------------------

def _verify_from_probs(probs, drafts, proposer, mode, weights, u_acc, u_res, **kw):
    """probs: [n][B][gamma+1][V] strictly positive; fed as float32 logits = log(probs)."""
    logits = np.log(probs).astype(np.float32)
    return logits, O.verify(logits, O.DTYPE_F32, drafts, proposer, mode, weights, u_acc, u_res, **kw)


def _step_dists(logits, b, j, pi, mode, weights):
    """(q, r) of one position from the oracle's own step functions."""
    n = logits.shape[0]
    l = [O.row_to_f64(logits[m, b, j], O.DTYPE_F32) for m in range(n)]
    s = np.stack([O.softmax(x) for x in l])
    if mode == O.ENSEMBLE:
        r = O.combine_ensemble(s, weights)
    elif mode == O.LOGIT_MIX:
        r = O.combine_logit_mix(np.stack(l), weights)
    else:
        r, _ = O.combine_contrastive(l[0], l[1], weights[0], weights[1])
    return s[pi], r


# --------------------------------------------------------------------------
# App. A.1: the output law equals r  (pin (a))
# --------------------------------------------------------------------------

_LAW_WEIGHTS = {O.ENSEMBLE: [0.35, 0.65], O.CONTRASTIVE: [0.5, 0.1], O.LOGIT_MIX: [1.3, -0.4]}


@pytest.mark.parametrize("mode", [O.ENSEMBLE, O.CONTRASTIVE, O.LOGIT_MIX])
def test_output_law_exact_enumeration_V8(mode):
    """P(x) = sum_x' q(x') [a(x') 1{x = x'} + (1 - a(x')) res(x)] must equal r(x)."""
    rng = _rng(41 + mode)
    V, gamma, n = 8, 3, 2
    weights = np.array(_LAW_WEIGHTS[mode])
    logits = (rng.standard_normal((n, 1, gamma + 1, V)) * 2).astype(np.float32)
    for pi in range(n):
        for j in range(gamma):
            q, r = _step_dists(logits, 0, j, pi, mode, weights)
            f, F = O.sample_weights(r, q, residual=True)
            law = np.zeros(V)
            p_reject = 0.0
            for xp in range(V):
                ratio = O.accept(0.0, r[xp], q[xp])[1]
                a = min(1.0, ratio)                  # measure of {u in [0,1): u < min(1, ratio)}
                law[xp] += q[xp] * a
                p_reject += q[xp] * (1.0 - a)
            law += p_reject * f / F
            assert np.allclose(law, r, rtol=0, atol=1e-12)
            assert abs(p_reject - F) < 1e-12         # App. A.1: P(reject) = sum max(r - q, 0)


@pytest.mark.parametrize("mode", [O.ENSEMBLE, O.CONTRASTIVE, O.LOGIT_MIX])
def test_output_law_chi_square_monte_carlo_V8_gamma3(mode):
    """10^6 seeded trials through the full step: tokens at position k (given it was
    reached) follow r_k, and the bonus token follows r_gamma."""
    rng = _rng(51 + mode)
    V, gamma, n, B = 8, 3, 2, 1_000_000
    weights = np.array({O.ENSEMBLE: [0.4, 0.6], O.CONTRASTIVE: [0.5, 0.1], O.LOGIT_MIX: [0.7, 0.6]}[mode])
    row = (rng.standard_normal((n, 1, gamma + 1, V)) * 1.5).astype(np.float32)
    logits = np.ascontiguousarray(np.broadcast_to(row, (n, B, gamma + 1, V)))
    pi = 1
    proposer = np.full(B, pi, dtype=np.int32)
    drafts = np.empty((B, gamma), dtype=np.int32)
    dists = []
    for j in range(gamma + 1):
        q, r = _step_dists(logits, 0, j, pi, mode, weights)
        dists.append((q, r))
        if j < gamma:                                    # Eq. (1): drafts ~ q
            drafts[:, j] = rng.choice(V, size=B, p=q / q.sum())
    res = O.verify(logits, O.DTYPE_F32, drafts, proposer, mode, weights,
                   rng.random((B, gamma)), rng.random(B))
    assert res.status == 0
    alen = res.accepted_len
    for k in range(gamma + 1):
        reached = alen >= k
        toks = res.out_tokens[reached, k]
        assert np.all(toks >= 0)
        r = dists[k][1]
        counts = np.bincount(toks, minlength=V).astype(np.float64)
        keep = r > 0
        assert counts[~keep].sum() == 0                 # never a token outside the support of r
        if keep.sum() < 2:                              # a one-token mask leaves nothing to test
            continue
        chi2, pval = stats.chisquare(counts[keep], r[keep] / r[keep].sum() * counts.sum())
        assert pval > 1e-3, (k, pval)
    # first-rejection scan: P(accepted_len >= k) = prod_{j<k} alpha_j  (generalises App. A.2)
    surv = 1.0
    for k in range(1, gamma + 1):
        q, r = dists[k - 1]
        surv *= np.minimum(q, r).sum()
        phat = np.mean(alen >= k)
        sigma = math.sqrt(surv * (1 - surv) / B)
        assert abs(phat - surv) < 5 * sigma, (k, phat, surv)


# --------------------------------------------------------------------------
# r == q  =>  every draft accepted  (pin (b))
# --------------------------------------------------------------------------

def test_r_equals_q_accepts_everything():
    rng = _rng(61)
    V, gamma, B = 50, 4, 64
    u_acc = rng.random((B, gamma))
    u_acc[0, :] = np.nextafter(1.0, 0.0)                  # the largest u in [0,1)
    u_res = rng.random(B)
    drafts = rng.integers(0, V, (B, gamma)).astype(np.int32)
    one = (rng.standard_normal((1, B, gamma + 1, V)) * 3).astype(np.float32)
    other = (rng.standard_normal((1, B, gamma + 1, V)) * 3).astype(np.float32)
    # (i) identical logits for all models, any weights
    res = O.verify(np.concatenate([one, one, one]), O.DTYPE_F32, drafts, np.arange(B) % 3, O.ENSEMBLE,
                   [0.2, 0.5, 0.3], u_acc, u_res)
    assert np.all(res.accepted_len == gamma)
    assert np.array_equal(res.out_tokens[:, :gamma], drafts) and np.all(res.out_tokens[:, gamma] >= 0)
    # (ii) weights one-hot on the proposer
    res = O.verify(np.concatenate([one, other]), O.DTYPE_F32, drafts, np.ones(B, dtype=np.int32), O.ENSEMBLE,
                   [0.0, 1.0], u_acc, u_res)
    assert np.all(res.accepted_len == gamma)
    # (iii) contrastive with mu = 0, no mask, proposer = expert
    res = O.verify(np.concatenate([one, other]), O.DTYPE_F32, drafts, np.zeros(B, dtype=np.int32),
                   O.CONTRASTIVE, [0.0, 0.0], u_acc, u_res)
    assert np.all(res.accepted_len == gamma)
    # and the contrary: proposer = the other model gives rejections
    res = O.verify(np.concatenate([one, other]), O.DTYPE_F32, drafts, np.zeros(B, dtype=np.int32), O.ENSEMBLE,
                   [0.0, 1.0], u_acc, u_res)
    assert np.any(res.accepted_len < gamma)


# --------------------------------------------------------------------------
# lambda = 0  =>  textbook speculative sampling  (Sec. 3.2)
# --------------------------------------------------------------------------

def _textbook_speculative_sampling(p, q, drafts, u_acc, u_res):
    """Independent float64 re-derivation: target p[j], proposer q[j], j = 0..gamma."""
    gamma = len(drafts)
    out = []
    for j in range(gamma):
        d = drafts[j]
        if u_acc[j] < min(1.0, p[j][d] / q[j][d]):
            out.append(int(d))
            continue
        res = np.maximum(p[j] - q[j], 0.0)
        cdf = np.cumsum(res)
        return j, out + [int(np.searchsorted(cdf, u_res * cdf[-1], side="right"))]
    cdf = np.cumsum(p[gamma])
    return gamma, out + [int(np.searchsorted(cdf, u_res * cdf[-1], side="right"))]


def test_lambda0_reduces_to_vanilla_speculative_decoding():
    rng = _rng(71)
    V, gamma, B = 40, 5, 400
    probs = rng.dirichlet(np.ones(V) * 0.5, size=(2, B, gamma + 1)) + 1e-6
    probs /= probs.sum(-1, keepdims=True)
    drafts = rng.integers(0, V, (B, gamma)).astype(np.int32)
    u_acc, u_res = rng.random((B, gamma)), rng.random(B)
    proposer = np.zeros(B, dtype=np.int32)               # model 0 proposes, weight 0 on it: r = p_1
    logits, res = _verify_from_probs(probs, drafts, proposer, O.ENSEMBLE, [0.0, 1.0], u_acc, u_res)
    l64 = logits.astype(np.float64)
    sm = special.softmax(l64, axis=-1)
    lens = []
    for b in range(B):
        alen, toks = _textbook_speculative_sampling(sm[1, b], sm[0, b], drafts[b], u_acc[b], u_res[b])
        lens.append(alen)
        assert res.accepted_len[b] == alen
        assert list(res.out_tokens[b, :alen + 1]) == toks
        assert np.all(res.out_tokens[b, alen + 1:] == -1)
    assert len(set(lens)) == gamma + 1                   # every outcome 0..gamma occurred


# --------------------------------------------------------------------------
# first rejection: brute force on tiny inputs and App. A.2's expectation
# --------------------------------------------------------------------------

def test_first_rejection_brute_force_and_padding():
    rng = _rng(81)
    V, gamma, B, n = 6, 4, 500, 2
    logits = (rng.standard_normal((n, B, gamma + 1, V)) * 2).astype(np.float32)
    drafts = rng.integers(0, V, (B, gamma)).astype(np.int32)
    proposer = rng.integers(0, n, B).astype(np.int32)
    u_acc, u_res = rng.random((B, gamma)), rng.random(B)
    w = np.array([0.3, 0.7])
    res = O.verify(logits, O.DTYPE_F32, drafts, proposer, O.ENSEMBLE, w, u_acc, u_res, all_positions=True)
    res_seq = O.verify(logits, O.DTYPE_F32, drafts, proposer, O.ENSEMBLE, w, u_acc, u_res)
    assert np.array_equal(res.accepted_len, res_seq.accepted_len)       # diagnostics do not change decisions
    assert np.array_equal(res.out_tokens, res_seq.out_tokens)
    for b in range(B):
        flags = []
        for j in range(gamma):
            q, r = _step_dists(logits, b, j, proposer[b], O.ENSEMBLE, w)
            d = drafts[b, j]
            flags.append(u_acc[b, j] < min(1.0, r[d] / q[d]))
            assert res.r_at_draft[b, j] == r[d] and res.q_at_draft[b, j] == q[d]
        alen = flags.index(False) if False in flags else gamma
        assert res.accepted_len[b] == alen
        assert np.array_equal(res.out_tokens[b, :alen], drafts[b, :alen])
        assert 0 <= res.out_tokens[b, alen] < V
        assert np.all(res.out_tokens[b, alen + 1:] == -1)
        # the sampled token comes from the residual of position alen (or r at gamma)
        q, r = _step_dists(logits, b, alen, proposer[b], O.ENSEMBLE, w)
        f, F = O.sample_weights(r, q, residual=alen < gamma)
        assert res.out_tokens[b, alen] == O.inverse_cdf(f, F, u_res[b])[0]
        assert abs(res.sample_mass[b] - F) < 1e-15
        # positions after the first rejection were never evaluated in the sequential run
        assert np.all(np.isnan(res_seq.ratio[b, alen + 1:]))


def test_expected_tokens_per_cycle_app_a2():
    """E[#tokens] = (1 - alpha^gamma)/(1 - alpha) without the bonus token (App. A.2)."""
    rng = _rng(91)
    V, gamma, B, n = 8, 4, 400_000, 2
    row = (rng.standard_normal((n, 1, 1, V)) * 1.5).astype(np.float32)
    logits = np.ascontiguousarray(np.broadcast_to(row, (n, B, gamma + 1, V)))
    w = np.array([0.5, 0.5])
    q, r = _step_dists(logits, 0, 0, 0, O.ENSEMBLE, w)
    alpha = np.minimum(q, r).sum()
    assert abs(alpha - (1 - 0.5 * np.abs(q - r).sum())) < 1e-12          # Eq. (7)
    drafts = rng.choice(V, size=(B, gamma), p=q / q.sum()).astype(np.int32)
    res = O.verify(logits, O.DTYPE_F32, drafts, np.zeros(B, dtype=np.int32), O.ENSEMBLE, w,
                   rng.random((B, gamma)), rng.random(B))
    ntok = np.minimum(res.accepted_len + 1, gamma)                       # no bonus counted
    want = (1 - alpha ** gamma) / (1 - alpha)
    sigma = ntok.std() / math.sqrt(B)
    assert abs(ntok.mean() - want) < 5 * sigma


# --------------------------------------------------------------------------
# bf16 path, indexing, thread independence, argument checks
# --------------------------------------------------------------------------

def test_bf16_and_f32_storage_agree_on_bf16_representable_logits():
    rng = _rng(101)
    n, B, gamma, V = 3, 5, 3, 97
    l32 = _round_to_bf16(rng.standard_normal((n, B, gamma + 1, V)) * 3)
    drafts = rng.integers(0, V, (B, gamma)).astype(np.int32)
    proposer = (np.arange(B) % n).astype(np.int32)
    u_acc, u_res = rng.random((B, gamma)), rng.random(B)
    a = O.verify(l32, O.DTYPE_F32, drafts, proposer, O.ENSEMBLE, [0.5, 0.3, 0.2], u_acc, u_res)
    b = O.verify(_bf16_bits(l32), O.DTYPE_BF16, drafts, proposer, O.ENSEMBLE, [0.5, 0.3, 0.2], u_acc, u_res)
    assert np.array_equal(a.accepted_len, b.accepted_len) and np.array_equal(a.out_tokens, b.out_tokens)


def test_layout_is_model_batch_position_vocab():
    """Permuting batch rows permutes outputs; swapping two models with swapped weights
    and proposer indices changes nothing."""
    rng = _rng(111)
    n, B, gamma, V = 2, 6, 3, 33
    logits = (rng.standard_normal((n, B, gamma + 1, V)) * 2).astype(np.float32)
    drafts = rng.integers(0, V, (B, gamma)).astype(np.int32)
    proposer = rng.integers(0, n, B).astype(np.int32)
    u_acc, u_res = rng.random((B, gamma)), rng.random(B)
    w = np.array([0.3, 0.7])
    ref = O.verify(logits, O.DTYPE_F32, drafts, proposer, O.ENSEMBLE, w, u_acc, u_res)
    perm = rng.permutation(B)
    p = O.verify(logits[:, perm], O.DTYPE_F32, drafts[perm], proposer[perm], O.ENSEMBLE, w, u_acc[perm], u_res[perm])
    assert np.array_equal(p.out_tokens, ref.out_tokens[perm])
    s = O.verify(logits[::-1], O.DTYPE_F32, drafts, 1 - proposer, O.ENSEMBLE, w[::-1], u_acc, u_res)
    assert np.array_equal(s.out_tokens, ref.out_tokens)


def test_thread_count_does_not_change_results():
    rng = _rng(121)
    n, B, gamma, V = 2, 40, 3, 200
    logits = (rng.standard_normal((n, B, gamma + 1, V)) * 2).astype(np.float32)
    drafts = rng.integers(0, V, (B, gamma)).astype(np.int32)
    proposer = rng.integers(0, n, B).astype(np.int32)
    u_acc, u_res = rng.random((B, gamma)), rng.random(B)
    a = O.verify(logits, O.DTYPE_F32, drafts, proposer, O.CONTRASTIVE, [0.5, 0.1], u_acc, u_res, num_threads=1)
    b = O.verify(logits, O.DTYPE_F32, drafts, proposer, O.CONTRASTIVE, [0.5, 0.1], u_acc, u_res, num_threads=4)
    assert np.array_equal(a.out_tokens, b.out_tokens) and np.array_equal(a.cdf_hi, b.cdf_hi)


def test_argument_checks():
    rng = _rng(131)
    n, B, gamma, V = 2, 2, 2, 5
    logits = rng.standard_normal((n, B, gamma + 1, V)).astype(np.float32)
    drafts = np.zeros((B, gamma), dtype=np.int32)
    prop = np.zeros(B, dtype=np.int32)
    u_acc, u_res = rng.random((B, gamma)), rng.random(B)
    assert O.verify(logits, O.DTYPE_F32, drafts, prop, O.ENSEMBLE, [0.5, 0.6], u_acc, u_res).status == -5
    assert O.verify(logits, O.DTYPE_F32, drafts, prop, O.ENSEMBLE, [1.5, -0.5], u_acc, u_res).status == -5
    assert O.verify(logits, O.DTYPE_F32, drafts, prop, O.CONTRASTIVE, [0.5, 1.5], u_acc, u_res).status == -5
    assert O.verify(logits, O.DTYPE_F32, drafts, prop, 7, [0.5, 0.5], u_acc, u_res).status == -4
    bad = drafts.copy()
    bad[0, 0] = V
    assert O.verify(logits, O.DTYPE_F32, bad, prop, O.ENSEMBLE, [0.5, 0.5], u_acc, u_res).status == -2
    l3 = rng.standard_normal((3, B, gamma + 1, V)).astype(np.float32)
    assert O.verify(l3, O.DTYPE_F32, drafts, prop, O.CONTRASTIVE, [0.5, 0.1, 0.0], u_acc, u_res).status == -4
