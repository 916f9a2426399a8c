"""Pins of the oracle's extensions: temperature (Sec. 4.1), the verifier's own bonus token
(Sec. 3.1 / 3.3), per-position proposers (Alg. 2) and the acceptance rate of Eq. (7)."""
import math

import numpy as np
import pytest
from scipy import special, stats

from oracle import cos_oracle as O


def _rng(seed):
    return np.random.default_rng(seed)


def _inputs(rng, n, B, gamma, V, std=2.0):
    logits = (rng.standard_normal((n, B, gamma + 1, V)) * std).astype(np.float32)
    drafts = rng.integers(0, V, (B, gamma)).astype(np.int32)
    proposer = rng.integers(0, n, B).astype(np.int32)
    return logits, drafts, proposer, rng.random((B, gamma)), rng.random(B)


# ---- temperature -----------------------------------------------------------

def test_temperature_step_function_and_library_softmax():
    l = _rng(1).standard_normal(500) * 3
    for T in (0.5, 0.7, 1.0, 2.0):
        s = O.softmax(O.apply_temperature(l, T))
        assert np.allclose(s, special.softmax(l / T), rtol=1e-13)
    # T -> small sharpens, T -> large flattens
    assert O.softmax(O.apply_temperature(l, 0.25)).max() > O.softmax(l).max() > O.softmax(O.apply_temperature(l, 4.0)).max()


@pytest.mark.parametrize("mode,weights", [(O.ENSEMBLE, [0.3, 0.7]), (O.CONTRASTIVE, [0.5, 0.1])])
def test_temperature_equals_prescaled_logits(mode, weights):
    """T = 2 or 1/2 scales float32 logits exactly, so verify(l, T) == verify(l / T, 1) bit for bit."""
    rng = _rng(2 + mode)
    logits, drafts, proposer, ua, ur = _inputs(rng, 2, 200, 3, 64)
    for T in (2.0, 0.5):
        a = O.verify(logits, O.DTYPE_F32, drafts, proposer, mode, weights, ua, ur, temperature=T)
        b = O.verify((logits / np.float32(T)).astype(np.float32), O.DTYPE_F32, drafts, proposer, mode, weights, ua, ur)
        assert a.status == 0 and np.array_equal(a.out_tokens, b.out_tokens) and np.array_equal(a.cdf_hi, b.cdf_hi)
    c = O.verify(logits, O.DTYPE_F32, drafts, proposer, mode, weights, ua, ur, temperature=1.0)
    assert not np.array_equal(a.out_tokens, c.out_tokens)            # the temperature matters


def test_temperature_contrastive_is_softmax_of_scaled_difference():
    rng = _rng(4)
    V, T, mu = 300, 0.7, 0.4
    lp, lq = rng.standard_normal(V) * 3, rng.standard_normal(V) * 2
    r, _ = O.combine_contrastive(O.apply_temperature(lp, T), O.apply_temperature(lq, T), mu, 0.0)
    assert np.allclose(r, special.softmax((lp - mu * lq) / T), rtol=1e-12)


# ---- acceptance rate (Eq. 7) -------------------------------------------------

def test_acceptance_rate_closed_form_and_identity():
    q = np.array([1 / 4, 1 / 2, 1 / 4])
    r = np.array([4 / 16, 5 / 16, 7 / 16])
    assert abs(O.acceptance_rate(q, r) - 13 / 16) < 1e-15             # min = (4, 5, 4)/16, by hand
    rng = _rng(5)
    for _ in range(10):
        q = O.softmax(rng.standard_normal(200) * 3)
        r = O.softmax(rng.standard_normal(200) * 3)
        assert abs(O.acceptance_rate(q, r) - (1 - 0.5 * np.abs(q - r).sum())) < 1e-12   # Eq. (7)
        assert abs(O.acceptance_rate(q, q) - 1.0) < 1e-12


def test_alpha_output_of_the_whole_step():
    rng = _rng(6)
    logits, drafts, proposer, ua, ur = _inputs(rng, 3, 40, 4, 50)
    w = [0.5, 0.3, 0.2]
    res = O.verify(logits, O.DTYPE_F32, drafts, proposer, O.ENSEMBLE, w, ua, ur, all_positions=True, want_alpha=True)
    seq = O.verify(logits, O.DTYPE_F32, drafts, proposer, O.ENSEMBLE, w, ua, ur, want_alpha=True)
    for b in range(40):
        for j in range(4):
            s = np.stack([O.softmax(O.row_to_f64(logits[m, b, j], O.DTYPE_F32)) for m in range(3)])
            r = O.combine_ensemble(s, np.array(w))
            want = np.minimum(s[proposer[b]], r).sum()
            assert abs(res.alpha[b, j] - want) < 1e-12
            assert res.alpha[b, j] >= w[proposer[b]] - 1e-12            # Thm 3.2
            if j <= seq.accepted_len[b]:
                assert seq.alpha[b, j] == res.alpha[b, j]
            else:
                assert math.isnan(seq.alpha[b, j])                     # never evaluated


# ---- the verifier's own bonus token (Sec. 3.1 / 3.3) --------------------------

def test_verifier_bonus_follows_the_verifiers_distribution_and_ignores_other_rows():
    rng = _rng(7)
    n, B, gamma, V = 2, 50_000, 2, 8
    row = (rng.standard_normal((n, 1, gamma + 1, V)) * 1.5).astype(np.float32)
    logits = np.ascontiguousarray(np.broadcast_to(row, (n, B, gamma + 1, V))).copy()
    drafts = rng.integers(0, V, (B, gamma)).astype(np.int32)
    proposer = np.zeros(B, dtype=np.int32)
    bonus = np.ones(B, dtype=np.int32)                                 # verifier = model 1
    ua = np.zeros((B, gamma))                                          # u = 0: every draft with r(d) > 0 is accepted
    ur = rng.random(B)
    logits[0, :, gamma, :] = np.nan                                    # the proposer has no logits there yet
    res = O.verify(logits, O.DTYPE_F32, drafts, proposer, O.ENSEMBLE, [0.5, 0.5], ua, ur, bonus_idx=bonus)
    assert res.status == 0 and np.all(res.accepted_len == gamma)
    sv = O.softmax(O.row_to_f64(logits[1, 0, gamma], O.DTYPE_F32))
    cdf = np.cumsum(sv)
    want = np.searchsorted(cdf, ur * cdf[-1], side="right")
    assert np.array_equal(res.out_tokens[:, gamma], want)
    counts = np.bincount(res.out_tokens[:, gamma], minlength=V)
    assert stats.chisquare(counts, sv / sv.sum() * B).pvalue > 1e-3
    # -1 (or no bonus_idx) draws the bonus from r: with NaN rows that poisons the draw, without them not
    clean = logits.copy()
    clean[0, :, gamma, :] = row[0, 0, gamma]
    a = O.verify(clean, O.DTYPE_F32, drafts, proposer, O.ENSEMBLE, [0.5, 0.5], ua, ur, bonus_idx=-np.ones(B, dtype=np.int32))
    b = O.verify(clean, O.DTYPE_F32, drafts, proposer, O.ENSEMBLE, [0.5, 0.5], ua, ur)
    assert np.array_equal(a.out_tokens, b.out_tokens)
    assert not np.array_equal(a.out_tokens[:, gamma], res.out_tokens[:, gamma])


def test_verifier_bonus_does_not_change_rejected_rows():
    rng = _rng(8)
    logits, drafts, proposer, ua, ur = _inputs(rng, 2, 300, 3, 40)
    base = O.verify(logits, O.DTYPE_F32, drafts, proposer, O.ENSEMBLE, [0.4, 0.6], ua, ur)
    vb = O.verify(logits, O.DTYPE_F32, drafts, proposer, O.ENSEMBLE, [0.4, 0.6], ua, ur, bonus_idx=1 - proposer)
    rejected = base.accepted_len < 3
    assert rejected.any() and (~rejected).any()
    assert np.array_equal(base.accepted_len, vb.accepted_len)
    assert np.array_equal(base.out_tokens[rejected], vb.out_tokens[rejected])


# ---- per-position proposers (Alg. 2) -------------------------------------------

def test_per_position_proposers_against_an_independent_rederivation():
    rng = _rng(9)
    n, B, gamma, V = 3, 300, 4, 30
    logits, drafts, proposer, ua, ur = _inputs(rng, n, B, gamma, V)
    pos = rng.integers(0, n, (B, gamma)).astype(np.int32)
    w = np.array([0.2, 0.5, 0.3])
    res = O.verify(logits, O.DTYPE_F32, drafts, proposer, O.ENSEMBLE, w, ua, ur, proposer_pos=pos)
    sm = special.softmax(logits.astype(np.float64), axis=-1)
    for b in range(B):
        alen, tok = gamma, None
        for j in range(gamma):
            r = np.tensordot(w, sm[:, b, j], axes=1)
            q = sm[pos[b, j], b, j]
            d = drafts[b, j]
            if not ua[b, j] < min(1.0, r[d] / q[d]):
                cdf = np.cumsum(np.maximum(r - q, 0.0))
                alen, tok = j, int(np.searchsorted(cdf, ur[b] * cdf[-1], side="right"))
                break
        if tok is None:
            cdf = np.cumsum(np.tensordot(w, sm[:, b, gamma], axes=1))
            tok = int(np.searchsorted(cdf, ur[b] * cdf[-1], side="right"))
        assert res.accepted_len[b] == alen and res.out_tokens[b, alen] == tok
    # constant per-position proposers are the per-row case
    same = O.verify(logits, O.DTYPE_F32, drafts, proposer, O.ENSEMBLE, w, ua, ur,
                    proposer_pos=np.repeat(proposer[:, None], gamma, axis=1))
    base = O.verify(logits, O.DTYPE_F32, drafts, proposer, O.ENSEMBLE, w, ua, ur)
    assert np.array_equal(same.out_tokens, base.out_tokens)
    assert not np.array_equal(res.out_tokens, base.out_tokens)


def test_extension_argument_checks():
    rng = _rng(10)
    logits, drafts, proposer, ua, ur = _inputs(rng, 2, 4, 2, 10)
    assert O.verify(logits, O.DTYPE_F32, drafts, proposer, O.ENSEMBLE, [0.5, 0.5], ua, ur,
                    bonus_idx=np.full(4, 2)).status == -2
    assert O.verify(logits, O.DTYPE_F32, drafts, proposer, O.ENSEMBLE, [0.5, 0.5], ua, ur,
                    proposer_pos=np.full((4, 2), -1)).status == -2
    assert O.verify(logits, O.DTYPE_F32, drafts, proposer, O.ENSEMBLE, [0.5, 0.5], ua, ur,
                    temperature=-1.0).status == -5


# ---- temperature 0 (greedy), contrastive mode ------------------------------------

def test_greedy_argmax_against_numpy_and_ties():
    rng = _rng(20)
    for V in (1, 7, 500):
        lp, lq = rng.standard_normal(V) * 3, rng.standard_normal(V) * 2
        for mu, a in ((0.5, 0.0), (0.1, 0.1), (1.0, 0.5), (0.3, 1.0)):
            c = lp - mu * lq
            mask = lp - lp.max() >= (np.log(a) if a > 0 else -np.inf)
            want = int(np.flatnonzero(mask)[np.argmax(c[mask])])
            assert O.argmax_contrastive(lp, lq, mu, a) == want
    assert O.argmax_contrastive(np.array([1.0, 5.0, 5.0, 2.0]), np.zeros(4), 0.5, 0.0) == 1     # tie: lowest index
    assert O.argmax_contrastive(np.array([4.0, 3.0]), np.array([10.0, 0.0]), 0.5, 0.0) == 1     # 4-5 < 3-0
    assert O.argmax_contrastive(np.array([4.0, 3.0]), np.array([10.0, 0.0]), 0.5, 0.9) == 0     # masked out


def test_greedy_step_is_the_small_temperature_limit_without_mask():
    """With alpha_cd = 0 the greedy step equals the sampled step at a tiny temperature (1e-9), whatever
    the uniforms (r is numerically one-hot): a pin against the float64 sampler pinned elsewhere."""
    rng = _rng(21)
    n, B, gamma, V = 2, 300, 3, 40
    logits = (rng.standard_normal((n, B, gamma + 1, V)) * 2).astype(np.float32)
    # drafts: the contrastive argmax on a prefix of random length (accepted), random tokens after it
    drafts = rng.integers(0, V, (B, gamma)).astype(np.int32)
    for b in range(B):
        for j in range(int(rng.integers(0, gamma + 1))):
            drafts[b, j] = O.argmax_contrastive(logits[0, b, j].astype(np.float64), logits[1, b, j].astype(np.float64), 0.5, 0.0)
    proposer = np.ones(B, dtype=np.int32)
    st, alen, toks = O.verify_greedy(logits, O.DTYPE_F32, drafts, [0.5, 0.0])
    assert st == 0
    lim = O.verify(logits, O.DTYPE_F32, drafts, proposer, O.CONTRASTIVE, [0.5, 0.0], rng.random((B, gamma)),
                   rng.random(B), temperature=1e-9)
    assert np.array_equal(alen, lim.accepted_len) and np.array_equal(toks, lim.out_tokens)
    assert len(set(alen.tolist())) >= 3


def test_greedy_step_brute_force_with_mask_and_verifier_bonus():
    rng = _rng(22)
    B, gamma, V = 200, 4, 25
    logits = (rng.standard_normal((2, B, gamma + 1, V)) * 2).astype(np.float32)
    mu, a = 0.7, 0.2
    arg = np.empty((B, gamma + 1), dtype=np.int64)
    for b in range(B):
        for j in range(gamma + 1):
            lp, lq = logits[0, b, j].astype(np.float64), logits[1, b, j].astype(np.float64)
            c = np.where(lp - lp.max() >= np.log(a), lp - mu * lq, -np.inf)
            arg[b, j] = int(np.argmax(c))
    drafts = arg[:, :gamma].astype(np.int32)
    cut = rng.integers(0, gamma + 1, B)
    for b in range(B):
        if cut[b] < gamma:
            drafts[b, cut[b]] = (drafts[b, cut[b]] + 1) % V
    bonus = rng.integers(-1, 2, B).astype(np.int32)
    st, alen, toks = O.verify_greedy(logits, O.DTYPE_F32, drafts, [mu, a], bonus_idx=bonus)
    assert st == 0 and np.array_equal(alen, cut)
    for b in range(B):
        if cut[b] < gamma:
            assert toks[b, cut[b]] == arg[b, cut[b]]
        elif bonus[b] >= 0:
            assert toks[b, gamma] == int(np.argmax(logits[bonus[b], b, gamma]))
        else:
            assert toks[b, gamma] == arg[b, gamma]
        assert np.array_equal(toks[b, :cut[b]], drafts[b, :cut[b]]) and np.all(toks[b, cut[b] + 1:] == -1)


# ---- rows with fewer drafts (num_drafts) and no extra token (no_bonus) -----------------------

def _poison_after(logits, num_drafts, first_unread):
    """NaN in every position >= num_drafts[b] + first_unread (never read by a correct implementation)."""
    out = logits.copy()
    for b, k in enumerate(num_drafts):
        out[:, b, k + first_unread:, :] = np.nan
    return out


@pytest.mark.parametrize("mode,weights,n", [(O.ENSEMBLE, [0.5, 0.2, 0.3], 3), (O.CONTRASTIVE, [0.5, 0.1], 2)])
def test_ragged_rows_equal_calls_on_the_truncated_tensor(mode, weights, n):
    """Row b with K drafts must equal the base step (pinned on its own) on logits[:, b, :K+1] with gamma = K."""
    rng = _rng(40 + mode)
    B, gamma, V = 120, 4, 40
    logits, drafts, proposer, ua, ur = _inputs(rng, n, B, gamma, V, std=1.0)
    for b in range(B):                       # drafts from the proposer, so that lengths vary
        for j in range(gamma):
            s = O.softmax(O.row_to_f64(logits[proposer[b], b, j], O.DTYPE_F32))
            drafts[b, j] = min(np.searchsorted(np.cumsum(s), rng.random(), side="right"), V - 1)
    K = rng.integers(0, gamma + 1, B).astype(np.int32)
    res = O.verify(_poison_after(logits, K, 1), O.DTYPE_F32, drafts, proposer, mode, weights, ua, ur, num_drafts=K)
    assert res.status == 0
    seen = set()
    for b in range(B):
        k = int(K[b])
        if k == 0:
            # nothing to test: one draw from r_0 by the step functions
            l = [O.row_to_f64(logits[m, b, 0], O.DTYPE_F32) for m in range(n)]
            if mode == O.ENSEMBLE:
                r = O.combine_ensemble(np.stack([O.softmax(x) for x in l]), np.array(weights))
            else:
                r = O.combine_contrastive(l[0], l[1], weights[0], weights[1])[0]
            tok = O.inverse_cdf(r, r.sum(), ur[b])[0]
            assert res.accepted_len[b] == 0 and res.out_tokens[b, 0] == tok and (res.out_tokens[b, 1:] == -1).all()
            continue
        one = O.verify(np.ascontiguousarray(logits[:, b:b + 1, :k + 1]), O.DTYPE_F32, drafts[b:b + 1, :k],
                       proposer[b:b + 1], mode, weights, ua[b:b + 1, :k], ur[b:b + 1])
        assert one.status == 0
        assert res.accepted_len[b] == one.accepted_len[0]
        assert np.array_equal(res.out_tokens[b, :k + 1], one.out_tokens[0])
        assert (res.out_tokens[b, k + 1:] == -1).all()
        assert res.sample_mass[b] == one.sample_mass[0] and res.cdf_hi[b] == one.cdf_hi[0]
        assert res.flags[b] == one.flags[0] == 0
        assert np.array_equal(res.r_at_draft[b, :k], one.r_at_draft[0], equal_nan=True)
        assert np.isnan(res.r_at_draft[b, k:]).all()
        seen.add((k, int(one.accepted_len[0]) == k))
    assert {(k, True) for k in range(1, gamma + 1)} <= seen            # all-accepted rows of every length occurred
    assert {(k, False) for k in range(1, gamma + 1)} <= seen


def test_ragged_rows_with_a_verifier_bonus():
    """The verifier's own extra token moves with the row's length: position K, model bonus_idx[b] alone."""
    rng = _rng(42)
    B, gamma, V = 150, 3, 25
    logits, drafts, proposer, ua, ur = _inputs(rng, 2, B, gamma, V, std=0.4)
    K = rng.integers(1, gamma + 1, B).astype(np.int32)
    verifier = (1 - proposer).astype(np.int32)
    poisoned = _poison_after(logits, K, 1)
    for b in range(B):
        poisoned[proposer[b], b, K[b]] = np.nan                      # the proposer has no logits at the bonus position
    res = O.verify(poisoned, O.DTYPE_F32, drafts, proposer, O.ENSEMBLE, [0.5, 0.5], ua, ur, num_drafts=K,
                   bonus_idx=verifier)
    assert res.status == 0
    hit = 0
    for b in range(B):
        k = int(K[b])
        one = O.verify(np.ascontiguousarray(logits[:, b:b + 1, :k + 1]), O.DTYPE_F32, drafts[b:b + 1, :k],
                       proposer[b:b + 1], O.ENSEMBLE, [0.5, 0.5], ua[b:b + 1, :k], ur[b:b + 1], bonus_idx=verifier[b:b + 1])
        assert np.array_equal(res.out_tokens[b, :k + 1], one.out_tokens[0]) and res.accepted_len[b] == one.accepted_len[0]
        if res.accepted_len[b] == k:
            hit += 1
            sv = O.softmax(O.row_to_f64(logits[verifier[b], b, k], O.DTYPE_F32))
            assert res.out_tokens[b, k] == O.inverse_cdf(sv, sv.sum(), ur[b])[0]
    assert hit > 20


def test_no_bonus_only_drops_the_extra_token():
    rng = _rng(43)
    B, gamma, V = 200, 3, 30
    logits, drafts, proposer, ua, ur = _inputs(rng, 2, B, gamma, V, std=0.5)
    K = rng.integers(0, gamma + 1, B).astype(np.int32)
    w = [0.6, 0.4]
    full = O.verify(logits, O.DTYPE_F32, drafts, proposer, O.ENSEMBLE, w, ua, ur, num_drafts=K)
    nob = O.verify(_poison_after(logits, K, 0), O.DTYPE_F32, drafts, proposer, O.ENSEMBLE, w, ua, ur, num_drafts=K,
                   no_bonus=True)
    # (a rejected row stops at a position below K, so the poison is never read)
    assert full.status == 0 and nob.status == 0
    assert np.array_equal(full.accepted_len, nob.accepted_len)
    done = full.accepted_len == K
    assert done.sum() > 20 and (~done).sum() > 20
    for b in range(B):
        if done[b]:
            assert np.array_equal(nob.out_tokens[b, :K[b]], drafts[b, :K[b]]) and (nob.out_tokens[b, K[b]:] == -1).all()
            assert nob.sample_mass[b] == 0.0 and nob.flags[b] == 0
        else:
            assert np.array_equal(nob.out_tokens[b], full.out_tokens[b])
            assert nob.sample_mass[b] == full.sample_mass[b]
    # without num_drafts: the Naive-CoS step (the extra token discarded, Sec. 3.2)
    a = O.verify(logits, O.DTYPE_F32, drafts, proposer, O.ENSEMBLE, w, ua, ur, no_bonus=True)
    c = O.verify(logits, O.DTYPE_F32, drafts, proposer, O.ENSEMBLE, w, ua, ur)
    assert np.array_equal(a.accepted_len, c.accepted_len)
    assert np.array_equal(a.out_tokens[:, :gamma], c.out_tokens[:, :gamma])
    assert (a.out_tokens[:, gamma] == -1).all()


def test_greedy_ragged_rows_and_no_bonus():
    rng = _rng(44)
    B, gamma, V = 150, 4, 12
    logits = (rng.standard_normal((2, B, gamma + 1, V))).astype(np.float32)
    w = [0.5, 0.2]
    drafts = np.zeros((B, gamma), dtype=np.int32)
    for b in range(B):
        for j in range(gamma):
            a = O.argmax_contrastive(logits[0, b, j].astype(np.float64), logits[1, b, j].astype(np.float64), *w)
            drafts[b, j] = a if rng.random() < 0.7 else (a + 1) % V
    K = rng.integers(0, gamma + 1, B).astype(np.int32)
    st, alen, toks = O.verify_greedy(_poison_after(logits, K, 1), O.DTYPE_F32, drafts, w, num_drafts=K)
    st2, alen2, toks2 = O.verify_greedy(_poison_after(logits, K, 0), O.DTYPE_F32, drafts, w, num_drafts=K, no_bonus=True)
    st3, alen3, toks3 = O.verify_greedy(logits, O.DTYPE_F32, drafts, w, num_drafts=K, no_bonus=True)
    assert st == 0 and st2 == 0 and np.array_equal(alen, alen2)
    assert st3 == 0 and np.array_equal(alen3, alen2) and np.array_equal(toks3, toks2)    # unread means unread
    for b in range(B):
        k = int(K[b])
        if k == 0:
            a0 = O.argmax_contrastive(logits[0, b, 0].astype(np.float64), logits[1, b, 0].astype(np.float64), *w)
            assert alen[b] == 0 and toks[b, 0] == a0 and (toks2[b] == -1).all()
            continue
        s1, a1, t1 = O.verify_greedy(np.ascontiguousarray(logits[:, b:b + 1, :k + 1]), O.DTYPE_F32, drafts[b:b + 1, :k], w)
        assert s1 == 0 and alen[b] == a1[0] and np.array_equal(toks[b, :k + 1], t1[0]) and (toks[b, k + 1:] == -1).all()
        if a1[0] == k:
            assert np.array_equal(toks2[b, :k], drafts[b, :k]) and (toks2[b, k:] == -1).all()
        else:
            assert np.array_equal(toks2[b], toks[b])
    assert (alen == K).sum() > 10 and (alen < K).sum() > 10


def test_num_drafts_argument_checks():
    rng = _rng(45)
    logits, drafts, proposer, ua, ur = _inputs(rng, 2, 3, 2, 10)
    for bad in ([0, 3, 1], [-1, 2, 2]):
        assert O.verify(logits, O.DTYPE_F32, drafts, proposer, O.ENSEMBLE, [0.5, 0.5], ua, ur,
                        num_drafts=bad).status == -2
        assert O.verify_greedy(logits, O.DTYPE_F32, drafts, [0.5, 0.1], num_drafts=bad)[0] == -2
    # draft tokens beyond a row's length are not looked at
    drafts2 = drafts.copy()
    drafts2[0, 1] = 999
    assert O.verify(logits, O.DTYPE_F32, drafts2, proposer, O.ENSEMBLE, [0.5, 0.5], ua, ur, num_drafts=[1, 2, 2]).status == 0


# ---- logit-level linear combination (Eq. (3), C' on logits) ------------------------------------

def test_logit_mix_hand_example_library_softmax_and_special_cases():
    import os
    from fractions import Fraction
    g = {}
    with open(os.path.join(os.path.dirname(__file__), "golden", "logit_mix_hand.txt")) as fh:
        for line in fh:
            line = line.split("#")[0].strip()
            if line:
                key, vals = line.split(":")
                g[key.strip()] = np.array([float(Fraction(v)) for v in vals.split()])
    l = np.log(np.stack([g["p0"], g["p1"]]))
    assert np.allclose(O.combine_logit_mix(l, g["beta_a"]), g["r_a"], rtol=1e-14)
    assert np.allclose(O.combine_logit_mix(l, g["beta_b"]), g["r_b"], rtol=1e-14)
    rng = _rng(60)
    n, V = 4, 300
    l = rng.standard_normal((n, V)) * 3
    beta = np.array([0.7, -0.3, 1.1, 0.25])
    assert np.allclose(O.combine_logit_mix(l, beta), special.softmax(beta @ l), rtol=1e-12)      # library softmax
    for m in range(n):                                                                         # one-hot: that model
        assert np.array_equal(O.combine_logit_mix(l, np.eye(n)[m]), O.softmax(l[m]))
    # uniform 1/n: the normalised geometric mean of the models' distributions
    s = np.stack([O.softmax(x) for x in l])
    geo = np.exp(np.log(s).mean(axis=0))
    assert np.allclose(O.combine_logit_mix(l, np.full(n, 1 / n)), geo / geo.sum(), rtol=1e-12)
    # (1, -mu) is Eq. (5) without its mask, bit for bit
    for mu in (0.1, 0.5, 1.0):
        assert np.array_equal(O.combine_logit_mix(l[:2], [1.0, -mu]), O.combine_contrastive(l[0], l[1], mu, 0.0)[0])
    # a model with beta = 0 takes no part, whatever its logits
    l2 = l.copy()
    l2[1] = -np.inf
    assert np.array_equal(O.combine_logit_mix(l2, [0.5, 0.0, 0.2, 0.3]), O.combine_logit_mix(l, [0.5, 0.0, 0.2, 0.3]))
    # a token one model rules out (positive weight) has probability 0
    l3 = l.copy()
    l3[2, 7] = -np.inf
    assert O.combine_logit_mix(l3, [0.5, 0.1, 0.2, 0.3])[7] == 0.0


def test_logit_mix_whole_step_equals_contrastive_without_mask_and_checks_arguments():
    rng = _rng(61)
    logits, drafts, proposer, ua, ur = _inputs(rng, 2, 300, 3, 40, std=1.0)
    a = O.verify(logits, O.DTYPE_F32, drafts, proposer, O.LOGIT_MIX, [1.0, -0.5], ua, ur, all_positions=True, want_alpha=True)
    b = O.verify(logits, O.DTYPE_F32, drafts, proposer, O.CONTRASTIVE, [0.5, 0.0], ua, ur, all_positions=True, want_alpha=True)
    assert a.status == 0 and b.status == 0
    assert np.array_equal(a.out_tokens, b.out_tokens) and np.array_equal(a.r_at_draft, b.r_at_draft)
    assert np.array_equal(a.alpha, b.alpha) and len(set(a.accepted_len.tolist())) == 4
    # one-hot on the proposer: r == q, everything accepted; one-hot on the other model: textbook speculative sampling
    onehot = O.verify(logits, O.DTYPE_F32, drafts, np.zeros(300, dtype=np.int32), O.LOGIT_MIX, [1.0, 0.0], ua, ur)
    assert np.all(onehot.accepted_len == 3)
    sd = O.verify(logits, O.DTYPE_F32, drafts, np.zeros(300, dtype=np.int32), O.LOGIT_MIX, [0.0, 1.0], ua, ur)
    ens = O.verify(logits, O.DTYPE_F32, drafts, np.zeros(300, dtype=np.int32), O.ENSEMBLE, [0.0, 1.0], ua, ur)
    assert np.array_equal(sd.out_tokens, ens.out_tokens)
    assert O.verify(logits, O.DTYPE_F32, drafts, proposer, O.LOGIT_MIX, [1.0, float("inf")], ua, ur).status == -5
    assert O.verify(logits, O.DTYPE_F32, drafts, proposer, 3, [1.0, 0.5], ua, ur).status == -4
    three = _inputs(rng, 3, 10, 2, 20)
    assert O.verify(three[0], O.DTYPE_F32, three[1], three[2], O.LOGIT_MIX, [0.5, 0.7, -0.2], three[3], three[4]).status == 0


# ---- temperature 0 (greedy), logit mix -------------------------------------------

def test_greedy_logit_mix_argmax_against_numpy_and_special_cases():
    rng = _rng(40)
    for n, V in ((1, 9), (2, 300), (3, 41), (5, 1000)):
        l = rng.standard_normal((n, V)) * 3
        beta = rng.normal(0.0, 0.8, n)
        beta[0] = 1.0
        assert O.argmax_logit_mix(l, beta) == int(np.argmax((beta[:, None] * l).sum(0)))
        one = np.zeros(n)
        one[n - 1] = 2.5                                         # one-hot mix: that model's argmax
        assert O.argmax_logit_mix(l, one) == int(np.argmax(l[n - 1]))
    lp, lq = rng.standard_normal(200) * 3, rng.standard_normal(200) * 2
    assert O.argmax_logit_mix(np.stack([lp, lq]), [1.0, -0.5]) == O.argmax_contrastive(lp, lq, 0.5, 0.0)  # Eq. (5), no mask
    assert O.argmax_logit_mix(np.array([[1.0, 5.0, 5.0, 2.0], [0.0, 0.0, 0.0, 0.0]]), [1.0, 1.0]) == 1     # tie: lowest index
    assert O.argmax_logit_mix(np.array([[4.0, 3.0], [10.0, 0.0]]), [1.0, -0.5]) == 1                        # 4-5 < 3-0
    assert O.argmax_logit_mix(np.array([[4.0, 3.0], [10.0, 0.0]]), [1.0, 0.0]) == 0                         # beta = 0: no part
    assert O.argmax_logit_mix(np.array([[4.0, 3.0], [np.nan, 0.0]]), [1.0, 0.0]) == 0                       # ... not even its NaN


def test_greedy_logit_mix_step_is_the_small_temperature_limit():
    """The greedy step equals the sampled logit-mix step at a tiny temperature (1e-9), whatever the
    uniforms and the proposers: a pin against the float64 sampler that is pinned elsewhere."""
    rng = _rng(41)
    n, B, gamma, V = 3, 300, 3, 40
    beta = [0.9, 0.6, -0.4]
    logits = (rng.standard_normal((n, B, gamma + 1, V)) * 2).astype(np.float32)
    drafts = rng.integers(0, V, (B, gamma)).astype(np.int32)
    for b in range(B):
        for j in range(int(rng.integers(0, gamma + 1))):      # an accepted prefix of random length
            drafts[b, j] = O.argmax_logit_mix(logits[:, b, j].astype(np.float64), beta)
    st, alen, toks = O.verify_greedy(logits, O.DTYPE_F32, drafts, beta, mode=O.LOGIT_MIX)
    assert st == 0
    lim = O.verify(logits, O.DTYPE_F32, drafts, rng.integers(0, n, B).astype(np.int32), O.LOGIT_MIX, beta,
                   rng.random((B, gamma)), rng.random(B), temperature=1e-9)
    assert np.array_equal(alen, lim.accepted_len) and np.array_equal(toks, lim.out_tokens)
    assert len(set(alen.tolist())) >= 3


def test_greedy_logit_mix_brute_force_with_verifier_bonus_ragged_rows_and_no_bonus():
    rng = _rng(42)
    n, B, gamma, V = 4, 200, 4, 25
    beta = np.array([1.0, 0.5, 0.0, -0.3])
    logits = (rng.standard_normal((n, B, gamma + 1, V)) * 2).astype(np.float32)
    arg = np.argmax(np.einsum("m,mbjv->bjv", beta, logits.astype(np.float64)), axis=-1)
    K = rng.integers(0, gamma + 1, B).astype(np.int32)          # drafts per row
    drafts = arg[:, :gamma].astype(np.int32)
    cut = np.array([rng.integers(0, k + 1) for k in K])          # first mismatch (== K[b]: none)
    for b in range(B):
        if cut[b] < K[b]:
            drafts[b, cut[b]] = (drafts[b, cut[b]] + 1) % V
    bonus = rng.integers(-1, n, B).astype(np.int32)
    poisoned = logits.copy()
    for b in range(B):
        poisoned[:, b, K[b] + 1:] = np.nan                        # never read
    st, alen, toks = O.verify_greedy(poisoned, O.DTYPE_F32, drafts, beta, bonus_idx=bonus, num_drafts=K, mode=O.LOGIT_MIX)
    assert st == 0 and np.array_equal(alen, cut)
    for b in range(B):
        assert np.array_equal(toks[b, :cut[b]], drafts[b, :cut[b]]) and np.all(toks[b, cut[b] + 1:] == -1)
        if cut[b] < K[b] or bonus[b] < 0:
            assert toks[b, cut[b]] == arg[b, cut[b]]
        else:
            assert toks[b, cut[b]] == int(np.argmax(logits[bonus[b], b, K[b]]))
    for b in range(B):
        poisoned[:, b, K[b]:] = np.nan                            # without the extra token not even that position
    st2, alen2, toks2 = O.verify_greedy(poisoned, O.DTYPE_F32, drafts, beta, num_drafts=K, no_bonus=True, mode=O.LOGIT_MIX)
    assert st2 == 0 and np.array_equal(alen2, cut)
    full = cut == K
    assert np.all(toks2[full, :][np.arange(full.sum()), K[full]] == -1)
    assert np.array_equal(toks2[~full], toks[~full])
    # argument checks
    assert O.verify_greedy(logits, O.DTYPE_F32, drafts, [1.0, np.inf, 0.0, 0.0], mode=O.LOGIT_MIX)[0] == -5
    assert O.verify_greedy(logits, O.DTYPE_F32, drafts, beta, mode=O.ENSEMBLE)[0] == -4
    assert O.verify_greedy(logits, O.DTYPE_F32, drafts, [0.5, 0.1], mode=O.CONTRASTIVE)[0] == -4   # contrastive needs n == 2
    assert O.verify_greedy(logits, O.DTYPE_F32, drafts, beta, bonus_idx=np.full(B, n), mode=O.LOGIT_MIX)[0] == -2


# ---- temperature 0 (greedy), ensemble ---------------------------------------------

def test_softmax_t0_is_the_limit_of_the_softmax():
    rng = _rng(50)
    for V in (1, 5, 300):
        l = rng.standard_normal(V) * 3
        s = O.softmax_t0(l)
        assert s.sum() == 1.0 and s[np.argmax(l)] == 1.0
        assert np.array_equal(s, np.round(O.softmax(l / 1e-9)))          # numerically one-hot already at T = 1e-9
    assert np.array_equal(O.softmax_t0(np.array([1.0, 4.0, 4.0, -np.inf])), [0.0, 1.0, 0.0, 0.0])   # tie: lowest index


def test_greedy_ensemble_is_the_small_temperature_limit_of_the_step():
    """The whole step at temperature 0 equals the step at T = 1e-9 with the same uniforms (the softmaxes are
    one-hot there already): a pin against the sampler that is pinned elsewhere, with per-position proposers,
    verifier bonus tokens, ragged rows and the no-bonus variant."""
    rng = _rng(51)
    n, B, gamma, V = 3, 400, 3, 12                         # a small vocabulary: the models often agree
    w = [0.5, 0.3, 0.2]
    logits = (rng.standard_normal((n, B, gamma + 1, V)) * 2).astype(np.float32)
    logits[1, ::3] = logits[0, ::3]                         # ... and sometimes fully
    proposer = rng.integers(0, n, B).astype(np.int32)
    ppos = rng.integers(0, n, (B, gamma)).astype(np.int32)
    top = logits.argmax(-1)                                 # [n][B][gamma+1]
    drafts = rng.integers(0, V, (B, gamma)).astype(np.int32)
    for b in range(B):                                      # drafts as the paper has them: the proposer's own token
        for j in range(gamma):
            if rng.random() < 0.8:
                drafts[b, j] = top[ppos[b, j], b, j]
    ua, ur = rng.random((B, gamma)), rng.random(B)
    bonus = rng.integers(-1, n, B).astype(np.int32)
    nd = rng.integers(0, gamma + 1, B).astype(np.int32)
    for kw in ({}, {"proposer_pos": ppos}, {"bonus_idx": bonus}, {"num_drafts": nd}, {"num_drafts": nd, "no_bonus": True},
               {"proposer_pos": ppos, "bonus_idx": bonus, "num_drafts": nd}):
        g = O.verify(logits, O.DTYPE_F32, drafts, proposer, O.ENSEMBLE, w, ua, ur, greedy=True, all_positions=True, **kw)
        lim = O.verify(logits, O.DTYPE_F32, drafts, proposer, O.ENSEMBLE, w, ua, ur, temperature=1e-9, all_positions=True, **kw)
        assert g.status == 0 and lim.status == 0
        assert np.array_equal(g.accepted_len, lim.accepted_len) and np.array_equal(g.out_tokens, lim.out_tokens), kw
        assert np.array_equal(g.flags, lim.flags)
        assert len(set(g.accepted_len.tolist())) >= 3


def test_greedy_ensemble_by_cases():
    """Eq. (6) at temperature 0 by hand: q is one-hot at the proposer's token a_pi and r(x) is the weight of the
    models whose token is x.  A draft equal to a_pi is accepted with probability r(a_pi); any other draft is
    accepted iff some model votes for it; after a rejection the token is one of the other models' tokens, in
    proportion to their weights (by inverse CDF in token order); when every model agrees with the proposer a
    foreign draft is rejected and replaced by that token (residual without mass: the fall-back to r)."""
    V, gamma = 10, 1
    w = [0.5, 0.3, 0.2]

    def run(tokens, d, pi, u, ur=0.5):
        logits = np.zeros((3, 1, gamma + 1, V), dtype=np.float32)
        for m, t in enumerate(tokens):
            logits[m, 0, :, t] = 5.0
        return O.verify(logits, O.DTYPE_F32, [[d]], [pi], O.ENSEMBLE, w, [[u]], [ur], greedy=True)

    res = run((4, 4, 7), d=4, pi=0, u=0.79)                 # r(4) = 0.8
    assert res.accepted_len[0] == 1 and res.r_at_draft[0, 0] == 0.8 and res.q_at_draft[0, 0] == 1.0
    res = run((4, 4, 7), d=4, pi=0, u=0.81)                 # rejected: the residual is all on token 7
    assert res.accepted_len[0] == 0 and res.out_tokens[0, 0] == 7 and abs(res.sample_mass[0] - 0.2) < 1e-15
    res = run((4, 4, 7), d=7, pi=0, u=0.999)                # q(7) = 0 < r(7): always accepted
    assert res.accepted_len[0] == 1 and np.isinf(res.ratio[0, 0])
    res = run((4, 4, 7), d=2, pi=0, u=0.0)                  # nobody votes for 2: rejected even at u = 0
    assert res.accepted_len[0] == 0 and res.out_tokens[0, 0] == 7
    res = run((4, 6, 2), d=4, pi=0, u=0.6, ur=0.39)         # residual: token 2 (0.2) before token 6 (0.3): u*F = 0.195
    assert res.accepted_len[0] == 0 and res.out_tokens[0, 0] == 2
    res = run((4, 6, 2), d=4, pi=0, u=0.6, ur=0.41)         # 0.205 > 0.2: token 6
    assert res.out_tokens[0, 0] == 6
    res = run((4, 4, 4), d=9, pi=1, u=0.0)                  # all agree; a foreign draft: r = q, fall back to r
    assert res.accepted_len[0] == 0 and res.out_tokens[0, 0] == 4 and res.flags[0] & O.FLAG_RESIDUAL_FALLBACK
    res = run((4, 6, 2), d=4, pi=0, u=0.1, ur=0.75)         # accepted; bonus from r in token order: 2 (.2), 4 (.5), 6 (.3)
    assert res.accepted_len[0] == 1 and res.out_tokens[0, 1] == 6
    # only the ensemble is combined at the probability level; the logit-level modes have their own step
    lg = np.zeros((2, 1, 2, V), dtype=np.float32)
    assert O.verify(lg, O.DTYPE_F32, [[1]], [0], O.CONTRASTIVE, [0.5, 0.1], [[0.5]], [0.5], greedy=True).status == -4
