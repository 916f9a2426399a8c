"""The n-model CoS scheduler (Alg. 2, Sec. 3.4) around the verification step.

CPU: with the oracle as verify back end the generated tokens must follow the combined distribution r
(App. A.1 applied along Alg. 2), and the schedule must be the one the paper walks through for three
models.  GPU: the same driver with cos_verify must produce the same sequences token for token."""
import numpy as np
import pytest
import torch
from scipy import stats

from oracle import cos_oracle as O
from paper_2502_01662_amd import apf
from paper_2502_01662_amd import cos_scheduler as S
from paper_2502_01662_amd import workloads as W


def oracle_verify(logits, drafts, proposer, mode, weights, u_acc, u_res, proposer_pos=None, num_drafts=None,
                  no_bonus=False, temperature=1.0, greedy=False):
    dt = O.DTYPE_F32 if logits.dtype == torch.float32 else O.DTYPE_BF16
    if greedy and mode != O.ENSEMBLE:                       # temperature 0, logit-level modes: their own oracle step
        st, alen, toks = O.verify_greedy(W.host_logits(logits), dt, drafts.cpu().numpy(), weights, mode=mode,
                                         num_drafts=None if num_drafts is None else num_drafts.cpu().numpy(),
                                         no_bonus=no_bonus)
        assert st == 0
        return torch.from_numpy(alen), torch.from_numpy(toks)
    res = O.verify(W.host_logits(logits), dt, drafts.cpu().numpy(), proposer.cpu().numpy(), mode, weights,
                   u_acc.cpu().numpy(), u_res.cpu().numpy(), temperature=temperature, greedy=greedy,
                   proposer_pos=None if proposer_pos is None else proposer_pos.cpu().numpy(),
                   num_drafts=None if num_drafts is None else num_drafts.cpu().numpy(), no_bonus=no_bonus)
    assert res.status == 0
    return torch.from_numpy(res.accepted_len), torch.from_numpy(res.out_tokens)


def _exact_joint_law(lm, ctx0, mode, weights, depth):
    """P(x_1..x_depth | ctx0) when every token is drawn from r: plain collaborative decoding."""
    law = {}

    def r_of(ctx):
        c = torch.tensor([ctx[-2:]], dtype=torch.int32)
        l = [lm.logits(m, c)[0].to(torch.float64).numpy() for m in range(lm.n_models)]
        if mode == O.ENSEMBLE:
            return O.combine_ensemble(np.stack([O.softmax(x) for x in l]), np.asarray(weights, dtype=np.float64))
        if mode == O.LOGIT_MIX:
            return O.combine_logit_mix(np.stack(l), np.asarray(weights, dtype=np.float64))
        return O.combine_contrastive(l[0], l[1], weights[0], weights[1])[0]

    def rec(ctx, prob, toks):
        if len(toks) == depth:
            law[tuple(toks)] = prob
            return
        r = r_of(ctx)
        for x in range(lm.V):
            if r[x] > 0:
                rec(ctx + [x], prob * r[x], toks + [x])

    rec(list(ctx0), 1.0, [])
    return law


@pytest.mark.parametrize("n,gammas,mode,weights", [(3, (2, 1, 1), O.ENSEMBLE, [0.5, 0.3, 0.2]),
                                                  (3, (1, 2, 1), O.LOGIT_MIX, [0.6, 0.5, -0.1]),
                                                  (3, (1, 1, 1), O.ENSEMBLE, [0.2, 0.2, 0.6]),
                                                  (2, (2, 2), O.CONTRASTIVE, [0.5, 0.05]),
                                                  (4, (1, 2, 1, 1), O.ENSEMBLE, [0.25, 0.25, 0.25, 0.25])])
def test_generated_tokens_follow_the_combined_distribution(n, gammas, mode, weights):
    V, B, depth = 5, 50_000, 3
    lm = apf.HashedBigramLM(n, V, buckets=64, base_std=1.0, noise_std=0.7, seed=3 + n, device="cpu", dtype=torch.float32)
    prefix = torch.tensor([[1, 3]], dtype=torch.int32).repeat(B, 1)
    seqs, st = S.collaborative_speculation_decode(lm, prefix, iterations=4 * n + 4, gammas=gammas, combine_mode=mode,
                                                  weights=weights, verify=oracle_verify, seed=17)
    assert st.rejections > 0 and st.accepted > 0
    assert min(len(s) for s in seqs) >= 2 + depth
    law = _exact_joint_law(lm, [1, 3], mode, weights, depth)
    keys = sorted(law)
    index = {k: i for i, k in enumerate(keys)}
    counts = np.zeros(len(keys))
    for s in seqs:
        counts[index[tuple(s[2:2 + depth])]] += 1          # a token outside the support would raise
    expected = np.array([law[k] for k in keys]) * B
    keep = expected >= 5
    obs, exp = counts[keep], expected[keep]
    if (~keep).any():
        obs, exp = np.append(obs, counts[~keep].sum()), np.append(exp, expected[~keep].sum())
    chi2, pval = stats.chisquare(obs, exp)
    assert pval > 1e-3, pval


def _identical_models(n, V):
    lm = apf.HashedBigramLM(n, V, buckets=32, seed=1, device="cpu", dtype=torch.float32)
    lm.tables = [lm.tables[0] for _ in range(n)]           # r == q: every draft is accepted
    return lm


def test_schedule_of_the_three_model_walkthrough():
    """Proposal lengths (3, 2, 1), everything accepted (App. B.2's example): M1 drafts x1..x3; M2 scores
    them, adds x4 and drafts x5; M3 scores x1..x5 and adds x6, x1..x3 are verified; M1 scores x4..x6, adds
    x7, x4 and x5 are verified, M1 drafts x8, x9."""
    B = 7
    lm = _identical_models(3, 11)
    prefix = torch.tensor([[2, 5]], dtype=torch.int32).repeat(B, 1)
    want = {1: ([3, 0, 0], 0, 3), 2: ([3, 2, 0], 0, 5), 3: ([3, 2, 1], 3, 6), 4: ([6, 2, 1], 5, 6)}
    for it, (calls, tokens, longest) in want.items():
        seqs, st = S.collaborative_speculation_decode(lm, prefix, it, (3, 2, 1), O.ENSEMBLE, [0.5, 0.3, 0.2],
                                                      oracle_verify, seed=5)
        assert st.model_calls == [c * B for c in calls], (it, st)
        assert st.tokens_out == tokens * B and st.rejections == 0 and st.max_window == longest
        assert all(len(s) == 2 + tokens for s in seqs)


def test_three_models_of_length_one_reach_one_token_per_call():
    """Sec. 3.4's sketch: after the pipeline fills, every model call yields one accepted token, against
    three calls per token for plain collaboration."""
    B = 4
    lm = _identical_models(3, 9)
    prefix = torch.tensor([[0, 1]], dtype=torch.int32).repeat(B, 1)
    _, st = S.collaborative_speculation_decode(lm, prefix, 12, (1, 1, 1), O.ENSEMBLE, [1 / 3, 1 / 3, 1 / 3],
                                               oracle_verify, seed=1)
    assert st.model_calls == [4 * B] * 3 and st.tokens_out == 10 * B
    assert st.modelled_speedup([1.0, 1.0, 1.0]) == pytest.approx(2.5)


def test_rejection_clears_the_window_and_restarts_from_the_default_proposer():
    V, B = 6, 3000
    lm = apf.HashedBigramLM(3, V, buckets=16, base_std=0.5, noise_std=3.0, seed=2, device="cpu", dtype=torch.float32)
    prefix = torch.tensor([[1, 2]], dtype=torch.int32).repeat(B, 1)
    seqs, st = S.collaborative_speculation_decode(lm, prefix, 9, (2, 1, 1), O.ENSEMBLE, [0.4, 0.3, 0.3],
                                                  oracle_verify, seed=3)
    assert st.rejections > 0.2 * B
    assert st.verified == st.accepted + st.rejections
    assert st.tokens_out == st.accepted + st.rejections == sum(len(s) - 2 for s in seqs)
    # never slower than plain collaboration in model calls per token (every call can yield a token)
    assert st.modelled_speedup([1.0, 1.0, 1.0]) > 1.0


def test_argument_checks():
    lm = _identical_models(2, 5)
    prefix = torch.tensor([[0, 1]], dtype=torch.int32)
    with pytest.raises(ValueError):
        S.collaborative_speculation_decode(lm, prefix, 1, (1,), O.ENSEMBLE, [0.5, 0.5], oracle_verify)
    with pytest.raises(ValueError):
        S.collaborative_speculation_decode(lm, prefix, 1, (1, 0), O.ENSEMBLE, [0.5, 0.5], oracle_verify)
    with pytest.raises(ValueError):
        S.collaborative_speculation_decode(lm, prefix, 1, (9, 9), O.ENSEMBLE, [0.5, 0.5], oracle_verify)


@pytest.mark.gpu
@pytest.mark.parametrize("n,gammas,mode,weights", [(3, (3, 2, 1), O.ENSEMBLE, [0.5, 0.3, 0.2]),
                                                  (2, (2, 3), O.CONTRASTIVE, [0.5, 0.1]),
                                                  (4, (1, 1, 2, 1), O.ENSEMBLE, [0.4, 0.3, 0.2, 0.1]),
                                                  (3, (2, 1, 2), O.LOGIT_MIX, [0.5, 0.4, 0.1])])
def test_gpu_driver_matches_oracle_driver_token_for_token(n, gammas, mode, weights):
    from paper_2502_01662_amd import cos_verify as C
    V, B = 4096, 40
    lm_gpu = apf.HashedBigramLM(n, V, buckets=256, base_std=2.0, noise_std=0.6, seed=9, device="cuda")
    lm_cpu = apf.HashedBigramLM(n, V, buckets=256, base_std=2.0, noise_std=0.6, seed=9, device="cpu")
    prefix = torch.randint(0, V, (B, 4), dtype=torch.int32, generator=torch.Generator().manual_seed(4))
    want, st_o = S.collaborative_speculation_decode(lm_cpu, prefix, 14, gammas, mode, weights, oracle_verify, seed=21)
    got, st_g = S.collaborative_speculation_decode(lm_gpu, prefix.cuda(), 14, gammas, mode, weights, C.cos_verify, seed=21)
    assert got == want
    assert st_g == st_o and st_g.rejections > 0 and st_g.accepted > 100


@pytest.mark.parametrize("n,gammas,beta", [(2, (2, 1), [1.3, -0.3]), (3, (3, 2, 1), [0.8, 0.5, -0.3]), (4, (1, 1, 1, 1), [0.4, 0.3, 0.2, 0.1])])
def test_greedy_scheduler_is_lossless(n, gammas, beta):
    """Temperature 0 with a logit mix of n models: whatever the schedule, the text is the one that
    one-token-at-a-time greedy decoding of the mix writes."""
    V, B, iterations = 40, 48, 12
    lm = apf.HashedBigramLM(n, V, buckets=128, base_std=2.0, noise_std=0.5, seed=17, device="cpu", dtype=torch.float32)
    prefix = torch.randint(0, V, (B, 3), dtype=torch.int32, generator=torch.Generator().manual_seed(3))
    seqs, st = S.collaborative_speculation_decode(lm, prefix, iterations, gammas, O.LOGIT_MIX, beta, oracle_verify,
                                                  seed=7, greedy=True)
    for row, got in zip(prefix.tolist(), seqs):
        seq = list(row)
        while len(seq) < len(got):
            ctx = torch.tensor([seq[-2:]], dtype=torch.int32)
            rows = np.stack([lm.logits(m, ctx)[0].to(torch.float64).numpy() for m in range(n)])
            seq.append(O.argmax_logit_mix(rows, beta))
        assert got == seq
    assert st.accepted > 0 and st.rejections > 0 and st.tokens_out > B


@pytest.mark.gpu
@pytest.mark.parametrize("mode,weights,n", [(O.ENSEMBLE, [0.5, 0.3, 0.2], 3), (O.LOGIT_MIX, [0.8, 0.5, -0.3], 3),
                                            (O.CONTRASTIVE, [0.5, 0.1], 2)])
def test_gpu_greedy_scheduler_matches_oracle_scheduler_token_for_token(mode, weights, n):
    from paper_2502_01662_amd import cos_verify as C
    V, B = 2048, 24
    gammas = (3, 2, 1)[:n]
    lm_gpu = apf.HashedBigramLM(n, V, buckets=256, base_std=2.0, noise_std=0.6, seed=19, device="cuda")
    lm_cpu = apf.HashedBigramLM(n, V, buckets=256, base_std=2.0, noise_std=0.6, seed=19, device="cpu")
    prefix = torch.randint(0, V, (B, 4), dtype=torch.int32, generator=torch.Generator().manual_seed(6))
    want, st_o = S.collaborative_speculation_decode(lm_cpu, prefix, 10, gammas, mode, weights, oracle_verify, seed=23, greedy=True)
    got, st_g = S.collaborative_speculation_decode(lm_gpu, prefix.cuda(), 10, gammas, mode, weights, C.cos_verify, seed=23, greedy=True)
    assert got == want and st_g == st_o
    assert st_g.accepted > 0
