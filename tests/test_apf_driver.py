"""Alternate Proposal Framework (Alg. 1, Sec. 3.3) around the verification step.

CPU: the driver with the oracle as its verify back end must generate tokens that follow the combined
distribution r (the paper's central claim: App. A.1 applied along Alg. 1), with and without the bonus
token.  GPU: the same driver with cos_verify must produce the same sequences token for token."""
import numpy as np
import pytest
import torch
from scipy import stats

from oracle import cos_oracle as O
from paper_2502_01662_amd import apf
from paper_2502_01662_amd import workloads as W


def oracle_verify(logits, drafts, proposer, mode, weights, u_acc, u_res, bonus_idx=None, temperature=1.0, greedy=False):
    dt = O.DTYPE_F32 if logits.dtype == torch.float32 else O.DTYPE_BF16
    if greedy and mode != O.ENSEMBLE:                       # temperature 0, logit-level modes: their own oracle step
        st, alen, toks = O.verify_greedy(W.host_logits(logits), dt, drafts.cpu().numpy(), weights, mode=mode,
                                         bonus_idx=None if bonus_idx is None else bonus_idx.cpu().numpy())
        assert st == 0
        return torch.from_numpy(alen), torch.from_numpy(toks)
    res = O.verify(W.host_logits(logits), dt, drafts.cpu().numpy(), proposer.cpu().numpy(), mode, weights,
                   u_acc.cpu().numpy(), u_res.cpu().numpy(), temperature=temperature, greedy=greedy,
                   bonus_idx=None if bonus_idx is None else bonus_idx.cpu().numpy())
    assert res.status == 0
    return torch.from_numpy(res.accepted_len), torch.from_numpy(res.out_tokens)


def _exact_joint_law(lm, ctx0, mode, weights, depth):
    """P(x_1..x_depth | ctx0) when every token is drawn from r: vanilla collaborative decoding."""
    V = lm.V
    law = {}

    def r_of(ctx):
        c = torch.tensor([ctx[-2:]], dtype=torch.int32)
        l = [lm.logits(m, c)[0].to(torch.float64).numpy() for m in range(2)]
        s = np.stack([O.softmax(x) for x in l])
        if mode == O.ENSEMBLE:
            return O.combine_ensemble(s, np.asarray(weights, dtype=np.float64))
        return O.combine_contrastive(l[0], l[1], weights[0], weights[1])[0]

    def rec(ctx, prob, toks):
        if len(toks) == depth:
            law[tuple(toks)] = prob
            return
        r = r_of(ctx)
        for x in range(V):
            if r[x] > 0:
                rec(ctx + [x], prob * r[x], toks + [x])

    rec(list(ctx0), 1.0, [])
    return law


@pytest.mark.parametrize("use_bonus", [True, False])
@pytest.mark.parametrize("mode,weights", [(O.ENSEMBLE, [0.4, 0.6]), (O.CONTRASTIVE, [0.5, 0.05])])
def test_generated_tokens_follow_the_combined_distribution(mode, weights, use_bonus):
    V, gamma, B, depth = 5, 2, 60_000, 3
    lm = apf.HashedBigramLM(2, V, buckets=64, base_std=1.0, noise_std=0.7, seed=3, device="cpu", dtype=torch.float32)
    prefix = torch.tensor([[1, 3]], dtype=torch.int32).repeat(B, 1)
    seqs, st = apf.alternate_proposal_decode(lm, prefix, cycles=3, gamma=gamma, combine_mode=mode, weights=weights,
                                             verify=oracle_verify, seed=11, use_bonus=use_bonus)
    assert min(len(s) for s in seqs) >= 2 + depth
    if use_bonus:
        assert st.swapped_cycles > 0                       # the alternate path was exercised
    else:
        assert st.swapped_cycles == 0
    law = _exact_joint_law(lm, [1, 3], mode, weights, depth)
    keys = sorted(law)
    index = {k: i for i, k in enumerate(keys)}
    counts = np.zeros(len(keys))
    for s in seqs:
        counts[index[tuple(s[2:2 + depth])]] += 1          # a token outside the support would raise
    expected = np.array([law[k] for k in keys]) * B
    keep = expected >= 5
    obs, exp = counts[keep], expected[keep]
    if (~keep).any():                                      # pool the rare cells
        obs, exp = np.append(obs, counts[~keep].sum()), np.append(exp, expected[~keep].sum())
    chi2, pval = stats.chisquare(obs, exp)
    assert pval > 1e-3, pval


def test_alternation_saves_proposer_steps():
    """Thm 3.6's mechanism: a cycle that starts from a bonus token drafts one token fewer itself."""
    V, gamma, B = 50, 3, 2000
    lm = apf.HashedBigramLM(2, V, buckets=128, base_std=2.0, noise_std=0.3, seed=5, device="cpu", dtype=torch.float32)
    prefix = torch.randint(0, V, (B, 3), dtype=torch.int32, generator=torch.Generator().manual_seed(1))
    _, naive = apf.alternate_proposal_decode(lm, prefix, 6, gamma, O.ENSEMBLE, [0.5, 0.5], oracle_verify, seed=2,
                                             use_bonus=False)
    _, alt = apf.alternate_proposal_decode(lm, prefix, 6, gamma, O.ENSEMBLE, [0.5, 0.5], oracle_verify, seed=2,
                                           use_bonus=True)
    assert alt.swapped_cycles > 0.2 * B
    # same number of model calls per cycle, but every swapped cycle reuses one drafted token
    assert alt.tokens_out + 0 >= naive.tokens_out * 0.95


@pytest.mark.gpu
@pytest.mark.parametrize("mode,weights", [(O.ENSEMBLE, [0.5, 0.5]), (O.CONTRASTIVE, [0.5, 0.1])])
def test_gpu_driver_matches_oracle_driver_token_for_token(mode, weights):
    from paper_2502_01662_amd import cos_verify as C
    V, gamma, B = 4096, 4, 48
    lm_gpu = apf.HashedBigramLM(2, V, buckets=256, base_std=2.0, noise_std=0.6, seed=9, device="cuda")
    lm_cpu = apf.HashedBigramLM(2, V, buckets=256, base_std=2.0, noise_std=0.6, seed=9, device="cpu")
    prefix = torch.randint(0, V, (B, 4), dtype=torch.int32, generator=torch.Generator().manual_seed(4))
    want, st_o = apf.alternate_proposal_decode(lm_cpu, prefix, 8, gamma, mode, weights, oracle_verify, seed=21)
    got, st_g = apf.alternate_proposal_decode(lm_gpu, prefix.cuda(), 8, gamma, mode, weights, C.cos_verify, seed=21)
    assert got == want
    assert st_g == st_o and st_g.swapped_cycles > 0


def _vanilla_greedy(lm, prefix, steps, argmax_of_rows):
    """Plain collaborative decoding at temperature 0: one token at a time, the argmax of the combination."""
    out = []
    for row in prefix.tolist():
        seq = list(row)
        for _ in range(steps):
            ctx = torch.tensor([seq[-2:]], dtype=torch.int32)
            rows = [lm.logits(m, ctx)[0].to(torch.float64).numpy() for m in range(lm.n_models)]
            seq.append(int(argmax_of_rows(rows)))
        out.append(seq)
    return out


@pytest.mark.parametrize("use_bonus", [True, False])
@pytest.mark.parametrize("mode,weights", [(O.CONTRASTIVE, [0.5, 0.1]), (O.CONTRASTIVE, [1.0, 0.0]), (O.LOGIT_MIX, [1.3, -0.3])])
def test_greedy_decoding_is_lossless(mode, weights, use_bonus):
    """The paper's headline setting (contrastive decoding at T = 0): speculation changes the number of
    model calls, not the text -- the driver's output is exactly what one-token-at-a-time greedy
    collaborative decoding writes."""
    V, gamma, B, cycles = 40, 3, 64, 6
    lm = apf.HashedBigramLM(2, V, buckets=128, base_std=2.0, noise_std=0.5, seed=13, device="cpu", dtype=torch.float32)
    prefix = torch.randint(0, V, (B, 3), dtype=torch.int32, generator=torch.Generator().manual_seed(2))
    seqs, st = apf.alternate_proposal_decode(lm, prefix, cycles, gamma, mode, weights, oracle_verify, seed=5,
                                             use_bonus=use_bonus, greedy=True)
    if mode == O.CONTRASTIVE:
        pick = lambda rows: O.argmax_contrastive(rows[0], rows[1], weights[0], weights[1])
    else:
        pick = lambda rows: O.argmax_logit_mix(np.stack(rows), weights)
    want = _vanilla_greedy(lm, prefix, cycles * (gamma + 1), pick)
    for got, ref in zip(seqs, want):
        assert got == ref[:len(got)]
    assert st.accepted > 0 and st.accepted < st.drafted            # both accepted and rejected drafts occurred
    assert st.swapped_cycles == 0 or use_bonus                   # (how often all drafts pass depends on the combination)


@pytest.mark.gpu
@pytest.mark.parametrize("mode,weights", [(O.ENSEMBLE, [0.5, 0.5]), (O.CONTRASTIVE, [0.5, 0.1]), (O.LOGIT_MIX, [1.3, -0.3])])
def test_gpu_greedy_driver_matches_oracle_driver_token_for_token(mode, weights):
    from paper_2502_01662_amd import cos_verify as C
    V, gamma, B = 4096, 4, 48
    lm_gpu = apf.HashedBigramLM(2, V, buckets=256, base_std=2.0, noise_std=0.6, seed=9, device="cuda")
    lm_cpu = apf.HashedBigramLM(2, V, buckets=256, base_std=2.0, noise_std=0.6, seed=9, device="cpu")
    prefix = torch.randint(0, V, (B, 4), dtype=torch.int32, generator=torch.Generator().manual_seed(4))
    want, st_o = apf.alternate_proposal_decode(lm_cpu, prefix, 8, gamma, mode, weights, oracle_verify, seed=21, greedy=True)
    got, st_g = apf.alternate_proposal_decode(lm_gpu, prefix.cuda(), 8, gamma, mode, weights, C.cos_verify, seed=21, greedy=True)
    assert got == want
    assert st_g == st_o and st_g.swapped_cycles > 0
