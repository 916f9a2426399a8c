"""GPU parity of the logit-level linear combination r = softmax(sum_m beta_m l_m) (Eq. (3), C' on logits;
the form of decoding-time realignment, Sec. 2) -- same bar as the other combine modes."""
import numpy as np
import pytest
import torch

from oracle import cos_oracle as O
from paper_2502_01662_amd import cos_verify as C
from paper_2502_01662_amd import workloads as W
from tests import parity as P
from tests.test_gpu_parity import _check, _random_inputs

pytestmark = pytest.mark.gpu
MIX = C.COS_COMBINE_LOGIT_MIX

BETAS = {1: [1.3], 2: [1.5, -0.5], 3: [0.6, 0.6, -0.2], 4: [0.25, 0.25, 0.25, 0.25], 5: [1.0, -0.3, 0.2, 0.0, 0.4],
         8: [0.3, 0.2, -0.1, 0.15, 0.25, 0.0, 0.1, 0.2]}


def _likely_drafts(inp, beta, every=2):
    """Put the mix's argmax on every other row so that acceptances and rejections both occur."""
    gamma = inp["draft_tokens"].shape[1]
    c = sum(float(b) * inp["logits"][m, :, :gamma].float() for m, b in enumerate(beta) if b != 0)
    inp["draft_tokens"][::every] = c.argmax(-1).to(torch.int32)[::every]


@pytest.mark.parametrize("dtype", ["bf16", "f32", "f16"])
@pytest.mark.parametrize("n,B,gamma,V", [(1, 3, 2, 777), (2, 6, 3, 4099), (2, 4, 2, 33000), (3, 5, 4, 8192), (4, 4, 3, 20011),
                                         (5, 3, 2, 6000), (8, 2, 3, 2048), (3, 2, 31, 513), (2, 3, 2, 70001)])
def test_logit_mix_shapes(dtype, n, B, gamma, V):
    inp = _random_inputs(n, B, gamma, V, dtype, seed=500 + n + V, std=1.5)
    _likely_drafts(inp, BETAS[n])
    alen, toks, diag, rep = _check(f"mix n={n} B={B} gamma={gamma} V={V} {dtype}", inp, MIX, BETAS[n])
    assert rep.exact_rows + rep.excused_accept_ties + rep.excused_cdf_ties == B


def test_logit_mix_equals_contrastive_without_mask_on_the_gpu():
    inp = _random_inputs(2, 24, 3, 12007, "bf16", seed=520, std=2.0)
    _likely_drafts(inp, [1.0, -0.5])
    a = _check("mix (1, -0.5)", inp, MIX, [1.0, -0.5])
    b = _check("contrastive mu=0.5 no mask", inp, C.COS_COMBINE_CONTRASTIVE, [0.5, 0.0])
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    assert len(set(a[0].tolist())) >= 3


def test_logit_mix_one_hot_on_the_proposer_accepts_everything():
    inp = _random_inputs(3, 16, 4, 5000, "bf16", seed=521)
    inp["proposer_idx"][:] = 1
    alen, toks, _, _ = _check("mix one-hot", inp, MIX, [0.0, 1.0, 0.0])
    assert np.all(alen == 4)


def test_logit_mix_ignores_a_model_without_weight_and_handles_minus_inf():
    n, B, gamma, V = 3, 12, 3, 9001
    inp = _random_inputs(n, B, gamma, V, "bf16", seed=522, std=1.5)
    inp["logits"][1] = float("nan")                           # beta_1 = 0 and model 1 never proposes
    inp["proposer_idx"] = torch.tensor([0, 2] * (B // 2), dtype=torch.int32).cuda()
    dead = torch.arange(0, V, 7).cuda()
    inp["logits"][0][..., dead] = float("-inf")               # ruled out by model 0 (positive weight)
    beta = [0.7, 0.0, 0.5]
    _likely_drafts(inp, beta)
    alen, toks, _, _ = _check("mix, dead model and -inf logits", inp, MIX, beta)
    drawn = toks[np.arange(B), alen]
    assert np.all(drawn % 7 != 0)                             # never a token model 0 rules out


def test_logit_mix_with_every_extension():
    n, B, gamma, V = 3, 20, 4, 9001
    beta = [0.9, -0.3, 0.5]
    inp = _random_inputs(n, B, gamma, V, "bf16", seed=523, std=1.5)
    _likely_drafts(inp, beta)
    g = torch.Generator().manual_seed(8)
    inp["proposer_pos"] = torch.randint(0, n, (B, gamma), generator=g, dtype=torch.int32).cuda()
    inp["bonus_idx"] = ((inp["proposer_idx"] + 1) % n).to(torch.int32)
    inp["bonus_idx"][3] = -1
    inp["temperature"] = 0.8
    nd = torch.tensor([b % (gamma + 1) for b in range(B)], dtype=torch.int32)
    inp["num_drafts"] = nd.cuda()
    inp["u_accept"][::2] = 0.0
    for b in range(B):
        inp["logits"][:, b, int(nd[b]) + 1:] = float("nan")
        if int(inp["bonus_idx"][b]) >= 0:                      # only the verifier has logits at the bonus position
            for m in range(n):
                if m != int(inp["bonus_idx"][b]):
                    inp["logits"][m, b, int(nd[b])] = float("nan")
    base = _check("mix + proposer_pos + verifier bonus + T + ragged", inp, MIX, beta)
    assert (base[0] == nd.numpy()).sum() >= B // 3
    for w in (1, 2, 3):
        inp["stop_window"] = w
        alen, toks, _, _ = _check(f"mix + all, window {w}", inp, MIX, beta)
        assert np.array_equal(alen, base[0]) and np.array_equal(toks, base[1])
    inp["stop_window"] = 0
    inp["no_bonus"] = True
    alen, toks, _, _ = _check("mix + all, no bonus", inp, MIX, beta)
    assert np.array_equal(alen, base[0])


@pytest.mark.parametrize("n,dtype", [(2, "bf16"), (3, "f32"), (4, "bf16"), (6, "bf16")])
def test_logit_mix_acceptance_rates(n, dtype):
    from oracle import cos_oracle as O
    B, gamma, V = 8, 3, 20011
    beta = (BETAS[n] if n in BETAS else [0.4, 0.3, -0.2, 0.2, 0.2, 0.1])
    inp = _random_inputs(n, B, gamma, V, dtype, seed=530 + n, std=1.5)
    alpha = torch.full((B, gamma), -1.0, dtype=torch.float64, device="cuda")
    alen, toks = C.cos_verify(inp["logits"], inp["draft_tokens"], inp["proposer_idx"], MIX, beta,
                              inp["u_accept"], inp["u_resample"], alpha=alpha)
    torch.cuda.synchronize()
    ora = O.verify(W.host_logits(inp["logits"]), P.oracle_dtype(inp["logits"]), inp["draft_tokens"].cpu().numpy(),
                   inp["proposer_idx"].cpu().numpy(), MIX, beta, inp["u_accept"].cpu().numpy(),
                   inp["u_resample"].cpu().numpy(), all_positions=True, want_alpha=True)
    err = np.abs(alpha.cpu().numpy() - ora.alpha).max()
    print(f"[parity] mix alpha n={n} {dtype}: max abs err {err:.3e}", flush=True)
    assert err < 1e-6
    assert np.array_equal(alen.cpu().numpy(), ora.accepted_len) and np.array_equal(toks.cpu().numpy(), ora.out_tokens)


def test_logit_mix_at_the_c5_shape_and_argument_checks():
    w = W.C5.scaled(B=16)
    inp = W.generate(w, device="cuda")
    beta = [0.4, 0.3, 0.2, 0.1]
    alen, toks, _, rep = _check("c5 shape, logit mix", inp, MIX, beta)
    assert len(set(alen.tolist())) >= 3
    with pytest.raises(C.CosVerifyError):
        C.cos_verify(inp["logits"], inp["draft_tokens"], inp["proposer_idx"], MIX, [0.4, float("nan"), 0.2, 0.1],
                     inp["u_accept"], inp["u_resample"])
    with pytest.raises(C.CosVerifyError):
        C.cos_verify(inp["logits"], inp["draft_tokens"], inp["proposer_idx"], 3, beta, inp["u_accept"], inp["u_resample"])
    with pytest.raises(C.CosVerifyError):                    # temperature 0 has no acceptance rates to report
        C.cos_verify(inp["logits"], inp["draft_tokens"], inp["proposer_idx"], MIX, beta, inp["u_accept"],
                     inp["u_resample"], greedy=True, alpha=torch.empty((w.B, w.gamma), dtype=torch.float64, device="cuda"))


@pytest.mark.parametrize("dtype,shift", [("f32", 0.0), ("f32", 500.0), ("bf16", 0.0), ("f16", 0.0)])
def test_logit_level_modes_cancel_exactly_when_r_equals_q(dtype, shift):
    """A one-hot mix on the proposer (or contrastive mu = 0 with the expert proposing) makes r == q;
    a draft token of probability zero is still rejected, and the residual then has no mass at all:
    the kernels must see exactly zero (and draw from r, flagged), not rounding noise."""
    inp = _random_inputs(2, 6, 2, 3000, dtype, seed=33, std=2.0)
    if shift:
        inp["logits"] = (inp["logits"].double() + shift).to(inp["logits"].dtype)
    inp["proposer_idx"][:] = 0
    inp["draft_tokens"][:, 0] = 7
    inp["logits"][:, :, 0, 7] = float("-inf")
    for name, mode, w in (("mix one-hot", MIX, [1.0, 0.0]), ("contrastive mu=0", C.COS_COMBINE_CONTRASTIVE, [0.0, 0.0])):
        alen, toks, diag, rep = _check(f"{name}, zero residual mass, {dtype} shift {shift}", inp, mode, w)
        assert np.all(alen == 0)
        assert np.all(diag.flags.cpu().numpy() & C.COS_FLAG_RESIDUAL_FALLBACK)
        assert rep.flag_mismatches == 0


# ---------------------------------------------------------------------------
# temperature 0 (greedy) of the logit mix: bit-exact, no near-tie excuses
# ---------------------------------------------------------------------------

def _greedy_mix_inputs(n, B, gamma, V, dtype, seed, beta, std=2.0):
    """Random logits; drafts follow the argmax of the mix on a prefix of varying length."""
    inp = _random_inputs(n, B, gamma, V, dtype, seed=seed, std=std)
    host = W.host_logits(inp["logits"])
    odt = P.oracle_dtype(inp["logits"])
    drafts = inp["draft_tokens"].cpu().numpy().copy()
    for b in range(B):
        for j in range(b % (gamma + 1)):
            drafts[b, j] = O.argmax_logit_mix(np.stack([O.row_to_f64(host[m, b, j], odt) for m in range(n)]), beta)
    inp["draft_tokens"] = torch.from_numpy(drafts).cuda()
    return inp, host, odt


@pytest.mark.parametrize("dtype", ["bf16", "f32", "f16"])
@pytest.mark.parametrize("n,B,gamma,V,beta", [(1, 5, 2, 9, [1.7]), (2, 12, 3, 1000, [1.0, -0.5]), (3, 8, 2, 4099, [0.5, 0.3, 0.2]),
                                              (4, 10, 4, 33000, [0.9, 0.0, -0.3, 0.4]), (5, 7, 3, 70001, [0.2] * 5),
                                              (2, 16, 5, 128256, [1.5, -0.5]), (8, 6, 2, 20000, [0.3, 0.1, -0.2, 0.0, 0.5, 0.1, 0.1, 0.1])])
def test_greedy_logit_mix_is_bit_exact(dtype, n, B, gamma, V, beta):
    inp, host, odt = _greedy_mix_inputs(n, B, gamma, V, dtype, seed=V + B, beta=beta)
    for bonus in (None, torch.tensor([(b % (n + 1)) - 1 for b in range(B)], dtype=torch.int32).cuda()):
        if bonus is not None:                                 # with a verifier bonus the other rows are never read
            for b in range(B):
                if int(bonus[b]) >= 0:
                    for m in range(n):
                        if m != int(bonus[b]):
                            inp["logits"][m, b, gamma] = float("nan")
            host = W.host_logits(inp["logits"])
        alen, toks = C.cos_verify(inp["logits"], inp["draft_tokens"], inp["proposer_idx"], MIX, beta,
                                  inp["u_accept"], inp["u_resample"], greedy=True, bonus_idx=bonus)
        torch.cuda.synchronize()
        st, want_len, want_toks = O.verify_greedy(host, odt, inp["draft_tokens"].cpu().numpy(), beta, mode=O.LOGIT_MIX,
                                                  bonus_idx=None if bonus is None else bonus.cpu().numpy())
        assert st == 0
        assert np.array_equal(alen.cpu().numpy(), want_len)
        assert np.array_equal(toks.cpu().numpy(), want_toks)
        assert len(set(want_len.tolist())) == min(B, gamma + 1)


@pytest.mark.parametrize("no_bonus", [False, True])
def test_greedy_logit_mix_ragged_rows_odd_vocabulary_and_minus_inf(no_bonus):
    n, B, gamma, V, beta = 3, 21, 4, 33001, [0.6, 0.3, 0.4]
    inp, _, _ = _greedy_mix_inputs(n, B, gamma, V, "bf16", seed=77, beta=beta)
    inp["logits"][:, :, :, 5::7] = float("-inf")              # impossible tokens (non-negative weights)
    inp, host, odt = inp, W.host_logits(inp["logits"]), O.DTYPE_BF16
    drafts = inp["draft_tokens"].cpu().numpy().copy()
    for b in range(B):
        for j in range(b % (gamma + 1)):
            drafts[b, j] = O.argmax_logit_mix(np.stack([O.row_to_f64(host[m, b, j], odt) for m in range(n)]), beta)
    inp["draft_tokens"] = torch.from_numpy(drafts).cuda()
    nd = np.array([(b * 2) % (gamma + 1) for b in range(B)], dtype=np.int32)
    for b in range(B):
        inp["logits"][:, b, int(nd[b]) + (0 if no_bonus else 1):] = float("nan")
    host = W.host_logits(inp["logits"])
    alen, toks = C.cos_verify(inp["logits"], inp["draft_tokens"], inp["proposer_idx"], MIX, beta, inp["u_accept"],
                              inp["u_resample"], greedy=True, num_drafts=torch.from_numpy(nd).cuda(), no_bonus=no_bonus)
    torch.cuda.synchronize()
    st, want_len, want_toks = O.verify_greedy(host, odt, drafts, beta, num_drafts=nd, no_bonus=no_bonus, mode=O.LOGIT_MIX)
    assert st == 0
    assert np.array_equal(alen.cpu().numpy(), want_len) and np.array_equal(toks.cpu().numpy(), want_toks)
    assert (want_len == nd).sum() >= 4 and (want_len < nd).sum() >= 4


def test_greedy_logit_mix_ties_and_the_contrastive_special_case():
    B, gamma, V = 4, 2, 5000
    inp = _random_inputs(2, B, gamma, V, "bf16", seed=3)
    inp["logits"][:] = 0.0                                   # every token ties
    inp["logits"][0, :, :, 4000] = 1.0
    inp["logits"][0, :, :, 77] = 1.0                         # two maxima: the lower index wins
    inp["draft_tokens"][:] = 77
    alen, toks = C.cos_verify(inp["logits"], inp["draft_tokens"], inp["proposer_idx"], MIX, [1.0, -0.5],
                              inp["u_accept"], inp["u_resample"], greedy=True)
    torch.cuda.synchronize()
    assert np.all(alen.cpu().numpy() == gamma) and np.all(toks.cpu().numpy() == 77)
    # beta = (1, -mu) is Eq. (5) without its mask: the two greedy kernels agree
    inp = _random_inputs(2, 9, 3, 50000, "f32", seed=8, std=2.5)
    top = inp["logits"][0].double() - 0.5 * inp["logits"][1].double()
    inp["draft_tokens"][::2] = top[::2, :3].argmax(-1).to(torch.int32)
    a1, t1 = C.cos_verify(inp["logits"], inp["draft_tokens"], inp["proposer_idx"], MIX, [1.0, -0.5],
                          inp["u_accept"], inp["u_resample"], greedy=True)
    a2, t2 = C.cos_verify(inp["logits"], inp["draft_tokens"], inp["proposer_idx"], C.COS_COMBINE_CONTRASTIVE, [0.5, 0.0],
                          inp["u_accept"], inp["u_resample"], greedy=True)
    torch.cuda.synchronize()
    assert torch.equal(a1, a2) and torch.equal(t1, t2) and int(a1.max()) == 3
