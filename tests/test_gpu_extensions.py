"""GPU parity of the extensions of the step (cos_verify_ex): temperature, the verifier's own
bonus token, per-position proposers -- same bar as the base step."""
import numpy as np
import pytest
import torch

from oracle import cos_oracle as O
from paper_2502_01662_amd import cos_verify as C
from paper_2502_01662_amd import workloads as W
from tests import parity as P
from tests.test_gpu_parity import _check, _random_inputs

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("T", [0.5, 0.7, 1.3, 2.0])
@pytest.mark.parametrize("dtype", ["bf16", "f32", "f16"])
def test_temperature_ensemble_and_contrastive(T, dtype):
    inp = _random_inputs(3, 6, 3, 4099, dtype, seed=int(T * 100))
    inp["temperature"] = T
    _check(f"ens T={T} {dtype}", inp, C.COS_COMBINE_ENSEMBLE, [0.2, 0.5, 0.3])
    inp = _random_inputs(2, 6, 3, 33000, dtype, seed=int(T * 100) + 1, std=2.0)
    inp["temperature"] = T
    _check(f"cd T={T} {dtype}", inp, C.COS_COMBINE_CONTRASTIVE, [0.5, 0.1])


def test_temperature_changes_the_result_and_one_is_the_base_step():
    w = W.C3.scaled(B=8)
    inp = W.generate(w, device="cuda")
    base = P.run_gpu(inp, w.mode, w.weights)
    inp["temperature"] = 1.0
    same = P.run_gpu(inp, w.mode, w.weights)
    assert np.array_equal(base[0], same[0]) and np.array_equal(base[1], same[1])
    inp["temperature"] = 0.6
    alen, toks, diag, _ = _check("c3 T=0.6", inp, w.mode, w.weights)
    assert not np.array_equal(toks, base[1])


@pytest.mark.parametrize("mode,weights,n", [(C.COS_COMBINE_ENSEMBLE, [0.5, 0.5], 2),
                                            (C.COS_COMBINE_ENSEMBLE, [0.5, 0.3, 0.2], 3),
                                            (C.COS_COMBINE_CONTRASTIVE, [0.5, 0.1], 2)])
def test_verifier_bonus(mode, weights, n):
    """Accept everything (identical models would be trivial: use u_accept = 0 on half the rows), draw
    the bonus from the verifier alone, with NaN where the other models have no logits yet."""
    B, gamma, V = 12, 3, 5000
    inp = _random_inputs(n, B, gamma, V, "bf16", seed=77 + n + mode, std=1.5)
    inp["u_accept"][::2] = 0.0
    if mode == C.COS_COMBINE_CONTRASTIVE:       # keep the drafts inside the mask so they are accepted at u = 0
        top = inp["logits"][0, :, :gamma].float().argmax(-1).to(torch.int32)
        inp["draft_tokens"][::2] = top[::2]
    bonus = ((inp["proposer_idx"] + 1) % n).to(torch.int32)
    bonus[1] = -1                                # one row keeps the bonus from r
    inp["bonus_idx"] = bonus
    for b in range(B):
        if int(bonus[b]) >= 0:
            for m in range(n):
                if m != int(bonus[b]):
                    inp["logits"][m, b, gamma] = float("nan")
    # rows with bonus -1 need valid logits everywhere
    alen, toks, diag, rep = _check(f"verifier bonus mode={mode} n={n}", inp, mode, weights)
    assert (alen == gamma).sum() >= B // 2
    assert np.all(toks[np.arange(B), alen] >= 0)


def test_verifier_bonus_only_changes_fully_accepted_rows():
    inp = _random_inputs(2, 64, 2, 3000, "bf16", seed=5)
    base = P.run_gpu(inp, C.COS_COMBINE_ENSEMBLE, [0.4, 0.6])
    inp["bonus_idx"] = (1 - inp["proposer_idx"]).to(torch.int32)
    alen, toks, diag, _ = _check("bonus vs base", inp, C.COS_COMBINE_ENSEMBLE, [0.4, 0.6])
    rejected = base[0] < 2
    assert rejected.any() and (~rejected).any()
    assert np.array_equal(alen, base[0])
    assert np.array_equal(toks[rejected], base[1][rejected])
    assert not np.array_equal(toks[~rejected], base[1][~rejected])


@pytest.mark.parametrize("mode,weights,n", [(C.COS_COMBINE_ENSEMBLE, [0.2, 0.5, 0.3], 3),
                                            (C.COS_COMBINE_CONTRASTIVE, [0.3, 0.05], 2)])
def test_per_position_proposers(mode, weights, n):
    B, gamma, V = 24, 4, 8200
    inp = _random_inputs(n, B, gamma, V, "bf16", seed=31 + n, std=1.5)
    g = torch.Generator().manual_seed(9)
    inp["proposer_pos"] = torch.randint(0, n, (B, gamma), generator=g, dtype=torch.int32).cuda()
    alen, toks, diag, _ = _check(f"per-position proposers mode={mode}", inp, mode, weights)
    del inp["proposer_pos"]
    base = P.run_gpu(inp, mode, weights)
    assert not np.array_equal(base[1], toks)


def test_all_extensions_together_on_c5_shape():
    w = W.C5.scaled(B=16)
    inp = W.generate(w, device="cuda")
    g = torch.Generator().manual_seed(3)
    inp["temperature"] = 0.8
    inp["proposer_pos"] = torch.randint(0, w.n, (w.B, w.gamma), generator=g, dtype=torch.int32).cuda()
    inp["bonus_idx"] = torch.randint(-1, w.n, (w.B,), generator=g, dtype=torch.int32).cuda()
    inp["u_accept"][::3] = 0.0
    _check("c5 B=16 with every extension", inp, w.mode, w.weights)


def test_option_validation():
    inp = _random_inputs(2, 2, 2, 64, "bf16", seed=1)
    with pytest.raises(C.CosVerifyError):
        C.cos_verify(inp["logits"], inp["draft_tokens"], inp["proposer_idx"], 0, [0.5, 0.5], inp["u_accept"],
                     inp["u_resample"], temperature=-1.0)
    with pytest.raises(C.CosVerifyError):
        C.cos_verify(inp["logits"], inp["draft_tokens"], inp["proposer_idx"], 0, [0.5, 0.5], inp["u_accept"],
                     inp["u_resample"], temperature=float("nan"))


@pytest.mark.parametrize("mode,weights,n,dtype", [(C.COS_COMBINE_ENSEMBLE, [0.5, 0.3, 0.2], 3, "bf16"),
                                                  (C.COS_COMBINE_ENSEMBLE, [0.25] * 4, 4, "f32"),
                                                  (C.COS_COMBINE_ENSEMBLE, [0.1, 0.2, 0.3, 0.15, 0.25], 5, "bf16"),
                                                  (C.COS_COMBINE_CONTRASTIVE, [0.5, 0.1], 2, "bf16"),
                                                  (C.COS_COMBINE_CONTRASTIVE, [0.2, 0.0], 2, "f32")])
def test_acceptance_rate_output(mode, weights, n, dtype):
    """alpha = sum min(q, r) per draft position (Eq. 7) against the oracle: float32 terms of relative
    error ~1e-7 summed in float64, so 1e-6 absolute on a number in [0, 1]."""
    from oracle import cos_oracle as O
    B, gamma, V = 10, 3, 20011
    inp = _random_inputs(n, B, gamma, V, dtype, seed=91 + n, std=1.5)
    g = torch.Generator().manual_seed(4)
    inp["proposer_pos"] = torch.randint(0, n, (B, gamma), generator=g, dtype=torch.int32).cuda()
    inp["temperature"] = 0.9
    alpha = torch.full((B, gamma), -1.0, dtype=torch.float64, device="cuda")
    alen, toks = C.cos_verify(inp["logits"], inp["draft_tokens"], inp["proposer_idx"], mode, weights,
                              inp["u_accept"], inp["u_resample"], alpha=alpha, **P._gpu_ext(inp))
    torch.cuda.synchronize()
    ora = O.verify(W.host_logits(inp["logits"]), P.oracle_dtype(inp["logits"]), inp["draft_tokens"].cpu().numpy(),
                   inp["proposer_idx"].cpu().numpy(), mode, weights, inp["u_accept"].cpu().numpy(),
                   inp["u_resample"].cpu().numpy(), all_positions=True, temperature=0.9,
                   proposer_pos=inp["proposer_pos"].cpu().numpy(), want_alpha=True)
    got = alpha.cpu().numpy()
    err = np.abs(got - ora.alpha).max()
    print(f"[parity] alpha mode={mode} n={n} {dtype}: max abs err {err:.3e}", flush=True)
    assert err < 1e-6
    assert np.array_equal(alen.cpu().numpy(), ora.accepted_len) and np.array_equal(toks.cpu().numpy(), ora.out_tokens)
    if mode == C.COS_COMBINE_ENSEMBLE:          # Thm 3.2: alpha >= the proposer's weight
        w = np.asarray(weights)[inp["proposer_pos"].cpu().numpy()]
        assert np.all(got >= w - 1e-6)


def test_acceptance_rate_full_c4_shape():
    from oracle import cos_oracle as O
    w = W.C4.scaled(B=32)
    inp = W.generate(w, device="cuda")
    alpha = torch.empty((w.B, w.gamma), dtype=torch.float64, device="cuda")
    C.cos_verify(inp["logits"], inp["draft_tokens"], inp["proposer_idx"], w.mode, w.weights,
                 inp["u_accept"], inp["u_resample"], alpha=alpha)
    torch.cuda.synchronize()
    ora = O.verify(W.host_logits(inp["logits"]), O.DTYPE_BF16, inp["draft_tokens"].cpu().numpy(),
                   inp["proposer_idx"].cpu().numpy(), w.mode, list(w.weights), inp["u_accept"].cpu().numpy(),
                   inp["u_resample"].cpu().numpy(), all_positions=True, want_alpha=True)
    assert np.abs(alpha.cpu().numpy() - ora.alpha).max() < 1e-6


# ---------------------------------------------------------------------------
# stop_window: verify w positions per launch, never read past the first rejection
# ---------------------------------------------------------------------------

@pytest.mark.parametrize("window", [1, 2, 3, 5])
@pytest.mark.parametrize("name", ["c1", "c2", "c3", "c4", "c5"])
def test_stop_window_equals_the_one_launch_step(name, window):
    w = W.WORKLOADS[name]
    w = w.scaled(B=min(w.B, 12))
    inp = W.generate(w, device="cuda")
    base = P.run_gpu(inp, w.mode, w.weights)
    inp["stop_window"] = window
    alen, toks, diag, _ = _check(f"{name} stop_window={window}", inp, w.mode, w.weights)
    assert np.array_equal(alen, base[0]) and np.array_equal(toks, base[1])


@pytest.mark.parametrize("mode,weights,n", [(C.COS_COMBINE_ENSEMBLE, [0.2, 0.5, 0.3], 3),
                                            (C.COS_COMBINE_CONTRASTIVE, [0.3, 0.05], 2)])
def test_stop_window_never_reads_past_the_first_rejection(mode, weights, n):
    B, gamma, V = 32, 5, 8200
    inp = _random_inputs(n, B, gamma, V, "bf16", seed=61 + n, std=1.5)
    if mode == C.COS_COMBINE_CONTRASTIVE:
        # drafts at the expert's argmax are accepted, random ones are outside the mask: mix them so
        # that every accepted length occurs
        top = inp["logits"][0, :, :gamma].float().argmax(-1).to(torch.int32)
        cut = (torch.arange(B, device="cuda") % (gamma + 1))[:, None]
        keep = torch.arange(gamma, device="cuda")[None, :] < cut
        inp["draft_tokens"] = torch.where(keep, top, inp["draft_tokens"]).contiguous()
        inp["proposer_idx"][:] = 0
    base_alen, base_toks, _ = P.run_gpu(inp, mode, weights)
    assert len(set(base_alen.tolist())) >= 3
    for window in (1, 2):
        poisoned = dict(inp)
        poisoned["logits"] = inp["logits"].clone()
        for b in range(B):
            first_unread = (int(base_alen[b]) // window + 1) * window
            if first_unread <= gamma:
                poisoned["logits"][:, b, first_unread:] = float("nan")
        poisoned["stop_window"] = window
        alen, toks, _ = P.run_gpu(poisoned, mode, weights)
        assert np.array_equal(alen, base_alen) and np.array_equal(toks, base_toks), window


def test_stop_window_with_other_extensions():
    w = W.C5.scaled(B=16)
    inp = W.generate(w, device="cuda")
    g = torch.Generator().manual_seed(3)
    inp["temperature"] = 0.8
    inp["proposer_pos"] = torch.randint(0, w.n, (w.B, w.gamma), generator=g, dtype=torch.int32).cuda()
    inp["bonus_idx"] = torch.randint(-1, w.n, (w.B,), generator=g, dtype=torch.int32).cuda()
    inp["u_accept"][::3] = 0.0
    inp["stop_window"] = 2
    _check("c5 B=16, window 2, every extension", inp, w.mode, w.weights)
    alpha = torch.empty((w.B, w.gamma), dtype=torch.float64, device="cuda")
    with pytest.raises(C.CosVerifyError):     # acceptance rates of unread positions do not exist
        C.cos_verify(inp["logits"], inp["draft_tokens"], inp["proposer_idx"], w.mode, w.weights,
                     inp["u_accept"], inp["u_resample"], alpha=alpha, stop_window=2)


# ---------------------------------------------------------------------------
# temperature 0 (greedy), contrastive mode: bit-exact, no near-tie excuses
# ---------------------------------------------------------------------------

def _greedy_inputs(B, gamma, V, dtype, seed, mu, alpha):
    """Random logits; drafts follow the contrastive argmax on a prefix of varying length."""
    from oracle import cos_oracle as O
    inp = _random_inputs(2, B, gamma, V, dtype, seed=seed, std=2.0)
    host = W.host_logits(inp["logits"])
    odt = P.oracle_dtype(inp["logits"])
    drafts = inp["draft_tokens"].cpu().numpy().copy()
    for b in range(B):
        for j in range(b % (gamma + 1)):
            drafts[b, j] = O.argmax_contrastive(O.row_to_f64(host[0, b, j], odt), O.row_to_f64(host[1, b, j], odt), mu, alpha)
    inp["draft_tokens"] = torch.from_numpy(drafts).cuda()
    return inp, host, odt


@pytest.mark.parametrize("dtype", ["bf16", "f32", "f16"])
@pytest.mark.parametrize("B,gamma,V,mu,alpha", [(6, 2, 8, 0.5, 0.1), (12, 3, 1000, 0.1, 0.1), (8, 2, 4099, 0.5, 0.0),
                                                (10, 4, 33000, 1.0, 0.5), (7, 3, 70001, 0.3, 1.0),
                                                (16, 5, 128256, 0.5, 0.1)])
def test_greedy_contrastive_is_bit_exact(dtype, B, gamma, V, mu, alpha):
    from oracle import cos_oracle as O
    inp, host, odt = _greedy_inputs(B, gamma, V, dtype, seed=V + B, mu=mu, alpha=alpha)
    for bonus in (None, torch.tensor([(b % 3) - 1 for b in range(B)], dtype=torch.int32).cuda()):
        alen, toks = C.cos_verify(inp["logits"], inp["draft_tokens"], inp["proposer_idx"], C.COS_COMBINE_CONTRASTIVE,
                                  [mu, alpha], inp["u_accept"], inp["u_resample"], greedy=True, bonus_idx=bonus)
        torch.cuda.synchronize()
        st, want_len, want_toks = O.verify_greedy(host, odt, inp["draft_tokens"].cpu().numpy(), [mu, alpha],
                                                  bonus_idx=None if bonus is None else bonus.cpu().numpy())
        assert st == 0
        assert np.array_equal(alen.cpu().numpy(), want_len)
        assert np.array_equal(toks.cpu().numpy(), want_toks)
        assert len(set(want_len.tolist())) == min(B, gamma + 1)


def test_greedy_ties_go_to_the_lowest_index_and_unsupported_combinations():
    from oracle import cos_oracle as O
    B, gamma, V = 4, 2, 5000
    inp = _random_inputs(2, B, gamma, V, "bf16", seed=3)
    inp["logits"][:] = 0.0                                   # every token ties
    inp["logits"][0, :, :, 4000] = 1.0
    inp["logits"][0, :, :, 77] = 1.0                         # two maxima of c: the lower index wins
    inp["draft_tokens"][:] = 77
    alen, toks = C.cos_verify(inp["logits"], inp["draft_tokens"], inp["proposer_idx"], C.COS_COMBINE_CONTRASTIVE,
                              [0.5, 0.0], inp["u_accept"], inp["u_resample"], greedy=True)
    torch.cuda.synchronize()
    assert np.all(alen.cpu().numpy() == gamma) and np.all(toks.cpu().numpy() == 77)
    st, want_len, want_toks = O.verify_greedy(W.host_logits(inp["logits"]), O.DTYPE_BF16,
                                              inp["draft_tokens"].cpu().numpy(), [0.5, 0.0])
    assert np.array_equal(toks.cpu().numpy(), want_toks)
    with pytest.raises(C.CosVerifyError):                    # the one-hot r of Eq. (5) has no use for per-position proposers
        C.cos_verify(inp["logits"], inp["draft_tokens"], inp["proposer_idx"], C.COS_COMBINE_CONTRASTIVE, [0.5, 0.0],
                     inp["u_accept"], inp["u_resample"], greedy=True,
                     proposer_pos=torch.zeros((B, gamma), dtype=torch.int32, device="cuda"))
    with pytest.raises(C.CosVerifyError):
        C.cos_verify(inp["logits"], inp["draft_tokens"], inp["proposer_idx"], C.COS_COMBINE_CONTRASTIVE, [0.5, 0.0],
                     inp["u_accept"], inp["u_resample"], greedy=True, stop_window=1)


# ---------------------------------------------------------------------------
# rows with fewer drafts (num_drafts) and no extra token (no_bonus): what Alg. 2's VERIFY needs
# ---------------------------------------------------------------------------

def _ragged_inputs(n, B, gamma, V, dtype, seed, no_bonus, mode):
    """num_drafts cycles through 0..gamma; half the rows accept every draft (u_accept = 0, drafts
    inside the mask in contrastive mode); every position a correct kernel never reads holds NaN."""
    inp = _random_inputs(n, B, gamma, V, dtype, seed=seed, std=1.5)
    inp["u_accept"][::2] = 0.0
    if mode == C.COS_COMBINE_CONTRASTIVE:
        top = inp["logits"][0, :, :gamma].float().argmax(-1).to(torch.int32)
        inp["draft_tokens"][::2] = top[::2]
    nd = torch.tensor([(b // 2) % (gamma + 1) for b in range(B)], dtype=torch.int32)
    for b in range(B):
        inp["logits"][:, b, int(nd[b]) + (0 if no_bonus else 1):] = float("nan")
        inp["draft_tokens"][b, int(nd[b]):] = V - 1            # ignored
        inp["u_accept"][b, int(nd[b]):] = 0.0                  # ignored (would accept if it were read)
    inp["num_drafts"] = nd.cuda()
    inp["no_bonus"] = no_bonus
    return inp, nd.numpy()


@pytest.mark.parametrize("no_bonus", [False, True])
@pytest.mark.parametrize("mode,weights,n,dtype", [(C.COS_COMBINE_ENSEMBLE, [0.5, 0.3, 0.2], 3, "bf16"),
                                                  (C.COS_COMBINE_ENSEMBLE, [0.4, 0.6], 2, "f32"),
                                                  (C.COS_COMBINE_CONTRASTIVE, [0.5, 0.1], 2, "bf16"),
                                                  (C.COS_COMBINE_CONTRASTIVE, [0.3, 0.0], 2, "f32")])
def test_ragged_rows(mode, weights, n, dtype, no_bonus):
    B, gamma, V = 24, 5, 6007
    inp, nd = _ragged_inputs(n, B, gamma, V, dtype, seed=300 + n + mode, no_bonus=no_bonus, mode=mode)
    alen, toks, diag, rep = _check(f"ragged mode={mode} n={n} {dtype} no_bonus={no_bonus}", inp, mode, weights)
    assert np.all(alen <= nd)
    full = alen == nd
    assert full.sum() >= B // 2 and (~full).sum() >= 2
    drawn = toks[np.arange(B), alen]
    if no_bonus:
        assert np.all(drawn[full] == -1) and np.all(drawn[~full] >= 0)
        assert np.all(diag.sample_mass.cpu().numpy()[full] == 0.0)
    else:
        assert np.all(drawn >= 0)


def test_ragged_rows_with_every_other_extension():
    B, gamma, V, n = 20, 4, 9001, 3
    inp, nd = _ragged_inputs(n, B, gamma, V, "bf16", seed=321, no_bonus=False, mode=C.COS_COMBINE_ENSEMBLE)
    g = torch.Generator().manual_seed(8)
    inp["proposer_pos"] = torch.randint(0, n, (B, gamma), generator=g, dtype=torch.int32).cuda()
    inp["bonus_idx"] = ((inp["proposer_idx"] + 1) % n).to(torch.int32)
    inp["temperature"] = 0.8
    for b in range(B):                                           # only the verifier has logits at the bonus position
        for m in range(n):
            if m != int(inp["bonus_idx"][b]):
                inp["logits"][m, b, int(nd[b])] = float("nan")
    base = _check("ragged + proposer_pos + verifier bonus + T", inp, C.COS_COMBINE_ENSEMBLE, [0.2, 0.5, 0.3])
    for w in (1, 2, 3):
        inp["stop_window"] = w
        alen, toks, _, _ = _check(f"ragged + all, window {w}", inp, C.COS_COMBINE_ENSEMBLE, [0.2, 0.5, 0.3])
        assert np.array_equal(alen, base[0]) and np.array_equal(toks, base[1])


@pytest.mark.parametrize("window", [1, 2, 4])
@pytest.mark.parametrize("mode,weights,n", [(C.COS_COMBINE_ENSEMBLE, [0.5, 0.5], 2), (C.COS_COMBINE_CONTRASTIVE, [0.5, 0.1], 2)])
def test_ragged_rows_no_bonus_in_windows(mode, weights, n, window):
    inp, nd = _ragged_inputs(n, 18, 5, 4099, "bf16", seed=340 + mode, no_bonus=True, mode=mode)
    inp["stop_window"] = window
    alen, toks, _, _ = _check(f"ragged no_bonus window={window} mode={mode}", inp, mode, weights)
    assert (alen == nd).sum() >= 9


def test_ragged_acceptance_rates():
    from oracle import cos_oracle as O
    B, gamma, V, n = 12, 4, 12007, 3
    inp, nd = _ragged_inputs(n, B, gamma, V, "bf16", seed=350, no_bonus=True, mode=C.COS_COMBINE_ENSEMBLE)
    alpha = torch.full((B, gamma), -1.0, dtype=torch.float64, device="cuda")
    w = [0.2, 0.5, 0.3]
    alen, toks = C.cos_verify(inp["logits"], inp["draft_tokens"], inp["proposer_idx"], C.COS_COMBINE_ENSEMBLE, w,
                              inp["u_accept"], inp["u_resample"], alpha=alpha, **P._gpu_ext(inp))
    torch.cuda.synchronize()
    ora = O.verify(W.host_logits(inp["logits"]), O.DTYPE_BF16, inp["draft_tokens"].cpu().numpy(),
                   inp["proposer_idx"].cpu().numpy(), C.COS_COMBINE_ENSEMBLE, w, inp["u_accept"].cpu().numpy(),
                   inp["u_resample"].cpu().numpy(), all_positions=True, want_alpha=True, num_drafts=nd, no_bonus=True)
    got = alpha.cpu().numpy()
    has = np.arange(gamma)[None, :] < nd[:, None]
    assert np.isnan(got[~has]).all() and np.isnan(ora.alpha[~has]).all()
    assert np.abs(got[has] - ora.alpha[has]).max() < 1e-6
    assert np.array_equal(alen.cpu().numpy(), ora.accepted_len) and np.array_equal(toks.cpu().numpy(), ora.out_tokens)


@pytest.mark.parametrize("no_bonus", [False, True])
def test_ragged_greedy(no_bonus):
    from oracle import cos_oracle as O
    B, gamma, V, mu, a = 21, 4, 33000, 0.5, 0.1
    inp, host, odt = _greedy_inputs(B, gamma, V, "bf16", seed=360, mu=mu, alpha=a)
    nd = np.array([(b * 2) % (gamma + 1) for b in range(B)], dtype=np.int32)
    for b in range(B):
        inp["logits"][:, b, int(nd[b]) + (0 if no_bonus else 1):] = float("nan")
    host = W.host_logits(inp["logits"])
    alen, toks = C.cos_verify(inp["logits"], inp["draft_tokens"], inp["proposer_idx"], C.COS_COMBINE_CONTRASTIVE,
                              [mu, a], inp["u_accept"], inp["u_resample"], greedy=True,
                              num_drafts=torch.from_numpy(nd).cuda(), no_bonus=no_bonus)
    torch.cuda.synchronize()
    st, want_len, want_toks = O.verify_greedy(host, odt, inp["draft_tokens"].cpu().numpy(), [mu, a], num_drafts=nd,
                                              no_bonus=no_bonus)
    assert st == 0
    assert np.array_equal(alen.cpu().numpy(), want_len) and np.array_equal(toks.cpu().numpy(), want_toks)
    assert (want_len == nd).sum() >= 4 and (want_len < nd).sum() >= 4


def test_ragged_rows_at_the_c5_shape():
    w = W.C5.scaled(B=24)
    inp = W.generate(w, device="cuda")
    nd = torch.tensor([b % (w.gamma + 1) for b in range(w.B)], dtype=torch.int32)
    for b in range(w.B):
        inp["logits"][:, b, int(nd[b]):] = float("nan")
    inp["num_drafts"] = nd.cuda()
    inp["no_bonus"] = True
    alen, toks, _, _ = _check("c5 shape, ragged, no bonus", inp, w.mode, w.weights)
    assert np.all(alen <= nd.numpy())
    base = W.generate(w, device="cuda")
    full = P.run_gpu(base, w.mode, w.weights)
    # a shorter row is a prefix of the full row's verification
    assert np.array_equal(alen, np.minimum(full[0], nd.numpy()))


# ---------------------------------------------------------------------------
# r close to q (acceptance rates above 97 %), rejection forced: the default path, no option set
# ---------------------------------------------------------------------------

def _nearly_identical_models(n, B, gamma, V, noise, seed, dtype="f32", proposer=0):
    """n models that differ from one base by Gaussian noise of the given size; every first draft is the
    proposer's favourite token and u_accept -> 1 forces the rejections that hardly ever happen otherwise
    (a slightly flatter r gives that token less than q does)."""
    inp = _random_inputs(1, B, gamma, V, "f32", seed=seed, std=2.5)
    g = torch.Generator().manual_seed(seed + 1)
    base = inp["logits"][0].double().cpu()
    tdt = {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}[dtype]
    inp["logits"] = torch.stack([(base + torch.randn(base.shape, generator=g, dtype=torch.float64) * noise).to(tdt)
                                 for _ in range(n)]).cuda()
    inp["proposer_idx"] = torch.full((B,), proposer, dtype=torch.int32).cuda()
    inp["u_accept"][:] = 1.0 - 1e-12
    inp["draft_tokens"][:, 0] = inp["logits"][proposer, :, 0].argmax(-1).to(torch.int32)
    return inp


@pytest.mark.parametrize("noise", [0.03, 0.003, 0.0003])
@pytest.mark.parametrize("mode,weights,n", [(C.COS_COMBINE_ENSEMBLE, [0.5, 0.5], 2),
                                            (C.COS_COMBINE_ENSEMBLE, [0.4, 0.35, 0.25], 3),
                                            (C.COS_COMBINE_CONTRASTIVE, [0.002, 0.0], 2),   # mu -> 0: r -> softmax(l_0)
                                            (C.COS_COMBINE_CONTRASTIVE, [0.002, 1e-6], 2),  # the same behind a wide mask
                                            (C.COS_COMBINE_LOGIT_MIX, [0.5, 0.5], 2)])
@pytest.mark.parametrize("refine_kernels", [0, 1])
def test_residual_of_nearly_identical_models(mode, weights, n, noise, refine_kernels):
    """Models that differ by a little noise: the residual mass is 1e-2 ... 1e-5 of a probability, far below
    what term-by-term float32 resolves.  The step evaluates such residuals in their difference form by
    itself (no option): every drawn token must be the float64 reference's, in every combine mode -- by the
    route a row-set of this size takes by default (the sequence's last sampling workgroup alone) and by the
    two refinement launches that large row-sets take."""
    B, gamma, V = 256, 2, 32000
    inp = _nearly_identical_models(n, B, gamma, V, noise, seed=5, proposer=1 if mode != C.COS_COMBINE_ENSEMBLE else 0)
    diag = C.Diagnostics.allocate(B, gamma, "cuda")
    alen, toks = C.cos_verify(inp["logits"], inp["draft_tokens"], inp["proposer_idx"], mode, weights,
                              inp["u_accept"], inp["u_resample"], diag=diag,
                              shape=C.LaunchShape(refine_kernels=refine_kernels) if refine_kernels else None)
    torch.cuda.synchronize()
    rep = P.compare(inp, mode, weights, alen.cpu().numpy(), toks.cpu().numpy(), diag)
    flags = diag.flags.cpu().numpy()
    print(f"[parity] nearly identical models, noise {noise}, mode {mode}, refinement launches {refine_kernels}: {rep.summary()}, refined "
          f"{int((flags & C.COS_FLAG_RESIDUAL_REFINED != 0).sum())}/{B}, median F {np.median(diag.sample_mass.cpu().numpy()):.2e}", flush=True)
    assert rep.ok, rep.failures[:3]
    assert (flags & C.COS_FLAG_RESIDUAL_REFINED != 0).sum() > B // 4
    # the residual spreads over most of the vocabulary here, so the 1e-6 windows around its 32000 CDF edges
    # cover several percent of [0, 1): a few draws land in one and may take the neighbouring token
    assert rep.excused_accept_ties + rep.excused_cdf_ties <= B // 50


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
def test_residual_of_nearly_identical_models_in_16_bit_formats(dtype):
    """The same with stored 16-bit logits, where 'nearly identical' means many logits are bit-identical and
    the others differ by one step of the format."""
    B, gamma, V = 128, 2, 40000
    for mode, weights, n in ((C.COS_COMBINE_ENSEMBLE, [0.3, 0.3, 0.4], 3), (C.COS_COMBINE_LOGIT_MIX, [0.7, 0.3], 2)):
        inp = _nearly_identical_models(n, B, gamma, V, 0.004, seed=11, dtype=dtype)
        diag = C.Diagnostics.allocate(B, gamma, "cuda")
        alen, toks = C.cos_verify(inp["logits"], inp["draft_tokens"], inp["proposer_idx"], mode, weights,
                                  inp["u_accept"], inp["u_resample"], diag=diag)
        torch.cuda.synchronize()
        rep = P.compare(inp, mode, weights, alen.cpu().numpy(), toks.cpu().numpy(), diag)
        print(f"[parity] nearly identical {dtype} models, mode {mode}: {rep.summary()}, median F "
              f"{np.median(diag.sample_mass.cpu().numpy()):.2e}", flush=True)
        assert rep.ok, rep.failures[:3]
        assert rep.excused_accept_ties + rep.excused_cdf_ties <= 3, rep.summary()


@pytest.mark.parametrize("mode,weights,n,B,V,dtype", [
    (C.COS_COMBINE_ENSEMBLE, [0.25, 0.25, 0.25, 0.25], 4, 24, 262144, "bf16"),   # 2 MiB per row-set
    (C.COS_COMBINE_ENSEMBLE, [0.2] * 5, 5, 12, 150000, "bf16"),                  # the general model count
    (C.COS_COMBINE_LOGIT_MIX, [0.6, 0.4], 2, 24, 140000, "f32"),
    (C.COS_COMBINE_CONTRASTIVE, [0.002, 0.0], 2, 24, 300001, "f16"),             # unaligned rows
])
def test_large_row_sets_take_the_refinement_launches_by_default(mode, weights, n, B, V, dtype):
    """Above 256 KiB per row-set the default route is the two refinement launches; both routes must give the
    reference's tokens and the same outputs as each other (the tile sums do not depend on who computes them)."""
    gamma = 2
    inp = _nearly_identical_models(n, B, gamma, V, 0.004, seed=23, dtype=dtype,
                                   proposer=1 if mode != C.COS_COMBINE_ENSEMBLE else 0)
    assert n * V * inp["logits"].element_size() > 256 << 10
    outs = {}
    for route in (0, -1, 1):
        diag = C.Diagnostics.allocate(B, gamma, "cuda")
        alen, toks = C.cos_verify(inp["logits"], inp["draft_tokens"], inp["proposer_idx"], mode, weights,
                                  inp["u_accept"], inp["u_resample"], diag=diag,
                                  shape=C.LaunchShape(refine_kernels=route) if route else None)
        torch.cuda.synchronize()
        outs[route] = (alen.cpu().numpy(), toks.cpu().numpy(), diag.flags.cpu().numpy(), diag.sample_mass.cpu().numpy())
        rep = P.compare(inp, mode, weights, outs[route][0], outs[route][1], diag)
        print(f"[parity] large row-set, mode {mode}, n {n}, route {route}: {rep.summary()}, refined "
              f"{int((outs[route][2] & C.COS_FLAG_RESIDUAL_REFINED != 0).sum())}/{B}", flush=True)
        assert rep.ok, rep.failures[:3]
        assert rep.excused_accept_ties + rep.excused_cdf_ties <= 2, rep.summary()
    assert (outs[0][2] & C.COS_FLAG_RESIDUAL_REFINED != 0).sum() > B // 4
    for route in (-1, 1):
        assert np.array_equal(outs[route][0], outs[0][0]) and np.array_equal(outs[route][1], outs[0][1])
        assert np.array_equal(outs[route][2], outs[0][2])
        np.testing.assert_allclose(outs[route][3], outs[0][3], rtol=1e-12)


def test_refinement_launches_with_more_marked_sequences_than_a_thousand():
    """Every sequence of a batch of 3000 is marked: the refinement launches then have one workgroup per sequence."""
    n, B, gamma, V = 2, 3000, 1, 2000
    inp = _nearly_identical_models(n, B, gamma, V, 0.003, seed=91)
    inp["shape"] = C.LaunchShape(refine_kernels=1)
    alen, toks, diag = P.run_gpu(inp, C.COS_COMBINE_ENSEMBLE, [0.5, 0.5])
    rep = P.compare(inp, C.COS_COMBINE_ENSEMBLE, [0.5, 0.5], alen, toks, diag)
    flags = diag.flags.cpu().numpy()
    print(f"[parity] 3000 marked sequences: {rep.summary()}, refined {int((flags & C.COS_FLAG_RESIDUAL_REFINED != 0).sum())}", flush=True)
    assert rep.ok, rep.failures[:3]
    assert (flags & C.COS_FLAG_RESIDUAL_REFINED != 0).sum() > 1100          # more than the launch's usual thousand workgroups
    assert rep.excused_accept_ties + rep.excused_cdf_ties <= B // 50


def test_refinement_launches_in_a_captured_graph():
    """The refinement route under HIP graph capture: the list of marked sequences is built by atomics and
    emptied by the last workgroup, so every replay (eager work and garbage in the workspace in between) must
    reproduce the eager result."""
    n, B, gamma, V = 2, 24, 2, 70000
    inp = _nearly_identical_models(n, B, gamma, V, 0.003, seed=61)
    ws = C.allocate_workspace(n, B, gamma, V, C.COS_DTYPE_F32, C.COS_COMBINE_ENSEMBLE, "cuda")
    alen = torch.empty(B, dtype=torch.int32, device="cuda")
    toks = torch.empty((B, gamma + 1), dtype=torch.int32, device="cuda")
    diag = C.Diagnostics.allocate(B, gamma, "cuda")

    def call():
        C.cos_verify(inp["logits"], inp["draft_tokens"], inp["proposer_idx"], C.COS_COMBINE_ENSEMBLE, [0.5, 0.5],
                     inp["u_accept"], inp["u_resample"], accepted_len=alen, out_tokens=toks, workspace=ws, diag=diag)

    assert C.cos_verify_launch_info(n, B, gamma, V, C.COS_DTYPE_F32, C.COS_COMBINE_ENSEMBLE, [0.5, 0.5])["refine_launches"] == 1
    call()
    torch.cuda.synchronize()
    want = (alen.cpu().numpy().copy(), toks.cpu().numpy().copy())
    assert (diag.flags.cpu().numpy() & C.COS_FLAG_RESIDUAL_REFINED != 0).sum() > B // 4
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        call()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        call()
    for i in range(4):
        alen.fill_(-5)
        toks.fill_(-5)
        ws.fill_(i + 1)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert np.array_equal(alen.cpu().numpy(), want[0]) and np.array_equal(toks.cpu().numpy(), want[1]), i
    rep = P.compare(inp, C.COS_COMBINE_ENSEMBLE, [0.5, 0.5], want[0], want[1], None)
    assert rep.ok, rep.failures[:3]


def test_refinement_launches_leave_their_counters_at_zero():
    """The refinement kernels' arrival counters wrap like the others: a loop that promises a ready workspace
    gets the same outputs call after call, also when the set of marked sequences changes between calls."""
    n, B, gamma, V = 3, 40, 2, 20000
    inp = _nearly_identical_models(n, B, gamma, V, 0.003, seed=77)
    other = dict(inp)
    other["u_accept"] = inp["u_accept"].clone()
    other["u_accept"][::3] = 0.0                     # every third sequence accepts everything: no residual there
    ws = C.allocate_workspace(n, B, gamma, V, C.COS_DTYPE_F32, C.COS_COMBINE_ENSEMBLE, "cuda")
    ws.fill_(0xA5)
    want = {}
    for name, x in (("all", inp), ("some", other)):
        a, t = C.cos_verify(x["logits"], x["draft_tokens"], x["proposer_idx"], C.COS_COMBINE_ENSEMBLE, [0.5, 0.3, 0.2],
                            x["u_accept"], x["u_resample"], shape=C.LaunchShape(refine_kernels=-1))
        torch.cuda.synchronize()
        want[name] = (a.cpu().numpy(), t.cpu().numpy())
    for call, name in enumerate(("all", "some", "all", "all", "some")):
        x = inp if name == "all" else other
        a, t = C.cos_verify(x["logits"], x["draft_tokens"], x["proposer_idx"], C.COS_COMBINE_ENSEMBLE, [0.5, 0.3, 0.2],
                            x["u_accept"], x["u_resample"], workspace=ws,
                            shape=C.LaunchShape(refine_kernels=1, workspace_ready=1 if call else 0))
        torch.cuda.synchronize()
        assert np.array_equal(a.cpu().numpy(), want[name][0]) and np.array_equal(t.cpu().numpy(), want[name][1]), (call, name)


# ---------------------------------------------------------------------------
# temperature 0 (greedy), ensemble: r lives on the models' own tokens; bit-exact, nothing excused
# ---------------------------------------------------------------------------

def _greedy_ensemble_inputs(n, B, gamma, V, dtype, seed):
    """Models that often agree (a shared base plus a little noise); drafts are mostly the proposer's own
    token, sometimes another model's, sometimes a token nobody votes for."""
    g = torch.Generator().manual_seed(seed)
    tdt = {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}[dtype]
    base = torch.randn((1, B, gamma + 1, V), generator=g, dtype=torch.float64) * 2.0
    logits = (base + 0.7 * torch.randn((n, B, gamma + 1, V), generator=g, dtype=torch.float64)).to(tdt)
    inp = {"logits": logits.cuda(),
           "proposer_idx": torch.randint(0, n, (B,), generator=g, dtype=torch.int32).cuda(),
           "u_accept": torch.rand((B, gamma), generator=g, dtype=torch.float64).cuda(),
           "u_resample": torch.rand((B,), generator=g, dtype=torch.float64).cuda()}
    ppos = torch.randint(0, n, (B, gamma), generator=g, dtype=torch.int32)
    top = logits.double().argmax(-1)                              # [n][B][gamma+1], first maximum
    kind = torch.randint(0, 10, (B, gamma), generator=g)
    drafts = torch.randint(0, V, (B, gamma), generator=g, dtype=torch.int32)
    for b in range(B):
        for j in range(gamma):
            if kind[b, j] < 7:
                drafts[b, j] = top[ppos[b, j], b, j]              # the proposer's token
            elif kind[b, j] < 9:
                drafts[b, j] = top[(ppos[b, j] + 1) % n, b, j]    # another model's token
    inp["draft_tokens"] = drafts.cuda()
    inp["proposer_pos"] = ppos.cuda()
    return inp


@pytest.mark.parametrize("dtype", ["bf16", "f32", "f16"])
@pytest.mark.parametrize("n,B,gamma,V", [(1, 6, 2, 9), (2, 12, 3, 1000), (3, 9, 2, 4099), (4, 10, 4, 33000), (5, 7, 3, 70001),
                                         (8, 5, 2, 20000), (2, 16, 5, 128256)])
def test_greedy_ensemble_is_bit_exact(dtype, n, B, gamma, V):
    inp = _greedy_ensemble_inputs(n, B, gamma, V, dtype, seed=31 * V + n)
    w = np.random.default_rng(V + n).dirichlet(np.ones(n)).tolist()
    host, odt = W.host_logits(inp["logits"]), P.oracle_dtype(inp["logits"])
    common = (inp["draft_tokens"].cpu().numpy(), inp["proposer_idx"].cpu().numpy(), C.COS_COMBINE_ENSEMBLE, w,
              inp["u_accept"].cpu().numpy(), inp["u_resample"].cpu().numpy())
    bonus = torch.tensor([(b % (n + 1)) - 1 for b in range(B)], dtype=torch.int32).cuda()
    lens = set()
    for kw in ({}, {"proposer_pos": inp["proposer_pos"]}, {"bonus_idx": bonus}, {"proposer_pos": inp["proposer_pos"], "bonus_idx": bonus}):
        alen, toks = C.cos_verify(inp["logits"], inp["draft_tokens"], inp["proposer_idx"], C.COS_COMBINE_ENSEMBLE, w,
                                  inp["u_accept"], inp["u_resample"], greedy=True, **kw)
        torch.cuda.synchronize()
        ora = O.verify(host, odt, *common, greedy=True, **{k: v.cpu().numpy() for k, v in kw.items()})
        assert ora.status == 0
        assert np.array_equal(alen.cpu().numpy(), ora.accepted_len), kw.keys()
        assert np.array_equal(toks.cpu().numpy(), ora.out_tokens), kw.keys()
        lens |= set(ora.accepted_len.tolist())
    assert n == 1 or len(lens) >= min(3, gamma + 1)


@pytest.mark.parametrize("no_bonus", [False, True])
def test_greedy_ensemble_ragged_rows_odd_vocabulary_agreeing_models_and_zero_weights(no_bonus):
    n, B, gamma, V = 3, 24, 4, 33001
    inp = _greedy_ensemble_inputs(n, B, gamma, V, "bf16", seed=99)
    inp["logits"][1, ::2] = inp["logits"][0, ::2]              # two models agree on every other row
    inp["logits"][2, ::4] = inp["logits"][0, ::4]              # ... all three on every fourth: r == q, the fall-back
    w = [0.7, 0.3, 0.0]                                         # a model without weight still proposes
    nd = np.array([(b * 2) % (gamma + 1) for b in range(B)], dtype=np.int32)
    for b in range(B):
        inp["logits"][:, b, int(nd[b]) + (0 if no_bonus else 1):] = float("nan")
    host = W.host_logits(inp["logits"])
    alen, toks = C.cos_verify(inp["logits"], inp["draft_tokens"], inp["proposer_idx"], C.COS_COMBINE_ENSEMBLE, w,
                              inp["u_accept"], inp["u_resample"], greedy=True, proposer_pos=inp["proposer_pos"],
                              num_drafts=torch.from_numpy(nd).cuda(), no_bonus=no_bonus)
    torch.cuda.synchronize()
    ora = O.verify(host, O.DTYPE_BF16, inp["draft_tokens"].cpu().numpy(), inp["proposer_idx"].cpu().numpy(),
                   C.COS_COMBINE_ENSEMBLE, w, inp["u_accept"].cpu().numpy(), inp["u_resample"].cpu().numpy(), greedy=True,
                   proposer_pos=inp["proposer_pos"].cpu().numpy(), num_drafts=nd, no_bonus=no_bonus)
    assert ora.status == 0
    assert np.array_equal(alen.cpu().numpy(), ora.accepted_len) and np.array_equal(toks.cpu().numpy(), ora.out_tokens)
    assert (ora.flags & O.FLAG_RESIDUAL_FALLBACK).any()         # the degenerate case did occur


# ---------------------------------------------------------------------------
# masked contrastive mode in one read of the logits: candidate lists, and what happens when they do not fit
# ---------------------------------------------------------------------------

def _masked_inputs(B, gamma, V, dtype, seed, flat=False, std=3.0):
    inp = _random_inputs(2, B, gamma, V, dtype, seed=seed, std=std)
    if flat:          # an expert row with very many tokens at (nearly) the same top value: the mask is not sparse
        g = torch.Generator().manual_seed(seed + 7)
        top = (torch.rand((B, gamma + 1, V), generator=g) < 0.4).cuda()
        inp["logits"][0] = torch.where(top, torch.full_like(inp["logits"][0], 4.0), inp["logits"][0].clamp(max=3.0))
    # drafts the combination likes on half of the rows, so that lengths vary
    c = inp["logits"][0, :, :gamma].float() - 0.5 * inp["logits"][1, :, :gamma].float()
    inp["draft_tokens"][::2] = c.argmax(-1).to(torch.int32)[::2]
    return inp


@pytest.mark.parametrize("dtype", ["bf16", "f32", "f16"])
@pytest.mark.parametrize("flat,alpha_cd", [(False, 0.1), (False, 1e-4), (True, 0.5), (False, 1.0)])
def test_masked_contrastive_candidate_lists_and_their_overflow(dtype, flat, alpha_cd):
    """alpha_cd = 0.1 on Gaussian logits keeps a few dozen tokens (the candidate lists carry the whole step);
    alpha_cd = 1e-4, or an expert row with 40 % of its tokens at the top, keeps thousands (no list fits: the
    finishing workgroup reads the rows again and draws from the full row); alpha_cd = 1 keeps the expert's
    top token alone.  Same outputs as the reference either way, with acceptance rates, a verifier's bonus
    token, per-position proposers, one-position windows -- and the same tokens as the two-pass route."""
    B, gamma, V = 12, 3, 40000
    inp = _masked_inputs(B, gamma, V, dtype, seed=77, flat=flat)
    mode, weights = C.COS_COMBINE_CONTRASTIVE, [0.5, alpha_cd]
    auto = _check(f"masked {dtype} flat={flat} alpha_cd={alpha_cd}, route by the mask's width", inp, mode, weights)
    one_read = C.LaunchShape(two_pass_mask=-1)       # (a wide mask takes the two passes by itself)
    inp["shape"] = one_read
    alen, toks, diag, rep = _check(f"masked one-pass {dtype} flat={flat} alpha_cd={alpha_cd}", inp, mode, weights)
    assert np.array_equal(auto[0], alen) and np.array_equal(auto[1], toks)
    # the two-pass route gives the same tokens (near-ties aside: none at these seeds)
    a2, t2 = C.cos_verify(inp["logits"], inp["draft_tokens"], inp["proposer_idx"], mode, weights, inp["u_accept"],
                          inp["u_resample"], shape=C.LaunchShape(two_pass_mask=1))
    torch.cuda.synchronize()
    assert np.array_equal(a2.cpu().numpy(), alen) and np.array_equal(t2.cpu().numpy(), toks)
    # acceptance rates from the candidate lists (or the second read) against the oracle's
    alpha = torch.full((B, gamma), -1.0, dtype=torch.float64, device="cuda")
    C.cos_verify(inp["logits"], inp["draft_tokens"], inp["proposer_idx"], mode, weights, inp["u_accept"], inp["u_resample"],
                 alpha=alpha, shape=one_read)
    torch.cuda.synchronize()
    ora = O.verify(W.host_logits(inp["logits"]), P.oracle_dtype(inp["logits"]), inp["draft_tokens"].cpu().numpy(),
                   inp["proposer_idx"].cpu().numpy(), mode, weights, inp["u_accept"].cpu().numpy(),
                   inp["u_resample"].cpu().numpy(), all_positions=True, want_alpha=True)
    assert np.abs(alpha.cpu().numpy() - ora.alpha).max() < 1e-6
    # extensions on top
    g = torch.Generator().manual_seed(5)
    inp["proposer_pos"] = torch.randint(0, 2, (B, gamma), generator=g, dtype=torch.int32).cuda()
    inp["bonus_idx"] = torch.randint(-1, 2, (B,), generator=g, dtype=torch.int32).cuda()
    inp["u_accept"][B // 2:] = 0.0                               # these rows reach the bonus position
    inp["draft_tokens"][B // 2:] = (inp["logits"][0, B // 2:, :gamma].float() - 0.5 * inp["logits"][1, B // 2:, :gamma].float()).argmax(-1).to(torch.int32)
    for window in (0, 1, 2):
        inp["stop_window"] = window
        base = _check(f"masked one-pass {dtype} flat={flat} alpha_cd={alpha_cd} + extensions, window {window}", inp, mode, weights)
        # a verifier's own bonus token by the finishing workgroup alone, and by the cooperative draw kernel
        for route in (-1, 1):
            inp["shape"] = C.LaunchShape(two_pass_mask=-1, refine_kernels=route)
            other = _check(f"masked one-pass {dtype} flat={flat} alpha_cd={alpha_cd} + extensions, window {window}, "
                           f"refinement launches {route}", inp, mode, weights)
            assert np.array_equal(other[0], base[0]) and np.array_equal(other[1], base[1])
        inp["shape"] = one_read


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_masked_contrastive_with_many_chunks_of_a_huge_vocabulary(dtype):
    """Eight positions of 600 000 tokens in 37 chunks each: what the chunks leave (every token within reach of its
    own chunk's maximum: thousands per sequence) does not fit the finishing workgroup's list, what passes against
    the rows' true maxima (a few dozen per position) does -- the list is sized by a first counting sweep."""
    B, gamma, V = 4, 7, 600000
    inp = _masked_inputs(B, gamma, V, dtype, seed=131)
    inp["shape"] = C.LaunchShape(two_pass_mask=-1)
    mode, weights = C.COS_COMBINE_CONTRASTIVE, [0.5, 0.1]
    info = C.cos_verify_launch_info(2, B, gamma, V, {"bf16": C.COS_DTYPE_BF16, "f32": C.COS_DTYPE_F32}[dtype], mode, weights,
                                    shape=inp["shape"])
    assert info["one_read_mask"] == 1 and info["chunks_per_row"] >= 30
    alen, toks, diag, rep = _check(f"masked one-pass {dtype}, 600k tokens in {info['chunks_per_row']} chunks", inp, mode, weights)
    alpha = torch.full((B, gamma), -1.0, dtype=torch.float64, device="cuda")
    C.cos_verify(inp["logits"], inp["draft_tokens"], inp["proposer_idx"], mode, weights, inp["u_accept"], inp["u_resample"],
                 alpha=alpha, shape=inp["shape"])
    torch.cuda.synchronize()
    ora = O.verify(W.host_logits(inp["logits"]), P.oracle_dtype(inp["logits"]), inp["draft_tokens"].cpu().numpy(),
                   inp["proposer_idx"].cpu().numpy(), mode, weights, inp["u_accept"].cpu().numpy(),
                   inp["u_resample"].cpu().numpy(), all_positions=True, want_alpha=True)
    assert np.abs(alpha.cpu().numpy() - ora.alpha).max() < 1e-6
    two = C.cos_verify(inp["logits"], inp["draft_tokens"], inp["proposer_idx"], mode, weights, inp["u_accept"],
                       inp["u_resample"], shape=C.LaunchShape(two_pass_mask=1))
    torch.cuda.synchronize()
    assert np.array_equal(two[0].cpu().numpy(), alen) and np.array_equal(two[1].cpu().numpy(), toks)


def test_masked_contrastive_is_deterministic():
    """Candidates are collected in whatever order the wavefronts find them and sorted by token before anything
    is summed: two calls give the same bits, diagnostics included."""
    inp = _masked_inputs(16, 4, 128256, "bf16", seed=3)
    outs = []
    for _ in range(3):
        diag = C.Diagnostics.allocate(16, 4, "cuda")
        a, t = C.cos_verify(inp["logits"], inp["draft_tokens"], inp["proposer_idx"], C.COS_COMBINE_CONTRASTIVE, [0.5, 0.1],
                            inp["u_accept"], inp["u_resample"], diag=diag)
        torch.cuda.synchronize()
        outs.append((a, t, diag))
    for a, t, d in outs[1:]:
        assert torch.equal(a, outs[0][0]) and torch.equal(t, outs[0][1])
        for name in ("r_at_draft", "q_at_draft", "sample_mass", "cdf_lo", "cdf_hi", "flags"):
            assert torch.equal(getattr(d, name), getattr(outs[0][2], name)), name
