"""The n-model CoS scheduler (Alg. 2, Sec. 3.4) as a batched host-side driver around ``cos_verify``.

Every sequence keeps a window of pending tokens ``S_c`` and, per model, the distributions that model
has already computed for the leading positions of that window (the paper's caches ``C_i``).  One
iteration of the loop is one invocation of one model per sequence:

* empty window: the default proposer (model 0) drafts ``gamma_0`` tokens;
* otherwise the model with the fewest cached distributions scores the pending tokens it has not seen,
  which also yields its own next-token distribution, from which it draws a bonus token that joins the
  window as its proposal; every leading token that all models have now scored is verified against the
  combined distribution r (one ``cos_verify`` call with ``num_drafts`` = that count, ``proposer_pos`` =
  who proposed each token, ``no_bonus``); accepted tokens leave the window, a rejection replaces the
  token by a draw from the residual and clears the window and the caches; the model then drafts
  ``gamma_i - 1`` more tokens (skipped after a rejection: the text of Sec. 3.4 restarts from the default
  proposer then, while the printed listing would let the model draft onto the empty window).

The cache of logits rows is laid out ``[n][B][L][V]`` — exactly the layout ``cos_verify`` reads — so a
verification call takes the cache itself as its logits argument and copies nothing; positions no model
has filled yet hold NaN and are never read.  All random numbers come from one seeded host generator in
fixed-size blocks per iteration, so two runs with different ``verify`` back ends (the GPU library, or a
reference implementation in a test) can be compared token for token.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Callable, List, Sequence

import torch

from .apf import first_argmax, sample_from_logits


@dataclass
class SchedulerStats:
    iterations: int = 0
    model_calls: List[int] = field(default_factory=list)   # forward passes per model (a scoring pass counts once)
    verified: int = 0          # tokens put to the acceptance test
    accepted: int = 0
    rejections: int = 0
    tokens_out: int = 0
    max_window: int = 0        # longest pending window seen

    def modelled_speedup(self, costs: Sequence[float]) -> float:
        """Plain collaboration pays every model once per token (Sec. 3.2's cost model, verification
        free); this run paid ``model_calls``."""
        spent = sum(c * k for c, k in zip(costs, self.model_calls))
        return self.tokens_out * sum(costs) / spent if spent else float("nan")


def collaborative_speculation_decode(lm, prefix: torch.Tensor, iterations: int, gammas: Sequence[int],
                                     combine_mode: int, weights: Sequence[float], verify: Callable[..., tuple],
                                     seed: int = 0, temperature: float = 1.0, greedy: bool = False):
    """Run ``iterations`` model invocations per sequence of Alg. 2.

    lm       object with ``n_models``, ``V``, ``tables`` and ``logits_multi(models [R], contexts [R, 2])``
             (``apf.HashedBigramLM``); model 0 is the default proposer.
    prefix   [B, L0] int32, L0 >= 2, on the device of ``lm``.
    gammas   proposal length of every model (each >= 1).
    verify   callable with the signature of ``cos_verify.cos_verify``; it is called with the keyword
             arguments ``proposer_pos``, ``num_drafts``, ``no_bonus`` and ``temperature``.
    greedy   temperature 0: every model drafts its largest logit and ``verify`` is called with
             ``greedy=True`` instead of ``temperature`` (with ``proposer_pos`` only where the
             verification looks at the proposers: the ensemble).
    Returns (list of per-row token lists, SchedulerStats).
    """
    n = lm.n_models
    if len(gammas) != n or min(gammas) < 1:
        raise ValueError("one proposal length >= 1 per model")
    dev = prefix.device
    B, L0 = prefix.shape
    V = lm.V
    gmax = max(gammas)
    cap = 2 * sum(gammas) + 2                    # positions the cache holds; the window stays far below
    if cap - 1 > 31:
        raise ValueError("proposal lengths too long for one verification call")
    g_call = cap - 1                             # gamma of every verification call (static shapes)
    gam = torch.tensor(list(gammas), dtype=torch.int64, device=dev)
    gen = torch.Generator(device="cpu").manual_seed(seed)
    dtype = lm.tables[0].dtype
    rows = torch.arange(B, device=dev)

    seq = torch.zeros((B, L0 + iterations * (gmax + 1) + 2), dtype=torch.int32, device=dev)
    seq[:, :L0] = prefix
    seq_len = torch.full((B,), L0, dtype=torch.int64, device=dev)
    window = torch.zeros((B, cap), dtype=torch.int32, device=dev)         # S_c
    proposer = torch.zeros((B, cap), dtype=torch.int32, device=dev)       # who proposed each pending token
    win_len = torch.zeros((B,), dtype=torch.int64, device=dev)
    have = torch.zeros((B, n), dtype=torch.int64, device=dev)             # |C_i|
    cache = torch.full((n, B, cap, V), float("nan"), dtype=dtype, device=dev)
    stats = SchedulerStats(model_calls=[0] * n)

    def context_at(pos: torch.Tensor) -> torch.Tensor:
        """[B, 2]: the two tokens before pending position ``pos[b]`` (committed tokens, then the window)."""
        tail = seq[rows[:, None], (seq_len[:, None] + torch.tensor([-2, -1], device=dev)[None, :])]
        hist = torch.cat([tail, window], dim=1)                            # pending position p sits at p + 2
        return hist[rows[:, None], pos[:, None] + torch.tensor([0, 1], device=dev)[None, :]]

    def distributions(model: torch.Tensor, pos: torch.Tensor, active: torch.Tensor) -> torch.Tensor:
        """Logits rows of ``model[b]`` at pending position ``pos[b]``; cached for the active rows."""
        out = lm.logits_multi(model, context_at(pos))
        sel = active.nonzero(as_tuple=True)[0]
        cache[model[sel], sel, pos[sel]] = out[sel]
        return out

    def draft(model: torch.Tensor, count: torch.Tensor, u: torch.Tensor) -> None:
        """``count[b]`` tokens by ``model[b]``, one after the other (Eq. 1), appended to the window.
        (The caller does the accounting of forward passes.)"""
        for t in range(int(count.max()) if B else 0):
            active = count > t
            pos = torch.where(active, win_len, torch.zeros_like(win_len))
            if int(pos.max()) >= cap - 1:
                raise RuntimeError("pending window outgrew the cache")
            out = distributions(model, pos, active)
            tok = first_argmax(out) if greedy else sample_from_logits(out.float() / temperature, u[:, t])
            sel = active.nonzero(as_tuple=True)[0]
            window[sel, pos[sel]] = tok[sel]
            proposer[sel, pos[sel]] = model[sel].to(torch.int32)
            win_len[sel] += 1
            have[sel, model[sel]] = win_len[sel]

    for _ in range(iterations):
        u_draft = torch.rand((B, 2 * gmax), generator=gen, dtype=torch.float64)
        u_acc = torch.rand((B, g_call), generator=gen, dtype=torch.float64).to(dev)
        u_res = torch.rand((B,), generator=gen, dtype=torch.float64).to(dev)
        empty = win_len == 0
        # the model to invoke: the default proposer on an empty window, else the one furthest behind
        behind_most = torch.argmin(have * n + torch.arange(n, device=dev)[None, :], dim=1)   # ties: lowest index
        model = torch.where(empty, torch.zeros_like(win_len), behind_most)
        # ---- SCORE: the pending tokens this model has not seen (one forward pass, counted once below) ----
        behind = have[rows, model]
        for p in range(int(win_len.max()) if B else 0):
            active = (~empty) & (behind <= p) & (p < win_len)
            if bool(active.any()):
                distributions(model, torch.full_like(win_len, p), active)
        # ---- its own next token: gamma_0 drafts on an empty window, else the bonus token ----
        first = torch.where(empty, gam[model], torch.ones_like(win_len))
        draft(model, first, u_draft[:, :gmax])
        for m in range(n):          # scoring and the bonus token come out of one forward pass
            sel = model == m
            stats.model_calls[m] += int((sel & ~empty).sum()) + int(gammas[m] * (sel & empty).sum())
        stats.max_window = max(stats.max_window, int(win_len.max()) if B else 0)
        # ---- VERIFY every leading token that all models have scored ----
        K = have.min(dim=1).values
        how = {"temperature": temperature}
        if greedy:
            how = {"greedy": True}
        if not greedy or combine_mode == 0:              # at temperature 0 only the ensemble looks at the proposers
            how["proposer_pos"] = proposer[:, :g_call].contiguous()
        alen, toks = verify(cache, window[:, :g_call].contiguous(), torch.zeros(B, dtype=torch.int32, device=dev),
                            combine_mode, list(weights), u_acc, u_res, num_drafts=K.to(torch.int32),
                            no_bonus=True, **how)
        alen = alen.to(dev).to(torch.int64)
        toks = toks.to(dev)
        rejected = alen < K
        for j in range(int(alen.max()) if B else 0):          # accepted tokens join the sequence
            sel = (alen > j).nonzero(as_tuple=True)[0]
            seq[sel, seq_len[sel] + j] = window[sel, j]
        rsel = rejected.nonzero(as_tuple=True)[0]
        seq[rsel, seq_len[rsel] + alen[rsel]] = toks[rsel, alen[rsel]]      # the resampled token
        seq_len += alen + rejected.to(torch.int64)
        stats.verified += int(torch.minimum(alen + 1, K).sum())
        stats.accepted += int(alen.sum())
        stats.rejections += int(rejected.sum())
        stats.tokens_out += int((alen + rejected.to(torch.int64)).sum())
        # accepted tokens leave the window and the caches; a rejection clears both
        shift = torch.where(rejected, torch.zeros_like(K), K)
        idx = (torch.arange(cap, device=dev)[None, :] + shift[:, None]).clamp(max=cap - 1)
        window = window.gather(1, idx)
        proposer = proposer.gather(1, idx)
        cache = cache.gather(2, idx[None, :, :, None].expand(n, B, cap, V)).contiguous()
        win_len = torch.where(rejected, torch.zeros_like(win_len), win_len - K)
        have = torch.where(rejected[:, None], torch.zeros_like(have), have - K[:, None])
        # ---- PROPOSE: gamma_i - 1 more tokens, unless the window was just cleared or just started ----
        more = torch.where(empty | rejected, torch.zeros_like(win_len), gam[model] - 1)
        draft(model, more, u_draft[:, gmax:])
        for m in range(n):
            stats.model_calls[m] += int(more[model == m].sum())
        stats.max_window = max(stats.max_window, int(win_len.max()) if B else 0)
        stats.iterations += 1

    lens = seq_len.cpu().tolist()
    host = seq.cpu()
    return [host[b, :lens[b]].tolist() for b in range(B)], stats
