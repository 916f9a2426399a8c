"""Alternate Proposal Framework (Alg. 1, Sec. 3.3) as a host-side driver around ``cos_verify``.

Two models take turns: the proposer drafts ``gamma`` tokens, the verifier scores them in one pass,
``cos_verify`` accepts a prefix under the combined distribution r.  If every draft is accepted, the
verifier's own extra token (drawn from its distribution alone, ``bonus_idx``) is cached, the roles
swap, and the cached token becomes the first draft of the next cycle; after a rejection the cache is
cleared and the default proposer takes over.  Every token appended to a sequence follows r.

The driver is batched: every row keeps its own roles, which is why the verification step takes a
per-row ``proposer_idx``.  Models are anything with ``logits(model_index, contexts) -> [B, V]``; the
toy ``HashedBigramLM`` below stands in for real LLMs (none are available here).  All random numbers
come from one seeded host generator, so a run is reproducible and two runs with different ``verify``
back ends (the GPU library, or a reference implementation in a test) can be compared token by token.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Callable, List, Optional, Sequence

import torch


class HashedBigramLM:
    """Toy pair (or tuple) of correlated language models over a vocabulary of size V.

    logits_m(x | context) = base[h][x] + noise_m[h][x], h = hash of the last two tokens: the models
    share ``base`` (so they agree often, as a proposer and its verifier do) and differ by ``noise``.
    """

    def __init__(self, n_models: int, V: int, buckets: int, base_std: float = 2.0, noise_std: float = 1.0,
                 seed: int = 0, device: str = "cuda", dtype: torch.dtype = torch.bfloat16):
        g = torch.Generator(device="cpu").manual_seed(seed)
        self.V, self.buckets, self.n_models = V, buckets, n_models
        base = torch.randn((buckets, V), generator=g, dtype=torch.float64) * base_std
        self.tables = [(base + torch.randn((buckets, V), generator=g, dtype=torch.float64) * noise_std)
                       .to(dtype).to(device) for _ in range(n_models)]

    def bucket(self, contexts: torch.Tensor) -> torch.Tensor:
        a = contexts[:, -2].to(torch.int64)
        b = contexts[:, -1].to(torch.int64)
        return (a * 1000003 + b * 7919 + 12345) % self.buckets

    def logits(self, model: int, contexts: torch.Tensor) -> torch.Tensor:
        """[B, V] logits of ``model`` after ``contexts`` ([B, L], L >= 2)."""
        return self.tables[model][self.bucket(contexts)]

    def logits_multi(self, models: torch.Tensor, contexts: torch.Tensor) -> torch.Tensor:
        """[R, V]: logits of ``models[r]`` after ``contexts[r]`` (a different model per row)."""
        if getattr(self, "_stack", None) is None:
            self._stack = torch.stack(self.tables)
        return self._stack[models.to(torch.int64), self.bucket(contexts)]


def sample_from_logits(logits: torch.Tensor, u: torch.Tensor) -> torch.Tensor:
    """Eq. (1): one token per row from softmax(logits) by inverse CDF with the uniforms ``u``."""
    p = torch.softmax(logits.to(torch.float64), dim=-1)
    cdf = torch.cumsum(p, dim=-1)
    t = (u.to(cdf.device) * cdf[:, -1]).unsqueeze(1)
    return torch.searchsorted(cdf, t, right=True).squeeze(1).clamp_(max=logits.shape[1] - 1).to(torch.int32)


def first_argmax(logits: torch.Tensor) -> torch.Tensor:
    """Temperature 0: the index of each row's largest logit, the lowest one among equals."""
    top = logits.max(dim=-1, keepdim=True).values
    index = torch.arange(logits.shape[-1], device=logits.device).expand_as(logits)
    return torch.where(logits == top, index, logits.shape[-1]).min(dim=-1).values.to(torch.int32)


@dataclass
class APFStats:
    cycles: int = 0
    drafted: int = 0
    accepted: int = 0
    swapped_cycles: int = 0      # cycles that started from a cached bonus token
    tokens_out: int = 0


VerifyFn = Callable[..., tuple]


def alternate_proposal_decode(lm, prefix: torch.Tensor, cycles: int, gamma: int, combine_mode: int,
                              weights: Sequence[float], verify: VerifyFn, seed: int = 0,
                              default_proposer: int = 0, temperature: float = 1.0,
                              use_bonus: bool = True, greedy: bool = False):
    """Run ``cycles`` propose/score/verify cycles of Alg. 1 for a batch of sequences.

    prefix  [B, L0] int32 (L0 >= 2), on the device of ``lm``.
    verify  callable with the signature of ``cos_verify.cos_verify`` (keyword arguments
            ``bonus_idx`` and ``temperature`` included) returning (accepted_len, out_tokens).
    use_bonus = False gives Naive-CoS (Sec. 3.2): the verifier's extra token is discarded and the
            default proposer proposes every cycle.
    greedy  temperature 0 (the T = 0 runs of Sec. 4.1): the proposer drafts its largest logit and
            ``verify`` is called with ``greedy=True`` instead of ``temperature``.
    Returns (list of per-row token lists, APFStats).
    """
    dev = prefix.device
    B = prefix.shape[0]
    V = lm.V
    gen = torch.Generator(device="cpu").manual_seed(seed)
    seqs: List[List[int]] = [row.tolist() for row in prefix.cpu()]
    proposer = torch.full((B,), default_proposer, dtype=torch.int32)
    cache_tok = torch.full((B,), -1, dtype=torch.int32)          # C of Alg. 1 (-1 = empty)
    cache_row = torch.zeros((B, V), dtype=lm.tables[0].dtype, device=dev)   # its proposer-side logits
    stats = APFStats()
    nan = float("nan")

    def contexts(extra: Optional[torch.Tensor]) -> torch.Tensor:
        tail = torch.tensor([s[-2:] for s in seqs], dtype=torch.int32, device=dev)
        if extra is None or extra.shape[1] == 0:
            return tail
        return torch.cat([tail, extra], dim=1)[:, -2:]

    for _ in range(cycles):
        verifier = 1 - proposer
        p_dev, v_dev = proposer.to(dev), verifier.to(dev)
        has_cache = cache_tok >= 0
        stats.swapped_cycles += int(has_cache.sum())
        logits = torch.full((2, B, gamma + 1, V), nan, dtype=lm.tables[0].dtype, device=dev)
        drafts = torch.zeros((B, gamma), dtype=torch.int32, device=dev)
        rows = torch.arange(B, device=dev)
        # ---- PROPOSE: gamma tokens from the row's proposer (the cached bonus token first) ----
        for j in range(gamma):
            ctx = contexts(drafts[:, :j])
            both = torch.stack([lm.logits(0, ctx), lm.logits(1, ctx)])          # [2, B, V]
            prow = both[p_dev.long(), rows]
            u = torch.rand((B,), generator=gen, dtype=torch.float64)
            tok = first_argmax(prow) if greedy else sample_from_logits(prow.float() / temperature, u)
            if j == 0 and bool(has_cache.any()):
                hc = has_cache.to(dev)
                tok = torch.where(hc, cache_tok.to(dev), tok)
                prow = torch.where(hc[:, None], cache_row, prow)
            drafts[:, j] = tok
            logits[p_dev.long(), rows, j] = prow
            # ---- SCORE: the verifier's logits at the same position ----
            logits[v_dev.long(), rows, j] = both[v_dev.long(), rows]
        ctx = contexts(drafts)
        vrow = torch.stack([lm.logits(0, ctx), lm.logits(1, ctx)])[v_dev.long(), rows]
        logits[v_dev.long(), rows, gamma] = vrow      # the proposer has no logits here: left as NaN
        # ---- VERIFY ----
        u_acc = torch.rand((B, gamma), generator=gen, dtype=torch.float64).to(dev)
        u_res = torch.rand((B,), generator=gen, dtype=torch.float64).to(dev)
        how = {"greedy": True} if greedy else {"temperature": temperature}
        alen, toks = verify(logits, drafts, p_dev, combine_mode, list(weights), u_acc, u_res,
                            bonus_idx=v_dev.contiguous(), **how)
        alen_h, toks_h = alen.cpu(), toks.cpu()
        # ---- state update (Alg. 1) ----
        for b in range(B):
            a = int(alen_h[b])
            stats.drafted += gamma
            stats.accepted += a
            if a == gamma:                         # all accepted: cache the verifier's token, swap roles
                seqs[b].extend(toks_h[b, :gamma].tolist())
                stats.tokens_out += gamma
                if use_bonus:
                    cache_tok[b] = toks_h[b, gamma]
                    cache_row[b] = vrow[b]
                    proposer[b] = 1 - proposer[b]
                else:
                    cache_tok[b] = -1
            else:                                  # rejection: resampled token, default proposer again
                seqs[b].extend(toks_h[b, :a + 1].tolist())
                stats.tokens_out += a + 1
                cache_tok[b] = -1
                proposer[b] = default_proposer
        stats.cycles += 1
    return seqs, stats


def _demo() -> None:
    """Small end-to-end run on the GPU: APF against Naive-CoS, same seeds."""
    import time
    from . import cos_verify as C
    dev = "cuda"
    lm = HashedBigramLM(2, V=32000, buckets=512, seed=1, device=dev)
    prefix = torch.randint(0, 32000, (64, 4), dtype=torch.int32, device=dev)
    for use_bonus in (False, True):
        t0 = time.time()
        seqs, st = alternate_proposal_decode(lm, prefix, cycles=20, gamma=3, combine_mode=C.COS_COMBINE_ENSEMBLE,
                                             weights=[0.5, 0.5], verify=C.cos_verify, seed=7, use_bonus=use_bonus)
        torch.cuda.synchronize()
        print(f"{'alternate proposal' if use_bonus else 'naive CoS':>18}: {st.tokens_out} tokens in {st.cycles} cycles, "
              f"acceptance {st.accepted / st.drafted:.3f}, cycles started from a bonus token {st.swapped_cycles}, "
              f"{time.time() - t0:.2f} s")


if __name__ == "__main__":
    _demo()
