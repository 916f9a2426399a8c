"""Seeded synthetic inputs for the CoS verification step.

This module only draws random numbers: it holds none of the arithmetic of the
verification step (no softmax, no combine, no acceptance test, no CDF), so the
GPU library and the CPU oracle can both be fed from it without sharing code.

The five workloads stand in for the paper's model pairs (Sec. 4.1, Table 1):
only the vocabulary sizes (32000, 128256, 152064, and a 256000 one), the
proposal lengths and the combine settings are taken over; logits are seeded
Gaussian / Zipf-shaped tensors because neither the datasets nor the weights
are available.  Draft tokens follow Eq. (1): each is a draw from the row's
proposer distribution, obtained with the Gumbel-max identity
(argmax_x l(x) - ln(-ln U_x) is a sample of softmax(l)), which needs no
normalisation.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, Optional, Tuple

import torch

ENSEMBLE = 0
CONTRASTIVE = 1


@dataclass(frozen=True)
class Workload:
    name: str
    n: int
    B: int
    gamma: int
    V: int
    dtype: str                    # "f32" | "bf16"
    mode: int                     # ENSEMBLE | CONTRASTIVE
    weights: Tuple[float, ...]    # ensemble: w_m ; contrastive: (mu, alpha_cd)
    recipe: str                   # "noisy_copy" | "scaled_copy" | "shared_base" | "zipf"
    base_std: float
    noise_std: float
    scale: float = 1.0            # scaled_copy: l_1 = scale * l_0 + noise
    proposer: str = "mod"         # "mod" (b mod n) | "const:<k>" | "uniform" | "step" (set by caller)
    seed: int = 20250201

    @property
    def rows(self) -> int:
        return self.n * self.B * (self.gamma + 1)

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == "f32" else 2

    @property
    def logit_bytes(self) -> int:
        """Algorithmic bytes of one call: every logit once."""
        return self.rows * self.V * self.elem_bytes

    @property
    def positions(self) -> int:
        """Verified (draft) positions per call."""
        return self.B * self.gamma

    def scaled(self, **kw) -> "Workload":
        return replace(self, **kw)


# The five configurations, in the order the baseline file lists them.
C1 = Workload("c1_ens2_b1_g5_v32000_f32", 2, 1, 5, 32000, "f32", ENSEMBLE, (0.5, 0.5),
              "noisy_copy", 2.5, 1.0, proposer="step", seed=20250201)
C2 = Workload("c2_cd_b16_g5_v128256_bf16", 2, 16, 5, 128256, "bf16", CONTRASTIVE, (0.5, 0.1),
              "scaled_copy", 3.0, 1.5, scale=0.7, proposer="const:1", seed=20250202)
C3 = Workload("c3_ens3_b64_g4_v152064_bf16", 3, 64, 4, 152064, "bf16", ENSEMBLE, (0.5, 0.3, 0.2),
              "shared_base", 2.5, 1.0, proposer="mod", seed=20250203)
C4 = Workload("c4_ens2_b256_g8_v128256_bf16_zipf", 2, 256, 8, 128256, "bf16", ENSEMBLE, (0.6, 0.4),
              "zipf", 0.5, 0.8, proposer="mod", seed=20250204)
C5 = Workload("c5_ens4_b512_g6_v256000_bf16", 4, 512, 6, 256000, "bf16", ENSEMBLE,
              (0.25, 0.25, 0.25, 0.25), "shared_base", 3.0, 1.2, proposer="uniform", seed=20250205)

WORKLOADS: Dict[str, Workload] = {"c1": C1, "c2": C2, "c3": C3, "c4": C4, "c5": C5}


def _normal(shape, std, gen, device):
    return torch.randn(shape, generator=gen, device=device, dtype=torch.float64) * std


def _store(x64: torch.Tensor, dtype: str) -> torch.Tensor:
    """Round-to-nearest-even from float64 to the storage dtype."""
    return x64.to(torch.float32 if dtype == "f32" else torch.bfloat16)


def _logits(w: Workload, gen, device) -> torch.Tensor:
    n, B, g1, V = w.n, w.B, w.gamma + 1, w.V
    tdt = torch.float32 if w.dtype == "f32" else torch.bfloat16
    out = torch.empty((n, B, g1, V), dtype=tdt, device=device)
    # one batch row at a time keeps the float64 temporaries small
    for b in range(B):
        if w.recipe == "noisy_copy":          # l_0 ~ N(0, s^2); l_m = l_0 + N(0, t^2)
            base = _normal((g1, V), w.base_std, gen, device)
            out[0, b] = _store(base, w.dtype)
            for m in range(1, n):
                out[m, b] = _store(base + _normal((g1, V), w.noise_std, gen, device), w.dtype)
        elif w.recipe == "scaled_copy":       # l_0 ~ N(0, s^2); l_m = a l_0 + N(0, t^2)
            base = _normal((g1, V), w.base_std, gen, device)
            out[0, b] = _store(base, w.dtype)
            for m in range(1, n):
                out[m, b] = _store(w.scale * base + _normal((g1, V), w.noise_std, gen, device), w.dtype)
        elif w.recipe == "shared_base":       # l_m = base + N(0, t^2) for every m
            base = _normal((g1, V), w.base_std, gen, device)
            for m in range(n):
                out[m, b] = _store(base + _normal((g1, V), w.noise_std, gen, device), w.dtype)
        elif w.recipe == "zipf":              # l_0 = -1.1 ln(rank) + N(0, s^2) over a random permutation
            key = torch.rand((g1, V), generator=gen, device=device, dtype=torch.float64)
            rank = torch.argsort(torch.argsort(key, dim=1), dim=1).to(torch.float64) + 1.0
            base = -1.1 * torch.log(rank) + _normal((g1, V), w.base_std, gen, device)
            out[0, b] = _store(base, w.dtype)
            for m in range(1, n):
                out[m, b] = _store(base + _normal((g1, V), w.noise_std, gen, device), w.dtype)
        else:
            raise ValueError(w.recipe)
    return out


def _proposers(w: Workload, gen, device, step: int) -> torch.Tensor:
    if w.proposer == "mod":
        p = torch.arange(w.B, device=device) % w.n
    elif w.proposer.startswith("const:"):
        p = torch.full((w.B,), int(w.proposer.split(":")[1]), device=device)
    elif w.proposer == "uniform":
        p = torch.randint(0, w.n, (w.B,), generator=gen, device=device)
    elif w.proposer == "step":                # the proposer alternates from call to call
        p = torch.full((w.B,), step % w.n, device=device)
    else:
        raise ValueError(w.proposer)
    return p.to(torch.int32)


def _drafts(w: Workload, logits: torch.Tensor, proposer_idx: torch.Tensor, gen, device) -> torch.Tensor:
    """Eq. (1): d[b][j] ~ softmax(logits[proposer_idx[b], b, j, :]) by Gumbel-max."""
    B, gamma, V = w.B, w.gamma, w.V
    out = torch.empty((B, gamma), dtype=torch.int32, device=device)
    tiny = torch.finfo(torch.float64).tiny
    for b in range(B):
        rows = logits[int(proposer_idx[b]), b, :gamma, :].to(torch.float64)
        u = torch.rand((gamma, V), generator=gen, device=device, dtype=torch.float64).clamp_min(tiny)
        out[b] = torch.argmax(rows - torch.log(-torch.log(u)), dim=1).to(torch.int32)
    return out


def generate(w: Workload, device: str = "cpu", step: int = 0,
             seed: Optional[int] = None) -> Dict[str, torch.Tensor]:
    """All inputs of one ``cos_verify`` call, on ``device``, from one seed.

    ``step`` offsets the seed (fresh tensors per step) and drives the
    alternating proposer of ``proposer == "step"`` workloads.
    """
    gen = torch.Generator(device=device)
    gen.manual_seed((w.seed if seed is None else seed) + 1000003 * step)
    logits = _logits(w, gen, device)
    proposer_idx = _proposers(w, gen, device, step)
    draft_tokens = _drafts(w, logits, proposer_idx, gen, device)
    u_accept = torch.rand((w.B, w.gamma), generator=gen, device=device, dtype=torch.float64)
    u_resample = torch.rand((w.B,), generator=gen, device=device, dtype=torch.float64)
    return {"logits": logits, "draft_tokens": draft_tokens, "proposer_idx": proposer_idx,
            "u_accept": u_accept, "u_resample": u_resample}


def host_logits(logits: torch.Tensor):
    """Host view for the oracle: float32 array, or uint16 array of bf16 / float16 bits."""
    t = logits.detach().cpu().contiguous()
    if t.dtype in (torch.bfloat16, torch.float16):
        return t.view(torch.int16).numpy().view("uint16")
    return t.numpy()
