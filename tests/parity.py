"""GPU-vs-oracle comparison shared by the GPU tests, the smoke check and the benchmark.

Contract (decisions are integers decided by floating point, so near-ties are
excused, counted and reported; everything else must be bit-exact):

* accepted_len and out_tokens identical on every row that is not excused;
* a row is excused when the first differing accept decision has
  |u - ratio| < 1e-5 (oracle ratio), or when the lengths agree, the drawn token
  differs, the GPU's token has mass, and every boundary of the oracle's
  normalised CDF that separates the two tokens lies within 1e-6 of u_resample
  (the decision between them is then a CDF near-tie; tokens of mass below 1e-6
  may lie in between);
* r(d), q(d) agree to 1e-5 relative (absolute 1e-35 below 1e-30).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence

import numpy as np
import torch

from oracle import cos_oracle as O
from paper_2502_01662_amd import cos_verify as C
from paper_2502_01662_amd import workloads as W

RATIO_TIE = 1e-5
CDF_TIE = 1e-6
PROB_RTOL = 1e-5


@dataclass
class ParityReport:
    rows: int = 0
    exact_rows: int = 0
    excused_accept_ties: int = 0
    excused_cdf_ties: int = 0
    failures: List[str] = field(default_factory=list)
    max_rel_err_r: float = 0.0
    max_rel_err_q: float = 0.0
    flag_mismatches: int = 0

    @property
    def ok(self) -> bool:
        return not self.failures and self.flag_mismatches == 0

    def summary(self) -> Dict:
        return {"rows": self.rows, "exact_rows": self.exact_rows,
                "excused_accept_ties": self.excused_accept_ties,
                "excused_cdf_ties": self.excused_cdf_ties, "failures": len(self.failures),
                "max_rel_err_r": self.max_rel_err_r, "max_rel_err_q": self.max_rel_err_q,
                "flag_mismatches": self.flag_mismatches}


def oracle_dtype(logits: torch.Tensor) -> int:
    return {torch.float32: O.DTYPE_F32, torch.bfloat16: O.DTYPE_BF16, torch.float16: O.DTYPE_F16}[logits.dtype]


def _gpu_ext(inp):
    """Extensions of the step carried in the input dict (all optional)."""
    return {"temperature": float(inp.get("temperature", 1.0)), "bonus_idx": inp.get("bonus_idx"),
            "proposer_pos": inp.get("proposer_pos"), "stop_window": int(inp.get("stop_window", 0)),
            "num_drafts": inp.get("num_drafts"), "no_bonus": bool(inp.get("no_bonus", False)),
            "shape": inp.get("shape")}


def run_gpu(inp: Dict[str, torch.Tensor], mode: int, weights: Sequence[float], with_diag: bool = True):
    B, gamma = inp["draft_tokens"].shape
    diag = C.Diagnostics.allocate(B, gamma, inp["logits"].device) if with_diag else None
    alen, toks = C.cos_verify(inp["logits"], inp["draft_tokens"], inp["proposer_idx"], mode, weights,
                              inp["u_accept"], inp["u_resample"], diag=diag, **_gpu_ext(inp))
    torch.cuda.synchronize()
    return alen.cpu().numpy(), toks.cpu().numpy(), diag


def run_oracle(inp: Dict[str, torch.Tensor], mode: int, weights: Sequence[float],
               rows: Optional[Sequence[int]] = None, all_positions: bool = True, num_threads: int = 0):
    """Oracle on all batch rows, or on the subset ``rows`` (copied to the host first)."""
    logits = inp["logits"]
    sel = slice(None) if rows is None else torch.as_tensor(list(rows), device=logits.device)
    lg = logits[:, sel].contiguous()
    bonus = inp.get("bonus_idx")
    ppos = inp.get("proposer_pos")
    nd = inp.get("num_drafts")
    return lg, O.verify(W.host_logits(lg), oracle_dtype(lg), inp["draft_tokens"][sel].cpu().numpy(),
                        inp["proposer_idx"][sel].cpu().numpy(), mode, list(weights),
                        inp["u_accept"][sel].cpu().numpy(), inp["u_resample"][sel].cpu().numpy(),
                        all_positions=all_positions, num_threads=num_threads,
                        temperature=float(inp.get("temperature", 1.0)),
                        bonus_idx=None if bonus is None else bonus[sel].cpu().numpy(),
                        proposer_pos=None if ppos is None else ppos[sel].cpu().numpy(),
                        num_drafts=None if nd is None else nd[sel].cpu().numpy(),
                        no_bonus=bool(inp.get("no_bonus", False)))


def _rel_err(got: np.ndarray, want: np.ndarray) -> float:
    big = want >= 1e-30
    err = 0.0
    if big.any():
        err = float(np.max(np.abs(got[big] - want[big]) / want[big]))
    if (~big).any() and float(np.max(np.abs(got[~big] - want[~big]))) > 1e-35:
        err = max(err, 1.0)
    return err


def _sample_weights_of_row(host_lg, dtype, b, j, pi, mode, weights, residual, temperature=1.0, bonus=-1):
    n = host_lg.shape[0]
    l = [O.apply_temperature(O.row_to_f64(host_lg[m, b, j], dtype), temperature) for m in range(n)]
    if bonus >= 0 and not residual:
        s_v = O.softmax(l[bonus])
        return s_v, float(s_v.sum())
    s = np.stack([O.softmax(x) for x in l])
    if mode == O.ENSEMBLE:
        r = O.combine_ensemble(s, np.asarray(weights, dtype=np.float64))
    elif mode == O.LOGIT_MIX:
        r = O.combine_logit_mix(np.stack(l), np.asarray(weights, dtype=np.float64))
    else:
        r, _ = O.combine_contrastive(l[0], l[1], weights[0], weights[1])
    return O.sample_weights(r, s[pi], residual)


def compare(inp: Dict[str, torch.Tensor], mode: int, weights: Sequence[float], gpu_alen: np.ndarray,
            gpu_toks: np.ndarray, diag, rows: Optional[Sequence[int]] = None,
            num_threads: int = 0) -> ParityReport:
    """Compare GPU outputs with the oracle (on the batch rows ``rows``, default all)."""
    rep = ParityReport()
    lg, ora = run_oracle(inp, mode, weights, rows=rows, num_threads=num_threads)
    assert ora.status == 0, ora.status
    idx = np.arange(gpu_alen.shape[0]) if rows is None else np.asarray(list(rows))
    g_alen, g_toks = gpu_alen[idx], gpu_toks[idx]
    u_acc = inp["u_accept"].cpu().numpy()[idx]
    u_res = inp["u_resample"].cpu().numpy()[idx]
    prop = inp["proposer_idx"].cpu().numpy()[idx]
    ppos = None if inp.get("proposer_pos") is None else inp["proposer_pos"].cpu().numpy()[idx]
    bonus = None if inp.get("bonus_idx") is None else inp["bonus_idx"].cpu().numpy()[idx]
    gamma = u_acc.shape[1]
    # drafts per row: the row's bonus position takes the role of position gamma
    ndr = np.full(len(idx), gamma) if inp.get("num_drafts") is None else inp["num_drafts"].cpu().numpy()[idx]
    host_lg = None
    rep.rows = len(idx)
    if diag is not None:
        gr = diag.r_at_draft.cpu().numpy()[idx]
        gq = diag.q_at_draft.cpu().numpy()[idx]
        want_r, want_q = ora.r_at_draft, ora.q_at_draft
        has_draft = np.arange(gamma)[None, :] < ndr[:, None]
        read = np.ones_like(has_draft)
        w = int(inp.get("stop_window", 0))
        if 0 < w <= gamma:
            # only the windows up to the one holding the first rejection are read (and written)
            read = np.arange(gamma)[None, :] < ((np.minimum(g_alen, ora.accepted_len) // w + 1) * w)[:, None]
        if not (np.isnan(gr[read & ~has_draft]).all() and np.isnan(gq[read & ~has_draft]).all()):
            rep.failures.append("r(d) / q(d) of a position without a draft is not NaN")
        has_draft &= read
        gr, gq, want_r, want_q = gr[has_draft], gq[has_draft], want_r[has_draft], want_q[has_draft]
        rep.max_rel_err_r = _rel_err(gr, want_r)
        rep.max_rel_err_q = _rel_err(gq, want_q)
        if rep.max_rel_err_r > PROB_RTOL:
            rep.failures.append(f"r(d) relative error {rep.max_rel_err_r:.3e} > {PROB_RTOL}")
        if rep.max_rel_err_q > PROB_RTOL:
            rep.failures.append(f"q(d) relative error {rep.max_rel_err_q:.3e} > {PROB_RTOL}")
        gflags = diag.flags.cpu().numpy()[idx]
    for i in range(len(idx)):
        if g_alen[i] == ora.accepted_len[i] and np.array_equal(g_toks[i], ora.out_tokens[i]):
            rep.exact_rows += 1
            if diag is not None and (gflags[i] & 1) != (ora.flags[i] & 1):
                rep.flag_mismatches += 1
            continue
        where = f"row {idx[i]}: gpu len {g_alen[i]} tokens {g_toks[i].tolist()} vs oracle len " \
                f"{ora.accepted_len[i]} tokens {ora.out_tokens[i].tolist()}"
        if g_alen[i] != ora.accepted_len[i]:
            j = int(min(g_alen[i], ora.accepted_len[i]))       # first differing decision
            ratio = ora.ratio[i, j]
            if j < ndr[i] and abs(u_acc[i, j] - min(1.0, ratio)) < RATIO_TIE and \
                    np.array_equal(g_toks[i, :j], ora.out_tokens[i, :j]):
                rep.excused_accept_ties += 1
            else:
                rep.failures.append(where + f" (u={u_acc[i, j] if j < ndr[i] else None}, ratio={ratio})")
            continue
        j = int(ora.accepted_len[i])
        if not np.array_equal(np.delete(g_toks[i], j), np.delete(ora.out_tokens[i], j)):
            rep.failures.append(where + " (prefix or padding differs)")
            continue
        edge = min(abs(u_res[i] - ora.cdf_lo[i]), abs(u_res[i] - ora.cdf_hi[i]))
        if edge >= CDF_TIE:
            rep.failures.append(where + f" (u_resample {u_res[i]} is {edge:.3e} from the CDF edge)")
            continue
        if host_lg is None:
            host_lg = W.host_logits(lg)
        residual = j < ndr[i] and not (ora.flags[i] & O.FLAG_RESIDUAL_FALLBACK)
        pi = int(prop[i]) if (ppos is None or j >= ndr[i]) else int(ppos[i, j])
        f, F = _sample_weights_of_row(host_lg, oracle_dtype(lg), i, j, pi, mode, weights, residual,
                                      float(inp.get("temperature", 1.0)),
                                      -1 if bonus is None else int(bonus[i]))
        g, k = int(g_toks[i, j]), int(ora.out_tokens[i, j])
        # the boundary furthest from u among those between the two tokens: the lower edge of the GPU's
        # token if it lies above the oracle's, its upper edge if below (prefix sums in index order)
        far = float(np.sum(f[:g]) / F) if g > k else float(np.sum(f[:g + 1]) / F)
        if 0 <= g < len(f) and f[g] > 0 and abs(far - u_res[i]) < CDF_TIE:
            rep.excused_cdf_ties += 1
        else:
            rep.failures.append(where + f" (the CDF boundary at the GPU's token is {abs(far - u_res[i]):.3e} from "
                                        f"u_resample, or that token has no mass)")
    return rep


def check_workload(w: W.Workload, device: str = "cuda", step: int = 0, rows: Optional[Sequence[int]] = None,
                   inp: Optional[Dict[str, torch.Tensor]] = None) -> ParityReport:
    if inp is None:
        inp = W.generate(w, device=device, step=step)
    alen, toks, diag = run_gpu(inp, w.mode, w.weights)
    return compare(inp, w.mode, w.weights, alen, toks, diag, rows=rows)
