"""ctypes front end of the float64 CPU oracle (``cos_oracle.c``).

TEST INFRASTRUCTURE ONLY: the tests, the smoke check and the benchmark's
CPU-baseline leg may import this module; the product path never does.  The
module holds no arithmetic of its own: every number comes from the C file.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "cos_oracle.c")
_LIB = os.path.join(_HERE, "libcos_oracle.so")
# The mutation test of the pins (tests/test_oracle_mutations.py) points this at a library built from a
# deliberately wrong copy of the C file; such a library is loaded as it is, never rebuilt.
_OVERRIDE = os.environ.get("COS_ORACLE_LIBRARY")

DTYPE_F32 = 0
DTYPE_BF16 = 1
DTYPE_F16 = 2
ENSEMBLE = 0
CONTRASTIVE = 1
LOGIT_MIX = 2
FLAG_RESIDUAL_FALLBACK = 1
FLAG_TAIL_CLAMP = 2


def build(force: bool = True) -> str:
    """Compile the oracle with gcc (plain C99, OpenMP over batch rows)."""
    if _OVERRIDE:
        return _OVERRIDE
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-std=c99", "-O2", "-Wall", "-Wextra", "-fopenmp", "-shared", "-fPIC",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


class _Options(ctypes.Structure):
    _fields_ = [("temperature", ctypes.c_double), ("bonus_idx", ctypes.POINTER(ctypes.c_int32)),
                ("proposer_pos", ctypes.POINTER(ctypes.c_int32)), ("alpha", ctypes.POINTER(ctypes.c_double)),
                ("num_drafts", ctypes.POINTER(ctypes.c_int32)), ("no_bonus", ctypes.c_int), ("greedy", ctypes.c_int)]


_lib = None


def _load():
    global _lib
    if _lib is None:
        build(force=False)
        lib = ctypes.CDLL(_OVERRIDE or _LIB)
        dp = ctypes.POINTER(ctypes.c_double)
        ip = ctypes.POINTER(ctypes.c_int32)
        vp = ctypes.c_void_p
        ci = ctypes.c_int
        lib.cos_oracle_row_to_f64.argtypes = [vp, ci, ci, dp]
        lib.cos_oracle_row_to_f64.restype = None
        lib.cos_oracle_softmax_t0.argtypes = [dp, ci, dp]
        lib.cos_oracle_softmax_t0.restype = None
        lib.cos_oracle_softmax.argtypes = [dp, ci, dp]
        lib.cos_oracle_softmax.restype = None
        lib.cos_oracle_combine_ensemble.argtypes = [dp, dp, ci, ci, dp]
        lib.cos_oracle_combine_ensemble.restype = None
        lib.cos_oracle_combine_logit_mix.argtypes = [dp, dp, ci, ci, dp]
        lib.cos_oracle_combine_logit_mix.restype = None
        lib.cos_oracle_combine_contrastive.argtypes = [dp, dp, ctypes.c_double, ctypes.c_double, ci, dp]
        lib.cos_oracle_combine_contrastive.restype = ci
        lib.cos_oracle_accept.argtypes = [ctypes.c_double, ctypes.c_double, ctypes.c_double, dp]
        lib.cos_oracle_accept.restype = ci
        lib.cos_oracle_sample_weights.argtypes = [dp, dp, ci, ci, dp]
        lib.cos_oracle_sample_weights.restype = ctypes.c_double
        lib.cos_oracle_inverse_cdf.argtypes = [dp, ci, ctypes.c_double, ctypes.c_double,
                                               ctypes.POINTER(ci), dp, dp]
        lib.cos_oracle_inverse_cdf.restype = ci
        lib.cos_oracle_verify.argtypes = [vp, ci, ci, ci, ci, ci, ip, ip, ci, dp, dp, dp, ip, ip,
                                          dp, dp, dp, dp, dp, dp, ip, ci, ci]
        lib.cos_oracle_verify.restype = ci
        lib.cos_oracle_verify_ex.argtypes = lib.cos_oracle_verify.argtypes + [ctypes.POINTER(_Options)]
        lib.cos_oracle_verify_ex.restype = ci
        lib.cos_oracle_apply_temperature.argtypes = [dp, ci, ctypes.c_double]
        lib.cos_oracle_apply_temperature.restype = None
        lib.cos_oracle_acceptance_rate.argtypes = [dp, dp, ci]
        lib.cos_oracle_acceptance_rate.restype = ctypes.c_double
        lib.cos_oracle_argmax_contrastive.argtypes = [dp, dp, ctypes.c_double, ctypes.c_double, ci]
        lib.cos_oracle_argmax_contrastive.restype = ci
        lib.cos_oracle_argmax.argtypes = [dp, ci]
        lib.cos_oracle_argmax.restype = ci
        lib.cos_oracle_verify_greedy_mode.argtypes = [vp, ci, ci, ci, ci, ci, ip, ci, dp, ip, ip, ci, ip, ip, ci]
        lib.cos_oracle_verify_greedy_mode.restype = ci
        lib.cos_oracle_argmax_logit_mix.argtypes = [dp, dp, ci, ci]
        lib.cos_oracle_argmax_logit_mix.restype = ci
        lib.cos_oracle_max_threads.argtypes = []
        lib.cos_oracle_max_threads.restype = ci
        _lib = lib
    return _lib


def _dp(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _ip(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


# ---- step functions (one vocabulary row each) -----------------------------

def row_to_f64(row: np.ndarray, dtype: int) -> np.ndarray:
    """Widen one stored row (float32 array, or uint16 array of bf16 / binary16 bits)."""
    row = np.ascontiguousarray(row)
    assert row.dtype == (np.float32 if dtype == DTYPE_F32 else np.uint16)
    out = np.empty(row.shape[0], dtype=np.float64)
    _load().cos_oracle_row_to_f64(row.ctypes.data_as(ctypes.c_void_p), dtype, row.shape[0], _dp(out))
    return out


def apply_temperature(l, T: float) -> np.ndarray:
    out = _f64(l).copy()
    _load().cos_oracle_apply_temperature(_dp(out), out.shape[0], T)
    return out


def acceptance_rate(q, r) -> float:
    q = _f64(q)
    r = _f64(r)
    return _load().cos_oracle_acceptance_rate(_dp(q), _dp(r), q.shape[0])


def softmax(l) -> np.ndarray:
    l = _f64(l)
    s = np.empty_like(l)
    _load().cos_oracle_softmax(_dp(l), l.shape[0], _dp(s))
    return s


def softmax_t0(l) -> np.ndarray:
    """softmax(l / T) for T -> 0: one-hot at the largest entry (ties to the lowest index)."""
    l = _f64(l)
    s = np.empty_like(l)
    _load().cos_oracle_softmax_t0(_dp(l), l.shape[0], _dp(s))
    return s


def combine_ensemble(s, w) -> np.ndarray:
    s = _f64(s)
    w = _f64(w)
    n, V = s.shape
    assert w.shape == (n,)
    r = np.empty(V, dtype=np.float64)
    _load().cos_oracle_combine_ensemble(_dp(s), _dp(w), n, V, _dp(r))
    return r


def combine_contrastive(l_p, l_q, mu: float, alpha_cd: float):
    l_p = _f64(l_p)
    l_q = _f64(l_q)
    V = l_p.shape[0]
    r = np.empty(V, dtype=np.float64)
    count = _load().cos_oracle_combine_contrastive(_dp(l_p), _dp(l_q), mu, alpha_cd, V, _dp(r))
    return r, count


def accept(u: float, r_d: float, q_d: float):
    ratio = ctypes.c_double()
    acc = _load().cos_oracle_accept(u, r_d, q_d, ctypes.byref(ratio))
    return bool(acc), ratio.value


def sample_weights(r, q, residual: bool):
    r = _f64(r)
    q = _f64(q)
    f = np.empty_like(r)
    F = _load().cos_oracle_sample_weights(_dp(r), _dp(q), r.shape[0], int(residual), _dp(f))
    return f, F


def inverse_cdf(f, F: float, u: float):
    f = _f64(f)
    clamped = ctypes.c_int()
    lo = ctypes.c_double()
    hi = ctypes.c_double()
    tok = _load().cos_oracle_inverse_cdf(_dp(f), f.shape[0], F, u, ctypes.byref(clamped),
                                         ctypes.byref(lo), ctypes.byref(hi))
    return tok, bool(clamped.value), lo.value, hi.value


# ---- the whole step --------------------------------------------------------

@dataclass
class OracleResult:
    status: int
    accepted_len: np.ndarray      # [B] int32
    out_tokens: np.ndarray        # [B][gamma+1] int32
    r_at_draft: np.ndarray        # [B][gamma] float64 (NaN where never reached)
    q_at_draft: np.ndarray
    ratio: np.ndarray
    sample_mass: np.ndarray       # [B]
    cdf_lo: np.ndarray            # [B]
    cdf_hi: np.ndarray            # [B]
    flags: np.ndarray             # [B] int32
    alpha: Optional[np.ndarray] = None   # [B][gamma] acceptance rates (Eq. 7), NaN where not evaluated


def verify(logits: np.ndarray, dtype: int, draft_tokens, proposer_idx, mode: int, weights,
           u_accept, u_resample, all_positions: bool = False, num_threads: int = 0,
           temperature: float = 1.0, bonus_idx=None, proposer_pos=None,
           want_alpha: bool = False, num_drafts=None, no_bonus: bool = False, greedy: bool = False) -> OracleResult:
    """Run ``cos_oracle_verify_ex`` (the base step when no extension is given).

    ``logits`` is a host array of shape [n][B][gamma+1][V]: float32, or uint16
    holding bf16 bit patterns.
    """
    logits = np.ascontiguousarray(logits)
    assert logits.ndim == 4
    assert logits.dtype == (np.float32 if dtype == DTYPE_F32 else np.uint16), logits.dtype   # 16-bit formats as raw bits
    n, B, g1, V = logits.shape
    gamma = g1 - 1
    draft_tokens = np.ascontiguousarray(draft_tokens, dtype=np.int32).reshape(B, gamma)
    proposer_idx = np.ascontiguousarray(proposer_idx, dtype=np.int32).reshape(B)
    weights = _f64(weights)
    u_accept = _f64(u_accept).reshape(B, gamma)
    u_resample = _f64(u_resample).reshape(B)
    res = OracleResult(
        status=0,
        accepted_len=np.full(B, -7, dtype=np.int32),
        out_tokens=np.full((B, gamma + 1), -7, dtype=np.int32),
        r_at_draft=np.empty((B, gamma)), q_at_draft=np.empty((B, gamma)), ratio=np.empty((B, gamma)),
        sample_mass=np.empty(B), cdf_lo=np.empty(B), cdf_hi=np.empty(B),
        flags=np.zeros(B, dtype=np.int32))
    opt = _Options()
    opt.temperature = float(temperature)
    keep = []
    if bonus_idx is not None:
        bi = np.ascontiguousarray(bonus_idx, dtype=np.int32).reshape(B)
        keep.append(bi)
        opt.bonus_idx = _ip(bi)
    if proposer_pos is not None:
        pp = np.ascontiguousarray(proposer_pos, dtype=np.int32).reshape(B, gamma)
        keep.append(pp)
        opt.proposer_pos = _ip(pp)
    if want_alpha:
        res.alpha = np.empty((B, gamma))
        opt.alpha = _dp(res.alpha)
    if num_drafts is not None:
        nd = np.ascontiguousarray(num_drafts, dtype=np.int32).reshape(B)
        keep.append(nd)
        opt.num_drafts = _ip(nd)
    opt.no_bonus = int(bool(no_bonus))
    opt.greedy = int(bool(greedy))     # temperature 0, ensemble mode: every softmax one-hot at its largest logit
    res.status = _load().cos_oracle_verify_ex(
        logits.ctypes.data_as(ctypes.c_void_p), dtype, n, B, gamma, V,
        _ip(draft_tokens), _ip(proposer_idx), mode, _dp(weights), _dp(u_accept), _dp(u_resample),
        _ip(res.accepted_len), _ip(res.out_tokens), _dp(res.r_at_draft), _dp(res.q_at_draft),
        _dp(res.ratio), _dp(res.sample_mass), _dp(res.cdf_lo), _dp(res.cdf_hi), _ip(res.flags),
        int(all_positions), int(num_threads), ctypes.byref(opt))
    return res


def combine_logit_mix(l, beta):
    """l [n][V] logits, beta [n]: softmax of the linear combination of the logits."""
    l = _f64(l)
    beta = _f64(beta)
    n, V = l.shape
    assert beta.shape == (n,)
    r = np.empty(V)
    _load().cos_oracle_combine_logit_mix(_dp(l), _dp(beta), n, V, _dp(r))
    return r


def argmax_contrastive(l_p, l_q, mu: float, alpha_cd: float) -> int:
    l_p = _f64(l_p)
    l_q = _f64(l_q)
    return _load().cos_oracle_argmax_contrastive(_dp(l_p), _dp(l_q), mu, alpha_cd, l_p.shape[0])


def argmax_logit_mix(l, beta) -> int:
    """Temperature 0 of the logit mix: index of the largest sum_m beta_m l_m (ties to the lowest index)."""
    l = _f64(l)
    beta = _f64(beta)
    n, V = l.shape
    assert beta.shape == (n,)
    return _load().cos_oracle_argmax_logit_mix(_dp(l), _dp(beta), n, V)


def verify_greedy(logits: np.ndarray, dtype: int, draft_tokens, weights, bonus_idx=None, num_threads: int = 0,
                  num_drafts=None, no_bonus: bool = False, mode: int = CONTRASTIVE):
    """Temperature-0 step of a logit-level mode (contrastive, or logit mix); returns (status, accepted_len, out_tokens)."""
    logits = np.ascontiguousarray(logits)
    assert logits.ndim == 4
    assert logits.dtype == (np.float32 if dtype == DTYPE_F32 else np.uint16), logits.dtype   # 16-bit formats as raw bits
    n, B, g1, V = logits.shape
    gamma = g1 - 1
    draft_tokens = np.ascontiguousarray(draft_tokens, dtype=np.int32).reshape(B, gamma)
    weights = _f64(weights)
    assert weights.shape[0] >= (2 if mode == CONTRASTIVE else n)
    bi = None if bonus_idx is None else np.ascontiguousarray(bonus_idx, dtype=np.int32).reshape(B)
    nd = None if num_drafts is None else np.ascontiguousarray(num_drafts, dtype=np.int32).reshape(B)
    alen = np.full(B, -7, dtype=np.int32)
    toks = np.full((B, gamma + 1), -7, dtype=np.int32)
    st = _load().cos_oracle_verify_greedy_mode(logits.ctypes.data_as(ctypes.c_void_p), dtype, n, B, gamma, V,
                                               _ip(draft_tokens), int(mode), _dp(weights),
                                               _ip(bi) if bi is not None else None,
                                               _ip(nd) if nd is not None else None, int(bool(no_bonus)),
                                               _ip(alen), _ip(toks), int(num_threads))
    return st, alen, toks


def max_threads() -> int:
    return _load().cos_oracle_max_threads()
