"""Seeded random sweep of shapes, dtypes, combine modes and extensions: GPU against the oracle."""
import numpy as np
import pytest
import torch

from paper_2502_01662_amd import cos_verify as C
from tests import parity as P
from tests.test_gpu_parity import _random_inputs

pytestmark = pytest.mark.gpu


def _case(seed):
    rng = np.random.default_rng(seed)
    contrastive = bool(rng.integers(0, 3) == 0)
    n = 2 if contrastive else int(rng.integers(1, 9))
    B = int(rng.integers(1, 17))
    gamma = int(rng.integers(1, 9))
    V = int(rng.choice([rng.integers(1, 600), rng.integers(600, 9000), 8 * rng.integers(64, 3000), rng.integers(9000, 60000)]))
    dtype = "bf16" if rng.integers(0, 2) else "f32"
    std = float(rng.choice([0.5, 1.5, 3.0]))
    inp = _random_inputs(n, B, gamma, V, dtype, seed=seed, std=std)
    if rng.integers(0, 4) == 0 and V > 4:                       # some tokens impossible under every model
        dead = torch.from_numpy(rng.integers(0, V, max(1, V // 7))).cuda()
        inp["logits"][..., dead] = float("-inf")
        alive = torch.from_numpy(np.setdiff1d(np.arange(V), dead.cpu().numpy())[:1]).cuda()
        inp["logits"][..., alive] = 1.0                         # at least one finite logit per row
    if contrastive:
        weights = [float(rng.choice([0.0, 0.1, 0.5, 1.0])), float(rng.choice([0.0, 0.05, 0.1, 0.5]))]
        mode = C.COS_COMBINE_CONTRASTIVE
        if rng.integers(0, 2):                                   # give acceptance a chance: drafts at the expert's argmax
            top = inp["logits"][0, :, :gamma].float().argmax(-1).to(torch.int32)
            keep = torch.from_numpy(rng.integers(0, 2, (B, gamma)).astype(bool)).cuda()
            inp["draft_tokens"] = torch.where(keep, top, inp["draft_tokens"]).contiguous()
    else:
        weights = rng.dirichlet(np.ones(n)).tolist()
        if rng.integers(0, 5) == 0:
            weights = [0.0] * n
            weights[int(rng.integers(0, n))] = 1.0
        mode = C.COS_COMBINE_ENSEMBLE
    if rng.integers(0, 2):
        inp["temperature"] = float(rng.choice([0.5, 0.8, 1.0, 1.7]))
    if rng.integers(0, 2):
        inp["proposer_pos"] = torch.from_numpy(rng.integers(0, n, (B, gamma)).astype(np.int32)).cuda()
    if rng.integers(0, 2):
        inp["bonus_idx"] = torch.from_numpy(rng.integers(-1, n, B).astype(np.int32)).cuda()
    if rng.integers(0, 2):
        inp["stop_window"] = int(rng.integers(1, gamma + 2))
    if rng.integers(0, 3) == 0:
        inp["u_accept"][rng.integers(0, B)] = 0.0
    if rng.integers(0, 3) == 0:                                  # rows with fewer drafts; what follows is never read
        nd = rng.integers(0, gamma + 1, B).astype(np.int32)
        inp["num_drafts"] = torch.from_numpy(nd).cuda()
        for b in range(B):
            inp["logits"][:, b, int(nd[b]) + 1:] = float("nan")
    if rng.integers(0, 4) == 0:
        inp["no_bonus"] = True
    return inp, mode, weights, dict(n=n, B=B, gamma=gamma, V=V, dtype=dtype, mode=mode,
                                    ext={k: (v if not torch.is_tensor(v) else "tensor") for k, v in inp.items()
                                         if k in ("temperature", "proposer_pos", "bonus_idx", "stop_window",
                                                  "num_drafts", "no_bonus")})


@pytest.mark.parametrize("seed", range(100))
def test_random_configuration(seed):
    inp, mode, weights, desc = _case(1000 + seed)
    alen, toks, diag = P.run_gpu(inp, mode, weights)
    rep = P.compare(inp, mode, weights, alen, toks, diag)
    print(f"[fuzz] {desc}: {rep.summary()}", flush=True)
    assert rep.ok, (desc, rep.failures[:3])
    assert rep.excused_accept_ties + rep.excused_cdf_ties <= 1, (desc, rep.summary())


@pytest.mark.parametrize("seed", range(50))
def test_random_logit_mix_configuration(seed):
    """The same random shapes and extensions with the logit-level linear combination (Eq. (3))."""
    inp, _, _, desc = _case(5000 + seed)
    rng = np.random.default_rng(9000 + seed)
    n = desc["n"]
    beta = rng.normal(0.0, 0.8, n)
    beta[rng.integers(0, n)] = float(rng.choice([1.0, 0.5, 1.5]))        # at least one clearly positive weight
    if n > 1 and rng.integers(0, 3) == 0:
        beta[rng.integers(0, n)] = 0.0                                   # a model that takes no part
    if torch.isinf(inp["logits"]).any():
        beta = np.abs(beta)                                              # -inf logits need non-negative weights
    if rng.integers(0, 2):                                               # drafts the mix likes, so that some are accepted
        c = sum(float(beta[m]) * inp["logits"][m, :, :desc["gamma"]].float() for m in range(n) if beta[m] != 0)
        keep = torch.from_numpy(rng.integers(0, 2, c.shape[:2]).astype(bool)).cuda()
        inp["draft_tokens"] = torch.where(keep, c.argmax(-1).to(torch.int32), inp["draft_tokens"]).contiguous()
    desc["mode"], desc["beta"] = C.COS_COMBINE_LOGIT_MIX, beta.round(3).tolist()
    alen, toks, diag = P.run_gpu(inp, C.COS_COMBINE_LOGIT_MIX, beta.tolist())
    rep = P.compare(inp, C.COS_COMBINE_LOGIT_MIX, beta.tolist(), alen, toks, diag)
    print(f"[fuzz] {desc}: {rep.summary()}", flush=True)
    assert rep.ok, (desc, rep.failures[:3])
    assert rep.excused_accept_ties + rep.excused_cdf_ties <= 1, (desc, rep.summary())


@pytest.mark.parametrize("seed", range(40))
def test_random_float16_configuration(seed):
    """The same random shapes, modes and extensions with IEEE binary16 logits."""
    inp, mode, weights, desc = _case(7000 + seed)
    inp["logits"] = inp["logits"].to(torch.float16)                # -inf and NaN poison survive the conversion
    desc["dtype"] = "f16"
    alen, toks, diag = P.run_gpu(inp, mode, weights)
    rep = P.compare(inp, mode, weights, alen, toks, diag)
    print(f"[fuzz] {desc}: {rep.summary()}", flush=True)
    assert rep.ok, (desc, rep.failures[:3])
    assert rep.excused_accept_ties + rep.excused_cdf_ties <= 1, (desc, rep.summary())


@pytest.mark.parametrize("seed", range(60))
def test_random_greedy_configuration(seed):
    """Temperature 0 on the same random shapes, every combine mode: bit-exact, nothing excused."""
    from oracle import cos_oracle as O
    from paper_2502_01662_amd import workloads as W
    inp, mode, weights, desc = _case(11000 + seed)
    rng = np.random.default_rng(12000 + seed)
    n, B, gamma, V = desc["n"], desc["B"], desc["gamma"], desc["V"]
    if mode == C.COS_COMBINE_ENSEMBLE and seed % 2:               # every other ensemble case: its shape for a logit mix
        mode = C.COS_COMBINE_LOGIT_MIX
        weights = rng.normal(0.0, 0.8, n)
        weights[rng.integers(0, n)] = 1.0
        if torch.isinf(inp["logits"]).any():
            weights = np.abs(weights)
        weights = weights.tolist()
    host, odt = W.host_logits(inp["logits"]), P.oracle_dtype(inp["logits"])
    drafts = inp["draft_tokens"].cpu().numpy().copy()
    ppos = inp.get("proposer_pos")
    prop = inp["proposer_idx"].cpu().numpy()
    for b in range(B):                                            # a likely prefix of random length
        for j in range(int(rng.integers(0, gamma + 1))):
            rows = [O.row_to_f64(host[m, b, j], odt) for m in range(n)]
            if np.isnan(rows[0]).any():
                break                                             # poisoned: beyond this row's drafts
            if mode == C.COS_COMBINE_CONTRASTIVE:
                drafts[b, j] = O.argmax_contrastive(rows[0], rows[1], weights[0], weights[1])
            elif mode == C.COS_COMBINE_LOGIT_MIX:
                drafts[b, j] = O.argmax_logit_mix(np.stack(rows), weights)
            else:                                                 # the proposer's own token, or another model's
                pi = int(prop[b]) if ppos is None else int(ppos[b, j])
                drafts[b, j] = int(np.argmax(rows[(pi + int(rng.integers(0, 2))) % n]))
    inp["draft_tokens"] = torch.from_numpy(drafts).cuda()
    nd, bonus = inp.get("num_drafts"), inp.get("bonus_idx")
    ens = mode == C.COS_COMBINE_ENSEMBLE
    alen, toks = C.cos_verify(inp["logits"], inp["draft_tokens"], inp["proposer_idx"], mode, weights, inp["u_accept"],
                              inp["u_resample"], greedy=True, bonus_idx=bonus, num_drafts=nd,
                              proposer_pos=ppos if ens else None, no_bonus=bool(inp.get("no_bonus", False)))
    torch.cuda.synchronize()
    opts = dict(bonus_idx=None if bonus is None else bonus.cpu().numpy(), num_drafts=None if nd is None else nd.cpu().numpy(),
                no_bonus=bool(inp.get("no_bonus", False)))
    if ens:
        ora = O.verify(host, odt, drafts, prop, mode, weights, inp["u_accept"].cpu().numpy(), inp["u_resample"].cpu().numpy(),
                       greedy=True, proposer_pos=None if ppos is None else ppos.cpu().numpy(), **opts)
        st, want_len, want_toks = ora.status, ora.accepted_len, ora.out_tokens
    else:
        st, want_len, want_toks = O.verify_greedy(host, odt, drafts, weights, mode=mode, **opts)
    desc["mode"] = mode
    print(f"[fuzz] greedy {desc}: accepted lengths {np.bincount(want_len, minlength=gamma + 1).tolist()}", flush=True)
    assert st == 0
    assert np.array_equal(alen.cpu().numpy(), want_len), desc
    assert np.array_equal(toks.cpu().numpy(), want_toks), desc


@pytest.mark.parametrize("seed", range(40))
def test_random_configuration_with_random_chunking(seed):
    """The same random cases with the launch shape drawn at random as well: chunk length, how many of the last
    sequences of the grid get how much shorter chunks, the route of the masked contrastive mode and who refines
    residuals of little mass.  Outputs must not depend on it."""
    inp, mode, weights, desc = _case(15000 + seed)
    rng = np.random.default_rng(16000 + seed)
    if mode == C.COS_COMBINE_ENSEMBLE and rng.integers(0, 2):
        mode, weights = C.COS_COMBINE_LOGIT_MIX, np.abs(rng.normal(0.5, 0.5, desc["n"])).tolist()
    knobs = (int(rng.choice([0, 256, 512, 1024, 2048])), int(rng.integers(0, desc["B"] + 2)), int(rng.choice([1, 2, 3, 4, 8, 16])),
             int(rng.integers(-1, 2)), int(rng.integers(-1, 2)))      # ... and the routes of a wide mask and of small residuals
    inp["shape"] = C.LaunchShape(chunk_vectors=knobs[0], tail_sequences=knobs[1] if knobs[1] else -1, tail_factor=knobs[2],
                                 two_pass_mask=knobs[3], refine_kernels=knobs[4])
    alen, toks, diag = P.run_gpu(inp, mode, weights)
    rep = P.compare(inp, mode, weights, alen, toks, diag)
    print(f"[fuzz] chunking {knobs} {desc}: {rep.summary()}", flush=True)
    assert rep.ok, (desc, knobs, rep.failures[:3])
    assert rep.excused_accept_ties + rep.excused_cdf_ties <= 1, (desc, rep.summary())


@pytest.mark.parametrize("seed", range(36))
def test_random_nearly_identical_models(seed):
    """The regime speculation is built for: models that nearly agree (noise 0.3, 0.03 or 0.003 on a shared
    base; acceptance rates of ~80 % up to above 99.9 %), with rejections forced at a random position so
    that residuals of little mass are drawn from.  Default path, no option: every row must be the
    reference's or an excused near-tie."""
    rng = np.random.default_rng(21000 + seed)
    noise = [0.3, 0.03, 0.003][seed % 3]
    mode = [C.COS_COMBINE_ENSEMBLE, C.COS_COMBINE_CONTRASTIVE, C.COS_COMBINE_LOGIT_MIX][(seed // 3) % 3]
    n = 2 if mode == C.COS_COMBINE_CONTRASTIVE else int(rng.integers(2, 6))
    B, gamma = int(rng.integers(8, 65)), int(rng.integers(1, 6))
    V = int(rng.choice([8 * rng.integers(500, 5000), rng.integers(3000, 50000)]))
    dtype = ["f32", "bf16", "f16"][int(rng.integers(0, 3))]
    tdt = {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}[dtype]
    g = torch.Generator().manual_seed(22000 + seed)
    base = torch.randn((B, gamma + 1, V), generator=g, dtype=torch.float64) * float(rng.choice([1.5, 2.5, 3.5]))
    logits = torch.stack([(base + torch.randn(base.shape, generator=g, dtype=torch.float64) * noise).to(tdt)
                          for _ in range(n)]).cuda()
    prop = torch.from_numpy(rng.integers(0, n, B).astype(np.int32)).cuda()
    # drafts: the proposer's favourite token, which a slightly flatter r rejects when u -> 1
    pl = logits[prop.long(), torch.arange(B, device="cuda")]                    # [B][gamma+1][V]
    drafts = pl[:, :gamma].float().argmax(-1).to(torch.int32).contiguous()
    u_acc = torch.rand((B, gamma), generator=g, dtype=torch.float64) * 0.5      # accepted when ratio >= 0.5 ...
    forced = torch.from_numpy(rng.integers(0, gamma + 1, B))                    # ... up to the forced position
    for b in range(B):
        if forced[b] < gamma:
            u_acc[b, forced[b]] = 1.0 - 1e-12
    inp = {"logits": logits, "draft_tokens": drafts, "proposer_idx": prop, "u_accept": u_acc.cuda(),
           "u_resample": torch.rand((B,), generator=g, dtype=torch.float64).cuda()}
    if mode == C.COS_COMBINE_ENSEMBLE:
        weights = rng.dirichlet(np.ones(n) * 3).tolist()
    elif mode == C.COS_COMBINE_CONTRASTIVE:
        weights = [float(rng.choice([0.0, 0.001, 0.01])), float(rng.choice([0.0, 1e-7, 1e-3]))]
    else:
        weights = rng.dirichlet(np.ones(n) * 3).tolist()                         # a logit-level average of the models
    route = int(rng.integers(-1, 2))      # the lone workgroup, by size, or the two refinement launches
    if route:
        inp["shape"] = C.LaunchShape(refine_kernels=route)
    desc = dict(noise=noise, mode=mode, n=n, B=B, gamma=gamma, V=V, dtype=dtype, weights=np.round(weights, 4).tolist(),
                refine_kernels=route)
    alen, toks, diag = P.run_gpu(inp, mode, weights)
    rep = P.compare(inp, mode, weights, alen, toks, diag)
    flags = diag.flags.cpu().numpy()
    mass = diag.sample_mass.cpu().numpy()
    print(f"[fuzz] nearly identical {desc}: {rep.summary()}, refined {int((flags & C.COS_FLAG_RESIDUAL_REFINED != 0).sum())}/{B}, "
          f"smallest residual mass {mass[alen < gamma].min() if (alen < gamma).any() else None}", flush=True)
    assert rep.ok, (desc, rep.failures[:3])
    assert rep.excused_accept_ties + rep.excused_cdf_ties <= 1, (desc, rep.summary())
