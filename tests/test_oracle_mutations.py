"""Do the oracle's pins catch a plausible mistake?  Each case below plants one mistake in a copy of the oracle's
C file -- a dropped term, a wrong sign, a transposed operand or index, a missing logarithm, an off-by-one --
compiles the copy on the CPU and runs the pin tests against it in a child process; the pins must fail.  The
unchanged copy must pass by the same route.  Nothing here touches a GPU or the HIP library.

The mistakes are planted in the oracle only; every substitution is checked to apply exactly as many times as
stated, so that an edit of the C file that moves a line makes the case fail loudly instead of going stale."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

_ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
_SRC = os.path.join(_ROOT, "oracle", "cos_oracle.c")
_PINS = ["tests/test_oracle_pins.py", "tests/test_oracle_extension_pins.py"]

# (name, passage the mistaken step follows, text, replacement, expected number of occurrences)
MUTANTS = [
    ("softmax_not_normalised", "Sec. 3.2 softmax",
     "for (x = 0; x < V; ++x) s[x] /= Z;", "(void)Z;", 1),
    ("softmax_max_skips_last", "Sec. 3.2 softmax",
     "  double M = l[0], Z = 0.0;\n  int x;\n  for (x = 1; x < V; ++x)",
     "  double M = l[0], Z = 0.0;\n  int x;\n  for (x = 1; x < V - 1; ++x)", 1),
    ("softmax_sum_skips_first", "Sec. 3.2 softmax",
     "  for (x = 0; x < V; ++x) {\n    s[x] = exp(l[x] - M);\n    Z += s[x];",
     "  for (x = 0; x < V; ++x) {\n    s[x] = exp(l[x] - M);\n    if (x) Z += s[x];", 1),
    ("ensemble_weights_reversed", "Eq. (4)",
     "acc += w[m] * s[(size_t)m * V + x];", "acc += w[n - 1 - m] * s[(size_t)m * V + x];", 1),
    ("ensemble_drops_last_model", "Eq. (4)",
     "for (m = 0; m < n; ++m) acc += w[m]", "for (m = 0; m + 1 < n || m == 0; ++m) acc += w[m]", 1),
    ("contrastive_sign_of_mu", "Eq. (5)",
     "double c = l_p[x] - mu * l_q[x];", "double c = l_p[x] + mu * l_q[x];", 3),
    ("contrastive_operands_swapped", "Eq. (5)",
     "double c = l_p[x] - mu * l_q[x];", "double c = l_q[x] - mu * l_p[x];", 3),
    ("contrastive_threshold_without_log", "plausibility mask",
     "thr = (alpha_cd > 0.0) ? log(alpha_cd) : -INFINITY;", "thr = (alpha_cd > 0.0) ? alpha_cd : -INFINITY;", 2),
    ("contrastive_mask_on_amateur", "plausibility mask",
     "(l_p[x] - Mp >= thr)", "(l_q[x] - Mp >= thr)", 3),
    ("contrastive_normaliser_over_all_tokens", "Eq. (5) on the mask",
     "    } else {\n      r[x] = 0.0;\n    }", "    } else {\n      r[x] = 0.0;\n      Zc += exp(l_p[x] - mu * l_q[x] - Mc);\n    }", 1),
    ("logit_mix_ignores_coefficients", "Eq. (3)",
     "      if (beta[m] != 0.0) c += beta[m] * l[(size_t)m * V + x];\n    r[x] = c;",
     "      if (beta[m] != 0.0) c += l[(size_t)m * V + x];\n    r[x] = c;", 1),
    ("accept_ratio_inverted", "Eq. (6)",
     "ratio = r_d / q_d;", "ratio = q_d / r_d;", 1),
    ("accept_not_strict", "Eq. (6), u < min(1, ratio)",
     "return u < bound;", "return u <= bound;", 1),
    ("accept_zero_q_rejects", "Eq. (6), q(d) = 0 < r(d)",
     "ratio = INFINITY;", "ratio = 0.0;", 1),
    ("residual_sign", "Sec. 3.2 residual max(0, r - q)",
     "double v = residual ? r[x] - q[x] : r[x];", "double v = residual ? q[x] - r[x] : r[x];", 1),
    ("residual_without_clamp", "Sec. 3.2 residual max(0, r - q)",
     "f[x] = v > 0.0 ? v : 0.0;", "f[x] = v > 0.0 ? v : -v;", 1),
    ("residual_never_used", "Sec. 3.2: after a rejection the draw is from the residual",
     "residual = jstar < gb;", "residual = 0;", 1),
    ("inverse_cdf_not_strict", "inverse CDF, first k with prefix > t",
     "if (cum > t) {", "if (cum >= t) {", 1),
    ("inverse_cdf_exclusive_prefix", "inverse CDF, inclusive prefix",
     "if (cum > t) {", "if (prev > t) {", 1),
    ("acceptance_rate_takes_max", "Eq. (7)",
     "a += q[x] < r[x] ? q[x] : r[x];", "a += q[x] < r[x] ? r[x] : q[x];", 1),
    ("temperature_multiplies", "Sec. 4.1 temperature",
     "l[x] = l[x] / T;", "l[x] = l[x] * T;", 1),
    ("proposer_ignored", "q is the proposer's softmax (Sec. 3.2)",
     "q = s + (size_t)pi * V;", "q = s;", 1),
    ("layout_batch_major", "logits are [model][sequence][position][token]",
     "size_t row = ((size_t)m * B + b) * (size_t)(gamma + 1) + j;",
     "size_t row = ((size_t)b * n + m) * (size_t)(gamma + 1) + j;", 2),
    ("scan_goes_on_after_a_rejection", "Sec. 3.2: stop at the first rejection",
     "if (acc) continue;    /* accepted", "if (!acc) continue;    /* accepted", 1),
    ("accepted_prefix_off_by_one", "the accepted drafts precede the drawn token",
     "          if (x < jstar)\n            *o = draft_tokens",
     "          if (x < jstar - 1)\n            *o = draft_tokens", 1),
    ("bonus_row_from_the_combination", "Sec. 3.1 / 3.3: the verifier's own extra token",
     "memcpy(r, s + (size_t)bonus_from * V, sizeof(double) * (size_t)V);",
     "cos_oracle_combine_ensemble(s, weights, n, V, r);", 1),
    ("bf16_read_as_low_half", "bfloat16 storage",
     "uint32_t bits = (uint32_t)h << 16;", "uint32_t bits = (uint32_t)h << 15;", 1),
    ("f16_exponent_bias", "binary16 storage",
     "v = ldexp((double)(1024 + frac), e - 25);", "v = ldexp((double)(1024 + frac), e - 24);", 1),
    ("greedy_softmax_ties_to_last", "temperature 0: ties to the lowest index",
     "    if (l[x] > l[arg]) arg = x;\n  for (x = 0; x < V; ++x) s[x] = 0.0;",
     "    if (l[x] >= l[arg]) arg = x;\n  for (x = 0; x < V; ++x) s[x] = 0.0;", 1),
    ("greedy_contrast_without_mask", "temperature 0 keeps the plausibility mask",
     "    if (in) {\n      double c = l_p[x] - mu * l_q[x];\n      if (arg < 0 || c > best) {",
     "    if (in || 1) {\n      double c = l_p[x] - mu * l_q[x];\n      if (arg < 0 || c > best) {", 1),
]


def _build(tmp, name, source):
    c = os.path.join(tmp, name + ".c")
    so = os.path.join(tmp, name + ".so")
    with open(c, "w") as fh:
        fh.write(source)
    subprocess.run(["gcc", "-std=c99", "-O1", "-w", "-fopenmp", "-shared", "-fPIC", "-o", so, c, "-lm"], check=True)
    return so


def _run_pins(library):
    env = dict(os.environ, COS_ORACLE_LIBRARY=library, OMP_NUM_THREADS="2")
    return subprocess.run([sys.executable, "-m", "pytest", *_PINS, "-x", "-q", "-p", "no:cacheprovider"],
                          cwd=_ROOT, env=env, capture_output=True, text=True, timeout=600)


def _first_failure(out):
    for line in out.splitlines():
        if line.startswith("FAILED "):
            return line[7:].split(" - ")[0]
    return "?"


def test_every_planted_mistake_fails_a_pin(tmp_path):
    source = open(_SRC).read()
    tmp = str(tmp_path)
    libs = []
    for name, _, text, repl, count in MUTANTS:
        assert source.count(text) == count, f"{name}: the oracle's text changed ({source.count(text)} != {count})"
        libs.append(_build(tmp, name, source.replace(text, repl)))
    control = _build(tmp, "unchanged", source)

    with ThreadPoolExecutor(max_workers=4) as pool:
        results = list(pool.map(_run_pins, libs + [control]))
    ok = results.pop()
    assert ok.returncode == 0, "the unchanged copy must pass its pins:\n" + ok.stdout[-2000:]

    survivors = []
    for (name, passage, *_), res in zip(MUTANTS, results):
        if res.returncode == 1:
            print(f"[mutation] {name:42s} ({passage}): caught by {_first_failure(res.stdout)}", flush=True)
        elif res.returncode == 0:
            survivors.append(name)
        else:   # a crash or a collection error is not a pin doing its work
            pytest.fail(f"{name}: pin run ended with {res.returncode}\n{res.stdout[-1500:]}\n{res.stderr[-1500:]}")
    assert not survivors, f"no pin notices: {survivors}"
