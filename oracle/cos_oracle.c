/*
 * cos_oracle.c -- plain float64 CPU oracle for the CoS verification step.
 *
 * TEST INFRASTRUCTURE ONLY.  This file defines what the verification step of
 * "Collaborative decoding via Speculation" computes, written as slowly and as
 * plainly as possible so that it can be checked against the paper by eye.  It
 * shares no code, header, table or constant with the GPU library and must
 * never be imported, linked or called by the product path; only the tests,
 * the smoke check and the benchmark's CPU-baseline leg use it.
 *
 * What is computed (paper notation: q = proposer distribution, p = the other
 * models' distributions, r = combined distribution, gamma = proposal length):
 *
 *   softmax            Sec. 3.2 ("let l^q, l^p be the corresponding logits"),
 *                      temperature 1 as in the weighted-ensemble setup (Sec. 4.1)
 *   weighted ensemble  Eq. (4), extended to n models with one coefficient per
 *                      model as in the three-model run of Sec. 4.1 / Alg. 2
 *   contrastive        Eq. (5), r = Softmax(l^p - mu l^q); the plausibility
 *                      mask (keep x iff p(x) >= alpha_cd * max p) is NOT in the
 *                      paper's Eq. (5): it is this build's reading, and
 *                      alpha_cd = 0 gives Eq. (5) exactly
 *   acceptance test    Eq. (2) / Eq. (6): accept iff u < min(1, r(x)/q(x))
 *                      (strict '<' with u in [0,1): differs from the paper's
 *                      '<=' on a null set and never accepts a token with r = 0)
 *   first rejection    Sec. 3.1: the first rejected position discards the rest
 *   residual resample  Sec. 3.2 / App. A.1: norm(max(0, r - q))
 *   bonus token        Sec. 3.1: all gamma accepted -> one more token, here
 *                      drawn from r at position gamma (the caller supplies every
 *                      model's logits at all gamma+1 positions)
 *   token draw         inverse CDF in ascending token index: smallest k with
 *                      sum_{x<=k} f(x) > u*F  (the paper names only the
 *                      distribution; the procedure is this build's)
 *
 *   logit mix          r = softmax(sum_m beta_m l_m)  (Eq. (3), the logit-level
 *                      combination C'; decoding-time realignment of Sec. 2)
 *   extensions         cos_oracle_verify_ex: temperature (Sec. 4.1), the
 *                      verifier's own bonus token (Sec. 3.1 / 3.3), a proposer
 *                      per draft position (Alg. 2), the acceptance rate of Eq. (7),
 *                      a draft count per row and verification without an extra
 *                      token (Alg. 2's VERIFY)
 *
 * Everything is float64; sums run in ascending index order; nothing is
 * blocked, fused or reordered.
 *
 * Pins (tests/test_oracle_pins.py): independent library softmax, hand-derived
 * closed forms, the App. A.1 output law by exact enumeration and chi-square
 * Monte Carlo, r == q => all accepted, residual mass = 1 - sum min(q, r) =
 * (1/2) sum |r - q|, Thm 3.2 (alpha >= lambda), lambda = 0 => textbook
 * speculative sampling, P(accepted_len >= k) = prod alpha_j, E[#tokens] of
 * App. A.2, brute-force inverse CDF; extensions (tests/test_oracle_extension_pins.py):
 * scipy softmax of l/T and exactly pre-scaled logits, the bonus law s_v by
 * searchsorted and chi-square, an independent per-position re-derivation, the
 * hand value 13/16 and Eq. (7) for alpha, rows with fewer drafts and the
 * no-extra-token mode against the base step on the truncated tensor, the logit
 * mix by a hand example, library softmax and its special cases.  No
 * function here is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_DTYPE_F32 = 0, ORACLE_DTYPE_BF16 = 1, ORACLE_DTYPE_F16 = 2 };
enum { ORACLE_ENSEMBLE = 0, ORACLE_CONTRASTIVE = 1, ORACLE_LOGIT_MIX = 2 };
enum {
  ORACLE_OK = 0,
  ORACLE_ERR_NULL = -1,
  ORACLE_ERR_SHAPE = -2,
  ORACLE_ERR_DTYPE = -3,
  ORACLE_ERR_MODE = -4,
  ORACLE_ERR_WEIGHTS = -5,
  ORACLE_ERR_NOMEM = -10
};
enum { ORACLE_FLAG_RESIDUAL_FALLBACK = 1, ORACLE_FLAG_TAIL_CLAMP = 2 };

/* ---- storage formats -> float64 (exact) -------------------------------- */

/* bfloat16 is the upper half of an IEEE binary32: widening is exact. */
static double bf16_to_f64(uint16_t h) {
  uint32_t bits = (uint32_t)h << 16;
  float f;
  memcpy(&f, &bits, sizeof f);
  return (double)f;
}

/* IEEE binary16: 1 sign, 5 exponent (bias 15), 10 fraction bits.  Every value
 * is a small integer times a power of two, so the float64 below is exact. */
static double f16_to_f64(uint16_t h) {
  const int sign = h >> 15, e = (h >> 10) & 0x1f, frac = h & 0x3ff;
  double v;
  if (e == 0)
    v = ldexp((double)frac, -24); /* zero and subnormals: frac * 2^-24 */
  else if (e == 31)
    v = frac ? NAN : INFINITY;
  else
    v = ldexp((double)(1024 + frac), e - 25); /* (1 + frac/1024) * 2^(e-15) */
  return sign ? -v : v;
}

void cos_oracle_row_to_f64(const void *row, int dtype, int V, double *out) {
  int x;
  if (dtype == ORACLE_DTYPE_F32) {
    const float *p = (const float *)row;
    for (x = 0; x < V; ++x) out[x] = (double)p[x];
  } else if (dtype == ORACLE_DTYPE_F16) {
    const uint16_t *p = (const uint16_t *)row;
    for (x = 0; x < V; ++x) out[x] = f16_to_f64(p[x]);
  } else {
    const uint16_t *p = (const uint16_t *)row;
    for (x = 0; x < V; ++x) out[x] = bf16_to_f64(p[x]);
  }
}

/* ---- Sec. 4.1: temperature T > 0 divides the logits before every softmax -- */
/* (The paper runs T = 1 and T = 0; how T enters Eq. (5) is not stated: here it
 * divides both l^p and l^q, i.e. every logit, before anything else.)        */
void cos_oracle_apply_temperature(double *l, int V, double T) {
  int x;
  for (x = 0; x < V; ++x) l[x] = l[x] / T;
}

/* ---- Eq. (7) / App. A.1: acceptance rate alpha = sum_x min(q(x), r(x)) ---- */
double cos_oracle_acceptance_rate(const double *q, const double *r, int V) {
  double a = 0.0;
  int x;
  for (x = 0; x < V; ++x) a += q[x] < r[x] ? q[x] : r[x];
  return a;
}

/* ---- Sec. 3.2: s = softmax(l), temperature 1 --------------------------- */
/* M = max_x l(x); Z = sum_x exp(l(x) - M); s(x) = exp(l(x) - M) / Z.       */
void cos_oracle_softmax(const double *l, int V, double *s) {
  double M = l[0], Z = 0.0;
  int x;
  for (x = 1; x < V; ++x)
    if (l[x] > M) M = l[x];
  for (x = 0; x < V; ++x) {
    s[x] = exp(l[x] - M);
    Z += s[x];
  }
  for (x = 0; x < V; ++x) s[x] /= Z;
}

/* ---- the same at temperature 0 (Sec. 4.1 runs T = 0 and T = 1) ----------- */
/* softmax(l / T) for T -> 0: all mass on the largest entry, ties to the lowest
 * index.                                                                     */
void cos_oracle_softmax_t0(const double *l, int V, double *s) {
  int x, arg = 0;
  for (x = 1; x < V; ++x)
    if (l[x] > l[arg]) arg = x;
  for (x = 0; x < V; ++x) s[x] = 0.0;
  s[arg] = 1.0;
}

/* ---- Eq. (4), n models: r(x) = sum_m w_m s_m(x) ------------------------ */
/* s is [n][V] row-major.                                                   */
void cos_oracle_combine_ensemble(const double *s, const double *w, int n, int V,
                                 double *r) {
  int x, m;
  for (x = 0; x < V; ++x) {
    double acc = 0.0;
    for (m = 0; m < n; ++m) acc += w[m] * s[(size_t)m * V + x];
    r[x] = acc;
  }
}

/* ---- Eq. (5) with plausibility mask ------------------------------------ */
/* l_p = expert (target) logits, l_q = amateur logits.
 * mask = { x : l_p(x) - max l_p >= log(alpha_cd) }  (every finite x if
 * alpha_cd == 0); c(x) = l_p(x) - mu l_q(x);
 * r(x) = exp(c(x) - M_c) / Z_c on the mask, 0 elsewhere, M_c and Z_c over the
 * mask only.  A token whose expert logit is -inf has probability 0 under the
 * expert and is never in the mask.  Returns the mask size.                  */
int cos_oracle_combine_contrastive(const double *l_p, const double *l_q,
                                   double mu, double alpha_cd, int V,
                                   double *r) {
  double Mp = l_p[0], thr, Mc = -INFINITY, Zc = 0.0;
  int x, count = 0;
  for (x = 1; x < V; ++x)
    if (l_p[x] > Mp) Mp = l_p[x];
  thr = (alpha_cd > 0.0) ? log(alpha_cd) : -INFINITY;
  /* M_c over the mask */
  for (x = 0; x < V; ++x) {
    int in = (l_p[x] > -INFINITY) && (l_p[x] - Mp >= thr);
    if (in) {
      double c = l_p[x] - mu * l_q[x];
      if (c > Mc) Mc = c;
      ++count;
    }
  }
  /* exp(c - M_c) on the mask, 0 off it; Z_c in index order */
  for (x = 0; x < V; ++x) {
    int in = (l_p[x] > -INFINITY) && (l_p[x] - Mp >= thr);
    if (in) {
      double c = l_p[x] - mu * l_q[x];
      r[x] = exp(c - Mc);
      Zc += r[x];
    } else {
      r[x] = 0.0;
    }
  }
  for (x = 0; x < V; ++x) r[x] /= Zc;
  return count;
}

/* ---- Eq. (3), logit level: a linear combination of the models' logits ----- */
/* c(x) = sum_m beta_m l_m(x), r = softmax(c): the form of decoding-time
 * realignment (Sec. 2), of logit-level ensembles (beta_m = 1/n), and of Eq. (5)
 * without its mask (beta = (1, -mu)).  l is [n][V] row-major.  Models with
 * beta_m == 0 take no part (so their logits may be -inf).  c is summed in
 * model order.                                                              */
void cos_oracle_combine_logit_mix(const double *l, const double *beta, int n, int V,
                                  double *r) {
  int x, m;
  for (x = 0; x < V; ++x) {
    double c = 0.0;
    for (m = 0; m < n; ++m)
      if (beta[m] != 0.0) c += beta[m] * l[(size_t)m * V + x];
    r[x] = c; /* softmax in place below */
  }
  cos_oracle_softmax(r, V, r);
}

/* ---- temperature 0 (greedy decoding, the T = 0 runs of Sec. 4.1) ---------- */
/* As T -> 0 a softmax becomes one-hot at its largest entry, so r of Eq. (5)
 * is one-hot at argmax_x (l_p(x) - mu l_q(x)).  The plausibility mask is kept
 * as defined at temperature 1 (l_p(x) - max l_p >= log(alpha_cd)): at T -> 0 it
 * would shrink to the expert's argmax and the contrast would do nothing.  Ties
 * go to the lowest index.  Returns the index, or -1 if the mask is empty
 * (every expert logit -inf).                                                */
int cos_oracle_argmax_contrastive(const double *l_p, const double *l_q, double mu,
                                  double alpha_cd, int V) {
  double Mp = l_p[0], thr, best = -INFINITY;
  int x, arg = -1;
  for (x = 1; x < V; ++x)
    if (l_p[x] > Mp) Mp = l_p[x];
  thr = (alpha_cd > 0.0) ? log(alpha_cd) : -INFINITY;
  for (x = 0; x < V; ++x) {
    int in = (l_p[x] > -INFINITY) && (l_p[x] - Mp >= thr);
    if (in) {
      double c = l_p[x] - mu * l_q[x];
      if (arg < 0 || c > best) {
        best = c;
        arg = x;
      }
    }
  }
  return arg;
}

/* Temperature 0 of the logit-level linear combination (Eq. (3)): the softmax of
 * c(x) = sum_m beta_m l_m(x) becomes one-hot at the largest c(x), ties to the
 * lowest index.  c is summed exactly as cos_oracle_combine_logit_mix sums it
 * (model order, models with beta_m = 0 left out).  l is [n][V].              */
int cos_oracle_argmax_logit_mix(const double *l, const double *beta, int n, int V) {
  double best = -INFINITY;
  int x, m, arg = -1;
  for (x = 0; x < V; ++x) {
    double c = 0.0;
    for (m = 0; m < n; ++m)
      if (beta[m] != 0.0) c += beta[m] * l[(size_t)m * V + x];
    if (arg < 0 || c > best) {
      best = c;
      arg = x;
    }
  }
  return arg;
}

/* argmax of one row, ties to the lowest index */
int cos_oracle_argmax(const double *l, int V) {
  int x, arg = 0;
  for (x = 1; x < V; ++x)
    if (l[x] > l[arg]) arg = x;
  return arg;
}

/* ---- Eq. (6): accept iff u < min(1, r(d)/q(d)) ------------------------- */
/* q(d) = 0 and r(d) > 0 -> ratio = +inf (accept); r(d) = 0 -> ratio = 0
 * (reject, also when q(d) = 0).  Returns 1 = accept, writes the ratio.      */
int cos_oracle_accept(double u, double r_d, double q_d, double *ratio_out) {
  double ratio, bound;
  if (r_d <= 0.0)
    ratio = 0.0;
  else if (q_d <= 0.0)
    ratio = INFINITY;
  else
    ratio = r_d / q_d;
  if (ratio_out) *ratio_out = ratio;
  bound = ratio < 1.0 ? ratio : 1.0;
  return u < bound;
}

/* ---- Sec. 3.2 / App. A.1: unnormalised sampling weights ---------------- */
/* residual != 0: f = max(0, r - q) (a draft was rejected);
 * residual == 0: f = r (bonus token).  Returns F = sum_x f(x).              */
double cos_oracle_sample_weights(const double *r, const double *q, int V,
                                 int residual, double *f) {
  double F = 0.0;
  int x;
  for (x = 0; x < V; ++x) {
    double v = residual ? r[x] - q[x] : r[x];
    f[x] = v > 0.0 ? v : 0.0;
    F += f[x];
  }
  return F;
}

/* ---- inverse CDF -------------------------------------------------------- */
/* t = u F; token = smallest k with sum_{x<=k} f(x) > t.  If rounding leaves
 * no such k, the last x with f(x) > 0 is taken and *clamped is set.
 * cdf_lo / cdf_hi receive the normalised CDF just before / after the token. */
int cos_oracle_inverse_cdf(const double *f, int V, double F, double u,
                           int *clamped, double *cdf_lo, double *cdf_hi) {
  double t = u * F, cum = 0.0, prev = 0.0;
  int x, last_pos = -1;
  double last_lo = 0.0, last_hi = 0.0;
  if (clamped) *clamped = 0;
  for (x = 0; x < V; ++x) {
    prev = cum;
    cum += f[x];
    if (f[x] > 0.0) {
      last_pos = x;
      last_lo = prev;
      last_hi = cum;
    }
    if (cum > t) {
      if (cdf_lo) *cdf_lo = prev / F;
      if (cdf_hi) *cdf_hi = cum / F;
      return x;
    }
  }
  if (clamped) *clamped = 1;
  if (cdf_lo) *cdf_lo = last_lo / F;
  if (cdf_hi) *cdf_hi = last_hi / F;
  return last_pos;
}

/* ---- argument checks ----------------------------------------------------- */
static int check_weights(int mode, int n, const double *w) {
  int m;
  if (mode == ORACLE_ENSEMBLE) {
    double sum = 0.0;
    for (m = 0; m < n; ++m) {
      if (!(w[m] >= 0.0) || !isfinite(w[m])) return ORACLE_ERR_WEIGHTS;
      sum += w[m];
    }
    if (fabs(sum - 1.0) > 1e-9) return ORACLE_ERR_WEIGHTS;
    return ORACLE_OK;
  }
  if (mode == ORACLE_CONTRASTIVE) {
    if (n != 2) return ORACLE_ERR_MODE;
    if (!isfinite(w[0])) return ORACLE_ERR_WEIGHTS;
    if (!(w[1] >= 0.0 && w[1] <= 1.0)) return ORACLE_ERR_WEIGHTS;
    return ORACLE_OK;
  }
  if (mode == ORACLE_LOGIT_MIX) {
    for (m = 0; m < n; ++m)
      if (!isfinite(w[m])) return ORACLE_ERR_WEIGHTS;
    return ORACLE_OK;
  }
  return ORACLE_ERR_MODE;
}

/* ---- the whole verification step, one call per batch -------------------- */
/*
 * logits        host, [n][B][gamma+1][V] contiguous, dtype f32, bf16 or f16 (IEEE binary16)
 * draft_tokens  [B][gamma]   proposal tokens (Eq. 1), each in [0, V)
 * proposer_idx  [B]          which model's softmax is q for that row
 * mode/weights  ensemble: w[0..n-1];  contrastive (n == 2, model 0 = expert,
 *               model 1 = amateur): w[0] = mu, w[1] = alpha_cd;  logit mix:
 *               beta[0..n-1], any finite values
 * u_accept      [B][gamma]   uniforms in [0,1) for Eq. (6)
 * u_resample    [B]          one uniform in [0,1) for the residual or bonus draw
 * accepted_len  out [B]      number of accepted drafts, in [0, gamma]
 * out_tokens    out [B][gamma+1]: accepted drafts, then the sampled token,
 *               then -1 padding
 * Optional diagnostics (NULL = not wanted):
 *   r_at_draft, q_at_draft, ratio  [B][gamma]  (NaN for positions the
 *                                  sequential procedure never reached, unless
 *                                  all_positions != 0)
 *   sample_mass [B]  F of the sampled row;  cdf_lo / cdf_hi [B]  normalised
 *   CDF edges of the drawn token;  flags [B]  bit0 residual fallback, bit1
 *   tail clamp.
 * all_positions != 0 fills the [B][gamma] diagnostics for every position; the
 * decisions are unaffected.  num_threads <= 0 uses the OpenMP default; rows of
 * the batch are independent and each is processed sequentially by one thread,
 * so the result does not depend on the thread count.
 */
/*
 * Extensions beyond the base step (every member optional):
 *   temperature    T > 0 (0 or unset = 1): cos_oracle_apply_temperature on every row
 *   bonus_idx      [B] or NULL: when all gamma drafts are accepted, the extra
 *                  token is drawn from s_v, v = bonus_idx[b] >= 0 -- the
 *                  verifier's own distribution, as in Sec. 3.1 / 3.3, for which
 *                  the other models' logits at position gamma are not needed and
 *                  not read; -1 (or NULL) draws it from r at position gamma
 *   proposer_pos   [B][gamma] or NULL: the proposer of each draft position
 *                  (tokens of one window can come from different models, Alg. 2);
 *                  overrides proposer_idx
 *   alpha          out [B][gamma] or NULL: acceptance rate of every evaluated
 *                  position, Eq. (7) (NaN where never evaluated)
 *   num_drafts     [B] or NULL: row b carries only num_drafts[b] in [0, gamma]
 *                  drafts (rows of a batch, and the windows Alg. 2 verifies, differ
 *                  in length); position num_drafts[b] takes the role of position
 *                  gamma, later positions are never read, accepted_len[b] is in
 *                  [0, num_drafts[b]]
 *   no_bonus       != 0: when every draft of a row is accepted nothing is drawn
 *                  (Alg. 2's VERIFY only tests and resamples; Naive-CoS discards the
 *                  extra token): out_tokens[b][num_drafts[b]] = -1 and the logits of
 *                  that position are not read; sample_mass, cdf edges and flags of
 *                  such a row are 0
 *   greedy         != 0: temperature 0 for the ensemble of Eq. (4): every model's
 *                  softmax is one-hot at its largest logit (cos_oracle_softmax_t0),
 *                  so r = sum_m w_m e_{a_m} has at most n tokens and q = e_{a_pi};
 *                  every later step (Eq. (6), residual, inverse CDF) is unchanged and
 *                  still consumes the uniforms; `temperature` is not used.  Ensemble
 *                  mode only (the logit-level modes: cos_oracle_verify_greedy_mode)
 */
typedef struct cos_oracle_options {
  double temperature;
  const int32_t *bonus_idx;
  const int32_t *proposer_pos;
  double *alpha;
  const int32_t *num_drafts;
  int no_bonus;
  int greedy;
} cos_oracle_options;

int cos_oracle_verify_ex(const void *logits, int dtype, int n, int B, int gamma,
                         int V, const int32_t *draft_tokens,
                         const int32_t *proposer_idx, int mode,
                         const double *weights, const double *u_accept,
                         const double *u_resample, int32_t *accepted_len,
                         int32_t *out_tokens, double *r_at_draft,
                         double *q_at_draft, double *ratio, double *sample_mass,
                         double *cdf_lo, double *cdf_hi, int32_t *flags,
                         int all_positions, int num_threads,
                         const cos_oracle_options *opt) {
  int status, b, failed = 0;
  size_t esize;
  const double T = (opt && opt->temperature > 0.0) ? opt->temperature : 1.0;
  const int32_t *bonus_idx = opt ? opt->bonus_idx : NULL;
  const int32_t *proposer_pos = opt ? opt->proposer_pos : NULL;
  double *alpha = opt ? opt->alpha : NULL;
  const int32_t *num_drafts = opt ? opt->num_drafts : NULL;
  const int no_bonus = opt ? opt->no_bonus : 0;
  const int greedy = opt ? opt->greedy : 0;
  if (!logits || !draft_tokens || !proposer_idx || !weights || !u_accept ||
      !u_resample || !accepted_len || !out_tokens)
    return ORACLE_ERR_NULL;
  if (n < 1 || B < 0 || gamma < 1 || V < 1) return ORACLE_ERR_SHAPE;
  if (dtype != ORACLE_DTYPE_F32 && dtype != ORACLE_DTYPE_BF16 && dtype != ORACLE_DTYPE_F16)
    return ORACLE_ERR_DTYPE;
  status = check_weights(mode, n, weights);
  if (status != ORACLE_OK) return status;
  if (greedy && mode != ORACLE_ENSEMBLE) return ORACLE_ERR_MODE;
  esize = dtype == ORACLE_DTYPE_F32 ? 4 : 2;
  if (opt && !(opt->temperature >= 0.0) ) return ORACLE_ERR_WEIGHTS;
  for (b = 0; b < B; ++b) {
    int j;
    if (proposer_idx[b] < 0 || proposer_idx[b] >= n) return ORACLE_ERR_SHAPE;
    if (bonus_idx && (bonus_idx[b] < -1 || bonus_idx[b] >= n)) return ORACLE_ERR_SHAPE;
    if (num_drafts && (num_drafts[b] < 0 || num_drafts[b] > gamma)) return ORACLE_ERR_SHAPE;
    for (j = 0; j < (num_drafts ? num_drafts[b] : gamma); ++j) {
      int32_t d = draft_tokens[(size_t)b * gamma + j];
      if (d < 0 || d >= V) return ORACLE_ERR_SHAPE;
      if (proposer_pos && (proposer_pos[(size_t)b * gamma + j] < 0 ||
                           proposer_pos[(size_t)b * gamma + j] >= n))
        return ORACLE_ERR_SHAPE;
    }
  }
#ifdef _OPENMP
  if (num_threads > 0) omp_set_num_threads(num_threads);
#endif
#pragma omp parallel
  {
    /* per-thread scratch: logits l[n][V], softmaxes s[n][V], r[V], f[V] */
    double *l = (double *)malloc(sizeof(double) * (size_t)n * V);
    double *s = (double *)malloc(sizeof(double) * (size_t)n * V);
    double *r = (double *)malloc(sizeof(double) * (size_t)V);
    double *f = (double *)malloc(sizeof(double) * (size_t)V);
    if (!l || !s || !r || !f) {
#pragma omp atomic write
      failed = 1;
    }
#pragma omp for schedule(dynamic, 1)
    for (b = 0; b < B; ++b) {
      int pi, j, m, jstar, alive, x, clamped = 0, flag = 0, residual, token, bonus_from;
      const int gb = num_drafts ? num_drafts[b] : gamma; /* drafts of this row */
      const double *q;
      double F, lo = 0.0, hi = 0.0;
      if (failed) continue;
      alive = 1; /* no draft of this row rejected so far */
      jstar = -1;
      bonus_from = bonus_idx ? bonus_idx[b] : -1;
      for (j = 0; j < gamma; ++j) {
        size_t k = (size_t)b * gamma + j;
        if (r_at_draft) r_at_draft[k] = NAN;
        if (q_at_draft) q_at_draft[k] = NAN;
        if (ratio) ratio[k] = NAN;
        if (alpha) alpha[k] = NAN;
      }
      /* positions 0..gb-1 carry a draft; position gb is the bonus row */
      for (j = 0; j <= gb; ++j) {
        const int verifier_bonus = (j == gb) && bonus_from >= 0;
        if (!alive && !(all_positions && j < gb)) break;
        if (j == gb && no_bonus) {
          /* every draft accepted and no extra token wanted: nothing is read or drawn */
          accepted_len[b] = gb;
          for (x = 0; x <= gamma; ++x)
            out_tokens[(size_t)b * (gamma + 1) + x] =
                x < gb ? draft_tokens[(size_t)b * gamma + x] : -1;
          if (sample_mass) sample_mass[b] = 0.0;
          if (cdf_lo) cdf_lo[b] = 0.0;
          if (cdf_hi) cdf_hi[b] = 0.0;
          if (flags) flags[b] = 0;
          break;
        }
        for (m = 0; m < n; ++m) {
          size_t row = ((size_t)m * B + b) * (size_t)(gamma + 1) + j;
          const char *src = (const char *)logits + row * (size_t)V * esize;
          if (verifier_bonus && m != bonus_from) continue; /* not needed, not read */
          cos_oracle_row_to_f64(src, dtype, V, l + (size_t)m * V);
          if (greedy) {
            cos_oracle_softmax_t0(l + (size_t)m * V, V, s + (size_t)m * V);
            continue;
          }
          if (T != 1.0) cos_oracle_apply_temperature(l + (size_t)m * V, V, T);
          cos_oracle_softmax(l + (size_t)m * V, V, s + (size_t)m * V);
        }
        if (verifier_bonus) {
          /* Sec. 3.1 / 3.3: the bonus token follows the verifier's own distribution */
          memcpy(r, s + (size_t)bonus_from * V, sizeof(double) * (size_t)V);
        } else if (mode == ORACLE_ENSEMBLE) {
          cos_oracle_combine_ensemble(s, weights, n, V, r);
        } else if (mode == ORACLE_LOGIT_MIX) {
          cos_oracle_combine_logit_mix(l, weights, n, V, r);
        } else {
          cos_oracle_combine_contrastive(l, l + V, weights[0], weights[1], V, r);
        }
        if (j < gb) {
          size_t k = (size_t)b * gamma + j;
          int d = draft_tokens[k];
          double rt;
          int acc;
          pi = proposer_pos ? proposer_pos[k] : proposer_idx[b];
          q = s + (size_t)pi * V;
          acc = cos_oracle_accept(u_accept[k], r[d], q[d], &rt);
          if (r_at_draft) r_at_draft[k] = r[d];
          if (q_at_draft) q_at_draft[k] = q[d];
          if (ratio) ratio[k] = rt;
          if (alpha) alpha[k] = cos_oracle_acceptance_rate(q, r, V);
          if (!alive) continue; /* diagnostics only: row already decided */
          if (acc) continue;    /* accepted: go on to the next draft */
        } else {
          q = r; /* unused: the bonus draw takes f = r */
        }
        /* here j is the first rejected position, or j == gb (all accepted:
         * bonus token).  r, q hold the distributions of that position.      */
        jstar = j;
        alive = 0;
        residual = jstar < gb;
        F = cos_oracle_sample_weights(r, q, V, residual, f);
        if (!(F > 0.0) || !isfinite(F)) {
          /* cannot happen in exact arithmetic: fall back to r itself */
          F = cos_oracle_sample_weights(r, q, V, 0, f);
          flag |= ORACLE_FLAG_RESIDUAL_FALLBACK;
        }
        token = cos_oracle_inverse_cdf(f, V, F, u_resample[b], &clamped, &lo, &hi);
        if (clamped) flag |= ORACLE_FLAG_TAIL_CLAMP;
        accepted_len[b] = jstar;
        for (x = 0; x <= gamma; ++x) {
          int32_t *o = out_tokens + (size_t)b * (gamma + 1) + x;
          if (x < jstar)
            *o = draft_tokens[(size_t)b * gamma + x];
          else if (x == jstar)
            *o = token;
          else
            *o = -1;
        }
        if (sample_mass) sample_mass[b] = F;
        if (cdf_lo) cdf_lo[b] = lo;
        if (cdf_hi) cdf_hi[b] = hi;
        if (flags) flags[b] = flag;
      }
    }
    free(l);
    free(s);
    free(r);
    free(f);
  }
  return failed ? ORACLE_ERR_NOMEM : ORACLE_OK;
}

/* ---- the step at temperature 0, logit-level modes --------------------------
 * r is one-hot at a_j -- cos_oracle_argmax_contrastive (mode contrastive, n = 2,
 * weights = (mu, alpha_cd)) or cos_oracle_argmax_logit_mix (mode logit mix,
 * weights = beta[0..n-1]) of position j -- so Eq. (6) accepts d_j iff d_j == a_j
 * whatever q is (r(d) = 0 otherwise), the residual norm(max(0, r - q)) and its
 * fall-back r are both one-hot at a_j, and the bonus token is a_gamma -- or, with
 * bonus_idx[b] = v >= 0, the argmax of l_v alone (Sec. 3.3).  No random numbers
 * are consumed.  num_drafts / no_bonus as in cos_oracle_options.              */
int cos_oracle_verify_greedy_mode(const void *logits, int dtype, int n, int B, int gamma, int V,
                                  const int32_t *draft_tokens, int mode, const double *weights,
                                  const int32_t *bonus_idx, const int32_t *num_drafts,
                                  int no_bonus, int32_t *accepted_len,
                                  int32_t *out_tokens, int num_threads) {
  int b, failed = 0;
  size_t esize;
  if (!logits || !draft_tokens || !weights || !accepted_len || !out_tokens) return ORACLE_ERR_NULL;
  if (n < 1 || B < 0 || gamma < 1 || V < 1) return ORACLE_ERR_SHAPE;
  if (dtype != ORACLE_DTYPE_F32 && dtype != ORACLE_DTYPE_BF16 && dtype != ORACLE_DTYPE_F16)
    return ORACLE_ERR_DTYPE;
  if (mode != ORACLE_CONTRASTIVE && mode != ORACLE_LOGIT_MIX) return ORACLE_ERR_MODE;
  if (mode == ORACLE_CONTRASTIVE && n != 2) return ORACLE_ERR_MODE;
  if (check_weights(mode, n, weights) != ORACLE_OK) return ORACLE_ERR_WEIGHTS;
  esize = dtype == ORACLE_DTYPE_F32 ? 4 : 2;
  for (b = 0; b < B; ++b) {
    if (num_drafts && (num_drafts[b] < 0 || num_drafts[b] > gamma)) return ORACLE_ERR_SHAPE;
    if (bonus_idx && bonus_idx[b] >= n) return ORACLE_ERR_SHAPE;
  }
#ifdef _OPENMP
  if (num_threads > 0) omp_set_num_threads(num_threads);
#endif
#pragma omp parallel
  {
    double *l = (double *)malloc(sizeof(double) * (size_t)n * V);
    if (!l) {
#pragma omp atomic write
      failed = 1;
    }
#pragma omp for schedule(dynamic, 1)
    for (b = 0; b < B; ++b) {
      const int gb = num_drafts ? num_drafts[b] : gamma; /* drafts of this row */
      int j, m, x, jstar = gb, token = -1;
      if (failed) continue;
      for (j = 0; j <= gb; ++j) {
        const int v = (j == gb && bonus_idx) ? bonus_idx[b] : -1;
        int a;
        if (j == gb && no_bonus) break; /* all accepted, no extra token: nothing read */
        for (m = 0; m < n; ++m) {
          size_t row = ((size_t)m * B + b) * (size_t)(gamma + 1) + j;
          if (v >= 0 && m != v) continue; /* not needed, not read */
          cos_oracle_row_to_f64((const char *)logits + row * (size_t)V * esize, dtype, V,
                                l + (size_t)m * V);
        }
        if (v >= 0)
          a = cos_oracle_argmax(l + (size_t)v * V, V);
        else if (mode == ORACLE_CONTRASTIVE)
          a = cos_oracle_argmax_contrastive(l, l + V, weights[0], weights[1], V);
        else
          a = cos_oracle_argmax_logit_mix(l, weights, n, V);
        if (j < gb && draft_tokens[(size_t)b * gamma + j] == a) continue; /* accepted */
        jstar = j;
        token = a;
        break;
      }
      accepted_len[b] = jstar;
      for (x = 0; x <= gamma; ++x) {
        int32_t *o = out_tokens + (size_t)b * (gamma + 1) + x;
        *o = x < jstar ? draft_tokens[(size_t)b * gamma + x] : (x == jstar ? token : -1);
      }
    }
    free(l);
  }
  return failed ? ORACLE_ERR_NOMEM : ORACLE_OK;
}

/* The contrastive mode of the above (n = 2, weights = (mu, alpha_cd)). */
int cos_oracle_verify_greedy(const void *logits, int dtype, int B, int gamma, int V,
                             const int32_t *draft_tokens, const double *weights,
                             const int32_t *bonus_idx, const int32_t *num_drafts,
                             int no_bonus, int32_t *accepted_len,
                             int32_t *out_tokens, int num_threads) {
  return cos_oracle_verify_greedy_mode(logits, dtype, 2, B, gamma, V, draft_tokens,
                                       ORACLE_CONTRASTIVE, weights, bonus_idx, num_drafts,
                                       no_bonus, accepted_len, out_tokens, num_threads);
}

/* The base step: no extensions. */
int cos_oracle_verify(const void *logits, int dtype, int n, int B, int gamma,
                      int V, const int32_t *draft_tokens,
                      const int32_t *proposer_idx, int mode,
                      const double *weights, const double *u_accept,
                      const double *u_resample, int32_t *accepted_len,
                      int32_t *out_tokens, double *r_at_draft,
                      double *q_at_draft, double *ratio, double *sample_mass,
                      double *cdf_lo, double *cdf_hi, int32_t *flags,
                      int all_positions, int num_threads) {
  return cos_oracle_verify_ex(logits, dtype, n, B, gamma, V, draft_tokens, proposer_idx, mode,
                              weights, u_accept, u_resample, accepted_len, out_tokens, r_at_draft,
                              q_at_draft, ratio, sample_mass, cdf_lo, cdf_hi, flags,
                              all_positions, num_threads, NULL);
}

/* number of threads an OpenMP parallel region would use right now */
int cos_oracle_max_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}
