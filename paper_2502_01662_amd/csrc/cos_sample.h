// cos_sample.h -- the sampling weights f = max(0, r - q) or r (App. A.1), the tile
// sums, the inverse-CDF draw, and the acceptance-rate kernel (Eq. (7)).
#pragma once

#include "cos_device.h"

namespace {

// ---------------------------------------------------------------------------
// sampling weights f(x) of one 16-byte vector per model
// ---------------------------------------------------------------------------

// Ensemble: f = max(0, sum_m a_m 2^(l_m*log2e - K_m)); the a_m carry the
// ensemble weights, minus one for the proposer when a residual is wanted
// (App. A.1), times 2^(K_m - log2-sum-exp) so that the K_m are integers.  Each
// product is rounded before it is added (no fused multiply-add), so that terms
// of identical models cancel exactly and r == q leaves no residual mass.
template <int NCAP, int N>
__device__ __forceinline__ void eval_f_ensemble(const float (&x)[NCAP][N], int n, float scale,
                                                const float (&coef)[NCAP], const float (&off)[NCAP],
                                                float (&f)[N]) {
#pragma unroll
  for (int k = 0; k < N; ++k) {
    float s = 0.0f;
#pragma unroll
    for (int m = 0; m < NCAP; ++m)
      if (m < n) s += coef[m] * fast_exp2(fmaf(x[m][k], scale, -off[m]));
    f[k] = fmaxf(s, 0.0f);
  }
}

// Contrastive: r = [mask] coef[0] 2^(c*scale - off[0]), q = coef[1] 2^(l_pi*scale - off[1]);
// f = max(0, r - q) on the mask (coef[1] = 0 for a bonus draw from r), 0 off it.
// plain >= 0 (the verifier's own bonus token): f = coef[1] 2^(l_plain*scale - off[1]), no mask.
template <typename T, int N>
__device__ __forceinline__ void eval_f_contrastive(const float (&x0)[N], const float (&x1)[N],
                                                   int pi, int plain, float m0, const Params& p,
                                                   const float (&coef)[2], const float (&off)[2],
                                                   const float (&ref)[2], float (&f)[N]) {
  const int qsel = __builtin_amdgcn_readfirstlane(plain >= 0 ? plain : pi);  // uniform: a scalar branch
  float q[N];
  if (qsel) {
#pragma unroll
    for (int k = 0; k < N; ++k) q[k] = coef[1] * fast_exp2(fmaf(x1[k] - ref[1], p.scale, -off[1]));
  } else {
#pragma unroll
    for (int k = 0; k < N; ++k) q[k] = coef[1] * fast_exp2(fmaf(x0[k] - ref[0], p.scale, -off[1]));
  }
#pragma unroll
  for (int k = 0; k < N; ++k) {
    if (plain >= 0) {
      f[k] = q[k];
    } else {
      const bool in = in_mask<T>(x0[k], m0, p.thr32, p.thr64);
      const float c = contrast(x0[k], x1[k], p.mu_hi, p.mu_lo, ref[0], ref[1]);
      const float r = coef[0] * fast_exp2(fmaf(c, p.scale, -off[0]));
      f[k] = in ? fmaxf(r - q[k], 0.0f) : 0.0f;
    }
  }
}

// Logit mix: r = coef[0] 2^(c*scale - off[0]), q = coef[1] 2^(l_pi*scale - off[1]);
// f = max(0, r - q) (coef[1] = 0 for a bonus draw from r).
// plain >= 0 (the verifier's own bonus token): f = coef[1] 2^(l_plain*scale - off[1]).
template <int NCAP, int N>
__device__ __forceinline__ void eval_f_mix(const float (&x)[NCAP][N], int n, int pi, int plain,
                                           const Params& p, const float (&coef)[NCAP],
                                           const float (&off)[NCAP], const float (&ref)[NCAP],
                                           float (&f)[N]) {
  static_assert(NCAP >= 2, "two coefficients");
  const int qsel = __builtin_amdgcn_readfirstlane(plain >= 0 ? plain : pi);  // uniform: a scalar branch
  // the shifted rows and their combination (mix_shifted_rows: mix_one's numbers at less arithmetic)
  float d[NCAP][N], c[N];
  mix_shifted_rows<NCAP, N>(p, n, x, ref, plain < 0, d, c);
  float q[N];
#pragma unroll
  for (int m = 0; m < NCAP; ++m)
    if (m == qsel) {
#pragma unroll
      for (int k = 0; k < N; ++k) q[k] = coef[1] * fast_exp2(fmaf(d[m][k], p.scale, -off[1]));
    }
#pragma unroll
  for (int k = 0; k < N; ++k) {
    if (plain >= 0) {
      f[k] = q[k];
    } else {
      const float r = coef[0] * fast_exp2(fmaf(c[k], p.scale, -off[0]));
      f[k] = fmaxf(r - q[k], 0.0f);
    }
  }
}

// ---------------------------------------------------------------------------
// the residual in its difference form, for r close to q
// ---------------------------------------------------------------------------
//
// max(0, r - q) evaluated term by term rounds each softmax value to float32 on its
// own: an absolute error of ~1e-7 of the value, harmless unless r - q is a small
// fraction of it everywhere, i.e. unless the residual mass F = 1 - alpha is small.
// Then the last workgroup of the sequence evaluates the residual once more as
//   ensemble:     q(x) * sum_{m != pi} w_m (2^delta_m - 1),  delta_m = log2(s_m(x) / s_pi(x))
//   logit level:  q(x) * (2^delta - 1),                      delta   = log2(r(x) / q(x))
// (the ensemble form uses sum_m w_m = 1), whose error is relative to the small
// differences themselves.  delta needs the difference of two log-normalisers, and the
// streaming kernel's float32 sums give each of them to ~1e-7 only -- an absolute
// error in delta, hence a relative one of 1e-7 / F in the residual.  The workgroup
// therefore first takes that difference itself, again in difference form: with
// E(x) = 2^(l_pi(x)*scale - K) and one offset K for both rows,
//   Z_m / Z_pi - 1 = sum_x E(x) (2^d0_m(x) - 1) / sum_x E(x),   d0_m = (l_m - l_pi)*scale
// (logit level: d0 = (c - l_pi)*scale; tokens outside the mask contribute -E(x)),
// which is what makes sum_x (r - q) vanish: the refined residual then carries a
// relative error of ~1e-7 whatever its mass.

// What the difference form needs beside the plain coefficients.
template <int NCAP>
struct Refine {
  float coef_q, off_q;  // q(x) = coef_q 2^(l_pi(x)*scale - off_q)
  float w[NCAP];        // ensemble: w_m (0 for the proposer); logit level: unused
  float dlse[NCAP];     // ensemble: lse2_m - lse2_pi; logit level: slot 0 = lse2_r - lse2_q
  float wsum_m1;        // sum of the weights - 1 (ensemble: within 1e-9 of zero, kept so the form is
                        // exact; logit mix: sum_m beta_m - 1)
};

// 2^d - 1 for |d| <= 1 with an error relative to the result.
__device__ __forceinline__ float exp2m1(float d) {
  const float y = d * 0.69314718055994531f;
  const float poly =
      y * fmaf(y, fmaf(y, fmaf(y, fmaf(y, fmaf(y, 1.0f / 720.0f, 1.0f / 120.0f), 1.0f / 24.0f), 1.0f / 6.0f), 0.5f), 1.0f);
  return fabsf(y) < 0.125f ? poly : fast_exp2(d) - 1.0f;
}

template <int NCAP, int MODE>
__device__ __forceinline__ void plan_refine(const Params& p, const SeqPlan& plan, int n, Refine<NCAP>& rf) {
  double lq;  // log2-sum-exp2 of the proposer's row
  rf.wsum_m1 = 0.0f;
  if constexpr (MODE == kEns) {
    lq = plan.lse2[0];
    double wsum = 0.0;
#pragma unroll
    for (int m = 1; m < NCAP; ++m) {
      const double v = plan.lse2[m];  // value first, then the choice: no indexed access
      lq = (m == plan.pi) ? v : lq;
    }
#pragma unroll
    for (int m = 0; m < NCAP; ++m) {
      const bool on = m < n && m != plan.pi && p.w[m] != 0.0;
      rf.w[m] = on ? (float)p.w[m] : 0.0f;
      rf.dlse[m] = on ? (float)(plan.lse2[m] - lq) : 0.0f;
      if (m < n) wsum += p.w[m];
    }
    rf.wsum_m1 = (float)(wsum - 1.0);
  } else if constexpr (MODE == kMix) {
    lq = plan.lse2[0];
    double bsum = 0.0;
#pragma unroll
    for (int m = 0; m < NCAP; ++m) {
      rf.w[m] = rf.dlse[m] = 0.0f;
      if (m < n) bsum += p.w[m];
    }
    rf.wsum_m1 = (float)(bsum - 1.0);  // sum_m beta_m - 1
    rf.dlse[0] = (float)(plan.lse2[1] - lq);
  } else {
    const double l0 = plan.lse2[0], l1 = plan.lse2[1];
    lq = plan.pi ? l1 : l0;
#pragma unroll
    for (int m = 0; m < NCAP; ++m) rf.w[m] = rf.dlse[m] = 0.0f;
    rf.dlse[0] = (float)(plan.lse2[2] - lq);
  }
  const double K = rint(lq);
  rf.off_q = (float)K;
  rf.coef_q = (float)exp2(K - lq);
}

// The residual of one vector in its difference form.  `plainf` is the term-by-term
// value, kept wherever the difference form does not apply (q(x) = 0, or a ratio
// beyond a factor of two, where nothing cancels).  A term whose numerator is 0
// (a -inf logit, a token outside the mask) has delta = -inf and 2^delta - 1 = -1
// without any special case.
template <typename T, int NCAP, int N, int MODE>
__device__ __forceinline__ void eval_f_refined(const Params& p, const float (&x)[NCAP][N], int n, int pi,
                                               float m0, const float (&ref)[NCAP], const Refine<NCAP>& rf,
                                               const float (&plainf)[N], float (&f)[N]) {
  float refq = ref[0];
#pragma unroll
  for (int m = 1; m < NCAP; ++m) refq = (m == pi) ? ref[m] : refq;
#pragma unroll
  for (int k = 0; k < N; ++k) {
    const float lp = pick_row<NCAP, N>(x, pi, k);
    const float q = rf.coef_q * fast_exp2(fmaf(lp - refq, p.scale, -rf.off_q));
    float acc = rf.wsum_m1;
    float far = 0.0f;  // largest finite |delta| of this element
    if constexpr (MODE == kEns) {
#pragma unroll
      for (int m = 0; m < NCAP; ++m)
        if (m < n && rf.w[m] != 0.0f) {
          const float d = fmaf(x[m][k] - lp, p.scale, -rf.dlse[m]);
          far = fmaxf(far, d == -INFINITY ? 0.0f : fabsf(d));
          acc = fmaf(rf.w[m], exp2m1(d), acc);
        }
    } else {
      // c(x) - l_pi(x) on the shifted logits, from differences between the models so that it
      // rounds at their scale: sum_m beta_m (v_m - v_pi) + (sum_m beta_m - 1) v_pi
      const float vp = lp - refq;
      float cd;
      if constexpr (MODE == kMix) {
        cd = rf.wsum_m1 * vp;
        bool dead = false;
#pragma unroll
        for (int m = 0; m < NCAP; ++m)
          if (m < n && (p.beta_hi[m] != 0.0f || p.beta_lo[m] != 0.0f)) {
            dead = dead || x[m][k] == -INFINITY;
            // (l_m - l_pi) - (ref_m - ref_pi): both differences are exact for nearby rows
            const float dv = (x[m][k] - lp) - (ref[m] - refq);
            cd = fmaf(p.beta_lo[m], dv, fmaf(p.beta_hi[m], dv, cd));
          }
        cd = dead ? -INFINITY : cd;
      } else {
        const float v1 = x[1][k] - ref[1];
        cd = fmaf(-p.mu_lo, v1, fmaf(-p.mu_hi, v1, (x[0][k] - lp) - (ref[0] - refq)));
        cd = in_mask<T>(x[0][k], m0, p.thr32, p.thr64) ? cd : -INFINITY;
      }
      const float d = fmaf(cd, p.scale, -rf.dlse[0]);
      far = d == -INFINITY ? 0.0f : fabsf(d);
      acc = exp2m1(d);
    }
    // (NaN in `far` -- q(x) = 0 -- fails the comparison and keeps the plain value)
    f[k] = (far <= 1.0f) ? fmaxf(q * acc, 0.0f) : plainf[k];
  }
}

// First pass of the difference form: this lane's contributions, over one vector, to
// Q = sum_x E(x) and A[t] = sum_x (E_t(x) - E(x)) for every term t of r (ensemble: the models with
// weight other than the proposer; logit level: slot 0), E_t being the term's own 2^(. - K).
template <typename T, int NCAP, int N, int MODE>
__device__ __forceinline__ void refine_sums(const Params& p, const float (&x)[NCAP][N], int n, int pi, float m0,
                                            const float (&ref)[NCAP], const Refine<NCAP>& rf, double& Q,
                                            double (&A)[NCAP]) {
  float refq = ref[0];
#pragma unroll
  for (int m = 1; m < NCAP; ++m) refq = (m == pi) ? ref[m] : refq;
#pragma unroll
  for (int k = 0; k < N; ++k) {
    const float lp = pick_row<NCAP, N>(x, pi, k);
    const float vp = lp - refq;
    const float E = fast_exp2(fmaf(vp, p.scale, -rf.off_q));
    Q += (double)E;
    if constexpr (MODE == kEns) {
#pragma unroll
      for (int m = 0; m < NCAP; ++m)
        if (m < n && rf.w[m] != 0.0f) {
          const float d0 = (x[m][k] - lp) * p.scale;
          // beyond a factor of two nothing cancels: the term's own value minus E (a -inf logit: -E)
          const float t = (fabsf(d0) <= 1.0f) ? E * exp2m1(d0) : fast_exp2(fmaf(x[m][k], p.scale, -rf.off_q)) - E;
          A[m] += (double)t;
        }
    } else {
      float cd, c;  // c(x) - l_pi(x) and c(x), both on the shifted logits
      bool in = true;
      if constexpr (MODE == kMix) {
        cd = rf.wsum_m1 * vp;
        bool dead = false;
#pragma unroll
        for (int m = 0; m < NCAP; ++m)
          if (m < n && (p.beta_hi[m] != 0.0f || p.beta_lo[m] != 0.0f)) {
            dead = dead || x[m][k] == -INFINITY;
            // (l_m - l_pi) - (ref_m - ref_pi): both differences are exact for nearby rows
            const float dv = (x[m][k] - lp) - (ref[m] - refq);
            cd = fmaf(p.beta_lo[m], dv, fmaf(p.beta_hi[m], dv, cd));
          }
        float l[NCAP];
#pragma unroll
        for (int m = 0; m < NCAP; ++m) l[m] = x[m][k];
        c = mix_one<NCAP>(p, n, l, ref);
        in = !dead;
      } else {
        const float v1 = x[1][k] - ref[1];
        cd = fmaf(-p.mu_lo, v1, fmaf(-p.mu_hi, v1, (x[0][k] - lp) - (ref[0] - refq)));
        c = contrast(x[0][k], x[1][k], p.mu_hi, p.mu_lo, ref[0], ref[1]);
        in = in_mask<T>(x[0][k], m0, p.thr32, p.thr64);
      }
      const float d0 = cd * p.scale;
      float t;
      if (!in)
        t = -E;
      else if (fabsf(d0) <= 1.0f)  // false for NaN (a proposer logit of -inf)
        t = E * exp2m1(d0);
      else
        t = fast_exp2(fmaf(c, p.scale, -rf.off_q)) - E;
      A[0] += (double)t;
    }
  }
}

// Coefficients and integer offsets of the sampling weights from a sequence's plan.
template <int NCAP, int MODE>
__device__ __forceinline__ void plan_coefficients(const Params& p, const SeqPlan& plan, bool residual,
                                                  int n, float (&coef)[NCAP], float (&off)[NCAP]) {
#pragma unroll
  for (int m = 0; m < NCAP; ++m) {
    // A term without weight must vanish whatever its logits are: with the offset far up,
    // 2^(l*scale - off) is 0 for every finite l (with offset 0 a large logit would overflow
    // to +inf, and 0 * inf would poison the sum).
    coef[m] = 0.0f;
    off[m] = kOffNever;
    if (m < n || (MODE == kMix && m < 2)) {
      double a, lse;
      const bool plain = !residual && plan.bonus >= 0;  // bonus token from one model's softmax alone
      if constexpr (MODE == kEns) {
        a = plain ? (m == plan.bonus ? 1.0 : 0.0) : p.w[m] - ((residual && m == plan.pi) ? 1.0 : 0.0);
        lse = plan.lse2[m];
      } else if constexpr (MODE == kMix) {
        // slot 0: r from the mixed logits (statistic 1); slot 1: q (statistic 0); others unused
        a = (m == 0) ? (plain ? 0.0 : 1.0) : ((m == 1 && (residual || plain)) ? 1.0 : 0.0);
        lse = plan.lse2[m == 0 ? 1 : 0];
      } else {
        a = (m == 0) ? 1.0 : ((residual || plain) ? 1.0 : 0.0);
        const double lse_q0 = plan.lse2[0], lse_q1 = plan.lse2[1];  // values first, then the choice
        lse = m == 0 ? plan.lse2[2] : ((plain ? plan.bonus : plan.pi) ? lse_q1 : lse_q0);
      }
      if (a != 0.0) {  // a model without weight may have no statistic at all (lse = -inf)
        const double K = rint(lse);
        off[m] = (float)K;
        coef[m] = (float)(a * exp2(K - lse));
      }
    }
  }
}

// Raw vectors of one tile (64 lanes x one 16-byte vector per model) for this lane.
// Tiles past the row's end are redirected to the last vector (masked in tile_eval).
template <typename T, bool ALIGNED, int NCAP>
__device__ __forceinline__ void tile_load(const Params& p, const T* const (&rows)[NCAP], int n, int tile,
                                          float (&x)[NCAP][VecOf<T>::N]) {
  const int vc = min(tile * 64 + lane_id(), p.nvec - 1);
#pragma unroll
  for (int m = 0; m < NCAP; ++m)
    if (m < n) load_vec<T, ALIGNED>(rows[m], vc, p.V, x[m]);
}

// f of the loaded tile for this lane; 0 past the row's end.
template <typename T, int NCAP, int MODE>
__device__ __forceinline__ void tile_eval(const Params& p, const float (&x)[NCAP][VecOf<T>::N], int n,
                                          int tile, int pi, int plain, float m0,
                                          const float (&coef)[NCAP], const float (&off)[NCAP],
                                          const float (&ref)[NCAP], float (&f)[VecOf<T>::N],
                                          bool refined, const Refine<NCAP>& rf) {
  constexpr int N = VecOf<T>::N;
  if constexpr (MODE == kEns)
    eval_f_ensemble<NCAP, N>(x, n, p.scale, coef, off, f);
  else if constexpr (MODE == kMix)
    eval_f_mix<NCAP, N>(x, n, pi, plain, p, coef, off, ref, f);
  else
    eval_f_contrastive<T, N>(x[0], x[1], pi, plain, m0, p, coef, off, ref, f);
  if (refined) {  // wave-uniform: the residual once more, in its difference form
    float g[N];
    eval_f_refined<T, NCAP, N, MODE>(p, x, n, pi, m0, ref, rf, f, g);
#pragma unroll
    for (int k = 0; k < N; ++k) f[k] = g[k];
  }
  if (tile * 64 + lane_id() >= p.nvec) {
#pragma unroll
    for (int k = 0; k < N; ++k) f[k] = 0.0f;
  }
}

template <typename T, bool ALIGNED, int NCAP, int MODE>
__device__ __forceinline__ void tile_weights(const Params& p, const T* const (&rows)[NCAP], int n,
                                             int tile, int pi, int plain, float m0,
                                             const float (&coef)[NCAP], const float (&off)[NCAP],
                                             const float (&ref)[NCAP], float (&f)[VecOf<T>::N],
                                             bool refined, const Refine<NCAP>& rf) {
  float x[NCAP][VecOf<T>::N];
  tile_load<T, ALIGNED, NCAP>(p, rows, n, tile, x);
  tile_eval<T, NCAP, MODE>(p, x, n, tile, pi, plain, m0, coef, off, ref, f, refined, rf);
}

template <int N>
__device__ __forceinline__ double lane_mass(const float (&f)[N]) {
  double s = 0.0;
#pragma unroll
  for (int k = 0; k < N; ++k) s += (double)f[k];
  return s;
}

// ---------------------------------------------------------------------------
// final scan + inverse CDF of one sequence (wavefront 0 of the last sampling
// workgroup); tile_sum holds the ntiles tile sums in LDS.
// Returns kDrawn, or without drawing: kNoMass if the weights have no mass and
// may_retry is set, kLittleMass if their mass is below refine_below.
// ---------------------------------------------------------------------------
constexpr double kRefineBelow = 1.0 / 32.0;  // residual mass under which the difference form is used

template <typename T, bool ALIGNED, int NCAP, int MODE>
__device__ int draw_token(const Params& p, int b, const SeqPlan& plan, const T* const (&rows)[NCAP],
                          int n, const float (&coef)[NCAP], const float (&off)[NCAP],
                          const float (&ref)[NCAP], const double* tile_sum, bool may_retry, int flags,
                          double refine_below, bool refined, const Refine<NCAP>& rf) {
  constexpr int N = VecOf<T>::N;
  const int lane = lane_id();
  const int g1 = p.gamma + 1;
  // scan of the tile sums: each lane owns a contiguous segment
  const int per = (p.ntiles + 63) / 64;
  const int t0 = min(lane * per, p.ntiles), t1 = min(t0 + per, p.ntiles);
  double seg = 0.0;
  for (int t = t0; t < t1; ++t) seg += tile_sum[t];
  const double incl = wave_inclusive_scan(seg);
  const double F = __shfl(incl, 63, 64);
  const double up = __shfl_up(incl, 1, 64);
  const double excl = lane ? up : 0.0;
  const bool bad = !(F > 0.0) || !(F < INFINITY);
  if (bad && may_retry) return kNoMass;
  if (!bad && F < refine_below) return kLittleMass;

  const double target = p.u_resample[b] * F;
  // first tile whose inclusive prefix exceeds the target; else the last tile with mass
  int hit = -1, lastpos = -1;
  double hit_excl = 0.0, lastpos_excl = 0.0, runsum = excl;
  for (int t = t0; t < t1; ++t) {
    const double ts = tile_sum[t];
    const double nxt = runsum + ts;
    if (hit < 0 && nxt > target) {
      hit = t;
      hit_excl = runsum;
    }
    if (ts > 0.0) {
      lastpos = t;
      lastpos_excl = runsum;
    }
    runsum = nxt;
  }
  const unsigned long long hits = __ballot(hit >= 0);
  const unsigned long long poss = __ballot(lastpos >= 0);
  bool clamp = false;
  int tile = 0;
  double tile_excl = 0.0;
  if (hits) {
    const int src = __ffsll((long long)hits) - 1;
    tile = __shfl(hit, src, 64);
    tile_excl = __shfl(hit_excl, src, 64);
  } else {
    clamp = true;
    if (poss) {
      const int src = 63 - __clzll((long long)poss);
      tile = __shfl(lastpos, src, 64);
      tile_excl = __shfl(lastpos_excl, src, 64);
    }
  }

  // the same f values of that one tile, scanned element by element
  float f[N];
  tile_weights<T, ALIGNED, NCAP, MODE>(p, rows, n, tile, plan.pi, plan.bonus, plan.m0, coef, off, ref, f,
                                       refined, rf);
  const double lane_tot = lane_mass<N>(f);
  const double lincl = wave_inclusive_scan(lane_tot);
  const double lup = __shfl_up(lincl, 1, 64);
  const double lexcl = tile_excl + (lane ? lup : 0.0);
  int ksel = -1, klast = -1;
  double lo_sel = 0.0, hi_sel = 0.0, lo_last = 0.0, hi_last = 0.0, runl = lexcl;
#pragma unroll
  for (int k = 0; k < N; ++k) {
    const double nxt = runl + (double)f[k];
    if (ksel < 0 && nxt > target) {
      ksel = k;
      lo_sel = runl;
      hi_sel = nxt;
    }
    if (f[k] > 0.0f) {
      klast = k;
      lo_last = runl;
      hi_last = nxt;
    }
    runl = nxt;
  }
  const unsigned long long sel = clamp ? 0ull : __ballot(ksel >= 0);
  const unsigned long long pos = __ballot(klast >= 0);
  int src = 0, kk = 0;
  double lo = 0.0, hi = 0.0;
  if (sel) {
    src = __ffsll((long long)sel) - 1;
    kk = ksel;
    lo = lo_sel;
    hi = hi_sel;
  } else {
    // rounding left no prefix above the target inside this tile (or tail clamp):
    // take the last element with mass
    if (pos) src = 63 - __clzll((long long)pos);
    kk = klast < 0 ? 0 : klast;
    lo = lo_last;
    hi = hi_last;
    if (clamp) flags |= COS_FLAG_TAIL_CLAMP;
  }
  if (lane == src) {
    int token = (tile * 64 + lane) * N + kk;
    token = min(max(token, 0), p.V - 1);
    p.out_tokens[(size_t)b * g1 + plan.jstar] = token;
    if (p.diag.sample_mass) p.diag.sample_mass[b] = F;
    if (p.diag.cdf_lo) p.diag.cdf_lo[b] = lo / F;
    if (p.diag.cdf_hi) p.diag.cdf_hi[b] = hi / F;
    if (p.diag.flags) p.diag.flags[b] = flags;
  }
  return kDrawn;
}

// One workgroup over every tile of a row-set: body(t, x) for this wavefront's tiles t = wave,
// wave + kWaves, ...  (One tile per wavefront in flight: these passes are bound by the one workgroup's
// arithmetic, not by its loads; more in flight only cost the sampling kernel registers.)
template <typename T, bool ALIGNED, int NCAP, class Body>
__device__ __forceinline__ void for_each_tile(const Params& p, const T* const (&rows)[NCAP], int n, Body&& body) {
  constexpr int N = VecOf<T>::N;
  for (int t = threadIdx.x >> 6; t < p.ntiles; t += kWaves) {
    float x[NCAP][N];
    tile_load<T, ALIGNED, NCAP>(p, rows, n, t, x);
    body(t, x);
  }
}

// With every tile sum of the sampled position in tile_sum (LDS), the whole workgroup draws the
// sequence's token: the scan and the inverse CDF, and the two rare endings -- a residual of little
// mass (r close to q) is evaluated once more in its difference form, a residual without mass falls
// back to r.  Each ending recomputes every tile sum in this one workgroup (small row-sets, and the
// finishing kernel of the one-read contrastive mode; large row-sets: the refinement kernels below).
template <typename T, bool ALIGNED, int NCAP, int MODE>
__device__ __forceinline__ void finish_draw(const Params& p, int b, const SeqPlan& plan, const T* const (&rows)[NCAP],
                                            int n, float (&coef)[NCAP], float (&off)[NCAP], const float (&ref)[NCAP],
                                            double* tile_sum, int& s_flag, Refine<NCAP>& s_rf) {
  constexpr int N = VecOf<T>::N;
  const int lane = lane_id();
  const int wave = threadIdx.x >> 6;
  const Refine<NCAP> no_refine = {};  // the plain, term-by-term evaluation
  const bool residual = plan.residual != 0;
  int status = kDrawn;
  if (wave == 0)
    status = draw_token<T, ALIGNED, NCAP, MODE>(p, b, plan, rows, n, coef, off, ref, tile_sum, residual, 0,
                                                residual ? kRefineBelow : 0.0, false, no_refine);
  if (threadIdx.x == 0) s_flag = status;
  __syncthreads();
  status = s_flag;
  if (status == kDrawn) return;
  __syncthreads();  // s_flag is written again below

  if (status == kLittleMass) {
    // r is close to q: this one workgroup evaluates the residual of the whole row once more,
    // in its difference form, and draws from that
    if (threadIdx.x == 0) {
      // read the plan again rather than keeping its normalisers in registers across the
      // streaming loop above, which every sequence runs
      const SeqPlan again = p.plans[b];
      plan_refine<NCAP, MODE>(p, again, n, s_rf);
    }
    __syncthreads();
    const Refine<NCAP>& rf = s_rf;
    // first pass: the differences of the log-normalisers, themselves in difference form
    {
      double Q = 0.0, A[NCAP];
#pragma unroll
      for (int m = 0; m < NCAP; ++m) A[m] = 0.0;
      for_each_tile<T, ALIGNED, NCAP>(p, rows, n, [&](int t, const float (&x)[NCAP][N]) {
        if (t * 64 + lane < p.nvec) refine_sums<T, NCAP, N, MODE>(p, x, n, plan.pi, plan.m0, ref, rf, Q, A);
      });
      // the tile sums are not needed any more: their LDS takes the wavefronts' totals
      __syncthreads();
      Q = wave_sum(Q);
      if (lane == 0) tile_sum[wave * (NCAP + 1)] = Q;
#pragma unroll
      for (int m = 0; m < NCAP; ++m) {
        const double a = wave_sum(A[m]);
        if (lane == 0) tile_sum[wave * (NCAP + 1) + 1 + m] = a;
      }
      __syncthreads();
      if (threadIdx.x == 0) {
        double q = 0.0;
        for (int w = 0; w < kWaves; ++w) q += tile_sum[w * (NCAP + 1)];
#pragma unroll
        for (int m = 0; m < NCAP; ++m) {
          double a = 0.0;
          for (int w = 0; w < kWaves; ++w) a += tile_sum[w * (NCAP + 1) + 1 + m];
          const double ratio = a / q;  // Z_t / Z_pi - 1
          const bool used = MODE == kEns ? s_rf.w[m] != 0.0f : m == 0;
          // (not finite, or not above -1: models that are not close after all; the streamed value stays)
          if (used && ratio > -1.0 && ratio < INFINITY) s_rf.dlse[m] = (float)(log1p(ratio) * 1.4426950408889634);
        }
      }
      __syncthreads();
    }
    for_each_tile<T, ALIGNED, NCAP>(p, rows, n, [&](int t, const float (&x)[NCAP][N]) {
      float f[N];
      tile_eval<T, NCAP, MODE>(p, x, n, t, plan.pi, plan.bonus, plan.m0, coef, off, ref, f, true, rf);
      const double ts = wave_sum(lane_mass<N>(f));
      if (lane == 0) tile_sum[t] = ts;
    });
    __syncthreads();
    if (wave == 0)
      status = draw_token<T, ALIGNED, NCAP, MODE>(p, b, plan, rows, n, coef, off, ref, tile_sum, true,
                                                  COS_FLAG_RESIDUAL_REFINED, 0.0, true, rf);
    if (threadIdx.x == 0) s_flag = status;
    __syncthreads();
    if (s_flag == kDrawn) return;
  }

  // The residual has no mass (cannot happen in exact arithmetic): draw from r
  // itself.  Rare, so this one workgroup recomputes every tile sum.
  plan_coefficients<NCAP, MODE>(p, plan, false, n, coef, off);
  for_each_tile<T, ALIGNED, NCAP>(p, rows, n, [&](int t, const float (&x)[NCAP][N]) {
    float f[N];
    tile_eval<T, NCAP, MODE>(p, x, n, t, plan.pi, plan.bonus, plan.m0, coef, off, ref, f, false, no_refine);
    const double ts = wave_sum(lane_mass<N>(f));
    if (lane == 0) tile_sum[t] = ts;
  });
  __syncthreads();
  if (wave == 0)
    draw_token<T, ALIGNED, NCAP, MODE>(p, b, plan, rows, n, coef, off, ref, tile_sum, false,
                                       COS_FLAG_RESIDUAL_FALLBACK, 0.0, false, no_refine);
}

// Sampling kernel.  Workgroup index -> (b, c): tiles [c*tpc, (c+1)*tpc) of the
// sampled position's rows -> tile sums; the last workgroup of b draws the token.
// A residual of little mass (r close to q) is evaluated once more in its difference form: by the last
// workgroup of its sequence alone (LONE; two more passes over the row-set at the rate of one
// workgroup, which is fine for small row-sets), or -- the sequence only marked here -- by the two
// refinement kernels below, which split the marked sequences between about a thousand workgroups.
template <typename T, bool ALIGNED, int NM, int MODE, bool LONE>
__global__ void __launch_bounds__(kThreads) sample_kernel(Params p) {
  constexpr int N = VecOf<T>::N;
  constexpr bool CONTRASTIVE = MODE == kCd;
  // register rows; the logit mix keeps its two coefficients in slots 0 and 1
  constexpr int NCAP = CONTRASTIVE ? 2 : (NM ? (MODE == kMix && NM < 2 ? 2 : NM) : COS_MAX_MODELS);
  constexpr int TU = NCAP <= 4 ? 4 : 1;  // tiles in flight per wavefront
  extern __shared__ double tile_sum[];
  __shared__ int s_flag;
  // parameters of the rarely used difference form: kept in LDS, not in scalar registers, which
  // the streaming loop below needs for itself
  __shared__ Refine<NCAP> s_rf;

  const int b = blockIdx.x / p.C;
  const int c = blockIdx.x - b * p.C;
  const int lane = lane_id();
  const int wave = threadIdx.x >> 6;
  const int n = CONTRASTIVE ? 2 : (NM ? NM : p.n);
  const SeqPlan plan = p.plans[b];
  if (plan.skip) return;  // every draft accepted, no extra token: nothing to draw
  // A verifier bonus reads that one model's row only (the others carry a zero
  // coefficient and may hold anything, so every slot points at the valid row).
  const bool one_row = MODE == kEns && plan.residual == 0 && plan.bonus >= 0;
  const T* rows[NCAP];
#pragma unroll
  for (int m = 0; m < NCAP; ++m)
    rows[m] = row_ptr<T>(p, one_row ? plan.bonus : (m < n ? m : 0), b, plan.jstar);
  float coef[NCAP], off[NCAP];
  plan_coefficients<NCAP, MODE>(p, plan, plan.residual != 0, n, coef, off);
  float ref[NCAP];  // per-row reference of the logit-level combinations (unused by the ensemble)
#pragma unroll
  for (int m = 0; m < NCAP; ++m) ref[m] = (MODE != kEns && m < n) ? row_reference<T>(rows[m]) : 0.0f;

  const Refine<NCAP> no_refine = {};  // the plain, term-by-term evaluation
  HandOff<double>* sums = p.tile_sums + (size_t)b * p.ntiles;
  const int tb = c * p.tpc;
  const int te = min(tb + p.tpc, p.ntiles);
  // wavefront w takes tiles tb + w, tb + w + kWaves, ...; TU of them are in flight at once
  for (int t = tb + wave; t < te; t += kWaves * TU) {
    float x[TU][NCAP][N];
#pragma unroll
    for (int i = 0; i < TU; ++i)
      tile_load<T, ALIGNED, NCAP>(p, rows, n, min(t + i * kWaves, te - 1), x[i]);
#pragma unroll
    for (int i = 0; i < TU; ++i) {
      const int ti = t + i * kWaves;
      float f[N];
      tile_eval<T, NCAP, MODE>(p, x[i], n, min(ti, te - 1), plan.pi, plan.bonus, plan.m0, coef,
                               off, ref, f, false, no_refine);
      const double ts = wave_sum_to_lane63(lane_mass<N>(f));
      if (lane == 63 && ti < te) tile_sum[ti - tb] = ts;  // staged in LDS
    }
  }
  __syncthreads();
  // publish this workgroup's tile sums with coalesced write-through stores
  for (int i = threadIdx.x; i < te - tb; i += kThreads) sums[tb + i].publish(tile_sum[i]);
  wait_stores();
  if (!arrive_last(p.counters + ((size_t)p.nwin * p.B + b) * kCtrStride, p.C, &s_flag)) return;

  // last workgroup of this sequence: all tile sums are published
  for (int t = threadIdx.x; t < p.ntiles; t += kThreads) tile_sum[t] = sums[t].read();
  __syncthreads();
  if constexpr (LONE) {
    finish_draw<T, ALIGNED, NCAP, MODE>(p, b, plan, rows, n, coef, off, ref, tile_sum, s_flag, s_rf);
  } else {
    if (wave == 0) {
      const bool residual = plan.residual != 0;
      const int status = draw_token<T, ALIGNED, NCAP, MODE>(p, b, plan, rows, n, coef, off, ref, tile_sum, residual,
                                                            0, residual ? kRefineBelow : 0.0, false, no_refine);
      if (lane == 0 && status != kDrawn) {  // for the refinement kernels: mark the sequence, add it to their list
        p.plans[b].redo = status;
        const int slot = __hip_atomic_fetch_add(p.refine_ctl, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        p.refine_list[slot] = b;
      }
    }
  }
}

// The refinement kernels' work: the sequences the sampling kernel marked (refine_list), each split over
// as many workgroups as the launch has to spare -- with few marked sequences each gets many, so that its
// two extra passes over the row-set take microseconds instead of one workgroup's hundreds.  All
// workgroups see the same final count, hence the same split.
struct RefineTask {
  int count;  // marked sequences
  int cr;     // workgroups per marked sequence
  int b;      // this workgroup's sequence (-1: none)
  int c;      // its part of that sequence
  int slot;   // cr * (index in the list) + c
  int tb, te; // its tiles
};
__device__ __forceinline__ RefineTask refine_task(const Params& p) {
  RefineTask t;
  t.count = __hip_atomic_load(p.refine_ctl, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  t.b = -1;
  if (t.count <= 0) return t;
  t.cr = min(p.refine_cmax, max(1, p.refine_grid / t.count));
  const int i = blockIdx.x / t.cr;
  if (i >= t.count) return t;
  t.c = blockIdx.x - i * t.cr;
  t.slot = blockIdx.x;
  t.b = p.refine_list[i];
  const int per = (p.ntiles + t.cr - 1) / t.cr;
  t.tb = min(t.c * per, p.ntiles);
  t.te = min(t.tb + per, p.ntiles);
  return t;
}

// Refinement, first kernel (a launch of refine_grid workgroups that return at once when no sequence is
// marked): the sums that give the differences of the log-normalisers in difference form (refine_sums),
// every workgroup over its own tiles; the last one of the sequence combines them.
template <typename T, bool ALIGNED, int NM, int MODE>
__global__ void __launch_bounds__(kThreads) refine_sums_kernel(Params p) {
  constexpr int N = VecOf<T>::N;
  constexpr bool CONTRASTIVE = MODE == kCd;
  constexpr int NCAP = CONTRASTIVE ? 2 : (NM ? (MODE == kMix && NM < 2 ? 2 : NM) : COS_MAX_MODELS);
  constexpr int TU = NCAP <= 4 ? 2 : 1;  // tiles in flight per wavefront
  constexpr int NS = COS_MAX_MODELS + 1;
  __shared__ double s_part[kWaves][NCAP + 1];
  __shared__ int s_flag;
  __shared__ Refine<NCAP> s_rf;

  const RefineTask task = refine_task(p);
  if (task.b < 0) return;
  const int b = task.b;
  const SeqPlan plan = p.plans[b];
  if (plan.redo != kLittleMass) return;  // (no mass: nothing to refine, the second kernel draws from r)
  const int lane = lane_id();
  const int wave = threadIdx.x >> 6;
  const int n = CONTRASTIVE ? 2 : (NM ? NM : p.n);
  const T* rows[NCAP];
#pragma unroll
  for (int m = 0; m < NCAP; ++m) rows[m] = row_ptr<T>(p, m < n ? m : 0, b, plan.jstar);
  float ref[NCAP];
#pragma unroll
  for (int m = 0; m < NCAP; ++m) ref[m] = (MODE != kEns && m < n) ? row_reference<T>(rows[m]) : 0.0f;
  if (threadIdx.x == 0) plan_refine<NCAP, MODE>(p, plan, n, s_rf);
  __syncthreads();
  const Refine<NCAP>& rf = s_rf;

  double Q = 0.0, A[NCAP];
#pragma unroll
  for (int m = 0; m < NCAP; ++m) A[m] = 0.0;
  const int tb = task.tb, te = task.te;
  for (int t = tb + wave; t < te; t += kWaves * TU) {
    float x[TU][NCAP][N];
#pragma unroll
    for (int i = 0; i < TU; ++i) tile_load<T, ALIGNED, NCAP>(p, rows, n, min(t + i * kWaves, te - 1), x[i]);
#pragma unroll
    for (int i = 0; i < TU; ++i) {
      const int ti = t + i * kWaves;
      if (ti < te && ti * 64 + lane < p.nvec)
        refine_sums<T, NCAP, N, MODE>(p, x[i], n, plan.pi, plan.m0, ref, rf, Q, A);
    }
  }
  Q = wave_sum(Q);
  if (lane == 0) s_part[wave][0] = Q;
#pragma unroll
  for (int m = 0; m < NCAP; ++m) {
    const double a = wave_sum(A[m]);
    if (lane == 0) s_part[wave][1 + m] = a;
  }
  __syncthreads();
  HandOff<double>* parts = p.refine_partials + (size_t)(task.slot - task.c) * NS;  // of this sequence
  if (threadIdx.x <= NCAP) {
    double v = 0.0;
    for (int w = 0; w < kWaves; ++w) v += s_part[w][threadIdx.x];
    parts[(size_t)task.c * NS + threadIdx.x].publish(v);
  }
  wait_stores();
  if (!arrive_last(p.counters + ((size_t)(p.nwin + 1) * p.B + b) * kCtrStride, task.cr, &s_flag)) return;

  // last workgroup of the sequence: the workgroups' sums added up (one partial per thread, so that the
  // reads are in flight together; wave_sum adds in a fixed order), Z_t / Z_pi - 1 for every term, then the
  // log-normaliser differences
#pragma unroll
  for (int k = 0; k <= NCAP; ++k) {
    double v = 0.0;
    for (int i = threadIdx.x; i < task.cr; i += kThreads) v += parts[(size_t)i * NS + k].read();
    v = wave_sum(v);
    if (lane == 0) s_part[wave][k] = v;
  }
  __syncthreads();
  if (threadIdx.x < NCAP) {
    const int m = threadIdx.x;
    double q = 0.0, a = 0.0;
    for (int w = 0; w < kWaves; ++w) {
      q += s_part[w][0];
      a += s_part[w][1 + m];
    }
    const double ratio = a / q;
    const bool used = MODE == kEns ? rf.w[m] != 0.0f : m == 0;
    float d = rf.dlse[m];
    // (not finite, or not above -1: models that are not close after all; the streamed value stays)
    if (used && ratio > -1.0 && ratio < INFINITY) d = (float)(log1p(ratio) * 1.4426950408889634);
    p.refine_dlse[(size_t)b * COS_MAX_MODELS + m] = d;
  }
}

// Refinement, second kernel (the same launch shape and split): the tile sums of a marked sequence once
// more -- the residual in its difference form with the first kernel's normaliser differences, or r itself
// where the residual had no mass, or a verifier's own bonus token that the one-read contrastive mode left
// undrawn -- and the draw by the sequence's last workgroup.  The workgroup that finishes the last marked
// sequence empties the list for the next call.
template <typename T, bool ALIGNED, int NM, int MODE>
__global__ void __launch_bounds__(kThreads) refine_draw_kernel(Params p) {
  constexpr int N = VecOf<T>::N;
  constexpr bool CONTRASTIVE = MODE == kCd;
  constexpr int NCAP = CONTRASTIVE ? 2 : (NM ? (MODE == kMix && NM < 2 ? 2 : NM) : COS_MAX_MODELS);
  constexpr int TU = NCAP <= 4 ? 2 : 1;  // tiles in flight per wavefront
  extern __shared__ double tile_sum[];
  __shared__ int s_flag;
  __shared__ Refine<NCAP> s_rf;

  const RefineTask task = refine_task(p);
  if (task.b < 0) return;
  const int b = task.b;
  const SeqPlan plan = p.plans[b];
  const bool little = plan.redo == kLittleMass;
  const int lane = lane_id();
  const int wave = threadIdx.x >> 6;
  const int n = CONTRASTIVE ? 2 : (NM ? NM : p.n);
  const T* rows[NCAP];
#pragma unroll
  for (int m = 0; m < NCAP; ++m) rows[m] = row_ptr<T>(p, m < n ? m : 0, b, plan.jstar);
  float ref[NCAP];
#pragma unroll
  for (int m = 0; m < NCAP; ++m) ref[m] = (MODE != kEns && m < n) ? row_reference<T>(rows[m]) : 0.0f;
  float coef[NCAP], off[NCAP];
  plan_coefficients<NCAP, MODE>(p, plan, little, n, coef, off);  // no mass: the weights of r itself
  if (threadIdx.x == 0) {
    plan_refine<NCAP, MODE>(p, plan, n, s_rf);
    if (little) {
#pragma unroll
      for (int m = 0; m < NCAP; ++m) s_rf.dlse[m] = p.refine_dlse[(size_t)b * COS_MAX_MODELS + m];
    }
  }
  __syncthreads();
  const Refine<NCAP>& rf = s_rf;

  HandOff<double>* sums = p.tile_sums + (size_t)b * p.ntiles;
  const int tb = task.tb, te = task.te;
  for (int t = tb + wave; t < te; t += kWaves * TU) {
    float x[TU][NCAP][N];
#pragma unroll
    for (int i = 0; i < TU; ++i) tile_load<T, ALIGNED, NCAP>(p, rows, n, min(t + i * kWaves, te - 1), x[i]);
#pragma unroll
    for (int i = 0; i < TU; ++i) {
      const int ti = t + i * kWaves;
      float f[N];
      tile_eval<T, NCAP, MODE>(p, x[i], n, min(ti, te - 1), plan.pi, plan.bonus, plan.m0, coef, off, ref, f, little, rf);
      const double ts = wave_sum_to_lane63(lane_mass<N>(f));
      if (lane == 63 && ti < te) tile_sum[ti - tb] = ts;
    }
  }
  __syncthreads();
  for (int i = threadIdx.x; i < te - tb; i += kThreads) sums[tb + i].publish(tile_sum[i]);
  wait_stores();
  if (!arrive_last(p.counters + ((size_t)(p.nwin + 2) * p.B + b) * kCtrStride, task.cr, &s_flag)) return;

  for (int t = threadIdx.x; t < p.ntiles; t += kThreads) tile_sum[t] = sums[t].read();
  __syncthreads();
  int status = kDrawn;
  if (wave == 0)
    status = draw_token<T, ALIGNED, NCAP, MODE>(p, b, plan, rows, n, coef, off, ref, tile_sum, little,
                                                little ? COS_FLAG_RESIDUAL_REFINED
                                                       : (plan.redo == kWholeRow ? 0 : COS_FLAG_RESIDUAL_FALLBACK),
                                                0.0, little, rf);
  if (threadIdx.x == 0) s_flag = status;
  __syncthreads();
  if (s_flag != kDrawn) {
    __syncthreads();
    // The refined residual has no mass either (cannot happen in exact arithmetic): this one workgroup
    // recomputes every tile sum of r itself and draws from that.
    const Refine<NCAP> no_refine = {};
    plan_coefficients<NCAP, MODE>(p, plan, false, n, coef, off);
    for (int t = wave; t < p.ntiles; t += kWaves) {
      float f[N];
      tile_weights<T, ALIGNED, NCAP, MODE>(p, rows, n, t, plan.pi, plan.bonus, plan.m0, coef, off, ref, f, false,
                                           no_refine);
      const double ts = wave_sum(lane_mass<N>(f));
      if (lane == 0) tile_sum[t] = ts;
    }
    __syncthreads();
    if (wave == 0)
      draw_token<T, ALIGNED, NCAP, MODE>(p, b, plan, rows, n, coef, off, ref, tile_sum, false,
                                         COS_FLAG_RESIDUAL_FALLBACK, 0.0, false, no_refine);
  }
  // this sequence is done; whoever finishes the last one leaves the list empty (both control counters at
  // zero, as every arrival counter is left)
  if (threadIdx.x == 0) {
    const unsigned prev = __builtin_amdgcn_atomic_inc32(reinterpret_cast<unsigned*>(p.refine_ctl + kCtrStride),
                                                        (unsigned)(task.count - 1), __ATOMIC_RELAXED, "agent");
    if (prev == (unsigned)(task.count - 1))
      __hip_atomic_store(p.refine_ctl, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
}

// Acceptance-rate kernel (optional): alpha = sum_x min(q(x), r(x)) of Eq. (7) for
// every draft position.  Workgroup index -> (b, j, c); a second full read of the
// draft positions' rows, with the normalisers the streaming kernel left behind.
template <typename T, bool ALIGNED, int NM, int MODE>
__global__ void __launch_bounds__(kThreads) acceptance_rate_kernel(Params p) {
  constexpr int N = VecOf<T>::N;
  constexpr bool CONTRASTIVE = MODE == kCd;
  constexpr int NCAP = CONTRASTIVE ? 2 : (NM ? (MODE == kMix && NM < 2 ? 2 : NM) : COS_MAX_MODELS);
  __shared__ double wsum[kWaves];
  __shared__ int s_flag;

  const int per_b = p.gamma * p.CA;
  const int b = blockIdx.x / per_b;
  int rem = blockIdx.x - b * per_b;
  const int j = rem / p.CA;
  const int c = rem - j * p.CA;
  const int lane = lane_id();
  const int wave = threadIdx.x >> 6;
  const int n = CONTRASTIVE ? 2 : (NM ? NM : p.n);
  const int g1 = p.gamma + 1;
  if (j >= drafts_of(p, b)) {  // no draft at this position: no acceptance rate
    if (c == 0 && threadIdx.x == 0) p.alpha[(size_t)b * p.gamma + j] = NAN;
    return;
  }
  const int pi = __builtin_amdgcn_readfirstlane(p.proposer_pos ? p.proposer_pos[(size_t)b * p.gamma + j] : p.proposer[b]);
  const double* lse = p.lse_all + ((size_t)b * g1 + j) * p.nstat;
  const float m0 = CONTRASTIVE ? p.rowmax_all[(size_t)b * g1 + j] : 0.0f;

  // r = sum_m cr[m] 2^(l_m*scale - off[m]); q = cq 2^(l_pi*scale - off[pi])   (ensemble)
  // r = [mask] cr[0] 2^(c*scale - off[0]);  q = cq 2^(l_pi*scale - off[1])    (contrastive)
  // r = cr[0] 2^(mix*scale - off[0]);       q = cq 2^(l_pi*scale - off[1])    (logit mix)
  float cr[NCAP], off[NCAP], cq = 0.0f;
#pragma unroll
  for (int m = 0; m < NCAP; ++m) {
    cr[m] = 0.0f;
    off[m] = 0.0f;
    if (MODE == kMix ? m < 2 : m < n) {
      const double l2 = CONTRASTIVE ? lse[m == 0 ? 2 : pi] : (MODE == kMix ? lse[m == 0 ? 1 : 0] : lse[m]);
      const double K = rint(l2);
      const double unit = exp2(K - l2);
      off[m] = (float)K;
      if constexpr (CONTRASTIVE || MODE == kMix) {
        if (m == 0) cr[0] = (float)unit; else cq = (float)unit;
      } else {
        cr[m] = (float)(p.w[m] * unit);
        if (m == pi) cq = (float)unit;
      }
    }
  }
  const T* rows[NCAP];
#pragma unroll
  for (int m = 0; m < NCAP; ++m) rows[m] = row_ptr<T>(p, m < n ? m : 0, b, j);
  float ref[NCAP];
#pragma unroll
  for (int m = 0; m < NCAP; ++m) ref[m] = (MODE != kEns && m < n) ? row_reference<T>(rows[m]) : 0.0f;
  float refq = ref[0];  // the proposer row's reference
#pragma unroll
  for (int m = 1; m < NCAP; ++m) refq = (m == pi) ? ref[m] : refq;

  double acc = 0.0;
  const int tb = c * p.tpa;
  const int te = min(tb + p.tpa, p.ntiles);
  for (int t = tb + wave; t < te; t += kWaves) {
    float x[NCAP][N];
    tile_load<T, ALIGNED, NCAP>(p, rows, n, t, x);
    [[maybe_unused]] float d[NCAP][N], cm[N];
    if constexpr (MODE == kMix) mix_shifted_rows<NCAP, N>(p, n, x, ref, true, d, cm);
    if (t * 64 + lane < p.nvec) {
      [[maybe_unused]] float qm[N];
      if constexpr (MODE == kMix) {
#pragma unroll
        for (int m = 0; m < NCAP; ++m)
          if (m == pi) {  // uniform over the workgroup: a scalar branch
#pragma unroll
            for (int k = 0; k < N; ++k) qm[k] = cq * fast_exp2(fmaf(d[m][k], p.scale, -off[1]));
          }
      }
#pragma unroll
      for (int k = 0; k < N; ++k) {
        float r = 0.0f, q = 0.0f;
        if constexpr (MODE == kEns) {
#pragma unroll
          for (int m = 0; m < NCAP; ++m)
            if (m < n) {
              const float e = fast_exp2(fmaf(x[m][k], p.scale, -off[m]));
              r += cr[m] * e;
              if (m == pi) q = cq * e;
            }
        } else if constexpr (MODE == kMix) {
          r = cr[0] * fast_exp2(fmaf(cm[k], p.scale, -off[0]));
          q = qm[k];
        } else {
          const bool in = in_mask<T>(x[0][k], m0, p.thr32, p.thr64);
          const float cc = contrast(x[0][k], x[1][k], p.mu_hi, p.mu_lo, ref[0], ref[1]);
          r = in ? cr[0] * fast_exp2(fmaf(cc, p.scale, -off[0])) : 0.0f;
          q = cq * fast_exp2(fmaf((pi ? x[1][k] : x[0][k]) - refq, p.scale, -off[1]));
        }
        acc += (double)fminf(q, r);
      }
    }
  }
  const double ws = wave_sum(acc);
  if (lane == 0) wsum[wave] = ws;
  __syncthreads();
  HandOff<double>* parts = p.alpha_partials + ((size_t)b * p.gamma + j) * p.CA;
  if (threadIdx.x == 0) {
    double tot = 0.0;
    for (int w = 0; w < kWaves; ++w) tot += wsum[w];
    parts[c].publish(tot);
    wait_stores();
  }
  int* counter = p.counters + ((size_t)(p.nwin + 3) * p.B + 2 + (size_t)b * p.gamma + j) * kCtrStride;
  if (!arrive_last(counter, p.CA, &s_flag)) return;
  if (threadIdx.x == 0) {
    double tot = 0.0;
    for (int i = 0; i < p.CA; ++i) tot += parts[i].read();
    p.alpha[(size_t)b * p.gamma + j] = tot;
  }
}

}  // namespace
