// cos_stats.h -- the streaming kernels: softmax statistics of every logit row
// (Sec. 3.2), the decision of a sequence (Eq. (6), Sec. 3.1) by the workgroup that
// completes it, and the temperature-0 argmax kernel.
#pragma once

#include "cos_device.h"

namespace {

// ---------------------------------------------------------------------------
// streaming softmax statistics (Sec. 3.2)
// ---------------------------------------------------------------------------

// Running statistic of one wavefront: acc lanes hold sum 2^(l*log2e - o) with a
// wave-uniform integer offset o >= ceil(max l * log2e) seen so far.
struct Running {
  int o;
  float acc[4];
};

__device__ __forceinline__ void running_init(Running& r) {
  r.o = kNoOffset;
  r.acc[0] = r.acc[1] = r.acc[2] = r.acc[3] = 0.0f;
}

// Raise the offset to cover a new wave-wide maximum `wm` (wave-uniform).
// Offsets are integers, so the rescale by 2^(old - new) is exact.
__device__ __forceinline__ void running_cover(Running& r, float wm, float scale) {
  if (wm > -INFINITY) {
    float of = ceilf(wm * scale);
    of = fminf(fmaxf(of, -kMaxOffset), kMaxOffset);
    const int on = (int)of;
    if (on > r.o) {
      const int shift = r.o - on;
#pragma unroll
      for (int a = 0; a < 4; ++a) r.acc[a] = ldexpf(r.acc[a], shift);
      r.o = on;
    }
  }
}

__device__ __forceinline__ double running_total(const Running& r) {
  const double z = ((double)r.acc[0] + (double)r.acc[1]) + ((double)r.acc[2] + (double)r.acc[3]);
  return wave_sum(z);
}

template <int U, int N>
__device__ __forceinline__ void running_add(Running& run, const float (&x)[U][N], float scale) {
  float lm = -INFINITY;
#pragma unroll
  for (int u = 0; u < U; ++u)
#pragma unroll
    for (int k = 0; k < N; ++k) lm = fmaxf(lm, x[u][k]);
  running_cover(run, wave_max(lm), scale);
  const float neg_o = -(float)run.o;
#pragma unroll
  for (int u = 0; u < U; ++u)
#pragma unroll
    for (int k = 0; k < N; ++k) run.acc[k & 3] += fast_exp2(fmaf(x[u][k], scale, neg_o));
}

// The same for row `sel` of NR rows held in registers.  `sel` is uniform over the wavefront, so the row
// is chosen by a scalar branch around NR copies of the accumulation instead of a select per element.
template <int NR, int U, int N>
__device__ __forceinline__ void running_add_row(Running& run, const float (&x)[NR][U][N], int sel, float scale) {
  sel = __builtin_amdgcn_readfirstlane(sel);
#pragma unroll
  for (int m = 0; m < NR; ++m)
    if (m == sel) running_add<U, N>(run, x[m], scale);
}

// ---- raw-register variant for 16-byte aligned rows -------------------------
//
// For the 16-bit formats (bf16, binary16: both sign-magnitude) the maximum is taken on
// the raw bit patterns with packed 16-bit
// integer maxima: among non-negative floats integer order equals float order,
// and a pattern with the sign bit set never wins against one without, so
// whenever the wave-wide result is non-negative it is the true maximum;
// otherwise (every element negative) the float path below decides.

typedef short short2_t __attribute__((ext_vector_type(2)));

__device__ __forceinline__ int wave_max_i32(int v) {
#define COS_DPP_IMAX(ctrl, row_mask) \
  v = max(v, __builtin_amdgcn_update_dpp(v, v, ctrl, row_mask, 0xf, false));
  COS_DPP_IMAX(0x111, 0xf)  // row_shr:1
  COS_DPP_IMAX(0x112, 0xf)  // row_shr:2
  COS_DPP_IMAX(0x114, 0xf)  // row_shr:4
  COS_DPP_IMAX(0x118, 0xf)  // row_shr:8
  COS_DPP_IMAX(0x142, 0xa)  // row_bcast:15 into rows 1 and 3
  COS_DPP_IMAX(0x143, 0xc)  // row_bcast:31 into rows 2 and 3
#undef COS_DPP_IMAX
  return __builtin_amdgcn_readlane(v, 63);
}

// U raw vectors per lane starting at `base` (stride kThreads); vectors at or
// past v1 are redirected to the in-range vector v1 - 1 (masked by the caller).
template <typename T, bool ALIGNED, int U>
__device__ __forceinline__ void load_raw_group(const T* __restrict__ row, int base, int v1,
                                               uint4 (&raw)[U]) {
  constexpr int N = VecOf<T>::N;
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const size_t v = (size_t)min(base + u * kThreads + (int)threadIdx.x, v1 - 1);
    raw[u] = ALIGNED ? load_stream16(row + v * N) : load_stream16_unaligned<T>(row + v * N);
  }
}

// The last, partial vector of a row whose length is not a multiple of the vector
// width: its elements one by one, the rest of the vector -inf.
template <typename T>
__device__ __forceinline__ uint4 load_tail_raw(const T* __restrict__ row, int first, int V) {
  constexpr int N = VecOf<T>::N;
  uint32_t w[4];
  if constexpr (sizeof(T) == 4) {
#pragma unroll
    for (int k = 0; k < N; ++k)
      w[k] = (first + k < V) ? __float_as_uint(widen(row[first + k])) : 0xff800000u;
  } else {
    const uint32_t ninf = IsBf16<T>::value ? 0xff80u : 0xfc00u;
    const uint16_t* bits = reinterpret_cast<const uint16_t*>(row);
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const uint32_t lo = (first + 2 * k < V) ? bits[first + 2 * k] : ninf;
      const uint32_t hi = (first + 2 * k + 1 < V) ? bits[first + 2 * k + 1] : ninf;
      w[k] = lo | (hi << 16);
    }
  }
  return make_uint4(w[0], w[1], w[2], w[3]);
}

// Replace vectors at or past v1 by -inf (only the last, partial group needs it).
template <typename T, int U>
__device__ __forceinline__ void mask_raw_group(int base, int v1, uint4 (&raw)[U]) {
  const uint32_t ninf = sizeof(T) == 4 ? 0xff800000u : (IsBf16<T>::value ? 0xff80ff80u : 0xfc00fc00u);
#pragma unroll
  for (int u = 0; u < U; ++u)
    if (base + u * kThreads + (int)threadIdx.x >= v1) raw[u] = make_uint4(ninf, ninf, ninf, ninf);
}

template <typename T, int U>
__device__ __forceinline__ void running_add_raw(Running& run, const uint4 (&raw)[U], float scale) {
  constexpr int N = VecOf<T>::N;
  if constexpr (sizeof(T) == 2) {
    short2_t m = __builtin_bit_cast(short2_t, raw[0].x);
#pragma unroll
    for (int u = 0; u < U; ++u) {
      m = __builtin_elementwise_max(m, __builtin_bit_cast(short2_t, raw[u].x));
      m = __builtin_elementwise_max(m, __builtin_bit_cast(short2_t, raw[u].y));
      m = __builtin_elementwise_max(m, __builtin_bit_cast(short2_t, raw[u].z));
      m = __builtin_elementwise_max(m, __builtin_bit_cast(short2_t, raw[u].w));
    }
    const int wm16 = wave_max_i32(max((int)m.x, (int)m.y));
    if (wm16 >= 0) {
      running_cover(run, raw16_to_float<T>(wm16), scale);
    } else {
      float lm = -INFINITY;
#pragma unroll
      for (int u = 0; u < U; ++u) {
        float x[N];
        unpack<T>(raw[u], x);
#pragma unroll
        for (int k = 0; k < N; ++k) lm = fmaxf(lm, x[k]);
      }
      running_cover(run, wave_max(lm), scale);
    }
  } else {
    float lm = -INFINITY;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      float x[N];
      unpack<T>(raw[u], x);
#pragma unroll
      for (int k = 0; k < N; ++k) lm = fmaxf(lm, x[k]);
    }
    running_cover(run, wave_max(lm), scale);
  }
  const float neg_o = -(float)run.o;
#pragma unroll
  for (int u = 0; u < U; ++u) {
    float x[N];
    unpack<T>(raw[u], x);
#pragma unroll
    for (int k = 0; k < N; ++k) run.acc[k & 3] += fast_exp2(fmaf(x[k], scale, neg_o));
  }
}

// Statistic of vectors [v0, v1) of one row, per wavefront (all lanes return the
// wave's values).
template <typename T, bool ALIGNED>
__device__ __forceinline__ void chunk_stats(const T* __restrict__ row, int v0, int v1, int V,
                                            float scale, int& o_out, double& z_out) {
  constexpr int N = VecOf<T>::N;
  constexpr int kStep = kThreads * kUnroll;
  Running run;
  running_init(run);
  // vectors that lie inside the row; an odd vocabulary leaves one partial vector at its end
  const int vfull = ALIGNED ? v1 : min(v1, V / N);
  // all kUnroll loads of a group are issued before the first use; only the
  // last group of a chunk can be partial
  for (int base = v0; base < vfull; base += kStep) {
    uint4 a[kUnroll];
    load_raw_group<T, ALIGNED, kUnroll>(row, base, vfull, a);
    if (base + kStep > vfull) mask_raw_group<T, kUnroll>(base, vfull, a);
    running_add_raw<T, kUnroll>(run, a, scale);
  }
  if (!ALIGNED && v1 > vfull && threadIdx.x < 64) {
    // the partial vector belongs to this chunk: lane 0 of the first wavefront brings it in
    uint4 a[1];
    const uint32_t ninf = sizeof(T) == 4 ? 0xff800000u : (IsBf16<T>::value ? 0xff80ff80u : 0xfc00fc00u);
    a[0] = threadIdx.x == 0 ? load_tail_raw<T>(row, vfull * N, V) : make_uint4(ninf, ninf, ninf, ninf);
    running_add_raw<T, 1>(run, a, scale);
  }
  o_out = run.o;
  z_out = running_total(run);
}

// Statistics of the wavefronts of a workgroup, combined by thread 0.
struct WaveStat {
  double z;
  int o;
  int pad;
};

// ws is [slots][kWaves]; lane 0 of every wavefront publishes its statistic.
__device__ __forceinline__ void publish_wave_stat(WaveStat* ws, int slot, int o, double z) {
  const int wave = threadIdx.x >> 6;
  if (lane_id() == 0) {
    ws[slot * kWaves + wave].z = z;
    ws[slot * kWaves + wave].o = o;
  }
}

// Thread 0: combine the wavefronts' statistics of one slot and hand the partial
// to the workgroup that will finish the sequence.
__device__ __forceinline__ void store_partial(const WaveStat* ws, int slot, Partial* out) {
  int omax = kNoOffset;
  for (int w = 0; w < kWaves; ++w) {
    const WaveStat& s = ws[slot * kWaves + w];
    if (s.z > 0.0 && s.o > omax) omax = s.o;
  }
  double z = 0.0;
  for (int w = 0; w < kWaves; ++w) {
    const WaveStat& s = ws[slot * kWaves + w];
    if (s.z > 0.0) z += ldexp(s.z, s.o - omax);
  }
  out->Z.publish(z);
  out->o.publish(omax);
}

__device__ __forceinline__ void store_empty_partial(Partial* out) {
  out->Z.publish(0.0);
  out->o.publish(kNoOffset);
}

// ---------------------------------------------------------------------------
// decide one sequence (runs in the workgroup that arrived last on its counter)
// ---------------------------------------------------------------------------

struct DecideShared {
  double lse2[kMaxStatsPerSeq];     // log2-sum-exp2 per (position, statistic)
  float rowmax[COS_MAX_GAMMA + 1];  // contrastive: expert maximum per position
  int accept[COS_MAX_GAMMA + 1];
  // the outcome (written by thread 0 of decide_outcome): -1 = every draft of the window accepted and the
  // bonus position is not in it
  int jstar, residual, pi, bonus, skip;
};

// What one thread brings in for its draft position before the statistics are combined: the draft
// token, its proposer, its uniform, the n logits at the token and the rows' references.
struct DraftGather {
  int d, pi;
  double u_acc;
  double lgat[COS_MAX_MODELS], rgat[COS_MAX_MODELS];
};

// Thread tid < ndraft gathers for position j0 + tid.  These loads do not depend on the statistics, so
// they go out first and their latency (draft token, then the n logits at it) overlaps the combine.
// Two steps, so that a caller can put other loads between them: the side arrays, then -- once the
// draft token is there -- the logits at it.
__device__ __forceinline__ void gather_drafts_side(const Params& p, int b, int ndraft, DraftGather& g) {
  const int tid = threadIdx.x;
  g.d = 0;
  g.pi = 0;
  g.u_acc = 0.0;
#pragma unroll
  for (int m = 0; m < COS_MAX_MODELS; ++m) g.lgat[m] = g.rgat[m] = 0.0;
  if (tid < ndraft) {
    const size_t k = (size_t)b * p.gamma + p.j0 + tid;
    g.d = p.draft[k];
    g.pi = p.proposer_pos ? p.proposer_pos[k] : p.proposer[b];
    g.u_acc = p.u_accept[k];
  }
}

template <typename T, int MODE>
__device__ __forceinline__ void gather_drafts_logits(const Params& p, int b, int ndraft, DraftGather& g) {
  const int tid = threadIdx.x;
  if (tid < ndraft) {
    const int j = p.j0 + tid;
#pragma unroll
    for (int m = 0; m < COS_MAX_MODELS; ++m)
      if (m < p.n) {
        const T* row = row_ptr<T>(p, m, b, j);
        g.lgat[m] = (double)widen(row[g.d]);
        if constexpr (MODE != kEns) g.rgat[m] = (double)row_reference<T>(row);
      }
  }
}

template <typename T, int MODE>
__device__ __forceinline__ void gather_drafts(const Params& p, int b, int ndraft, DraftGather& g) {
  gather_drafts_side(p, b, ndraft, g);
  gather_drafts_logits<T, MODE>(p, b, ndraft, g);
}

// Combine the chunk partials of every (position, statistic) of the window in float64 into sh.lse2.
// A group of G lanes (a power of two >= S, at most a wavefront) shares the S partials of one
// statistic, so that a row cut into many chunks (small batches) costs a few dependent loads, not S
// of them; with whole rows (S = 1) it is one thread per statistic.
__device__ __forceinline__ void combine_partials(const Params& p, int b, DecideShared& sh) {
  const int tid = threadIdx.x;
  const int g1 = p.gamma + 1;
  const int nstat = p.nstat;
  const int j0 = p.j0;
  const int nrows = p.nj * nstat;  // statistics of this window
  const int Sb = splits_of(p, b);  // chunks per row of this sequence
  int G = 1;
  while (G < Sb && G < 64) G <<= 1;
  const int per_pass = kThreads / G;
  const int gl = tid & (G - 1);
  for (int r0 = 0; r0 < nrows; r0 += per_pass) {  // uniform trip count: every lane shuffles
    const int r = r0 + tid / G;
    int omax = kNoOffset;
    double zsum = 0.0;  // sum of Z 2^(o - omax) over the partials seen by this lane
    if (r < nrows) {
      const Partial* pp = p.partials + (((size_t)b * g1 + j0) * nstat + r) * p.S;
      for (int s = gl; s < Sb; s += G) {
        const double z = pp[s].Z.read();
        const int o = pp[s].o.read();
        if (z > 0.0) {
          if (o > omax) {
            zsum = ldexp(zsum, omax - o);  // exact: a power of two
            omax = o;
          }
          zsum += ldexp(z, o - omax);
        }
      }
    }
    for (int span = G >> 1; span >= 1; span >>= 1) {
      const int oo = __shfl_xor(omax, span, 64);
      const double zz = __shfl_xor(zsum, span, 64);
      const int om = max(omax, oo);
      zsum = (zsum > 0.0 ? ldexp(zsum, omax - om) : 0.0) + (zz > 0.0 ? ldexp(zz, oo - om) : 0.0);
      omax = om;
    }
    if (r < nrows && gl == 0) sh.lse2[r] = (zsum > 0.0) ? (double)omax + log2(zsum) : -INFINITY;
  }
}

// A logit minus its row's reference exactly as the streaming kernels take it: in float32.  For logits of
// large magnitude that subtraction rounds (1e-7 of the difference), and the statistics were summed over
// the rounded values, so what is normalised by them must be those same values: then a token that
// holds nearly all of a row's mass gets its probability to 1e-7 of its small complement, not of itself.
__device__ __forceinline__ double shifted(double logit, double ref) { return (double)((float)logit - (float)ref); }

// Eq. (6) for every draft position of the window (float64), the first rejection (Sec. 3.1), the
// accepted prefix and the padding, and the plan for the draw.  sh.lse2 and (contrastive) sh.rowmax
// must be complete and visible (a barrier after they were written).  The sequence stays undecided
// (sh.jstar = -1) if every draft of the window is accepted and the window does not contain the
// bonus position.  The outcome is in sh after the caller's next barrier.
template <typename T, int MODE>
__device__ __forceinline__ void decide_outcome(const Params& p, int b, DecideShared& sh, const DraftGather& g,
                                               int ndraft) {
  constexpr bool CONTRASTIVE = MODE == kCd;
  const int tid = threadIdx.x;
  const int g1 = p.gamma + 1;
  const int nstat = p.nstat;
  const int j0 = p.j0, nj = p.nj;
  const int nrows = nj * nstat;
  const int n = p.n;
  const int gb = drafts_of(p, b);
  const double log2e = (double)p.scale;  // log2(e) / T, the same constant the streaming kernel used
  if (tid >= ndraft && tid < nj && j0 + tid < p.gamma) {  // no draft here
    if (p.diag.r_at_draft) p.diag.r_at_draft[(size_t)b * p.gamma + j0 + tid] = NAN;
    if (p.diag.q_at_draft) p.diag.q_at_draft[(size_t)b * p.gamma + j0 + tid] = NAN;
  }
  if (tid < ndraft) {
    const int jj = tid;
    const int pi = g.pi;
    const size_t k = (size_t)b * p.gamma + j0 + tid;
    double rd = 0.0, qd = 0.0;
    if constexpr (MODE == kMix) {
      // statistic 0: the proposer's row; statistic 1: the mixed logits; both on logits
      // shifted by the row references, as the statistics were
      double c = 0.0, lq = 0.0;
#pragma unroll
      for (int m = 0; m < COS_MAX_MODELS; ++m)
        if (m < n) {
          const double v = shifted(g.lgat[m], g.rgat[m]);
          if (p.w[m] != 0.0) c += p.w[m] * v;
          lq = (m == pi) ? v : lq;
        }
      rd = exp2(c * log2e - sh.lse2[jj * nstat + 1]);
      qd = exp2(lq * log2e - sh.lse2[jj * nstat + 0]);
    } else if constexpr (MODE == kEns) {
#pragma unroll
      for (int m = 0; m < COS_MAX_MODELS; ++m)
        if (m < n) {
          const double s = exp2(g.lgat[m] * log2e - sh.lse2[jj * nstat + m]);
          rd += p.w[m] * s;
          qd = (m == pi) ? s : qd;
        }
    } else {
      const double l0 = g.lgat[0], l1 = g.lgat[1];
      const bool in = (l0 > -INFINITY) && (l0 - (double)sh.rowmax[jj] >= p.thr64);
      // on logits shifted by the row references, as both statistics were
      const double d0 = shifted(l0, g.rgat[0]);
      const double d1 = shifted(l1, g.rgat[1]);
      const double c = d0 - p.w[0] * d1;
      rd = in ? exp2(c * log2e - sh.lse2[jj * nstat + 2]) : 0.0;
      qd = exp2((pi ? d1 : d0) * log2e - sh.lse2[jj * nstat + pi]);
    }
    double ratio;
    if (!(rd > 0.0))
      ratio = 0.0;
    else if (!(qd > 0.0))
      ratio = INFINITY;
    else
      ratio = rd / qd;
    const double bound = ratio < 1.0 ? ratio : 1.0;
    sh.accept[jj] = g.u_acc < bound;
    if (p.diag.r_at_draft) p.diag.r_at_draft[k] = rd;
    if (p.diag.q_at_draft) p.diag.q_at_draft[k] = qd;
  }
  __syncthreads();
  if (p.alpha) {
    if (tid < nrows) p.lse_all[((size_t)b * g1 + j0) * nstat + tid] = sh.lse2[tid];
    if (CONTRASTIVE && tid < nj) p.rowmax_all[(size_t)b * g1 + j0 + tid] = sh.rowmax[tid];
  }

  // first rejection (Sec. 3.1) inside the window; -1: none, and the bonus position is not in it
  int jstar = (j0 + nj > gb) ? gb : -1;
  for (int jj = ndraft - 1; jj >= 0; --jj)
    if (!sh.accept[jj]) jstar = j0 + jj;
  if (jstar < 0) {  // undecided: a later window continues
    if (tid == 0) {
      sh.jstar = -1;
      p.plans[b].jstar = -1;
    }
    return;
  }

  // the drawn token's slot is filled by whoever draws, unless nothing is drawn
  const bool skip = p.no_bonus && jstar == gb;
  if (tid == 0) p.accepted_len[b] = jstar;
  if (tid < g1 && (tid != jstar || skip))
    p.out_tokens[(size_t)b * g1 + tid] = (tid < jstar) ? p.draft[(size_t)b * p.gamma + tid] : -1;

  // plan for the draw
  SeqPlan* plan = p.plans + b;
  if (tid == 0) {
    const bool residual = jstar < gb;
    plan->jstar = jstar;
    plan->residual = residual;
    plan->pi = (residual && p.proposer_pos) ? p.proposer_pos[(size_t)b * p.gamma + jstar] : p.proposer[b];
    plan->bonus = (!residual && p.bonus_idx) ? p.bonus_idx[b] : -1;
    plan->m0 = (CONTRASTIVE && !skip) ? sh.rowmax[jstar - j0] : 0.0f;
    plan->skip = skip;
    plan->redo = 0;
    sh.jstar = jstar;
    sh.residual = residual;
    sh.pi = plan->pi;
    sh.bonus = plan->bonus;
    sh.skip = skip;
    if (skip) {
      if (p.diag.sample_mass) p.diag.sample_mass[b] = 0.0;
      if (p.diag.cdf_lo) p.diag.cdf_lo[b] = 0.0;
      if (p.diag.cdf_hi) p.diag.cdf_hi[b] = 0.0;
      if (p.diag.flags) p.diag.flags[b] = 0;
    }
  }
  if (tid < nstat && !skip) plan->lse2[tid] = sh.lse2[(jstar - j0) * nstat + tid];
}

// Decides the window [j0, j0+nj) of a sequence that no earlier window has decided (runs in the
// workgroup that arrived last on the sequence's counter).
template <typename T, int MODE>
__device__ void decide_sequence(const Params& p, int b, DecideShared& sh) {
  const int tid = threadIdx.x;
  const int g1 = p.gamma + 1;
  const int gb = drafts_of(p, b);
  const int ndraft = max(min(p.j0 + p.nj, gb) - p.j0, 0);  // draft positions in the window
  DraftGather g;
  gather_drafts<T, MODE>(p, b, ndraft, g);
  combine_partials(p, b, sh);
  if (MODE == kCd && tid < p.nj) {
    // written by the row-max kernel, an earlier launch on the same stream
    const int Sb = splits_of(p, b);
    const float* rm = p.rowmax + ((size_t)b * g1 + p.j0 + tid) * p.S;
    float m0 = -INFINITY;
    for (int s = 0; s < Sb && p.masked; ++s) m0 = fmaxf(m0, rm[s]);
    sh.rowmax[tid] = p.masked ? m0 : 0.0f;
  }
  __syncthreads();
  decide_outcome<T, MODE>(p, b, sh, g, ndraft);
}

// ---------------------------------------------------------------------------
// kernels
// ---------------------------------------------------------------------------

// Zeroes the arrival counters and marks every sequence undecided.
__global__ void __launch_bounds__(kThreads) fill_zero_kernel(int* dst, int count, SeqPlan* plans, int B) {
  const int i = blockIdx.x * kThreads + threadIdx.x;
  if (i < count) dst[i] = 0;
  if (i < B) plans[i].jstar = -1;
}

// Ensemble streaming kernel.  Workgroup index -> (b, j, m, s), b slowest.
template <typename T, bool ALIGNED>
__global__ void __launch_bounds__(kThreads) ensemble_stats_kernel(Params p) {
  __shared__ WaveStat ws[kWaves];
  __shared__ DecideShared sh;
  __shared__ int s_flag;

  const int g1 = p.gamma + 1;
  const Place pl = place_of(p, p.nj * p.n);
  const int b = pl.b, per_b = pl.per_b;
  if (p.win > 0 && p.plans[b].jstar >= 0) return;  // decided by an earlier window: nothing more is read
  int rem = pl.rem;
  const int jj = rem / (p.n * pl.S);
  rem -= jj * p.n * pl.S;
  const int j = p.j0 + jj;
  const int m = rem / pl.S;
  const int s = rem - m * pl.S;

  Partial* out = p.partials + (((size_t)b * g1 + j) * p.n + m) * p.S + s;
  // With a verifier bonus the other models' logits at the bonus position are
  // not needed (they may not exist yet) and are not read.
  const int gb = drafts_of(p, b);
  const int only = (p.bonus_idx && j == gb) ? p.bonus_idx[b] : -1;
  if ((only >= 0 && m != only) || position_unread(p, gb, j)) {
    if (threadIdx.x == 0) {
      store_empty_partial(out);
      wait_stores();
    }
  } else {
    const T* row = row_ptr<T>(p, m, b, j);
    const int v0 = s * pl.cv;
    const int v1 = min(v0 + pl.cv, p.nvec);
    int o;
    double z;
    chunk_stats<T, ALIGNED>(row, v0, v1, p.V, p.scale, o, z);
    publish_wave_stat(ws, 0, o, z);
    __syncthreads();
    if (threadIdx.x == 0) {
      store_partial(ws, 0, out);
      wait_stores();
    }
  }
  if (arrive_last(p.counters + ((size_t)p.win * p.B + b) * kCtrStride, per_b, &s_flag))
    decide_sequence<T, kEns>(p, b, sh);
}

// Contrastive, kernel 1: partial maxima of the expert row (model 0).
template <typename T, bool ALIGNED>
__global__ void __launch_bounds__(kThreads) expert_rowmax_kernel(Params p) {
  constexpr int N = VecOf<T>::N;
  constexpr int kStep = kThreads * kUnroll;
  __shared__ float wmax[kWaves];
  const int g1 = p.gamma + 1;
  if (p.win == 0 && p.fill_count > 0) {
    // the first kernel of the call: nothing has used the counters or the plans yet, and the
    // kernels that do start after this one has ended
    for (int i = blockIdx.x * kThreads + threadIdx.x; i < p.fill_count; i += gridDim.x * kThreads) p.counters[i] = 0;
    for (int i = blockIdx.x * kThreads + threadIdx.x; i < p.B; i += gridDim.x * kThreads) p.plans[i].jstar = -1;
  }
  const Place pl = place_of(p, p.nj);
  const int b = pl.b;
  const int j = p.j0 + pl.rem / pl.S;
  const int s = pl.rem - (j - p.j0) * pl.S;
  if (p.win > 0 && p.plans[b].jstar >= 0) return;  // decided by an earlier window
  const int rs = b * g1 + j;
  if (position_unread(p, drafts_of(p, b), j)) {
    if (threadIdx.x == 0) p.rowmax[(size_t)rs * p.S + s] = -INFINITY;
    return;
  }
  const T* row = row_ptr<T>(p, 0, b, j);
  const int v0 = s * pl.cv;
  const int v1 = min(v0 + pl.cv, p.nvec);
  float lm = -INFINITY;
  for (int base = v0; base < v1; base += kStep) {
    float x[kUnroll][N];
    if (base + kStep <= v1)
      load_group<T, ALIGNED, false, kUnroll>(row, base, v1, p.V, x);
    else
      load_group<T, ALIGNED, true, kUnroll>(row, base, v1, p.V, x);
#pragma unroll
    for (int u = 0; u < kUnroll; ++u)
#pragma unroll
      for (int k = 0; k < N; ++k) lm = fmaxf(lm, x[u][k]);
  }
  const float wm = wave_max(lm);
  if (lane_id() == 0) wmax[threadIdx.x >> 6] = wm;
  __syncthreads();
  if (threadIdx.x == 0) {
    float mx = wmax[0];
    for (int w = 1; w < kWaves; ++w) mx = fmaxf(mx, wmax[w]);
    p.rowmax[(size_t)rs * p.S + s] = mx;
  }
}

// Contrastive, kernel 2.  Workgroup index -> (b, j, s); reads the chunk of both
// rows once and produces the proposer row's softmax statistic and the masked
// statistic of the contrastive logits (Eq. (5) restricted to the mask).
template <typename T, bool ALIGNED, bool MASKED>
__global__ void __launch_bounds__(kThreads) contrastive_stats_kernel(Params p) {
  constexpr int N = VecOf<T>::N;
  constexpr int U = kUnroll >= 2 ? kUnroll / 2 : 1;
  constexpr int kStep = kThreads * U;
  __shared__ WaveStat ws[2 * kWaves];
  __shared__ DecideShared sh;
  __shared__ int s_flag;
  __shared__ float s_m0[kWaves];

  const int g1 = p.gamma + 1;
  const Place pl = place_of(p, p.nj);
  const int b = pl.b, per_b = pl.per_b;
  if (p.win > 0 && p.plans[b].jstar >= 0) return;  // decided by an earlier window: nothing more is read
  const int j = p.j0 + pl.rem / pl.S;
  const int s = pl.rem - (j - p.j0) * pl.S;
  const int tid = threadIdx.x;
  // Whose softmax statistic this position needs: the proposer's at a draft
  // position; at the bonus position only a verifier bonus needs one at all.
  const int gb = drafts_of(p, b);
  int pi = p.proposer[b];
  if (j < gb) {
    if (p.proposer_pos) pi = p.proposer_pos[(size_t)b * p.gamma + j];
  } else if (p.bonus_idx && p.bonus_idx[b] >= 0) {
    pi = p.bonus_idx[b];
  }
  if (position_unread(p, gb, j)) {  // uniform over the workgroup
    if (tid == 0) {
      Partial* out = p.partials + (((size_t)b * g1 + j) * 3) * p.S + s;
      store_empty_partial(out);
      store_empty_partial(out + (size_t)p.S);
      store_empty_partial(out + (size_t)2 * p.S);
      wait_stores();
    }
    if (arrive_last(p.counters + ((size_t)p.win * p.B + b) * kCtrStride, per_b, &s_flag))
      decide_sequence<T, kCd>(p, b, sh);
    return;
  }

  // expert maximum of this position from the row-max kernel's partial maxima
  {
    const float* rm = p.rowmax + ((size_t)b * g1 + j) * p.S;
    float lm = -INFINITY;
    for (int i = tid; i < pl.S && MASKED; i += kThreads) lm = fmaxf(lm, rm[i]);
    const float wm = wave_max(lm);
    if (lane_id() == 0) s_m0[tid >> 6] = wm;
    __syncthreads();
  }
  float m0 = s_m0[0];
  for (int w = 1; w < kWaves; ++w) m0 = fmaxf(m0, s_m0[w]);
  if (!MASKED) m0 = 0.0f;  // no mask: every finite expert logit is in

  const T* row0 = row_ptr<T>(p, 0, b, j);
  const T* row1 = row_ptr<T>(p, 1, b, j);
  const float ref0 = row_reference<T>(row0), ref1 = row_reference<T>(row1);
  const int v0 = s * pl.cv;
  const int v1 = min(v0 + pl.cv, p.nvec);
  Running rq, rc;  // proposer row; masked contrastive logits
  running_init(rq);
  running_init(rc);
  for (int base = v0; base < v1; base += kStep) {
    float x[2][U][N];
    if (base + kStep <= v1) {
      load_group<T, ALIGNED, false, U>(row0, base, v1, p.V, x[0]);
      load_group<T, ALIGNED, false, U>(row1, base, v1, p.V, x[1]);
    } else {
      load_group<T, ALIGNED, true, U>(row0, base, v1, p.V, x[0]);
      load_group<T, ALIGNED, true, U>(row1, base, v1, p.V, x[1]);
    }
    float c[U][N];
    if constexpr (!MASKED) {
      // Eq. (5) as printed, no mask: the rows are shifted in place and c comes straight from them.  An
      // expert logit of -inf gives c = -inf by itself unless the amateur's is not finite either; only a
      // group in which some c comes out NaN or +inf pays for the explicit test.
      bool odd = false;
#pragma unroll
      for (int u = 0; u < U; ++u)
#pragma unroll
        for (int k = 0; k < N; ++k) {
          x[0][u][k] -= ref0;
          x[1][u][k] -= ref1;
          c[u][k] = fmaf(-p.mu_lo, x[1][u][k], fmaf(-p.mu_hi, x[1][u][k], x[0][u][k]));
          odd = odd || !(c[u][k] < INFINITY);
        }
      if (__ballot(odd)) {
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
          for (int k = 0; k < N; ++k) c[u][k] = (x[0][u][k] > -INFINITY) ? c[u][k] : -INFINITY;
      }
      // the proposer's statistic on the same shifted logits: with mu = 0 and the expert proposing,
      // r and q see the very same numbers and cancel exactly
      running_add_row<2, U, N>(rq, x, pi, p.scale);
      running_add<U, N>(rc, c, p.scale);
    } else {
      // proposer row statistic, on the shifted logits like the contrastive one
      float xq[U][N];
      const float refq = pi ? ref1 : ref0;
#pragma unroll
      for (int u = 0; u < U; ++u)
#pragma unroll
        for (int k = 0; k < N; ++k) xq[u][k] = (pi ? x[1][u][k] : x[0][u][k]) - refq;
      running_add<U, N>(rq, xq, p.scale);
      // masked contrastive statistic; the mask is sparse, so skip wave-wide when empty
      float lmc = -INFINITY;
#pragma unroll
      for (int u = 0; u < U; ++u)
#pragma unroll
        for (int k = 0; k < N; ++k) {
          const bool in = in_mask<T>(x[0][u][k], m0, p.thr32, p.thr64);
          c[u][k] = in ? contrast(x[0][u][k], x[1][u][k], p.mu_hi, p.mu_lo, ref0, ref1) : -INFINITY;
          lmc = fmaxf(lmc, c[u][k]);
        }
      if (__ballot(lmc > -INFINITY)) running_add<U, N>(rc, c, p.scale);
    }
  }
  const double zq = running_total(rq);
  const double zc = running_total(rc);
  publish_wave_stat(ws, 0, rq.o, zq);
  publish_wave_stat(ws, 1, rc.o, zc);
  __syncthreads();
  if (tid == 0) {
    Partial* out = p.partials + (((size_t)b * g1 + j) * 3) * p.S;
    store_partial(ws, 0, out + (size_t)pi * p.S + s);
    store_empty_partial(out + (size_t)(1 - pi) * p.S + s);
    store_partial(ws, 1, out + (size_t)2 * p.S + s);
    wait_stores();
  }
  if (arrive_last(p.counters + ((size_t)p.win * p.B + b) * kCtrStride, per_b, &s_flag))
    decide_sequence<T, kCd>(p, b, sh);
}

// Logit mix streaming kernel.  Workgroup index -> (b, j, s); reads the chunk of
// all n rows once and produces the proposer row's softmax statistic
// (statistic 0) and the statistic of the mixed logits sum_m beta_m l_m
// (statistic 1; Eq. (3), logit level).
template <typename T, bool ALIGNED, int NM>
__global__ void __launch_bounds__(kThreads) mix_stats_kernel(Params p) {
  constexpr int N = VecOf<T>::N;
  constexpr int NCAP = NM ? NM : COS_MAX_MODELS;
  constexpr int U = NCAP <= 2 ? 4 : (NCAP <= 4 ? 2 : 1);  // vectors per lane and row in flight
  constexpr int kStep = kThreads * U;
  __shared__ WaveStat ws[2 * kWaves];
  __shared__ DecideShared sh;
  __shared__ int s_flag;

  const int n = NM ? NM : p.n;
  const int g1 = p.gamma + 1;
  const Place pl = place_of(p, p.nj);
  const int b = pl.b, per_b = pl.per_b;
  if (p.win > 0 && p.plans[b].jstar >= 0) return;  // decided by an earlier window: nothing more is read
  const int j = p.j0 + pl.rem / pl.S;
  const int s = pl.rem - (j - p.j0) * pl.S;
  const int tid = threadIdx.x;
  const int gb = drafts_of(p, b);
  // Whose softmax statistic this position needs: the proposer's at a draft
  // position; at the bonus position only a verifier bonus needs one, and then
  // the mixed logits are not needed.
  int pi = p.proposer[b];
  bool plain = false;
  if (j < gb) {
    if (p.proposer_pos) pi = p.proposer_pos[(size_t)b * p.gamma + j];
  } else if (p.bonus_idx && p.bonus_idx[b] >= 0) {
    pi = p.bonus_idx[b];
    plain = true;
  }
  Partial* out = p.partials + (((size_t)b * g1 + j) * 2) * p.S + s;
  if (position_unread(p, gb, j)) {  // uniform over the workgroup
    if (tid == 0) {
      store_empty_partial(out);
      store_empty_partial(out + (size_t)p.S);
      wait_stores();
    }
    if (arrive_last(p.counters + ((size_t)p.win * p.B + b) * kCtrStride, per_b, &s_flag))
      decide_sequence<T, kMix>(p, b, sh);
    return;
  }

  const T* rows[NCAP];
#pragma unroll
  for (int m = 0; m < NCAP; ++m) rows[m] = row_ptr<T>(p, m < n ? m : 0, b, j);
  float ref[NCAP];
#pragma unroll
  for (int m = 0; m < NCAP; ++m) ref[m] = m < n ? row_reference<T>(rows[m]) : 0.0f;
  const int v0 = s * pl.cv;
  const int v1 = min(v0 + pl.cv, p.nvec);
  Running rq, rc;  // proposer row; mixed logits
  running_init(rq);
  running_init(rc);
  for (int base = v0; base < v1; base += kStep) {
    float x[NCAP][U][N];
    if (base + kStep <= v1) {
#pragma unroll
      for (int m = 0; m < NCAP; ++m)
        if (m < n) load_group<T, ALIGNED, false, U>(rows[m], base, v1, p.V, x[m]);
    } else {
#pragma unroll
      for (int m = 0; m < NCAP; ++m)
        if (m < n) load_group<T, ALIGNED, true, U>(rows[m], base, v1, p.V, x[m]);
    }
    // The rows are shifted in place; c = sum_m beta_m d_m in model order with the two multiply-adds per
    // model of mix_one.  A model with beta_m = 0 adds 0 * d_m = 0 when d_m is finite; a -inf (or
    // non-finite) logit shows as a c that is not finite, and only such a group pays for mix_one's tests.
    float c[U][N];
    bool odd = false;
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int k = 0; k < N; ++k) {
        float acc = 0.0f;
#pragma unroll
        for (int m = 0; m < NCAP; ++m)
          if (m < n) {
            x[m][u][k] -= ref[m];
            acc = fmaf(p.beta_lo[m], x[m][u][k], fmaf(p.beta_hi[m], x[m][u][k], acc));
          }
        c[u][k] = acc;
        odd = odd || !(fabsf(acc) < INFINITY);
      }
    // shifted like the mixed logits: a one-hot mix on the proposer cancels exactly
    running_add_row<NCAP, U, N>(rq, x, pi, p.scale);
    if (!plain) {
      if (__ballot(odd)) {
        const float zero[NCAP] = {};
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
          for (int k = 0; k < N; ++k) {
            float l[NCAP];
#pragma unroll
            for (int m = 0; m < NCAP; ++m) l[m] = x[m][u][k];
            c[u][k] = mix_one<NCAP>(p, n, l, zero);  // -inf stays -inf under the shift
          }
      }
      running_add<U, N>(rc, c, p.scale);
    }
  }
  const double zq = running_total(rq);
  const double zc = running_total(rc);
  publish_wave_stat(ws, 0, rq.o, zq);
  publish_wave_stat(ws, 1, rc.o, zc);
  __syncthreads();
  if (tid == 0) {
    store_partial(ws, 0, out);
    if (plain)
      store_empty_partial(out + (size_t)p.S);
    else
      store_partial(ws, 1, out + (size_t)p.S);
    wait_stores();
  }
  if (arrive_last(p.counters + ((size_t)p.win * p.B + b) * kCtrStride, per_b, &s_flag))
    decide_sequence<T, kMix>(p, b, sh);
}

// Temperature 0 (greedy), logit-level modes.  r is one-hot at a_j -- the masked
// argmax of c = l_0 - mu l_1 (Eq. (5)), or the argmax of c = sum_m beta_m l_m
// (Eq. (3), linear) -- so a draft is accepted iff d_j == a_j and the token drawn at
// the first mismatch (or the bonus token) is a_j itself: one streaming argmax per
// position, no sampling kernel, no random numbers.  c is evaluated in float64 with
// separate multiplies and adds so that every comparison is the one a float64
// reference makes; ties go to the lowest index.  Workgroup index -> (b, j, s).
// With a verifier bonus the bonus position takes the plain argmax of that model's row.
struct ArgBest {
  double val;
  int idx;  // -1: nothing eligible seen
};

__device__ __forceinline__ void arg_better(ArgBest& a, double val, int idx) {
  if (idx >= 0 && (a.idx < 0 || val > a.val || (val == a.val && idx < a.idx))) {
    a.val = val;
    a.idx = idx;
  }
}

// One lane's candidate: element `idx` with value `val` is taken if eligible, in
// range and larger than what the lane holds (ascending idx per lane, so strict).
__device__ __forceinline__ void arg_take(ArgBest& best, double val, int idx, bool eligible) {
  if (eligible && (best.idx < 0 || val > best.val)) {
    best.val = val;
    best.idx = idx;
  }
}

// A value of a plain row (or of a mix) is eligible unless it is NaN; a row of -inf
// still has an argmax, its first element.
__device__ __forceinline__ bool arg_plain_ok(const ArgBest& best, double val) {
  return val > -INFINITY || (best.idx < 0 && val == -INFINITY);
}

// Lanes -> wavefront -> workgroup -> the chunk's partial, then the arrival: true in the workgroup
// that completes the sequence.
__device__ __forceinline__ bool greedy_arrive(const Params& p, int b, ArgBest best, Partial* out, int per_b,
                                              ArgBest* wbest, int* s_flag) {
  const int tid = threadIdx.x;
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) {
    const double ov = __shfl_xor(best.val, d, 64);
    const int oi = __shfl_xor(best.idx, d, 64);
    arg_better(best, ov, oi);
  }
  if (lane_id() == 0) wbest[tid >> 6] = best;
  __syncthreads();
  if (tid == 0) {
    ArgBest bb = wbest[0];
    for (int w = 1; w < kWaves; ++w) arg_better(bb, wbest[w].val, wbest[w].idx);
    out->Z.publish(bb.val);
    out->o.publish(bb.idx);
    wait_stores();
  }
  return arrive_last(p.counters + (size_t)b * kCtrStride, per_b, s_flag);
}

// The argmax of statistic `stat` from its chunk partials (read by one thread).
__device__ __forceinline__ int greedy_combine(const Params& p, int b, int stat) {
  const Partial* pp = p.partials + ((size_t)b * (p.gamma + 1) * p.nstat + stat) * p.S;
  const int Sb = splits_of(p, b);
  ArgBest bb;
  bb.val = 0.0;
  bb.idx = -1;
  for (int i = 0; i < Sb; ++i) arg_better(bb, pp[i].Z.read(), pp[i].o.read());
  return bb.idx;
}

// r is one-hot at the argmax of every position: first mismatch, outputs.
__device__ __forceinline__ void greedy_decide_one_hot(const Params& p, int b, int gb, int* s_arg) {
  const int tid = threadIdx.x;
  const int g1 = p.gamma + 1;
  if (tid < g1) s_arg[tid] = greedy_combine(p, b, tid * p.nstat);
  __syncthreads();
  int jstar = gb;
  for (int jj = gb - 1; jj >= 0; --jj)
    if (p.draft[(size_t)b * p.gamma + jj] != s_arg[jj]) jstar = jj;
  const bool skip = p.no_bonus && jstar == gb;  // every draft accepted, no extra token
  if (tid == 0) p.accepted_len[b] = jstar;
  if (tid < g1)
    p.out_tokens[(size_t)b * g1 + tid] =
        tid < jstar ? p.draft[(size_t)b * p.gamma + tid] : ((tid == jstar && !skip) ? s_arg[jstar] : -1);
}

__device__ __forceinline__ void greedy_finish(const Params& p, int b, int gb, ArgBest best, Partial* out,
                                              int per_b, ArgBest* wbest, int* s_flag, int* s_arg) {
  if (greedy_arrive(p, b, best, out, per_b, wbest, s_flag)) greedy_decide_one_hot(p, b, gb, s_arg);
}

template <typename T, bool ALIGNED>
__global__ void __launch_bounds__(kThreads) greedy_contrastive_kernel(Params p) {
  constexpr int N = VecOf<T>::N;
  constexpr int U = 4;
  constexpr int kStep = kThreads * U;
  __shared__ ArgBest wbest[kWaves];
  __shared__ float s_m0[kWaves];
  __shared__ int s_flag;
  __shared__ int s_arg[COS_MAX_GAMMA + 1];

  const int g1 = p.gamma + 1;
  const Place pl = place_of(p, g1);
  const int b = pl.b, per_b = pl.per_b;
  const int j = pl.rem / pl.S;
  const int s = pl.rem - j * pl.S;
  const int tid = threadIdx.x;
  const int gb = drafts_of(p, b);
  const bool unread = position_unread(p, gb, j);
  const int plain = (j == gb && p.bonus_idx) ? p.bonus_idx[b] : -1;
  const double mu = p.w[0];

  {
    const float* rm = p.rowmax + ((size_t)b * g1 + j) * p.S;
    float lm = -INFINITY;
    for (int i = tid; i < pl.S && p.masked; i += kThreads) lm = fmaxf(lm, rm[i]);
    const float wm = wave_max(lm);
    if (lane_id() == 0) s_m0[tid >> 6] = wm;
    __syncthreads();
  }
  float m0 = s_m0[0];
  for (int w = 1; w < kWaves; ++w) m0 = fmaxf(m0, s_m0[w]);
  if (!p.masked) m0 = 0.0f;  // no mask: every finite expert logit is in

  const T* row0 = row_ptr<T>(p, 0, b, j);
  const T* row1 = row_ptr<T>(p, 1, b, j);
  const int v0 = s * pl.cv;
  const int v1 = min(v0 + pl.cv, p.nvec);
  ArgBest best;
  best.val = 0.0;
  best.idx = -1;
  for (int base = v0; base < v1 && !unread; base += kStep) {
    float x0[U][N], x1[U][N];
    if (base + kStep <= v1) {
      load_group<T, ALIGNED, false, U>(row0, base, v1, p.V, x0);
      load_group<T, ALIGNED, false, U>(row1, base, v1, p.V, x1);
    } else {
      load_group<T, ALIGNED, true, U>(row0, base, v1, p.V, x0);
      load_group<T, ALIGNED, true, U>(row1, base, v1, p.V, x1);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int first = (base + u * kThreads + tid) * N;  // element index of x[u][0]
      const bool inside = base + u * kThreads + tid < v1;
#pragma unroll
      for (int k = 0; k < N; ++k) {
        double val;
        bool ok;
        if (plain >= 0) {
          val = (double)(plain ? x1[u][k] : x0[u][k]);
          ok = arg_plain_ok(best, val);
        } else {
          ok = in_mask<T>(x0[u][k], m0, p.thr32, p.thr64);
          const double prod = mu * (double)x1[u][k];
          val = (double)x0[u][k] - prod;
        }
        arg_take(best, val, first + k, ok && inside && first + k < p.V);
      }
    }
  }
  Partial* out = p.partials + (((size_t)b * g1 + j) * p.nstat) * p.S + s;
  greedy_finish(p, b, gb, best, out, per_b, wbest, &s_flag, s_arg);
}

// The same for the logit mix: one workgroup reads the chunk of all n rows.
template <typename T, bool ALIGNED, int NM>
__global__ void __launch_bounds__(kThreads) greedy_mix_kernel(Params p) {
  constexpr int N = VecOf<T>::N;
  constexpr int NCAP = NM ? NM : COS_MAX_MODELS;
  constexpr int U = NCAP <= 2 ? 4 : (NCAP <= 4 ? 2 : 1);  // vectors per lane and row in flight
  constexpr int kStep = kThreads * U;
  __shared__ ArgBest wbest[kWaves];
  __shared__ int s_flag;
  __shared__ int s_arg[COS_MAX_GAMMA + 1];

  const int n = NM ? NM : p.n;
  const int g1 = p.gamma + 1;
  const Place pl = place_of(p, g1);
  const int b = pl.b, per_b = pl.per_b;
  const int j = pl.rem / pl.S;
  const int s = pl.rem - j * pl.S;
  const int tid = threadIdx.x;
  const int gb = drafts_of(p, b);
  const bool unread = position_unread(p, gb, j);
  const int plain = (j == gb && p.bonus_idx) ? p.bonus_idx[b] : -1;
  // a verifier bonus reads that model's row only (slot 0); the others need not be valid
  const int nload = plain >= 0 ? 1 : n;

  const T* rows[NCAP];
#pragma unroll
  for (int m = 0; m < NCAP; ++m) rows[m] = row_ptr<T>(p, plain >= 0 ? plain : (m < n ? m : 0), b, j);
  const int v0 = s * pl.cv;
  const int v1 = min(v0 + pl.cv, p.nvec);
  ArgBest best;
  best.val = 0.0;
  best.idx = -1;
  for (int base = v0; base < v1 && !unread; base += kStep) {
    float x[NCAP][U][N];
    if (base + kStep <= v1) {
#pragma unroll
      for (int m = 0; m < NCAP; ++m)
        if (m < nload) load_group<T, ALIGNED, false, U>(rows[m], base, v1, p.V, x[m]);
    } else {
#pragma unroll
      for (int m = 0; m < NCAP; ++m)
        if (m < nload) load_group<T, ALIGNED, true, U>(rows[m], base, v1, p.V, x[m]);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int first = (base + u * kThreads + tid) * N;  // element index of x[.][u][0]
      const bool inside = base + u * kThreads + tid < v1;
#pragma unroll
      for (int k = 0; k < N; ++k) {
        double val;
        if (plain >= 0) {
          val = (double)x[0][u][k];
        } else {
          // sum_m beta_m l_m in model order, each product rounded on its own, models without
          // weight left out: the float64 reference's operations
          val = 0.0;
#pragma unroll
          for (int m = 0; m < NCAP; ++m)
            if (m < n && p.w[m] != 0.0) {
              const double prod = p.w[m] * (double)x[m][u][k];
              val = val + prod;
            }
        }
        arg_take(best, val, first + k, arg_plain_ok(best, val) && inside && first + k < p.V);
      }
    }
  }
  Partial* out = p.partials + (((size_t)b * g1 + j) * p.nstat) * p.S + s;
  greedy_finish(p, b, gb, best, out, per_b, wbest, &s_flag, s_arg);
}

// ---------------------------------------------------------------------------
// Temperature 0, ensemble.  Every model's softmax is one-hot at its largest logit
// a_m (ties to the lowest index), so r = sum_m w_m e_{a_m} (Eq. (4)) lives on at
// most n tokens and q = e_{a_pi}.  One streaming argmax per row; the workgroup that
// completes the sequence then takes Eq. (6), the first rejection and the draw in
// float64 on those few tokens, with exactly the operations a float64 reference
// makes on the full vocabulary (sums in model order, then in token order; terms
// that are zero there are left out here), so the outputs are bit-exact.
// ---------------------------------------------------------------------------

// r(x) = sum of the weights of the models whose token is x, in model order.
__device__ __forceinline__ double t0_mass(const Params& p, const int* a, int x) {
  double r = 0.0;
  for (int m = 0; m < p.n; ++m)
    if (a[m] == x) r += p.w[m];
  return r;
}

__device__ void greedy_decide_ensemble(const Params& p, int b, int gb, int* s_arg, int* s_accept) {
  const int tid = threadIdx.x;
  const int g1 = p.gamma + 1, n = p.n;
  for (int i = tid; i < g1 * n; i += kThreads) s_arg[i] = greedy_combine(p, b, i);  // (position, model)
  __syncthreads();
  if (tid < gb) {  // Eq. (6) at draft position tid
    const size_t k = (size_t)b * p.gamma + tid;
    const int d = p.draft[k];
    const int pi = p.proposer_pos ? p.proposer_pos[k] : p.proposer[b];
    const int* a = s_arg + tid * n;
    const double rd = t0_mass(p, a, d);
    const double qd = (a[pi] == d) ? 1.0 : 0.0;
    double ratio;
    if (!(rd > 0.0))
      ratio = 0.0;
    else if (!(qd > 0.0))
      ratio = INFINITY;
    else
      ratio = rd / qd;
    const double bound = ratio < 1.0 ? ratio : 1.0;
    s_accept[tid] = p.u_accept[k] < bound;
  }
  __syncthreads();
  int jstar = gb;
  for (int jj = gb - 1; jj >= 0; --jj)
    if (!s_accept[jj]) jstar = jj;
  const bool skip = p.no_bonus && jstar == gb;  // every draft accepted, no extra token
  if (tid == 0) p.accepted_len[b] = jstar;
  if (tid < g1 && (tid != jstar || skip))
    p.out_tokens[(size_t)b * g1 + tid] = tid < jstar ? p.draft[(size_t)b * p.gamma + tid] : -1;
  if (tid != 0 || skip) return;

  // the draw at jstar: from norm(max(0, r - q)) after a rejection, else from r (or from the
  // verifier's own one-hot softmax), by inverse CDF in ascending token order
  const int* a = s_arg + jstar * n;
  const bool residual = jstar < gb;
  const int v = (!residual && p.bonus_idx) ? p.bonus_idx[b] : -1;
  int token = -1;
  if (v >= 0) {
    token = a[v];
  } else {
    const int pi = (residual && p.proposer_pos) ? p.proposer_pos[(size_t)b * p.gamma + jstar] : p.proposer[b];
    int tok[COS_MAX_MODELS];
    double rr[COS_MAX_MODELS], f[COS_MAX_MODELS];
    int cnt = 0;
    for (int m = 0; m < n; ++m) {  // the distinct tokens, ascending
      const int x = a[m];
      bool seen = x < 0;
      for (int i = 0; i < cnt; ++i) seen = seen || tok[i] == x;
      if (seen) continue;
      int at = cnt++;
      while (at > 0 && tok[at - 1] > x) {
        tok[at] = tok[at - 1];
        --at;
      }
      tok[at] = x;
    }
    double F = 0.0;
    for (int i = 0; i < cnt; ++i) {
      rr[i] = t0_mass(p, a, tok[i]);
      const double val = residual ? rr[i] - ((tok[i] == a[pi]) ? 1.0 : 0.0) : rr[i];
      f[i] = val > 0.0 ? val : 0.0;
      F += f[i];
    }
    if (!(F > 0.0) || !(F < INFINITY)) {  // r == q although a draft was rejected: draw from r
      F = 0.0;
      for (int i = 0; i < cnt; ++i) {
        f[i] = rr[i] > 0.0 ? rr[i] : 0.0;
        F += f[i];
      }
    }
    const double t = p.u_resample[b] * F;
    double cum = 0.0;
    int last = -1;
    for (int i = 0; i < cnt && token < 0; ++i) {
      cum += f[i];
      if (f[i] > 0.0) last = tok[i];
      if (cum > t) token = tok[i];
    }
    if (token < 0) token = last;  // rounding left no prefix above t: the last token with mass
  }
  p.out_tokens[(size_t)b * g1 + jstar] = token;
}

// Workgroup index -> (b, j, m, s): the argmax of one chunk of one row.
template <typename T, bool ALIGNED>
__global__ void __launch_bounds__(kThreads) greedy_ensemble_kernel(Params p) {
  constexpr int N = VecOf<T>::N;
  constexpr int U = kUnroll;
  constexpr int kStep = kThreads * U;
  __shared__ ArgBest wbest[kWaves];
  __shared__ int s_flag;
  __shared__ int s_arg[kMaxStatsPerSeq];
  __shared__ int s_accept[COS_MAX_GAMMA + 1];

  const int g1 = p.gamma + 1;
  const Place pl = place_of(p, g1 * p.n);
  const int b = pl.b;
  int rem = pl.rem;
  const int j = rem / (p.n * pl.S);
  rem -= j * p.n * pl.S;
  const int m = rem / pl.S;
  const int s = rem - m * pl.S;
  const int tid = threadIdx.x;
  const int gb = drafts_of(p, b);
  // a verifier bonus needs that model's row only; rows of positions never read are skipped
  const int only = (p.bonus_idx && j == gb) ? p.bonus_idx[b] : -1;
  const bool unread = position_unread(p, gb, j) || (only >= 0 && m != only);

  const T* row = row_ptr<T>(p, m, b, j);
  const int v0 = s * pl.cv;
  const int v1 = min(v0 + pl.cv, p.nvec);
  // The wavefront keeps its largest value so far and where it first occurred.  Per element this is
  // one maximum; the search for the place runs only when a group of loads raises the wavefront's
  // maximum (a handful of times per chunk).  Groups come in ascending order of index, so a strict
  // comparison keeps the lowest index among equal values; elements past the row's or the chunk's
  // end read as -inf, NaN never wins a maximum.
  float wave_val = -INFINITY;
  int wave_idx = -1;
  for (int base = v0; base < v1 && !unread; base += kStep) {
    float x[U][N];
    if (base + kStep <= v1)
      load_group<T, ALIGNED, false, U>(row, base, v1, p.V, x);
    else
      load_group<T, ALIGNED, true, U>(row, base, v1, p.V, x);
    float lm = -INFINITY;
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int k = 0; k < N; ++k) lm = fmaxf(lm, x[u][k]);
    const float wm = wave_max(lm);
    if (wm > wave_val) {  // wave-uniform
      int cand = 0x7fffffff;
      if (lm == wm) {
#pragma unroll
        for (int u = U - 1; u >= 0; --u)
#pragma unroll
          for (int k = N - 1; k >= 0; --k)
            if (x[u][k] == wm) cand = (base + u * kThreads + tid) * N + k;  // descending: the first one stays
      }
      wave_idx = -wave_max_i32(-cand);
      wave_val = wm;
    }
  }
  if (wave_idx < 0 && !unread) {
    // nothing above -inf in this wavefront's share: its first element stands for it (a row of
    // -inf still has an argmax, its first element)
    const int first_vec = v0 + (tid & ~63);
    if (first_vec < v1) wave_idx = first_vec * N;
  }
  ArgBest best;
  best.val = (double)wave_val;
  best.idx = wave_idx;
  Partial* out = p.partials + (((size_t)b * g1 + j) * p.n + m) * p.S + s;
  if (greedy_arrive(p, b, best, out, pl.per_b, wbest, &s_flag)) greedy_decide_ensemble(p, b, gb, s_arg, s_accept);
}

}  // namespace
