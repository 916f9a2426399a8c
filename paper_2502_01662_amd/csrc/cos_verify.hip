// cos_verify.hip -- gfx950 kernels and C ABI of the CoS verification step.
//
// Structure (one GPU, one HIP stream, no host round trip):
//
//   fill kernel       zeroes the per-sequence arrival counters in the workspace.
//   streaming kernel  one workgroup per chunk of one logit row; reads every logit
//                     exactly once and reduces it to a partial softmax statistic
//                     (offset o, Z = sum 2^(l*log2e - o)), Sec. 3.2.  The workgroup
//                     that completes a sequence (last arrival on its counter)
//                     combines the partials in float64, runs the acceptance test
//                     of Eq. (6) for the gamma drafts, finds the first rejection
//                     (Sec. 3.1) and leaves a small plan for the draw.
//   sampling kernel   C workgroups per sequence re-read only the n rows of the one
//                     position that is sampled and reduce f = max(0, r - q)
//                     (App. A.1) or f = r (bonus) to tile sums; the last of them
//                     scans the tile sums and locates the token by inverse CDF.
//
// Contrastive mode (Eq. (5) with a plausibility mask) needs the expert row's
// maximum before anything can be masked, so a row-max kernel runs first.
//
// Extensions (cos_verify_ex): temperature, the verifier's own bonus token
// (Sec. 3.3), per-position proposers (Alg. 2), the acceptance rates of Eq. (7)
// (one more kernel), and a position window per streaming launch so that logits
// after a sequence's first rejection are never read.
//
// Numerics: per-element work is float32 (v_exp_f32); all offsets are integers
// in the log2 domain so that rescaling is exact; every cross-lane, cross-wave
// and cross-workgroup combine, r(d), q(d), the accept decision, tile sums, the
// scan and the CDF comparison are float64.
//
// Cross-workgroup hand-off: values another workgroup will read are written with
// agent-scope atomic stores (write-through), the writer waits for them to
// complete, then bumps an agent-scope counter; the workgroup that sees the final
// count reads them back with agent-scope atomic loads.  No cache-wide fences.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <cstdlib>

#include "cos_verify.h"

namespace {

constexpr int kThreads = 256;  // 4 wavefronts of 64 lanes
constexpr int kWaves = kThreads / 64;
constexpr int kUnroll = 8;  // 16-byte loads in flight per lane and iteration
constexpr float kLog2e = 1.44269504088896340736f;
constexpr int kNoOffset = -(1 << 29);       // "no finite element seen yet"
constexpr float kMaxOffset = 268435456.0f;  // 2^28: clamp for absurd logits
constexpr int kMaxSplits = 128;             // upper bound on chunks per row (workspace sizing)
constexpr int kMaxStatsPerSeq = 256;        // (gamma+1) * statistics per position
constexpr int kMaxTiles = 4096;             // tiles per row the final scan can hold in LDS
constexpr int kMaxAlphaBlocks = 64;         // acceptance-rate workgroups per (sequence, position)
// Arrival counters are agent-scope atomics executed at the memory side; one
// counter per 128-byte line spreads them over the memory channels (packed
// counters serialise on one channel and slow every stream that crosses it).
constexpr int kCtrStride = 32;  // ints between two counters (one 128-byte line each)

// Combine modes as template arguments.
constexpr int kEns = 0;  // Eq. (4): r = sum_m w_m softmax(l_m)
constexpr int kCd = 1;   // Eq. (5) with the plausibility mask
constexpr int kMix = 2;  // Eq. (3), logit level: r = softmax(sum_m beta_m l_m)

// One partial softmax statistic: Z = sum_x 2^(l(x)*log2e - o) over a chunk.
struct Partial {
  double Z;
  int o;
  int pad;
};

// What the streaming kernel leaves for the sampling kernel, per sequence.
struct SeqPlan {
  int jstar;     // position that is sampled = accepted_len
  int residual;  // 1: f = max(0, r - q); 0: f = r (bonus)
  int pi;        // proposer of the sampled position
  int bonus;     // >= 0: the bonus token is drawn from this model's softmax alone (jstar == gamma)
  float m0;      // contrastive: expert maximum at jstar
  int skip;      // 1: every draft accepted and no extra token wanted: nothing is sampled
  double lse2[COS_MAX_MODELS];  // log2-sum-exp2 of the statistics at jstar
};

struct Params {
  const void* logits;
  int n, B, gamma, V;
  const int* draft;
  const int* proposer;
  const int* proposer_pos;  // optional [B][gamma]: proposer of each draft position
  const int* bonus_idx;     // optional [B]: model the bonus token is drawn from (-1: from r)
  const int* num_drafts;    // optional [B]: drafts of each row (NULL: gamma everywhere)
  int no_bonus;             // 1: no extra token when every draft is accepted
  const double* u_accept;
  const double* u_resample;
  int* accepted_len;
  int* out_tokens;
  // workspace
  int* counters;      // (stride kCtrStride) [gamma+1 windows][B] streaming arrivals, [B] sampling
                      // arrivals, [B][gamma] acceptance-rate arrivals
  Partial* partials;  // [B][gamma+1][nstat][S]
  float* rowmax;      // contrastive: [B][gamma+1][S] partial maxima of the expert row
  SeqPlan* plans;     // [B]
  double* tile_sums;  // [B][ntiles]
  // acceptance-rate output (optional)
  double* alpha;           // [B][gamma] out, or NULL
  double* lse_all;         // [B][gamma+1][nstat] log2-sum-exp2 of every position
  float* rowmax_all;       // contrastive: [B][gamma+1] expert maxima
  double* alpha_partials;  // [B][gamma][CA]
  int CA;                  // acceptance-rate workgroups per (sequence, position)
  int tpa;                 // tiles per acceptance-rate workgroup
  int S;              // chunks per row
  int cv;             // vectors per chunk
  int nvec;           // 16-byte vectors per row (last may be partial when unaligned)
  int ntiles;         // tiles (64 vectors) per row
  int nstat;          // statistics per position: n (ensemble) or 3 (contrastive)
  int C;              // sampling workgroups per sequence
  int tpc;            // tiles per sampling workgroup
  int j0;             // first position of this launch's window
  int nj;             // positions in this launch's window (gamma+1: the whole step in one launch)
  int win;            // window index (selects the arrival counters)
  double w[COS_MAX_MODELS];  // ensemble weights; contrastive: w[0] = mu, w[1] = alpha_cd
  float scale;               // log2(e) / temperature: logits times this are base-2 exponents
  float mu_hi, mu_lo;        // mu split into two floats
  float beta_hi[COS_MAX_MODELS], beta_lo[COS_MAX_MODELS];  // logit mix: beta_m split into two floats
  int masked;                // contrastive: alpha_cd > 0 (else no row-max pass runs and m0 is taken as 0)
  float thr32;               // smallest float >= T ln(alpha_cd)
  double thr64;              // T ln(alpha_cd)
  cos_diag_t diag;
};

// Drafts of row b; position drafts_of(p, b) plays the bonus position's role.
__device__ __forceinline__ int drafts_of(const Params& p, int b) {
  return p.num_drafts ? p.num_drafts[b] : p.gamma;
}

// Positions after the row's bonus position are never read, and neither is the
// bonus position itself when no extra token is wanted.
__device__ __forceinline__ bool position_unread(const Params& p, int gb, int j) {
  return j > gb || (j == gb && p.no_bonus);
}

// ---------------------------------------------------------------------------
// wavefront and hand-off primitives
// ---------------------------------------------------------------------------

__device__ __forceinline__ int lane_id() { return threadIdx.x & 63; }

// max over the 64 lanes, returned wave-uniform.  DPP row shifts reduce each row
// of 16 lanes into its lane 15, two row broadcasts carry the result to lane 63.
__device__ __forceinline__ float wave_max(float v) {
#define COS_DPP_MAX(ctrl, row_mask)                                                        \
  {                                                                                        \
    const int t = __builtin_amdgcn_update_dpp(__float_as_int(v), __float_as_int(v), ctrl, \
                                              row_mask, 0xf, false);                      \
    v = fmaxf(v, __int_as_float(t));                                                       \
  }
  COS_DPP_MAX(0x111, 0xf)  // row_shr:1
  COS_DPP_MAX(0x112, 0xf)  // row_shr:2
  COS_DPP_MAX(0x114, 0xf)  // row_shr:4
  COS_DPP_MAX(0x118, 0xf)  // row_shr:8
  COS_DPP_MAX(0x142, 0xa)  // row_bcast:15 into rows 1 and 3
  COS_DPP_MAX(0x143, 0xc)  // row_bcast:31 into rows 2 and 3
#undef COS_DPP_MAX
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d, 64);
  return v;
}

// Sum over the 64 lanes with DPP moves (no LDS traffic); the total is valid in
// lane 63 only.
__device__ __forceinline__ double wave_sum_to_lane63(double v) {
#define COS_DPP_DSUM(ctrl, row_mask)                                                            \
  {                                                                                             \
    const long long bits = __double_as_longlong(v);                                             \
    const int lo = __builtin_amdgcn_update_dpp(0, (int)bits, ctrl, row_mask, 0xf, false);       \
    const int hi = __builtin_amdgcn_update_dpp(0, (int)(bits >> 32), ctrl, row_mask, 0xf, false); \
    v += __longlong_as_double(((long long)hi << 32) | (unsigned int)lo);                        \
  }
  COS_DPP_DSUM(0x111, 0xf)  // row_shr:1  (lanes without a source add +0.0)
  COS_DPP_DSUM(0x112, 0xf)  // row_shr:2
  COS_DPP_DSUM(0x114, 0xf)  // row_shr:4
  COS_DPP_DSUM(0x118, 0xf)  // row_shr:8
  COS_DPP_DSUM(0x142, 0xa)  // row_bcast:15 into rows 1 and 3
  COS_DPP_DSUM(0x143, 0xc)  // row_bcast:31 into rows 2 and 3
#undef COS_DPP_DSUM
  return v;
}

__device__ __forceinline__ double wave_inclusive_scan(double v) {
  const int lane = lane_id();
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const double y = __shfl_up(v, d, 64);
    if (lane >= d) v += y;
  }
  return v;
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

template <typename U>
__device__ __forceinline__ void store_agent(U* p, U v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
template <typename U>
__device__ __forceinline__ U load_agent(const U* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Wait until this wavefront's outstanding stores have completed.
__device__ __forceinline__ void wait_stores() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// Last-arrival test.  Every wavefront must have called wait_stores() after its
// hand-off stores.  Returns true in every thread of exactly one workgroup per
// counter: the one that arrives after all `total` workgroups have published.
__device__ __forceinline__ bool arrive_last(int* counter, int total, int* s_flag) {
  __syncthreads();
  if (threadIdx.x == 0) {
    const int prev = __hip_atomic_fetch_add(counter, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    *s_flag = (prev == total - 1);
  }
  __syncthreads();
  return *s_flag != 0;
}

// ---------------------------------------------------------------------------
// 16-byte vector loads of logits, widened to float32
// ---------------------------------------------------------------------------

template <typename T>
struct VecOf {
  static constexpr int N = 16 / sizeof(T);
};

// Every logit is read once per pass: 16-byte loads carry the non-temporal hint,
// which measurably raises the sustained read rate of a streaming kernel here.
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 load_stream16(const void* p) {
  const u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p));
  return make_uint4(v.x, v.y, v.z, v.w);
}

__device__ __forceinline__ float widen(float x) { return x; }
__device__ __forceinline__ float widen(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }

template <typename T>
__device__ __forceinline__ void unpack(const uint4& raw, float (&x)[VecOf<T>::N]);

template <>
__device__ __forceinline__ void unpack<float>(const uint4& raw, float (&x)[4]) {
  x[0] = __uint_as_float(raw.x);
  x[1] = __uint_as_float(raw.y);
  x[2] = __uint_as_float(raw.z);
  x[3] = __uint_as_float(raw.w);
}

// bf16 is the upper half of a float32; the lower address is the low half-word.
template <>
__device__ __forceinline__ void unpack<uint16_t>(const uint4& raw, float (&x)[8]) {
  x[0] = __uint_as_float(raw.x << 16);
  x[1] = __uint_as_float(raw.x & 0xffff0000u);
  x[2] = __uint_as_float(raw.y << 16);
  x[3] = __uint_as_float(raw.y & 0xffff0000u);
  x[4] = __uint_as_float(raw.z << 16);
  x[5] = __uint_as_float(raw.z & 0xffff0000u);
  x[6] = __uint_as_float(raw.w << 16);
  x[7] = __uint_as_float(raw.w & 0xffff0000u);
}

// Vector `vec` of a row.  ALIGNED: the row is 16-byte aligned and V is a
// multiple of the vector width, so every vector is one full 16-byte load.
// Otherwise element loads with a bound check; elements past V read as -inf.
// The caller guarantees 0 <= vec < ceil(V / N).
template <typename T, bool ALIGNED>
__device__ __forceinline__ void load_vec(const T* __restrict__ row, int vec, int V,
                                         float (&x)[VecOf<T>::N]) {
  constexpr int N = VecOf<T>::N;
  if constexpr (ALIGNED) {
    const uint4 raw = load_stream16(row + (size_t)vec * N);
    unpack<T>(raw, x);
  } else {
    const int base = vec * N;
#pragma unroll
    for (int k = 0; k < N; ++k) x[k] = (base + k < V) ? widen(row[base + k]) : -INFINITY;
  }
}

// U vectors per lane starting at `base` (stride kThreads), all loads issued
// before any use.  GUARDED: vectors at or past v1 read as -inf; their loads are
// redirected to the in-range vector v1 - 1 so nothing is out of bounds.
template <typename T, bool ALIGNED, bool GUARDED, int U>
__device__ __forceinline__ void load_group(const T* __restrict__ row, int base, int v1, int V,
                                           float (&x)[U][VecOf<T>::N]) {
  constexpr int N = VecOf<T>::N;
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int v = base + u * kThreads + (int)threadIdx.x;
    load_vec<T, ALIGNED>(row, GUARDED ? min(v, v1 - 1) : v, V, x[u]);
  }
  if constexpr (GUARDED) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int v = base + u * kThreads + (int)threadIdx.x;
      if (v >= v1) {
#pragma unroll
        for (int k = 0; k < N; ++k) x[u][k] = -INFINITY;
      }
    }
  }
}

template <typename T>
__device__ __forceinline__ const T* row_ptr(const Params& p, int m, int b, int j) {
  const size_t row = ((size_t)m * p.B + b) * (size_t)(p.gamma + 1) + j;
  return reinterpret_cast<const T*>(p.logits) + row * (size_t)p.V;
}

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

// ---- raw-register variant for 16-byte aligned rows -------------------------
//
// For bf16 the maximum is taken on the raw bit patterns with packed 16-bit
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
template <typename T, int U>
__device__ __forceinline__ void load_raw_group(const T* __restrict__ row, int base, int v1,
                                               uint4 (&raw)[U]) {
  const uint4* src = reinterpret_cast<const uint4*>(row);
#pragma unroll
  for (int u = 0; u < U; ++u)
    raw[u] = load_stream16(src + min(base + u * kThreads + (int)threadIdx.x, v1 - 1));
}

// Replace vectors at or past v1 by -inf (only the last, partial group needs it).
template <typename T, int U>
__device__ __forceinline__ void mask_raw_group(int base, int v1, uint4 (&raw)[U]) {
  const uint32_t ninf = sizeof(T) == 2 ? 0xff80ff80u : 0xff800000u;
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
      running_cover(run, __uint_as_float((uint32_t)wm16 << 16), scale);
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
  if constexpr (ALIGNED) {
    // all kUnroll loads of a group are issued before the first use; only the
    // last group of a chunk can be partial
    for (int base = v0; base < v1; base += kStep) {
      uint4 a[kUnroll];
      load_raw_group<T, kUnroll>(row, base, v1, a);
      if (base + kStep > v1) mask_raw_group<T, kUnroll>(base, v1, a);
      running_add_raw<T, kUnroll>(run, a, scale);
    }
  } else {
    int base = v0;
    for (; base + kStep <= v1; base += kStep) {
      float x[kUnroll][N];
      load_group<T, ALIGNED, false, kUnroll>(row, base, v1, V, x);
      running_add<kUnroll, N>(run, x, scale);
    }
    if (base < v1) {
      float x[kUnroll][N];
      load_group<T, ALIGNED, true, kUnroll>(row, base, v1, V, x);
      running_add<kUnroll, N>(run, x, scale);
    }
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
  store_agent(&out->Z, z);
  store_agent(&out->o, omax);
}

__device__ __forceinline__ void store_empty_partial(Partial* out) {
  store_agent(&out->Z, 0.0);
  store_agent(&out->o, kNoOffset);
}

// ---------------------------------------------------------------------------
// decide one sequence (runs in the workgroup that arrived last on its counter)
// ---------------------------------------------------------------------------

struct DecideShared {
  double lse2[kMaxStatsPerSeq];     // log2-sum-exp2 per (position, statistic)
  float rowmax[COS_MAX_GAMMA + 1];  // contrastive: expert maximum per position
  int accept[COS_MAX_GAMMA + 1];
};

// Decides the window [j0, j0+nj) of a sequence that no earlier window has
// decided.  The sequence stays undecided if every draft of the window is
// accepted and the window does not contain the bonus position.
template <typename T, int MODE>
__device__ void decide_sequence(const Params& p, int b, DecideShared& sh) {
  constexpr bool CONTRASTIVE = MODE == kCd;
  const int tid = threadIdx.x;
  const int g1 = p.gamma + 1;
  const int nstat = p.nstat;
  const int j0 = p.j0, nj = p.nj;
  const int nrows = nj * nstat;  // statistics of this window
  const int n = p.n;
  const int gb = drafts_of(p, b);
  const double log2e = (double)p.scale;  // log2(e) / T, the same constant the streaming kernel used

  // 1. combine the chunk partials of every (position, statistic) of the window in float64.
  //    A group of G lanes (a power of two >= S, at most a wavefront) shares the S partials of
  //    one statistic, so that a row cut into many chunks (small batches) costs a few dependent
  //    loads, not S of them; with whole rows (S = 1) it is one thread per statistic.
  {
    int G = 1;
    while (G < p.S && G < 64) G <<= 1;
    const int per_pass = kThreads / G;
    const int gl = tid & (G - 1);
    for (int r0 = 0; r0 < nrows; r0 += per_pass) {  // uniform trip count: every lane shuffles
      const int r = r0 + tid / G;
      int omax = kNoOffset;
      double zsum = 0.0;  // sum of Z 2^(o - omax) over the partials seen by this lane
      if (r < nrows) {
        const Partial* pp = p.partials + (((size_t)b * g1 + j0) * nstat + r) * p.S;
        for (int s = gl; s < p.S; s += G) {
          const double z = load_agent(&pp[s].Z);
          const int o = load_agent(&pp[s].o);
          if (z > 0.0) {
            if (o > omax) {
              zsum = ldexp(zsum, omax - o);  // exact: a power of two
              omax = o;
            }
            zsum += ldexp(z, o - omax);
          }
        }
      }
      for (int d = G >> 1; d >= 1; d >>= 1) {
        const int oo = __shfl_xor(omax, d, 64);
        const double zz = __shfl_xor(zsum, d, 64);
        const int om = max(omax, oo);
        zsum = (zsum > 0.0 ? ldexp(zsum, omax - om) : 0.0) + (zz > 0.0 ? ldexp(zz, oo - om) : 0.0);
        omax = om;
      }
      if (r < nrows && gl == 0) sh.lse2[r] = (zsum > 0.0) ? (double)omax + log2(zsum) : -INFINITY;
    }
  }
  if (CONTRASTIVE && tid < nj) {
    // written by the row-max kernel, an earlier launch on the same stream
    const float* rm = p.rowmax + ((size_t)b * g1 + j0 + tid) * p.S;
    float m0 = -INFINITY;
    for (int s = 0; s < p.S && p.masked; ++s) m0 = fmaxf(m0, rm[s]);
    sh.rowmax[tid] = p.masked ? m0 : 0.0f;
  }
  __syncthreads();

  // 2. Eq. (6) for every draft position of the window, in float64
  const int ndraft = max(min(j0 + nj, gb) - j0, 0);  // draft positions in the window
  if (tid >= ndraft && tid < nj && j0 + tid < p.gamma) {  // no draft here
    if (p.diag.r_at_draft) p.diag.r_at_draft[(size_t)b * p.gamma + j0 + tid] = NAN;
    if (p.diag.q_at_draft) p.diag.q_at_draft[(size_t)b * p.gamma + j0 + tid] = NAN;
  }
  if (tid < ndraft) {
    const int jj = tid, j = j0 + tid;
    const size_t k = (size_t)b * p.gamma + j;
    const int d = p.draft[k];
    const int pi = p.proposer_pos ? p.proposer_pos[k] : p.proposer[b];
    double rd = 0.0, qd = 0.0;
    if constexpr (MODE == kMix) {
      // statistic 0: the proposer's row; statistic 1: the mixed logits
      double c = 0.0;
      for (int m = 0; m < n; ++m)
        if (p.w[m] != 0.0) c += p.w[m] * (double)widen(row_ptr<T>(p, m, b, j)[d]);
      const double lq = (double)widen(row_ptr<T>(p, pi, b, j)[d]);
      rd = exp2(c * log2e - sh.lse2[jj * nstat + 1]);
      qd = exp2(lq * log2e - sh.lse2[jj * nstat + 0]);
    } else if constexpr (MODE == kEns) {
      for (int m = 0; m < n; ++m) {
        const double l = (double)widen(row_ptr<T>(p, m, b, j)[d]);
        const double s = exp2(l * log2e - sh.lse2[jj * nstat + m]);
        rd += p.w[m] * s;
        if (m == pi) qd = s;
      }
    } else {
      const double l0 = (double)widen(row_ptr<T>(p, 0, b, j)[d]);
      const double l1 = (double)widen(row_ptr<T>(p, 1, b, j)[d]);
      const bool in = (l0 > -INFINITY) && (l0 - (double)sh.rowmax[jj] >= p.thr64);
      const double c = l0 - p.w[0] * l1;
      rd = in ? exp2(c * log2e - sh.lse2[jj * nstat + 2]) : 0.0;
      qd = exp2((pi ? l1 : l0) * log2e - sh.lse2[jj * nstat + pi]);
    }
    double ratio;
    if (!(rd > 0.0))
      ratio = 0.0;
    else if (!(qd > 0.0))
      ratio = INFINITY;
    else
      ratio = rd / qd;
    const double bound = ratio < 1.0 ? ratio : 1.0;
    sh.accept[jj] = p.u_accept[k] < bound;
    if (p.diag.r_at_draft) p.diag.r_at_draft[k] = rd;
    if (p.diag.q_at_draft) p.diag.q_at_draft[k] = qd;
  }
  __syncthreads();
  if (p.alpha) {
    if (tid < nrows) p.lse_all[((size_t)b * g1 + j0) * nstat + tid] = sh.lse2[tid];
    if (CONTRASTIVE && tid < nj) p.rowmax_all[(size_t)b * g1 + j0 + tid] = sh.rowmax[tid];
  }

  // 3. first rejection (Sec. 3.1) inside the window; -1: none, and the bonus position is not in it
  int jstar = (j0 + nj > gb) ? gb : -1;
  for (int jj = ndraft - 1; jj >= 0; --jj)
    if (!sh.accept[jj]) jstar = j0 + jj;
  if (jstar < 0) return;  // undecided: a later window continues

  // the drawn token's slot is filled by the sampling kernel, unless nothing is drawn
  const bool skip = p.no_bonus && jstar == gb;
  if (tid == 0) p.accepted_len[b] = jstar;
  if (tid < g1 && (tid != jstar || skip))
    p.out_tokens[(size_t)b * g1 + tid] = (tid < jstar) ? p.draft[(size_t)b * p.gamma + tid] : -1;

  // 4. plan for the sampling kernel (read after this launch has ended)
  SeqPlan* plan = p.plans + b;
  if (tid == 0) {
    const bool residual = jstar < gb;
    plan->jstar = jstar;
    plan->residual = residual;
    plan->pi = (residual && p.proposer_pos) ? p.proposer_pos[(size_t)b * p.gamma + jstar] : p.proposer[b];
    plan->bonus = (!residual && p.bonus_idx) ? p.bonus_idx[b] : -1;
    plan->m0 = (CONTRASTIVE && !skip) ? sh.rowmax[jstar - j0] : 0.0f;
    plan->skip = skip;
    if (skip) {
      if (p.diag.sample_mass) p.diag.sample_mass[b] = 0.0;
      if (p.diag.cdf_lo) p.diag.cdf_lo[b] = 0.0;
      if (p.diag.cdf_hi) p.diag.cdf_hi[b] = 0.0;
      if (p.diag.flags) p.diag.flags[b] = 0;
    }
  }
  if (tid < nstat && !skip) plan->lse2[tid] = sh.lse2[(jstar - j0) * nstat + tid];
}

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

// Contrastive logit c = l_0 - mu*l_1 with mu = mu_hi + mu_lo.
__device__ __forceinline__ float contrast(float l0, float l1, float mu_hi, float mu_lo) {
  return fmaf(-mu_lo, l1, fmaf(-mu_hi, l1, l0));
}

// Plausibility mask: l_0 - max l_0 >= ln(alpha_cd), and a finite expert logit.
// bf16 differences are exact in float32; float32 inputs compare in float64.
template <typename T>
__device__ __forceinline__ bool in_mask(float l0, float m0, float thr32, double thr64) {
  if constexpr (sizeof(T) == 2) {
    return (l0 > -INFINITY) && (l0 - m0 >= thr32);
  } else {
    return (l0 > -INFINITY) && ((double)l0 - (double)m0 >= thr64);
  }
}

// Contrastive: r = [mask] coef[0] 2^(c*scale - off[0]), q = coef[1] 2^(l_pi*scale - off[1]);
// f = max(0, r - q) on the mask (coef[1] = 0 for a bonus draw from r), 0 off it.
// plain >= 0 (the verifier's own bonus token): f = coef[1] 2^(l_plain*scale - off[1]), no mask.
template <typename T, int N>
__device__ __forceinline__ void eval_f_contrastive(const float (&x0)[N], const float (&x1)[N],
                                                   int pi, int plain, float m0, const Params& p,
                                                   const float (&coef)[2], const float (&off)[2],
                                                   float (&f)[N]) {
  const int qsel = plain >= 0 ? plain : pi;
#pragma unroll
  for (int k = 0; k < N; ++k) {
    const float lq = qsel ? x1[k] : x0[k];
    const float q = coef[1] * fast_exp2(fmaf(lq, p.scale, -off[1]));
    if (plain >= 0) {
      f[k] = q;
    } else {
      const bool in = in_mask<T>(x0[k], m0, p.thr32, p.thr64);
      const float c = contrast(x0[k], x1[k], p.mu_hi, p.mu_lo);
      const float r = coef[0] * fast_exp2(fmaf(c, p.scale, -off[0]));
      f[k] = in ? fmaxf(r - q, 0.0f) : 0.0f;
    }
  }
}

// Logit mix c = sum_m beta_m l_m with beta_m = hi + lo; models with beta_m == 0
// take no part.  A -inf logit makes c = -inf (probability 0) instead of the NaN
// that hi * (-inf) + lo * (-inf) gives when hi and lo differ in sign.
template <int NCAP>
__device__ __forceinline__ float mix_one(const Params& p, int n, const float (&l)[NCAP]) {
  float acc = 0.0f;
  bool dead = false;
#pragma unroll
  for (int m = 0; m < NCAP; ++m)
    if (m < n && (p.beta_hi[m] != 0.0f || p.beta_lo[m] != 0.0f)) {
      const bool ninf = l[m] == -INFINITY;
      dead = dead || ninf;
      const float v = ninf ? 0.0f : l[m];
      acc = fmaf(p.beta_lo[m], v, fmaf(p.beta_hi[m], v, acc));
    }
  return dead ? -INFINITY : acc;
}

// Element k of the row of model `sel` (wave-uniform) out of the loaded rows.
template <int NCAP, int N>
__device__ __forceinline__ float pick_row(const float (&x)[NCAP][N], int sel, int k) {
  float v = x[0][k];
#pragma unroll
  for (int m = 1; m < NCAP; ++m) {
    const float xm = x[m][k];  // read first: a select of values, never of addresses (which would
    v = (m == sel) ? xm : v;   // force the rows out of registers)
  }
  return v;
}

// Logit mix: r = coef[0] 2^(c*scale - off[0]), q = coef[1] 2^(l_pi*scale - off[1]);
// f = max(0, r - q) (coef[1] = 0 for a bonus draw from r).
// plain >= 0 (the verifier's own bonus token): f = coef[1] 2^(l_plain*scale - off[1]).
template <int NCAP, int N>
__device__ __forceinline__ void eval_f_mix(const float (&x)[NCAP][N], int n, int pi, int plain,
                                           const Params& p, const float (&coef)[NCAP],
                                           const float (&off)[NCAP], float (&f)[N]) {
  static_assert(NCAP >= 2, "two coefficients");
  const int qsel = plain >= 0 ? plain : pi;
#pragma unroll
  for (int k = 0; k < N; ++k) {
    const float q = coef[1] * fast_exp2(fmaf(pick_row<NCAP, N>(x, qsel, k), p.scale, -off[1]));
    if (plain >= 0) {
      f[k] = q;
    } else {
      float l[NCAP];
#pragma unroll
      for (int m = 0; m < NCAP; ++m) l[m] = x[m][k];
      const float r = coef[0] * fast_exp2(fmaf(mix_one<NCAP>(p, n, l), p.scale, -off[0]));
      f[k] = fmaxf(r - q, 0.0f);
    }
  }
}

// Coefficients and integer offsets of the sampling weights from a sequence's plan.
template <int NCAP, int MODE>
__device__ __forceinline__ void plan_coefficients(const Params& p, const SeqPlan& plan, bool residual,
                                                  int n, float (&coef)[NCAP], float (&off)[NCAP]) {
#pragma unroll
  for (int m = 0; m < NCAP; ++m) {
    coef[m] = 0.0f;
    off[m] = 0.0f;
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
                                          float (&f)[VecOf<T>::N]) {
  constexpr int N = VecOf<T>::N;
  if constexpr (MODE == kEns)
    eval_f_ensemble<NCAP, N>(x, n, p.scale, coef, off, f);
  else if constexpr (MODE == kMix)
    eval_f_mix<NCAP, N>(x, n, pi, plain, p, coef, off, f);
  else
    eval_f_contrastive<T, N>(x[0], x[1], pi, plain, m0, p, coef, off, f);
  if (tile * 64 + lane_id() >= p.nvec) {
#pragma unroll
    for (int k = 0; k < N; ++k) f[k] = 0.0f;
  }
}

template <typename T, bool ALIGNED, int NCAP, int MODE>
__device__ __forceinline__ void tile_weights(const Params& p, const T* const (&rows)[NCAP], int n,
                                             int tile, int pi, int plain, float m0,
                                             const float (&coef)[NCAP], const float (&off)[NCAP],
                                             float (&f)[VecOf<T>::N]) {
  float x[NCAP][VecOf<T>::N];
  tile_load<T, ALIGNED, NCAP>(p, rows, n, tile, x);
  tile_eval<T, NCAP, MODE>(p, x, n, tile, pi, plain, m0, coef, off, f);
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
// Returns false if the weights have no mass and may_retry is set.
// ---------------------------------------------------------------------------
template <typename T, bool ALIGNED, int NCAP, int MODE>
__device__ bool draw_token(const Params& p, int b, const SeqPlan& plan, const T* const (&rows)[NCAP],
                           int n, const float (&coef)[NCAP], const float (&off)[NCAP],
                           const double* tile_sum, bool may_retry, int flags) {
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
  if (bad && may_retry) return false;

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
  tile_weights<T, ALIGNED, NCAP, MODE>(p, rows, n, tile, plan.pi, plan.bonus, plan.m0, coef, off, f);
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
  return true;
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
  const int per_b = p.nj * p.n * p.S;
  const int b = blockIdx.x / per_b;
  if (p.plans[b].jstar >= 0) return;  // decided by an earlier window: nothing more is read
  int rem = blockIdx.x - b * per_b;
  const int jj = rem / (p.n * p.S);
  rem -= jj * p.n * p.S;
  const int j = p.j0 + jj;
  const int m = rem / p.S;
  const int s = rem - m * p.S;

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
    const int v0 = s * p.cv;
    const int v1 = min(v0 + p.cv, p.nvec);
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
  const int ws = blockIdx.x / p.S;  // b * nj + jj
  const int s = blockIdx.x - ws * p.S;
  const int b = ws / p.nj, j = p.j0 + (ws - b * p.nj);
  if (p.plans[b].jstar >= 0) return;  // decided by an earlier window
  const int rs = b * g1 + j;
  if (position_unread(p, drafts_of(p, b), j)) {
    if (threadIdx.x == 0) p.rowmax[(size_t)rs * p.S + s] = -INFINITY;
    return;
  }
  const T* row = row_ptr<T>(p, 0, b, j);
  const int v0 = s * p.cv;
  const int v1 = min(v0 + p.cv, p.nvec);
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
template <typename T, bool ALIGNED>
__global__ void __launch_bounds__(kThreads) contrastive_stats_kernel(Params p) {
  constexpr int N = VecOf<T>::N;
  constexpr int U = kUnroll >= 2 ? kUnroll / 2 : 1;
  constexpr int kStep = kThreads * U;
  __shared__ WaveStat ws[2 * kWaves];
  __shared__ DecideShared sh;
  __shared__ int s_flag;
  __shared__ float s_m0[kWaves];

  const int g1 = p.gamma + 1;
  const int per_b = p.nj * p.S;
  const int b = blockIdx.x / per_b;
  if (p.plans[b].jstar >= 0) return;  // decided by an earlier window: nothing more is read
  int rem = blockIdx.x - b * per_b;
  const int j = p.j0 + rem / p.S;
  const int s = rem - (j - p.j0) * p.S;
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
    for (int i = tid; i < p.S && p.masked; i += kThreads) lm = fmaxf(lm, rm[i]);
    const float wm = wave_max(lm);
    if (lane_id() == 0) s_m0[tid >> 6] = wm;
    __syncthreads();
  }
  float m0 = s_m0[0];
  for (int w = 1; w < kWaves; ++w) m0 = fmaxf(m0, s_m0[w]);
  if (!p.masked) m0 = 0.0f;  // no mask: every finite expert logit is in

  const T* row0 = row_ptr<T>(p, 0, b, j);
  const T* row1 = row_ptr<T>(p, 1, b, j);
  const int v0 = s * p.cv;
  const int v1 = min(v0 + p.cv, p.nvec);
  Running rq, rc;  // proposer row; masked contrastive logits
  running_init(rq);
  running_init(rc);
  for (int base = v0; base < v1; base += kStep) {
    float x0[U][N], x1[U][N];
    if (base + kStep <= v1) {
      load_group<T, ALIGNED, false, U>(row0, base, v1, p.V, x0);
      load_group<T, ALIGNED, false, U>(row1, base, v1, p.V, x1);
    } else {
      load_group<T, ALIGNED, true, U>(row0, base, v1, p.V, x0);
      load_group<T, ALIGNED, true, U>(row1, base, v1, p.V, x1);
    }
    // proposer row statistic
    if (pi)
      running_add<U, N>(rq, x1, p.scale);
    else
      running_add<U, N>(rq, x0, p.scale);
    // masked contrastive statistic; the mask is sparse, so skip wave-wide when empty
    float c[U][N];
    float lmc = -INFINITY;
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int k = 0; k < N; ++k) {
        const bool in = in_mask<T>(x0[u][k], m0, p.thr32, p.thr64);
        c[u][k] = in ? contrast(x0[u][k], x1[u][k], p.mu_hi, p.mu_lo) : -INFINITY;
        lmc = fmaxf(lmc, c[u][k]);
      }
    if (__ballot(lmc > -INFINITY)) running_add<U, N>(rc, c, p.scale);
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
  const int per_b = p.nj * p.S;
  const int b = blockIdx.x / per_b;
  if (p.plans[b].jstar >= 0) return;  // decided by an earlier window: nothing more is read
  int rem = blockIdx.x - b * per_b;
  const int j = p.j0 + rem / p.S;
  const int s = rem - (j - p.j0) * p.S;
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
  const int v0 = s * p.cv;
  const int v1 = min(v0 + p.cv, p.nvec);
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
    float xq[U][N];
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int k = 0; k < N; ++k) {
        float v = x[0][u][k];
#pragma unroll
        for (int m = 1; m < NCAP; ++m) {
          const float xm = x[m][u][k];
          v = (m == pi) ? xm : v;
        }
        xq[u][k] = v;
      }
    running_add<U, N>(rq, xq, p.scale);
    if (!plain) {
      float c[U][N];
#pragma unroll
      for (int u = 0; u < U; ++u)
#pragma unroll
        for (int k = 0; k < N; ++k) {
          float l[NCAP];
#pragma unroll
          for (int m = 0; m < NCAP; ++m) l[m] = x[m][u][k];
          c[u][k] = mix_one<NCAP>(p, n, l);
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

// Sampling kernel.  Workgroup index -> (b, c): tiles [c*tpc, (c+1)*tpc) of the
// sampled position's rows -> tile sums; the last workgroup of b draws the token.
template <typename T, bool ALIGNED, int NM, int MODE>
__global__ void __launch_bounds__(kThreads) sample_kernel(Params p) {
  constexpr int N = VecOf<T>::N;
  constexpr bool CONTRASTIVE = MODE == kCd;
  // register rows; the logit mix keeps its two coefficients in slots 0 and 1
  constexpr int NCAP = CONTRASTIVE ? 2 : (NM ? (MODE == kMix && NM < 2 ? 2 : NM) : COS_MAX_MODELS);
  constexpr int TU = NCAP <= 4 ? 4 : 1;  // tiles in flight per wavefront
  extern __shared__ double tile_sum[];
  __shared__ int s_flag;

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

  double* sums = p.tile_sums + (size_t)b * p.ntiles;
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
                                      off, f);
      const double ts = wave_sum_to_lane63(lane_mass<N>(f));
      if (lane == 63 && ti < te) tile_sum[ti - tb] = ts;  // staged in LDS
    }
  }
  __syncthreads();
  // publish this workgroup's tile sums with coalesced write-through stores
  for (int i = threadIdx.x; i < te - tb; i += kThreads) store_agent(sums + tb + i, tile_sum[i]);
  wait_stores();
  if (!arrive_last(p.counters + ((size_t)(p.gamma + 1) * p.B + b) * kCtrStride, p.C, &s_flag)) return;

  // last workgroup of this sequence: all tile sums are published
  for (int t = threadIdx.x; t < p.ntiles; t += kThreads) tile_sum[t] = load_agent(sums + t);
  __syncthreads();
  bool done = false;
  if (wave == 0)
    done = draw_token<T, ALIGNED, NCAP, MODE>(p, b, plan, rows, n, coef, off, tile_sum,
                                                     plan.residual != 0, 0);
  if (threadIdx.x == 0) s_flag = done ? 0 : 1;
  __syncthreads();
  if (!s_flag) return;

  // The residual has no mass (cannot happen in exact arithmetic): draw from r
  // itself.  Rare, so this one workgroup recomputes every tile sum.
  plan_coefficients<NCAP, MODE>(p, plan, false, n, coef, off);
  for (int t = wave; t < p.ntiles; t += kWaves) {
    float f[N];
    tile_weights<T, ALIGNED, NCAP, MODE>(p, rows, n, t, plan.pi, plan.bonus, plan.m0, coef, off, f);
    const double ts = wave_sum(lane_mass<N>(f));
    if (lane == 0) tile_sum[t] = ts;
  }
  __syncthreads();
  if (wave == 0)
    draw_token<T, ALIGNED, NCAP, MODE>(p, b, plan, rows, n, coef, off, tile_sum, false,
                                              COS_FLAG_RESIDUAL_FALLBACK);
}

// Temperature 0 (greedy), contrastive mode.  r of Eq. (5) is one-hot at the
// masked argmax a_j of c = l_0 - mu l_1, so a draft is accepted iff d_j == a_j and
// the token drawn at the first mismatch (or the bonus token) is a_j itself: one
// streaming argmax per position, no sampling kernel, no random numbers.  c is
// evaluated in float64 with a separate multiply and subtract so that every
// comparison is the one a float64 reference makes; ties go to the lowest index.
// Workgroup index -> (b, j, s).  With a verifier bonus the bonus position takes
// the plain argmax of that model's row.
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
  const int per_b = g1 * p.S;
  const int b = blockIdx.x / per_b;
  int rem = blockIdx.x - b * per_b;
  const int j = rem / p.S;
  const int s = rem - j * p.S;
  const int tid = threadIdx.x;
  const int gb = drafts_of(p, b);
  const bool unread = position_unread(p, gb, j);
  const int plain = (j == gb && p.bonus_idx) ? p.bonus_idx[b] : -1;
  const double mu = p.w[0];

  {
    const float* rm = p.rowmax + ((size_t)b * g1 + j) * p.S;
    float lm = -INFINITY;
    for (int i = tid; i < p.S && p.masked; i += kThreads) lm = fmaxf(lm, rm[i]);
    const float wm = wave_max(lm);
    if (lane_id() == 0) s_m0[tid >> 6] = wm;
    __syncthreads();
  }
  float m0 = s_m0[0];
  for (int w = 1; w < kWaves; ++w) m0 = fmaxf(m0, s_m0[w]);
  if (!p.masked) m0 = 0.0f;  // no mask: every finite expert logit is in

  const T* row0 = row_ptr<T>(p, 0, b, j);
  const T* row1 = row_ptr<T>(p, 1, b, j);
  const int v0 = s * p.cv;
  const int v1 = min(v0 + p.cv, p.nvec);
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
#pragma unroll
      for (int k = 0; k < N; ++k) {
        double val;
        bool ok;
        if (plain >= 0) {
          val = (double)(plain ? x1[u][k] : x0[u][k]);
          ok = val > -INFINITY || (best.idx < 0 && val == -INFINITY);  // a row of -inf still has an argmax
        } else {
          ok = in_mask<T>(x0[u][k], m0, p.thr32, p.thr64);
          const double prod = mu * (double)x1[u][k];
          val = (double)x0[u][k] - prod;
        }
        if (ok && base + u * kThreads + tid < v1 && first + k < p.V && (best.idx < 0 || val > best.val)) {
          best.val = val;
          best.idx = first + k;
        }
      }
    }
  }
  // wavefront, then workgroup
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
    Partial* out = p.partials + (((size_t)b * g1 + j) * p.nstat) * p.S + s;
    store_agent(&out->Z, bb.val);
    store_agent(&out->o, bb.idx);
    wait_stores();
  }
  if (!arrive_last(p.counters + (size_t)b * kCtrStride, per_b, &s_flag)) return;

  // last workgroup of the sequence: argmax of every position, first mismatch, outputs
  if (tid < g1) {
    const Partial* pp = p.partials + (((size_t)b * g1 + tid) * p.nstat) * p.S;
    ArgBest bb;
    bb.val = 0.0;
    bb.idx = -1;
    for (int i = 0; i < p.S; ++i) arg_better(bb, load_agent(&pp[i].Z), load_agent(&pp[i].o));
    s_arg[tid] = bb.idx;
  }
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
  const int pi = p.proposer_pos ? p.proposer_pos[(size_t)b * p.gamma + j] : p.proposer[b];
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

  double acc = 0.0;
  const int tb = c * p.tpa;
  const int te = min(tb + p.tpa, p.ntiles);
  for (int t = tb + wave; t < te; t += kWaves) {
    float x[NCAP][N];
    tile_load<T, ALIGNED, NCAP>(p, rows, n, t, x);
    if (t * 64 + lane < p.nvec) {
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
          float l[NCAP];
#pragma unroll
          for (int m = 0; m < NCAP; ++m) l[m] = x[m][k];
          r = cr[0] * fast_exp2(fmaf(mix_one<NCAP>(p, n, l), p.scale, -off[0]));
          q = cq * fast_exp2(fmaf(pick_row<NCAP, N>(x, pi, k), p.scale, -off[1]));
        } else {
          const bool in = in_mask<T>(x[0][k], m0, p.thr32, p.thr64);
          const float cc = contrast(x[0][k], x[1][k], p.mu_hi, p.mu_lo);
          r = in ? cr[0] * fast_exp2(fmaf(cc, p.scale, -off[0])) : 0.0f;
          q = cq * fast_exp2(fmaf(pi ? x[1][k] : x[0][k], p.scale, -off[1]));
        }
        acc += (double)fminf(q, r);
      }
    }
  }
  const double ws = wave_sum(acc);
  if (lane == 0) wsum[wave] = ws;
  __syncthreads();
  double* parts = p.alpha_partials + ((size_t)b * p.gamma + j) * p.CA;
  if (threadIdx.x == 0) {
    double tot = 0.0;
    for (int w = 0; w < kWaves; ++w) tot += wsum[w];
    store_agent(parts + c, tot);
    wait_stores();
  }
  int* counter = p.counters + ((size_t)(p.gamma + 2) * p.B + (size_t)b * p.gamma + j) * kCtrStride;
  if (!arrive_last(counter, p.CA, &s_flag)) return;
  if (threadIdx.x == 0) {
    double tot = 0.0;
    for (int i = 0; i < p.CA; ++i) tot += load_agent(parts + i);
    p.alpha[(size_t)b * p.gamma + j] = tot;
  }
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------

int g_chunk_vectors = 0;  // 0 = heuristic
int g_sample_blocks = 0;  // 0 = heuristic

// Optional event ring around the streaming kernel (benchmarks only).
constexpr int kMaxProfileSlots = 1024;
hipEvent_t g_ev_start[kMaxProfileSlots], g_ev_stop[kMaxProfileSlots];
int g_ev_created = 0;   // event pairs that exist
int g_ev_slots = 0;     // pairs in use (0 = profiling off)
int g_ev_recorded = 0;  // calls recorded since the last enable

struct Plan {
  int nvec, ntiles, nstat;
  size_t off_counters, off_partials, off_rowmax, off_plans, off_tiles, off_lse_all, off_rowmax_all,
      off_alpha_partials, bytes;
};

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

bool shape_ok(int n, int B, int gamma, int V) {
  return n >= 1 && n <= COS_MAX_MODELS && B >= 0 && gamma >= 1 && gamma <= COS_MAX_GAMMA &&
         V >= 1 && V <= COS_MAX_VOCAB;
}

int alpha_blocks(int B, int gamma, int ntiles);

// Workspace layout for S chunks per row.
void plan_layout(int n, int B, int gamma, int V, cos_dtype_t dt, cos_combine_t mode, int S,
                 Plan* pl) {
  const int N = dt == COS_DTYPE_F32 ? 4 : 8;
  pl->nvec = (V + N - 1) / N;
  pl->ntiles = (pl->nvec + 63) / 64;
  pl->nstat = mode == COS_COMBINE_CONTRASTIVE ? 3 : (mode == COS_COMBINE_LOGIT_MIX ? 2 : n);
  const size_t g1 = (size_t)gamma + 1;
  size_t at = 0;
  pl->off_counters = at;
  at += align_up(((size_t)(gamma + 2) * B + (size_t)B * gamma) * kCtrStride * sizeof(int), 256);
  pl->off_plans = at;
  at += align_up((size_t)B * sizeof(SeqPlan), 256);
  pl->off_tiles = at;
  at += align_up((size_t)B * pl->ntiles * sizeof(double), 256);
  pl->off_lse_all = at;
  at += align_up((size_t)B * g1 * pl->nstat * sizeof(double), 256);
  pl->off_rowmax_all = at;
  at += align_up((size_t)B * g1 * sizeof(float), 256);
  pl->off_alpha_partials = at;
  at += align_up((size_t)B * gamma * alpha_blocks(B, gamma, pl->ntiles) * sizeof(double), 256);
  pl->off_rowmax = at;
  if (mode == COS_COMBINE_CONTRASTIVE) at += align_up((size_t)B * g1 * S * sizeof(float), 256);
  pl->off_partials = at;
  at += align_up((size_t)B * g1 * pl->nstat * S * sizeof(Partial), 256);
  pl->bytes = at;
}

int max_splits(int nvec) {
  const int s = (nvec + kThreads - 1) / kThreads;
  return s < kMaxSplits ? (s < 1 ? 1 : s) : kMaxSplits;
}

// Chunks per row.  A workgroup's start-up and hand-off cost is paid per chunk,
// so chunks are as long as possible: whole rows once there are a few thousand
// rows, otherwise just enough chunks to fill 256 CUs several times over.
void choose_split(int rows_total, int nvec, int* S_out, int* cv_out) {
  int cv;
  if (g_chunk_vectors > 0) {
    cv = g_chunk_vectors;
  } else {
    long s_want = (3072 + rows_total - 1) / (rows_total > 0 ? rows_total : 1);
    if (s_want < 1) s_want = 1;
    cv = (int)((nvec + s_want - 1) / s_want);
    // never less than one full group of loads per thread: shorter chunks only add hand-offs
    if (cv < kThreads * kUnroll) cv = kThreads * kUnroll;
  }
  cv = (cv + kThreads - 1) / kThreads * kThreads;
  if (cv < kThreads) cv = kThreads;
  int S = (nvec + cv - 1) / cv;
  const int smax = max_splits(nvec);
  if (S > smax) {
    S = smax;
    cv = (nvec + S - 1) / S;
    cv = (cv + kThreads - 1) / kThreads * kThreads;
    S = (nvec + cv - 1) / cv;
  }
  *S_out = S;
  *cv_out = cv;
}

// Acceptance-rate workgroups per (sequence, position): about 4096 in total, at
// least 4 tiles each, at most kMaxAlphaBlocks.
int alpha_blocks(int B, int gamma, int ntiles) {
  long ca = (4096 + (long)B * gamma - 1) / ((long)B * gamma > 0 ? (long)B * gamma : 1);
  const int cmax = (ntiles + 3) / 4;
  if (ca > cmax) ca = cmax;
  if (ca > kMaxAlphaBlocks) ca = kMaxAlphaBlocks;
  if (ca < 1) ca = 1;
  return (int)ca;
}

// Sampling workgroups per sequence: about 2048 in total, at least 4 tiles each.
void choose_sampling(int B, int ntiles, int* C_out, int* tpc_out) {
  const int target = g_sample_blocks > 0 ? g_sample_blocks : 2048;
  int C = (target + B - 1) / B;
  const int cmax = (ntiles + 3) / 4;
  if (C > cmax) C = cmax;
  if (C < 1) C = 1;
  const int tpc = (ntiles + C - 1) / C;
  *C_out = (ntiles + tpc - 1) / tpc;
  *tpc_out = tpc;
}

// Kernels that hold the rows of all n models in registers are specialised for
// n = 1..4 on the aligned path; everything else takes the generic instance.
template <typename T, bool ALIGNED, int MODE>
cos_status_t launch_sampling(const Params& p, size_t lds, hipStream_t st) {
  const long blocks = (long)p.B * p.C;
  if (blocks <= 0 || blocks > 0x7fffffffL) return COS_ERR_SHAPE;
  const dim3 grid((unsigned)blocks), block(kThreads);
  if constexpr (MODE == kCd) {
    hipLaunchKernelGGL((sample_kernel<T, ALIGNED, 2, kCd>), grid, block, lds, st, p);
  } else if constexpr (ALIGNED) {
    switch (p.n) {
      case 1: hipLaunchKernelGGL((sample_kernel<T, true, 1, MODE>), grid, block, lds, st, p); break;
      case 2: hipLaunchKernelGGL((sample_kernel<T, true, 2, MODE>), grid, block, lds, st, p); break;
      case 3: hipLaunchKernelGGL((sample_kernel<T, true, 3, MODE>), grid, block, lds, st, p); break;
      case 4: hipLaunchKernelGGL((sample_kernel<T, true, 4, MODE>), grid, block, lds, st, p); break;
      default: hipLaunchKernelGGL((sample_kernel<T, true, 0, MODE>), grid, block, lds, st, p); break;
    }
  } else {
    hipLaunchKernelGGL((sample_kernel<T, false, 0, MODE>), grid, block, lds, st, p);
  }
  return hipGetLastError() == hipSuccess ? COS_OK : COS_ERR_LAUNCH;
}

template <typename T, bool ALIGNED, int MODE>
cos_status_t launch_acceptance_rate(const Params& p, hipStream_t st) {
  const long blocks = (long)p.B * p.gamma * p.CA;
  if (blocks <= 0 || blocks > 0x7fffffffL) return COS_ERR_SHAPE;
  const dim3 grid((unsigned)blocks), block(kThreads);
  if constexpr (MODE == kCd) {
    hipLaunchKernelGGL((acceptance_rate_kernel<T, ALIGNED, 2, kCd>), grid, block, 0, st, p);
  } else if constexpr (ALIGNED) {
    switch (p.n) {
      case 1: hipLaunchKernelGGL((acceptance_rate_kernel<T, true, 1, MODE>), grid, block, 0, st, p); break;
      case 2: hipLaunchKernelGGL((acceptance_rate_kernel<T, true, 2, MODE>), grid, block, 0, st, p); break;
      case 3: hipLaunchKernelGGL((acceptance_rate_kernel<T, true, 3, MODE>), grid, block, 0, st, p); break;
      case 4: hipLaunchKernelGGL((acceptance_rate_kernel<T, true, 4, MODE>), grid, block, 0, st, p); break;
      default: hipLaunchKernelGGL((acceptance_rate_kernel<T, true, 0, MODE>), grid, block, 0, st, p); break;
    }
  } else {
    hipLaunchKernelGGL((acceptance_rate_kernel<T, false, 0, MODE>), grid, block, 0, st, p);
  }
  return hipGetLastError() == hipSuccess ? COS_OK : COS_ERR_LAUNCH;
}

template <typename T, bool ALIGNED>
void launch_mix_stats(const Params& p, dim3 grid, hipStream_t st) {
  const dim3 block(kThreads);
  if constexpr (ALIGNED) {
    switch (p.n) {
      case 1: hipLaunchKernelGGL((mix_stats_kernel<T, true, 1>), grid, block, 0, st, p); break;
      case 2: hipLaunchKernelGGL((mix_stats_kernel<T, true, 2>), grid, block, 0, st, p); break;
      case 3: hipLaunchKernelGGL((mix_stats_kernel<T, true, 3>), grid, block, 0, st, p); break;
      case 4: hipLaunchKernelGGL((mix_stats_kernel<T, true, 4>), grid, block, 0, st, p); break;
      default: hipLaunchKernelGGL((mix_stats_kernel<T, true, 0>), grid, block, 0, st, p); break;
    }
  } else {
    hipLaunchKernelGGL((mix_stats_kernel<T, false, 0>), grid, block, 0, st, p);
  }
}

// All launches of one call after the fill kernel.  `window` positions are
// verified per streaming launch; sequences decided by an earlier window are
// skipped by every later one (their workgroups return at once).
template <typename T, bool ALIGNED>
cos_status_t launch_all(Params p, int mode, int window, size_t lds, hipStream_t st,
                        hipEvent_t ev_start, hipEvent_t ev_stop) {
  const dim3 block(kThreads);
  const int g1 = p.gamma + 1;
  if (ev_start) (void)hipEventRecord(ev_start, st);
  p.win = 0;
  for (int j0 = 0; j0 < g1; j0 += window, ++p.win) {
    p.j0 = j0;
    p.nj = (j0 + window <= g1) ? window : g1 - j0;
    const long blocks = (long)p.B * p.nj * (mode == kEns ? p.n : 1) * p.S;
    if (blocks <= 0 || blocks > 0x7fffffffL) return COS_ERR_SHAPE;
    const dim3 grid((unsigned)blocks);
    if (mode == kEns) {
      hipLaunchKernelGGL((ensemble_stats_kernel<T, ALIGNED>), grid, block, 0, st, p);
    } else if (mode == kMix) {
      launch_mix_stats<T, ALIGNED>(p, grid, st);
    } else {
      // alpha_cd = 0 is Eq. (5) as printed: no mask, so no pass for the expert maxima
      if (p.masked) hipLaunchKernelGGL((expert_rowmax_kernel<T, ALIGNED>), grid, block, 0, st, p);
      hipLaunchKernelGGL((contrastive_stats_kernel<T, ALIGNED>), grid, block, 0, st, p);
    }
    if (hipGetLastError() != hipSuccess) return COS_ERR_LAUNCH;
  }
  if (ev_stop) (void)hipEventRecord(ev_stop, st);
  cos_status_t rc = mode == kEns   ? launch_sampling<T, ALIGNED, kEns>(p, lds, st)
                    : mode == kMix ? launch_sampling<T, ALIGNED, kMix>(p, lds, st)
                                   : launch_sampling<T, ALIGNED, kCd>(p, lds, st);
  if (rc != COS_OK || !p.alpha) return rc;
  return mode == kEns   ? launch_acceptance_rate<T, ALIGNED, kEns>(p, st)
         : mode == kMix ? launch_acceptance_rate<T, ALIGNED, kMix>(p, st)
                        : launch_acceptance_rate<T, ALIGNED, kCd>(p, st);
}

}  // namespace

extern "C" {

size_t cos_verify_workspace_bytes(int n, int B, int gamma, int V, cos_dtype_t dt,
                                  cos_combine_t mode) {
  if (!shape_ok(n, B, gamma, V)) return 0;
  if (dt != COS_DTYPE_F32 && dt != COS_DTYPE_BF16) return 0;
  if (mode != COS_COMBINE_ENSEMBLE && mode != COS_COMBINE_CONTRASTIVE && mode != COS_COMBINE_LOGIT_MIX)
    return 0;
  // Sized for one-position windows (stop_window = 1), which split rows the most.
  Plan pl;
  const int N = dt == COS_DTYPE_F32 ? 4 : 8;
  int S, cv;
  choose_split((mode == COS_COMBINE_ENSEMBLE ? n : 1) * (B > 0 ? B : 1), (V + N - 1) / N, &S, &cv);
  plan_layout(n, B, gamma, V, dt, mode, S, &pl);
  return pl.bytes < 256 ? 256 : pl.bytes;
}

cos_status_t cos_verify(const void* logits, cos_dtype_t dt, int n, int B, int gamma, int V,
                        const int32_t* draft_tokens, const int32_t* proposer_idx,
                        cos_combine_t combine_mode, const double* weights,
                        const double* u_accept, const double* u_resample,
                        int32_t* accepted_len, int32_t* out_tokens, void* workspace,
                        size_t workspace_bytes, const cos_diag_t* diag, void* hip_stream) {
  return cos_verify_ex(logits, dt, n, B, gamma, V, draft_tokens, proposer_idx, combine_mode, weights,
                       u_accept, u_resample, accepted_len, out_tokens, workspace, workspace_bytes,
                       diag, nullptr, hip_stream);
}

cos_status_t cos_verify_ex(const void* logits, cos_dtype_t dt, int n, int B, int gamma, int V,
                           const int32_t* draft_tokens, const int32_t* proposer_idx,
                           cos_combine_t combine_mode, const double* weights,
                           const double* u_accept, const double* u_resample,
                           int32_t* accepted_len, int32_t* out_tokens, void* workspace,
                           size_t workspace_bytes, const cos_diag_t* diag,
                           const cos_options_t* options, void* hip_stream) {
  // ---- host-side validation (no HIP call before it passes) ----
  double temperature = 1.0;
  if (options) {
    if (options->struct_bytes != sizeof(cos_options_t)) return COS_ERR_UNSUPPORTED;
    if (!(options->temperature >= 0.0) || !std::isfinite(options->temperature)) return COS_ERR_WEIGHTS;
    if (options->temperature > 0.0) temperature = options->temperature;
    if (options->stop_window < 0) return COS_ERR_SHAPE;
    if (options->greedy) {
      // temperature 0: built for the contrastive mode (the paper's T = 0 runs), whole step in one launch
      if (combine_mode != COS_COMBINE_CONTRASTIVE || options->alpha || options->proposer_pos ||
          (options->stop_window > 0 && options->stop_window <= gamma))
        return COS_ERR_UNSUPPORTED;
    }
    // acceptance rates of positions that were never read do not exist
    if (options->stop_window > 0 && options->stop_window <= gamma && options->alpha)
      return COS_ERR_UNSUPPORTED;
  }
  if (!shape_ok(n, B, gamma, V)) return COS_ERR_SHAPE;
  if (dt != COS_DTYPE_F32 && dt != COS_DTYPE_BF16) return COS_ERR_DTYPE;
  if (combine_mode != COS_COMBINE_ENSEMBLE && combine_mode != COS_COMBINE_CONTRASTIVE &&
      combine_mode != COS_COMBINE_LOGIT_MIX)
    return COS_ERR_MODE;
  const bool contrastive = combine_mode == COS_COMBINE_CONTRASTIVE;
  const bool mix = combine_mode == COS_COMBINE_LOGIT_MIX;
  const int mode = contrastive ? kCd : (mix ? kMix : kEns);
  if (contrastive && n != 2) return COS_ERR_MODE;
  if (!weights) return COS_ERR_NULL;
  if (mix) {
    for (int m = 0; m < n; ++m)
      if (!std::isfinite(weights[m])) return COS_ERR_WEIGHTS;
  } else if (!contrastive) {
    double sum = 0.0;
    for (int m = 0; m < n; ++m) {
      if (!(weights[m] >= 0.0) || !std::isfinite(weights[m])) return COS_ERR_WEIGHTS;
      sum += weights[m];
    }
    if (std::fabs(sum - 1.0) > 1e-9) return COS_ERR_WEIGHTS;
  } else {
    if (!std::isfinite(weights[0])) return COS_ERR_WEIGHTS;
    if (!(weights[1] >= 0.0 && weights[1] <= 1.0)) return COS_ERR_WEIGHTS;
  }
  if (B == 0) return COS_OK;
  if (!logits || !draft_tokens || !proposer_idx || !u_accept || !u_resample || !accepted_len ||
      !out_tokens)
    return COS_ERR_NULL;
  const size_t esize = dt == COS_DTYPE_F32 ? 4 : 2;
  if (reinterpret_cast<uintptr_t>(logits) % esize) return COS_ERR_ALIGN;
  const size_t need = cos_verify_workspace_bytes(n, B, gamma, V, dt, combine_mode);
  if (!workspace || reinterpret_cast<uintptr_t>(workspace) % 256 || workspace_bytes < need)
    return COS_ERR_WORKSPACE;
  if ((size_t)(gamma + 1) * (contrastive ? 3 : (mix ? 2 : n)) > kMaxStatsPerSeq) return COS_ERR_SHAPE;

  // ---- launch plan ----
  const int N = dt == COS_DTYPE_F32 ? 4 : 8;
  const int nvec = (V + N - 1) / N;
  int window = gamma + 1;  // positions per streaming launch
  if (options && options->stop_window > 0 && options->stop_window < window) window = options->stop_window;
  const int rows_total = (mode == kEns ? n : 1) * B * window;
  int S, cv;
  choose_split(rows_total, nvec, &S, &cv);
  Plan pl;
  plan_layout(n, B, gamma, V, dt, combine_mode, S, &pl);
  if (pl.bytes > workspace_bytes || pl.ntiles > kMaxTiles) return COS_ERR_WORKSPACE;

  Params p;
  p.logits = logits;
  p.n = n;
  p.B = B;
  p.gamma = gamma;
  p.V = V;
  p.draft = draft_tokens;
  p.proposer = proposer_idx;
  p.proposer_pos = options ? options->proposer_pos : nullptr;
  p.bonus_idx = options ? options->bonus_idx : nullptr;
  p.num_drafts = options ? options->num_drafts : nullptr;
  p.no_bonus = (options && options->no_bonus) ? 1 : 0;
  p.u_accept = u_accept;
  p.u_resample = u_resample;
  p.accepted_len = accepted_len;
  p.out_tokens = out_tokens;
  char* wsb = static_cast<char*>(workspace);
  p.counters = reinterpret_cast<int*>(wsb + pl.off_counters);
  p.partials = reinterpret_cast<Partial*>(wsb + pl.off_partials);
  p.rowmax = reinterpret_cast<float*>(wsb + pl.off_rowmax);
  p.plans = reinterpret_cast<SeqPlan*>(wsb + pl.off_plans);
  p.tile_sums = reinterpret_cast<double*>(wsb + pl.off_tiles);
  p.alpha = options ? options->alpha : nullptr;
  p.lse_all = reinterpret_cast<double*>(wsb + pl.off_lse_all);
  p.rowmax_all = reinterpret_cast<float*>(wsb + pl.off_rowmax_all);
  p.alpha_partials = reinterpret_cast<double*>(wsb + pl.off_alpha_partials);
  {
    const int ca = alpha_blocks(B, gamma, pl.ntiles);
    p.tpa = (pl.ntiles + ca - 1) / ca;
    p.CA = (pl.ntiles + p.tpa - 1) / p.tpa;  // <= ca
  }
  p.S = S;
  p.cv = cv;
  p.nvec = pl.nvec;
  p.ntiles = pl.ntiles;
  p.nstat = pl.nstat;
  choose_sampling(B, pl.ntiles, &p.C, &p.tpc);
  for (int m = 0; m < COS_MAX_MODELS; ++m) p.w[m] = m < n ? weights[m] : 0.0;
  p.scale = (float)((double)kLog2e / temperature);
  p.mu_hi = p.mu_lo = 0.0f;
  for (int m = 0; m < COS_MAX_MODELS; ++m) {
    p.beta_hi[m] = (mix && m < n) ? (float)weights[m] : 0.0f;
    p.beta_lo[m] = (mix && m < n) ? (float)(weights[m] - (double)p.beta_hi[m]) : 0.0f;
  }
  p.thr32 = -INFINITY;
  p.thr64 = -INFINITY;
  p.masked = (contrastive && weights[1] > 0.0) ? 1 : 0;
  if (contrastive) {
    p.mu_hi = (float)weights[0];
    p.mu_lo = (float)(weights[0] - (double)p.mu_hi);
    if (weights[1] > 0.0) {
      // (l_0 - max l_0) / T >= ln(alpha_cd)  <=>  l_0 - max l_0 >= T ln(alpha_cd)
      p.thr64 = temperature * std::log(weights[1]);
      float t = (float)p.thr64;  // smallest float >= thr64
      if ((double)t < p.thr64) t = std::nextafterf(t, INFINITY);
      p.thr32 = t;
    }
  }
  if (diag) {
    p.diag = *diag;
  } else {
    p.diag.r_at_draft = p.diag.q_at_draft = p.diag.sample_mass = nullptr;
    p.diag.cdf_lo = p.diag.cdf_hi = nullptr;
    p.diag.flags = nullptr;
  }

  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  const bool aligned = (reinterpret_cast<uintptr_t>(logits) % 16 == 0) && (V % N == 0);
  const size_t lds = (size_t)pl.ntiles * sizeof(double);
  const bool profile = g_ev_slots > 0;
  const int slot = profile ? g_ev_recorded % g_ev_slots : 0;
  hipEvent_t ev_start = profile ? g_ev_start[slot] : nullptr;
  hipEvent_t ev_stop = profile ? g_ev_stop[slot] : nullptr;

  // counters in use: one set per window, the sampling set, and the acceptance-rate set if wanted
  const int nctr = ((p.alpha ? 2 * gamma + 2 : gamma + 2) * B) * kCtrStride;
  hipLaunchKernelGGL(fill_zero_kernel, dim3((nctr + kThreads - 1) / kThreads), dim3(kThreads), 0, st,
                     p.counters, nctr, p.plans, B);
  if (hipGetLastError() != hipSuccess) return COS_ERR_LAUNCH;

  if (options && options->greedy) {
    p.j0 = 0;
    p.nj = gamma + 1;
    p.win = 0;
    const long blocks = (long)B * (gamma + 1) * S;
    if (blocks > 0x7fffffffL) return COS_ERR_SHAPE;
    const dim3 grid((unsigned)blocks), block(kThreads);
    if (profile) (void)hipEventRecord(ev_start, st);
    if (dt == COS_DTYPE_F32) {
      if (aligned) {
        if (p.masked) hipLaunchKernelGGL((expert_rowmax_kernel<float, true>), grid, block, 0, st, p);
        hipLaunchKernelGGL((greedy_contrastive_kernel<float, true>), grid, block, 0, st, p);
      } else {
        if (p.masked) hipLaunchKernelGGL((expert_rowmax_kernel<float, false>), grid, block, 0, st, p);
        hipLaunchKernelGGL((greedy_contrastive_kernel<float, false>), grid, block, 0, st, p);
      }
    } else {
      if (aligned) {
        if (p.masked) hipLaunchKernelGGL((expert_rowmax_kernel<uint16_t, true>), grid, block, 0, st, p);
        hipLaunchKernelGGL((greedy_contrastive_kernel<uint16_t, true>), grid, block, 0, st, p);
      } else {
        if (p.masked) hipLaunchKernelGGL((expert_rowmax_kernel<uint16_t, false>), grid, block, 0, st, p);
        hipLaunchKernelGGL((greedy_contrastive_kernel<uint16_t, false>), grid, block, 0, st, p);
      }
    }
    if (profile) {
      (void)hipEventRecord(ev_stop, st);
      ++g_ev_recorded;
    }
    return hipGetLastError() == hipSuccess ? COS_OK : COS_ERR_LAUNCH;
  }

  cos_status_t rc;
  if (dt == COS_DTYPE_F32)
    rc = aligned ? launch_all<float, true>(p, mode, window, lds, st, ev_start, ev_stop)
                 : launch_all<float, false>(p, mode, window, lds, st, ev_start, ev_stop);
  else
    rc = aligned ? launch_all<uint16_t, true>(p, mode, window, lds, st, ev_start, ev_stop)
                 : launch_all<uint16_t, false>(p, mode, window, lds, st, ev_start, ev_stop);
  if (profile) ++g_ev_recorded;
  return rc;
}

const char* cos_status_string(cos_status_t status) {
  switch (status) {
    case COS_OK: return "ok";
    case COS_ERR_NULL: return "a required pointer is NULL";
    case COS_ERR_SHAPE: return "n, B, gamma or V outside the supported range";
    case COS_ERR_DTYPE: return "unknown logits dtype";
    case COS_ERR_MODE: return "unknown combine mode, or contrastive mode with n != 2";
    case COS_ERR_WEIGHTS: return "invalid combine weights";
    case COS_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case COS_ERR_ALIGN: return "logits pointer not aligned to its element size";
    case COS_ERR_LAUNCH: return "a HIP call failed";
    case COS_ERR_UNSUPPORTED: return "not supported";
  }
  return "unknown status";
}

int cos_verify_version(void) { return 3; }

cos_status_t cos_profile_enable(int slots) {
  if (slots < 0 || slots > kMaxProfileSlots) return COS_ERR_SHAPE;
  while (g_ev_created < slots) {
    if (hipEventCreate(&g_ev_start[g_ev_created]) != hipSuccess) return COS_ERR_LAUNCH;
    if (hipEventCreate(&g_ev_stop[g_ev_created]) != hipSuccess) return COS_ERR_LAUNCH;
    ++g_ev_created;
  }
  g_ev_slots = slots;
  g_ev_recorded = 0;
  return COS_OK;
}

int cos_profile_recorded(void) { return g_ev_recorded < g_ev_slots ? g_ev_recorded : g_ev_slots; }

cos_status_t cos_profile_kernel_ms(int index, float* ms) {
  if (!ms) return COS_ERR_NULL;
  if (index < 0 || index >= cos_profile_recorded()) return COS_ERR_SHAPE;
  if (hipEventSynchronize(g_ev_stop[index]) != hipSuccess) return COS_ERR_LAUNCH;
  if (hipEventElapsedTime(ms, g_ev_start[index], g_ev_stop[index]) != hipSuccess) return COS_ERR_LAUNCH;
  return COS_OK;
}

void cos_tune_set_chunk_vectors(int vectors) { g_chunk_vectors = vectors > 0 ? vectors : 0; }

void cos_tune_set_sample_blocks(int blocks) { g_sample_blocks = blocks > 0 ? blocks : 0; }

}  // extern "C"
