// cos_device.h -- constants, the structures shared by the kernels, wavefront and
// hand-off primitives, logit loads and the logit-level combinations (gfx950).
#pragma once

#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>

#include "cos_verify.h"

// Constants and structures shared by the host side and the kernels' translation units.
namespace cosv {


constexpr int kThreads = 256;  // 4 wavefronts of 64 lanes
constexpr int kWaves = kThreads / 64;
constexpr int kUnroll = 8;  // 16-byte loads in flight per lane and iteration
constexpr float kLog2e = 1.44269504088896340736f;
constexpr int kNoOffset = -(1 << 29);       // "no finite element seen yet"
constexpr float kMaxOffset = 268435456.0f;  // 2^28: clamp for absurd logits
constexpr float kOffNever = 1.0e30f;         // offset of a term that must evaluate to 0
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

// A value that one workgroup hands to another inside one launch.  It can only be written by
// publish() -- an agent-scope atomic store, which gfx950 executes as a write-through store
// (global_store ... sc1) -- and only be read by read() -- an agent-scope atomic load
// (global_load ... sc1), which is served coherently at agent scope and never from a line another
// compute die's writes could have made stale.  There is no other access to the member, so a plain
// store or load of hand-off data (which the hand-off below would not cover) does not compile.
// Protocol (see wait_stores / arrive_last): publish, wait for the stores' completion, bump the
// counter; the workgroup that sees the last count reads.
template <typename U>
class HandOff {
 public:
#if defined(__HIPCC__)
  __device__ __forceinline__ void publish(U v) { __hip_atomic_store(&v_, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
  __device__ __forceinline__ U read() const { return __hip_atomic_load(&v_, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
#endif
 private:
  U v_;
};

// One partial softmax statistic: Z = sum_x 2^(l(x)*log2e - o) over a chunk.
struct Partial {
  HandOff<double> Z;
  HandOff<int> o;
  int pad;
};
static_assert(sizeof(Partial) == 16, "two partials per 32 bytes");

// A token that may lie in the plausibility mask of Eq. (5), with its two logits (masked contrastive
// mode: what the streaming kernel keeps of a row beside its statistics).
struct Cand {
  int idx;
  float l0, l1;
};
constexpr int kCandChunk = 256;  // candidates a chunk can leave in the workspace

// What the streaming kernel leaves for the sampling kernel, per sequence.
struct SeqPlan {
  int jstar;     // position that is sampled = accepted_len
  int residual;  // 1: f = max(0, r - q); 0: f = r (bonus)
  int pi;        // proposer of the sampled position
  int bonus;     // >= 0: the bonus token is drawn from this model's softmax alone (jstar == gamma)
  float m0;      // contrastive: expert maximum at jstar
  int skip;      // 1: every draft accepted and no extra token wanted: nothing is sampled
  int redo;      // left by the sampling kernel for the refinement kernels: 0 the token is drawn,
                 // kLittleMass: draw from the residual in its difference form, kNoMass: draw from r;
                 // kWholeRow (left by the one-read contrastive mode's finishing kernel): draw a
                 // verifier's own bonus token from its whole row
  int pad;
  double lse2[COS_MAX_MODELS];  // log2-sum-exp2 of the statistics at jstar
};
constexpr int kDrawn = 0, kNoMass = 1, kLittleMass = 2;  // what a draw reports (cos_sample.h)
constexpr int kWholeRow = 3;  // SeqPlan::redo only: nothing drawn yet, the weights of the plan as they are

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
  int* counters;      // (stride kCtrStride) [nwin windows][B] streaming arrivals, [B] sampling
                      // arrivals, 2 x [B] arrivals of the refinement kernels and their two control
                      // counters, [B][gamma] acceptance-rate arrivals
  Partial* partials;  // [B][gamma+1][nstat][S]
  float* rowmax;      // contrastive: [B][gamma+1][S] partial maxima of the expert row
  Cand* cand;         // masked contrastive, one-pass: [B][gamma+1][S][cand_cap] candidates of every chunk
  int* cand_count;    //   [B][gamma+1][S] how many (-1: they did not fit)
  int cand_cap;
  SeqPlan* plans;     // [B]
  HandOff<double>* tile_sums;  // [B][ntiles]
  // refinement kernels (a residual of little or no mass drawn from once more, by many workgroups)
  int* refine_ctl;                   // two counters (stride kCtrStride): marked sequences; those finished
  int* refine_list;                  // [B]: the marked sequences, in the order they were marked
  HandOff<double>* refine_partials;  // [refine_grid][COS_MAX_MODELS + 1]: every workgroup's sums of the first pass
  float* refine_dlse;                // [B][COS_MAX_MODELS]: differences of the log-normalisers it gives
  int whole_row_bonus;               // one-read contrastive mode: a verifier's own bonus token is left to
                                     // refine_draw_kernel (else the finishing workgroup draws it alone)
  int refine_grid;                   // workgroups of a refinement launch (>= B)
  int refine_cmax;                   // most workgroups one sequence is split over (>= 8 tiles each)
  // acceptance-rate output (optional)
  double* alpha;           // [B][gamma] out, or NULL
  double* lse_all;         // [B][gamma+1][nstat] log2-sum-exp2 of every position
  float* rowmax_all;       // contrastive: [B][gamma+1] expert maxima
  HandOff<double>* alpha_partials;  // [B][gamma][CA]
  int CA;                  // acceptance-rate workgroups per (sequence, position)
  int tpa;                 // tiles per acceptance-rate workgroup
  int S;              // stride of the per-chunk arrays: the larger of Sh and St
  int Sh, cvh;        // sequences before b_tail: chunks per row, vectors per chunk
  int St, cvt;        // sequences from b_tail on (the end of the grid, which runs while the GPU drains):
                      // more and shorter chunks
  int b_tail;         // first sequence cut the second way (B: none)
  int nvec;           // 16-byte vectors per row (last may be partial when unaligned)
  int ntiles;         // tiles (64 vectors) per row
  int nstat;          // statistics per position: n (ensemble) or 3 (contrastive)
  int C;              // sampling workgroups per sequence
  int tpc;            // tiles per sampling workgroup
  int j0;             // first position of this launch's window
  int nj;             // positions in this launch's window (gamma+1: the whole step in one launch)
  int win;            // window index (selects the arrival counters)
  int nwin;           // streaming launches of the call = sets of streaming arrival counters
  int fill_count;     // > 0: no fill kernel ran; the call's first kernel clears this many counter ints
                      // and marks the sequences undecided itself
  double w[COS_MAX_MODELS];  // ensemble weights; contrastive: w[0] = mu, w[1] = alpha_cd
  float scale;               // log2(e) / temperature: logits times this are base-2 exponents
  float mu_hi, mu_lo;        // mu split into two floats
  float beta_hi[COS_MAX_MODELS], beta_lo[COS_MAX_MODELS];  // logit mix: beta_m split into two floats
  int masked;                // contrastive: alpha_cd > 0 (else no row-max pass runs and m0 is taken as 0)
  float thr32;               // smallest float >= T ln(alpha_cd)
  double thr64;              // T ln(alpha_cd)
  cos_diag_t diag;
};

// How one call is launched: filled in by the host side of the ABI, consumed by the
// per-format translation units (cos_kernels_*.hip), which hold the kernels.
struct LaunchPlan {
  int mode;         // kEns, kCd or kMix
  int window;       // positions per streaming launch
  int greedy;       // temperature 0: one argmax kernel instead
  int onepass;      // masked contrastive mode in one read of the logits (candidate lists), no counters
  int ready;        // the caller promises zeroed arrival counters: no clearing kernel
  int refine_kernels;  // residuals of little mass are drawn from by two more launches (which do nothing
                       // when no sequence needs them) instead of by one workgroup
  int aligned;      // every row starts on a 16-byte boundary and V is a multiple of the vector width
  int counters;     // arrival counters (ints, with their stride) the fill kernel clears
  size_t lds;       // dynamic LDS of the sampling kernel (one double per tile)
  hipStream_t stream;
  hipEvent_t ev_start, ev_stop;  // optional: recorded around the streaming launches
};

// Enqueue every kernel of one call for logits stored as float32 / bfloat16 / binary16.
cos_status_t run_f32(const Params& p, const LaunchPlan& lp);
cos_status_t run_bf16(const Params& p, const LaunchPlan& lp);
cos_status_t run_f16(const Params& p, const LaunchPlan& lp);

}  // namespace cosv

using namespace cosv;

namespace {

// Drafts of row b; position drafts_of(p, b) plays the bonus position's role.
__device__ __forceinline__ int drafts_of(const Params& p, int b) {
  return p.num_drafts ? p.num_drafts[b] : p.gamma;
}

// Where a streaming workgroup works: its sequence, its index among that sequence's
// workgroups, and how the sequence's rows are cut.  The grid lists the sequences in
// order, rows_per_b rows each, every row cut into S chunks.
struct Place {
  int b, rem, S, cv, per_b;
};
__device__ __forceinline__ Place place_of(const Params& p, int rows_per_b) {
  Place pl;
  const int per_head = rows_per_b * p.Sh;
  const int head = p.b_tail * per_head;
  if ((int)blockIdx.x < head) {
    pl.S = p.Sh;
    pl.cv = p.cvh;
    pl.per_b = per_head;
    pl.b = blockIdx.x / per_head;
    pl.rem = blockIdx.x - pl.b * per_head;
  } else {
    const int i = blockIdx.x - head;
    pl.S = p.St;
    pl.cv = p.cvt;
    pl.per_b = rows_per_b * p.St;
    const int bb = i / pl.per_b;
    pl.b = p.b_tail + bb;
    pl.rem = i - bb * pl.per_b;
  }
  return pl;
}
__device__ __forceinline__ int splits_of(const Params& p, int b) { return b < p.b_tail ? p.Sh : p.St; }

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

// Wait until this wavefront's outstanding vector-memory operations have completed (vmcnt counts
// them down as they complete; for a write-through store that is the acknowledgement from the
// memory side it was written through to).  After a wavefront's publish() calls this is the release
// half of the hand-off: what it published is in place, for every compute die, before the wavefront
// goes on to the barrier and the counter bump of arrive_last().  It is the instruction sequence
// the compiler emits for an agent-scope release minus the cache write-back (buffer_wbl2), which
// only serves plain stores that may still sit dirty in a cache -- HandOff has none.
__device__ __forceinline__ void wait_stores() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// Last-arrival test.  Every wavefront must have called wait_stores() after its
// hand-off stores.  Returns true in every thread of exactly one workgroup per
// counter: the one that arrives after all `total` workgroups have published.
// The counter is bumped by an agent-scope atomic increment, executed where every compute die's atomics
// on that address are executed, so exactly one workgroup sees total - 1.  That workgroup's reads
// come after the barrier that follows the increment's returned value: they cannot be issued earlier, and
// being agent-scope loads (HandOff::read) they need no cache invalidation in front of them.
__device__ __forceinline__ bool arrive_last(int* counter, int total, int* s_flag) {
  __syncthreads();
  if (threadIdx.x == 0) {
    // increment that wraps to zero at the last arrival: the counter is left as it was found, so a
    // workspace whose counters were zero before a call has them zero after it
    const unsigned prev = __builtin_amdgcn_atomic_inc32(reinterpret_cast<unsigned*>(counter), (unsigned)(total - 1),
                                                        __ATOMIC_RELAXED, "agent");
    *s_flag = (prev == (unsigned)(total - 1));
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

// The same 16 bytes from an address that is only aligned to the element: one
// global_load_dwordx4 as well (unaligned access is enabled for compute on this GPU).
template <typename T>
__device__ __forceinline__ uint4 load_stream16_unaligned(const T* p) {
  typedef u32x4_t __attribute__((aligned(2))) u32x4_a2;
  typedef u32x4_t __attribute__((aligned(4))) u32x4_a4;
  u32x4_t v;
  if constexpr (sizeof(T) == 2)
    v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_a2*>(p));
  else
    v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_a4*>(p));
  return make_uint4(v.x, v.y, v.z, v.w);
}

__device__ __forceinline__ float widen(float x) { return x; }
__device__ __forceinline__ float widen(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }
__device__ __forceinline__ float widen(_Float16 h) { return (float)h; }

// Storage types: float, uint16_t = bfloat16 bit patterns, _Float16 = IEEE binary16.
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
template <typename T>
struct IsBf16 {
  static constexpr bool value = false;
};
template <>
struct IsBf16<uint16_t> {
  static constexpr bool value = true;
};

// A 16-bit pattern (a non-negative value of T) as float32.
template <typename T>
__device__ __forceinline__ float raw16_to_float(int bits) {
  if constexpr (IsBf16<T>::value)
    return __uint_as_float((uint32_t)bits << 16);
  else
    return (float)__builtin_bit_cast(_Float16, (uint16_t)bits);
}

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

// binary16 -> float32 is exact (v_cvt_f32_f16).
template <>
__device__ __forceinline__ void unpack<_Float16>(const uint4& raw, float (&x)[8]) {
  const half2_t a = __builtin_bit_cast(half2_t, raw.x), b = __builtin_bit_cast(half2_t, raw.y);
  const half2_t c = __builtin_bit_cast(half2_t, raw.z), d = __builtin_bit_cast(half2_t, raw.w);
  x[0] = (float)a.x;
  x[1] = (float)a.y;
  x[2] = (float)b.x;
  x[3] = (float)b.y;
  x[4] = (float)c.x;
  x[5] = (float)c.y;
  x[6] = (float)d.x;
  x[7] = (float)d.y;
}

// Vector `vec` of a row.  ALIGNED: the row is 16-byte aligned and V is a
// multiple of the vector width, so every vector is one full 16-byte load.
// Otherwise rows start anywhere (an odd vocabulary): a vector that lies inside
// the row is still one 16-byte load, from an element-aligned address; only the
// row's last, partial vector is read element by element, past V as -inf.
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
    if (base + N <= V) {
      const uint4 raw = load_stream16_unaligned<T>(row + base);
      unpack<T>(raw, x);
    } else {
#pragma unroll
      for (int k = 0; k < N; ++k) x[k] = (base + k < V) ? widen(row[base + k]) : -INFINITY;
    }
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
// logit-level combinations shared by the streaming and the sampling kernels
// ---------------------------------------------------------------------------

// Logit-level combinations are evaluated on logits shifted by a per-row reference (the row's
// first element, 0 if that is not finite): a softmax does not see a shift, and the float32
// result then rounds at the scale of the logits' spread, not of their magnitude.
template <typename T>
__device__ __forceinline__ float row_reference(const T* row) {
  const float v = widen(row[0]);
  return (fabsf(v) < INFINITY) ? v : 0.0f;  // false for NaN as well
}

// Contrastive logit c = (l_0 - ref_0) - mu*(l_1 - ref_1) with mu = mu_hi + mu_lo.
__device__ __forceinline__ float contrast(float l0, float l1, float mu_hi, float mu_lo, float ref0,
                                          float ref1) {
  const float d1 = l1 - ref1;
  return fmaf(-mu_lo, d1, fmaf(-mu_hi, d1, l0 - ref0));
}

// Plausibility mask: l_0 - max l_0 >= ln(alpha_cd), and a finite expert logit.
// bf16 differences are exact in float32; float32 and binary16 inputs compare in float64.
template <typename T>
__device__ __forceinline__ bool in_mask(float l0, float m0, float thr32, double thr64) {
  if constexpr (IsBf16<T>::value) {
    return (l0 > -INFINITY) && (l0 - m0 >= thr32);
  } else {
    return (l0 > -INFINITY) && ((double)l0 - (double)m0 >= thr64);
  }
}

// Logit mix c = sum_m beta_m (l_m - ref_m) with beta_m = hi + lo; models with beta_m == 0
// take no part.  A -inf logit makes c = -inf (probability 0) instead of the NaN
// that hi * (-inf) + lo * (-inf) gives when hi and lo differ in sign.
template <int NCAP>
__device__ __forceinline__ float mix_one(const Params& p, int n, const float (&l)[NCAP],
                                         const float (&ref)[NCAP]) {
  float acc = 0.0f;
  bool dead = false;
#pragma unroll
  for (int m = 0; m < NCAP; ++m)
    if (m < n && (p.beta_hi[m] != 0.0f || p.beta_lo[m] != 0.0f)) {
      const bool ninf = l[m] == -INFINITY;
      dead = dead || ninf;
      const float v = ninf ? 0.0f : l[m] - ref[m];
      acc = fmaf(p.beta_lo[m], v, fmaf(p.beta_hi[m], v, acc));
    }
  return dead ? -INFINITY : acc;
}

// The rows of one vector shifted by their references, d_m = l_m - ref_m, and their combination
// c = sum_m beta_m d_m, with mix_one's numbers: the same two multiply-adds per model in model
// order; a model with beta_m = 0 adds 0 * d_m = 0 when d_m is finite.  A -inf (or non-finite) logit
// shows as a c that is not finite; only a wavefront that sees one pays for mix_one's tests (-inf
// stays -inf under the shift).  want_c = false (uniform): only the shifted rows are wanted.
template <int NCAP, int N>
__device__ __forceinline__ void mix_shifted_rows(const Params& p, int n, const float (&x)[NCAP][N],
                                                 const float (&ref)[NCAP], bool want_c,
                                                 float (&d)[NCAP][N], float (&c)[N]) {
  bool odd = false;
#pragma unroll
  for (int k = 0; k < N; ++k) {
    float acc = 0.0f;
#pragma unroll
    for (int m = 0; m < NCAP; ++m) {
      d[m][k] = m < n ? x[m][k] - ref[m] : 0.0f;
      if (m < n) acc = fmaf(p.beta_lo[m], d[m][k], fmaf(p.beta_hi[m], d[m][k], acc));
    }
    c[k] = acc;
    odd = odd || !(fabsf(acc) < INFINITY);
  }
  if (want_c && __ballot(odd)) {
    const float zero[NCAP] = {};
#pragma unroll
    for (int k = 0; k < N; ++k) {
      float l[NCAP];
#pragma unroll
      for (int m = 0; m < NCAP; ++m) l[m] = d[m][k];
      c[k] = mix_one<NCAP>(p, n, l, zero);
    }
  }
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

}  // namespace
