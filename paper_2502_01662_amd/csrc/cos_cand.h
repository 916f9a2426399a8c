// cos_cand.h -- Eq. (5) with the plausibility mask in ONE read of the logits.
//
// The mask {x : l_0(x) - max l_0 >= T ln(alpha_cd)} needs the expert row's maximum, which is only
// known when the row has been read.  But the mask is sparse (a handful of tokens for alpha_cd
// around 0.1), and a token that passes the test against the final maximum also passes it against
// any earlier, smaller maximum.  So the streaming kernel keeps, per chunk, the candidates -- the
// tokens that pass against the largest expert logit seen so far -- with their two logits, and the
// chunk's own maximum; the finishing kernel (one workgroup per sequence) takes the true maximum of
// every position, drops the candidates that fail against it, and has the whole masked row in hand:
// its normaliser, r(d), the acceptance rate sum min(q, r) of Eq. (7), and -- since the residual
// max(0, r - q) and r itself vanish outside the mask -- the draw, all in float64 on at most a few
// hundred tokens.  Every logit is read once; there is no pass for the expert maxima, no sampling
// kernel and no acceptance-rate kernel.
//
// A chunk whose candidates do not fit (a mask that is not sparse: alpha_cd tiny, or a flat expert
// row) is marked; the finishing workgroup then reads that position's rows itself, once more, with
// the true maximum (the masked statistic, the acceptance rate), and draws from the full row with
// the tile sums of the general sampling path.  The bonus token of a verifier alone (no mask) takes
// that general path too.
#pragma once

#include "cos_device.h"
#include "cos_stats.h"
#include "cos_sample.h"

namespace {

constexpr int kCandStage = 1024;  // candidates one streaming workgroup can stage in LDS
constexpr int kCandRow = 2048;    // masked tokens of one position the finishing workgroup can hold

// ---------------------------------------------------------------------------
// streaming kernel: proposer statistic, chunk maximum of the expert row, candidates
// ---------------------------------------------------------------------------

// What a wavefront carries through its chunk.
struct OnePass {
  Running rq;  // the proposer row's statistic
  float wm0;   // largest expert logit the wavefront has seen (wave-uniform)
};

// The wavefront's largest element of U raw vectors per lane.  16-bit formats: on the raw bit patterns
// with packed integer maxima (among non-negative values integer order is float order, and a pattern
// with the sign bit set never wins against one without); if every element is negative, or the format
// is float32, on the widened values.
template <typename T, int U>
__device__ __forceinline__ float raw_wave_max(const uint4 (&raw)[U]) {
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
    if (wm16 >= 0) return raw16_to_float<T>(wm16);
  }
  float lm = -INFINITY;
#pragma unroll
  for (int u = 0; u < U; ++u) {
    float x[N];
    unpack<T>(raw[u], x);
#pragma unroll
    for (int k = 0; k < N; ++k) lm = fmaxf(lm, x[k]);
  }
  return wave_max(lm);
}

// U vectors per lane of both rows (raw; vector u holds tokens first + u * kThreads * N ...): the
// proposer row's statistic, the expert row's running maximum, and the tokens that pass the mask test
// against it.
template <typename T, int U>
__device__ __forceinline__ void onepass_group(const Params& p, OnePass& st, const uint4 (&a0)[U], const uint4 (&a1)[U],
                                              int first, int pi, float ref0, float ref1, int* s_count, Cand* s_cand) {
  constexpr int N = VecOf<T>::N;
  const float m0 = raw_wave_max<T, U>(a0);
  st.wm0 = fmaxf(st.wm0, m0);
  // the proposer's row on the shifted logits (as the finishing kernel evaluates q); the shift is
  // monotone, so the row's largest shifted logit is its largest logit shifted
  const float refq = pi ? ref1 : ref0;
  const float mq = pi ? raw_wave_max<T, U>(a1) : m0;
  running_cover(st.rq, mq - refq, p.scale);
  const float neg_o = -(float)st.rq.o;
  // a cut just below the mask's edge against the running maximum: what lies above it is looked at
  // exactly (vectors past the chunk's end and elements past the row's end read as -inf: never in)
  const float edge = st.wm0 + p.thr32;
  const float cut = edge - 2.0f * fabsf(edge) * 1.1920929e-7f - 1e-30f;
#pragma unroll
  for (int u = 0; u < U; ++u) {
    float x0[N], x1[N];
    unpack<T>(a0[u], x0);
    unpack<T>(a1[u], x1);
    bool any = false;
#pragma unroll
    for (int k = 0; k < N; ++k) {
      st.rq.acc[k & 3] += fast_exp2(fmaf((pi ? x1[k] : x0[k]) - refq, p.scale, neg_o));
      any = any || x0[k] >= cut;
    }
    if (any) {  // a few lanes per chunk
#pragma unroll
      for (int k = 0; k < N; ++k)
        if (in_mask<T>(x0[k], st.wm0, p.thr32, p.thr64)) {
          const int at = atomicAdd(s_count, 1);
          if (at < kCandStage) {
            s_cand[at].idx = first + u * kThreads * N + k;
            s_cand[at].l0 = x0[k];
            s_cand[at].l1 = x1[k];
          }
        }
    }
  }
}

// Workgroup index -> (b, j, s); reads the chunk of both rows once.
template <typename T, bool ALIGNED>
__global__ void __launch_bounds__(kThreads) contrastive_onepass_kernel(Params p) {
  constexpr int N = VecOf<T>::N;
  constexpr int U = kUnroll / 2;  // 16-byte loads in flight per lane and row
  constexpr int kStep = kThreads * U;
  __shared__ WaveStat ws[kWaves];
  __shared__ float s_m0[kWaves];
  __shared__ int s_count, s_out;
  __shared__ Cand s_cand[kCandStage];

  const int g1 = p.gamma + 1;
  const Place pl = place_of(p, p.nj);
  const int b = pl.b;
  if (p.win > 0 && p.plans[b].jstar >= 0) return;  // decided by an earlier window: nothing more is read
  const int j = p.j0 + pl.rem / pl.S;
  const int s = pl.rem - (j - p.j0) * pl.S;
  const int tid = threadIdx.x;
  const int lane = lane_id();
  const int gb = drafts_of(p, b);
  // Whose softmax statistic this position needs: the proposer's at a draft position; at the bonus
  // position only a verifier bonus needs one at all.
  int pi = p.proposer[b];
  if (j < gb) {
    if (p.proposer_pos) pi = p.proposer_pos[(size_t)b * p.gamma + j];
  } else if (p.bonus_idx && p.bonus_idx[b] >= 0) {
    pi = p.bonus_idx[b];
  }
  const size_t slot = ((size_t)b * g1 + j) * p.S + s;
  Partial* out = p.partials + (((size_t)b * g1 + j) * 3) * p.S + s;
  if (position_unread(p, gb, j)) {  // uniform over the workgroup
    if (tid == 0) {
      store_empty_partial(out);
      store_empty_partial(out + (size_t)p.S);
      store_empty_partial(out + (size_t)2 * p.S);
      p.rowmax[slot] = -INFINITY;
      p.cand_count[slot] = 0;
    }
    return;
  }
  if (tid == 0) {
    s_count = 0;
    s_out = 0;
  }
  __syncthreads();

  const T* row0 = row_ptr<T>(p, 0, b, j);
  const T* row1 = row_ptr<T>(p, 1, b, j);
  const float ref0 = row_reference<T>(row0), ref1 = row_reference<T>(row1);
  const int v0 = s * pl.cv;
  const int v1 = min(v0 + pl.cv, p.nvec);
  // vectors that lie inside the row; an odd vocabulary leaves one partial vector at its end
  const int vfull = ALIGNED ? v1 : min(v1, p.V / N);
  OnePass st;
  running_init(st.rq);
  st.wm0 = -INFINITY;
  for (int base = v0; base < vfull; base += kStep) {
    // all loads of both rows go out before the first use
    uint4 a0[U], a1[U];
    load_raw_group<T, ALIGNED, U>(row0, base, vfull, a0);
    load_raw_group<T, ALIGNED, U>(row1, base, vfull, a1);
    if (base + kStep > vfull) {
      mask_raw_group<T, U>(base, vfull, a0);
      mask_raw_group<T, U>(base, vfull, a1);
    }
    onepass_group<T, U>(p, st, a0, a1, (base + tid) * N, pi, ref0, ref1, &s_count, s_cand);
  }
  if (!ALIGNED && v1 > vfull && tid < 64) {
    // the partial vector belongs to this chunk: lane 0 of the first wavefront brings it in
    const uint32_t ninf = sizeof(T) == 4 ? 0xff800000u : (IsBf16<T>::value ? 0xff80ff80u : 0xfc00fc00u);
    const uint4 none = make_uint4(ninf, ninf, ninf, ninf);
    uint4 a0[1], a1[1];
    a0[0] = tid == 0 ? load_tail_raw<T>(row0, vfull * N, p.V) : none;
    a1[0] = tid == 0 ? load_tail_raw<T>(row1, vfull * N, p.V) : none;
    onepass_group<T, 1>(p, st, a0, a1, vfull * N, pi, ref0, ref1, &s_count, s_cand);
  }
  const double zq = running_total(st.rq);
  publish_wave_stat(ws, 0, st.rq.o, zq);
  if (lane == 0) s_m0[tid >> 6] = st.wm0;
  __syncthreads();
  float m_wg = s_m0[0];
  for (int w = 1; w < kWaves; ++w) m_wg = fmaxf(m_wg, s_m0[w]);
  if (tid == 0) {
    store_partial(ws, 0, out + (size_t)pi * p.S);
    store_empty_partial(out + (size_t)(1 - pi) * p.S);
    store_empty_partial(out + (size_t)2 * p.S);
    p.rowmax[slot] = m_wg;
  }
  // keep what passes against the chunk's own maximum (earlier, smaller maxima let more in)
  const int staged = s_count;
  Cand* dst = p.cand + slot * (size_t)p.cand_cap;
  for (int i = tid; i < min(staged, kCandStage); i += kThreads) {
    const Cand c = s_cand[i];
    if (in_mask<T>(c.l0, m_wg, p.thr32, p.thr64)) {
      const int at = atomicAdd(&s_out, 1);
      if (at < p.cand_cap) dst[at] = c;
    }
  }
  __syncthreads();
  if (tid == 0) p.cand_count[slot] = (staged > kCandStage || s_out > p.cand_cap) ? -1 : s_out;  // -1: did not fit
}

// ---------------------------------------------------------------------------
// finishing kernel: one workgroup per sequence
// ---------------------------------------------------------------------------

constexpr int kWin = COS_MAX_GAMMA + 1;  // positions a window can hold

struct FinishShared {
  Cand list[kCandRow];   // the masked tokens of the window's positions, one segment per position
  union {
    double f[kCandRow];  // draw: the sampling weights of the sampled position's tokens, ascending
    int pre[kWin * kMaxSplits];  // before: per position, the candidates of the chunks before each chunk
  };
  double red[kWaves];
  float m0[kWin];        // expert maximum per position
  float ref[kWin][2];    // row references per position
  int total[kWin];       // candidates per position before the test against the true maximum
  int off[kWin + 1];     // segment of each position in list
  int toff[kWin + 1];    // prefix of `total`: where each position's candidates start among all the window's
  int recount;           // 1: the totals do not fit the list; the segments are sized by the masked tokens
  int n[kWin];           // masked tokens per position
  int slow[kWin];        // 1: the position's candidates did not fit
  int flag;
};

__device__ __forceinline__ double block_sum(double v, double* red) {
  v = wave_sum(v);
  __syncthreads();
  if (lane_id() == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  double t = red[0];
  for (int w = 1; w < kWaves; ++w) t += red[w];
  return t;
}

__device__ __forceinline__ int wave_max_int(int v) {
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) v = max(v, __shfl_xor(v, d, 64));
  return v;
}
__device__ __forceinline__ long long wave_sum_ll(long long v) {
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d, 64);
  return v;
}

// Sums over a position's masked tokens must not depend on the order in which the wavefronts found
// them (a call gives the same bits every time): terms in [0, 1] are added as 2^-50 fixed-point
// integers, whose sum is exact in any order (at most kCandRow = 2^11 terms).
constexpr double kFix = 1125899906842624.0;  // 2^50
__device__ __forceinline__ long long to_fix(double v) { return (long long)(v * kFix + 0.5); }

// Ascending token index (the order of the inverse CDF): list[0 .. n).  Up to one token per thread each
// thread counts the tokens below its own and moves it there; longer lists take a bitonic merge sort
// whose comparators all put the smaller token first, so that positions past n need not exist.
__device__ __forceinline__ void sort_by_token(Cand* list, int n) {
  if (n <= kThreads) {
    Cand mine = {0, 0.0f, 0.0f};
    int rank = 0;
    if ((int)threadIdx.x < n) {
      mine = list[threadIdx.x];
      for (int i = 0; i < n; ++i) rank += list[i].idx < mine.idx;
    }
    __syncthreads();
    if ((int)threadIdx.x < n) list[rank] = mine;
    __syncthreads();
    return;
  }
  for (int k = 2; (k >> 1) < n; k <<= 1)
    for (int jj = k >> 1; jj > 0; jj >>= 1) {
      for (int i = threadIdx.x; i < n; i += kThreads) {
        const int partner = (jj == (k >> 1)) ? (i ^ (k - 1)) : (i ^ jj);
        if (partner > i && partner < n) {
          const Cand a = list[i], c = list[partner];
          if (a.idx > c.idx) {
            list[i] = c;
            list[partner] = a;
          }
        }
      }
      __syncthreads();
    }
}

// Contrastive logit on the shifted logits in float64, as decide_outcome evaluates it at a draft.
__device__ __forceinline__ double cand_c(const Params& p, const Cand& c, double ref0, double ref1) {
  return shifted(c.l0, ref0) - p.w[0] * shifted(c.l1, ref1);
}
// The proposer's shifted logit of a candidate, as its row's statistic was summed over.
__device__ __forceinline__ double cand_q(const Cand& c, int pi, double ref0, double ref1) {
  return pi ? shifted(c.l1, ref1) : shifted(c.l0, ref0);
}

// Masked statistic (and acceptance rate) of a position whose candidates did not fit: this one
// workgroup reads both rows again, with the true expert maximum.
template <typename T, bool ALIGNED>
__device__ __forceinline__ double slow_masked_lse(const Params& p, int b, int j, float m0, WaveStat* ws) {
  constexpr int N = VecOf<T>::N;
  constexpr int U = 4;
  constexpr int kStep = kThreads * U;
  const T* row0 = row_ptr<T>(p, 0, b, j);
  const T* row1 = row_ptr<T>(p, 1, b, j);
  const float ref0 = row_reference<T>(row0), ref1 = row_reference<T>(row1);
  Running rc;
  running_init(rc);
  for (int base = 0; base < p.nvec; base += kStep) {
    float x0[U][N], x1[U][N];
    load_group<T, ALIGNED, true, U>(row0, base, p.nvec, p.V, x0);
    load_group<T, ALIGNED, true, U>(row1, base, p.nvec, p.V, x1);
    float c[U][N];
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int k = 0; k < N; ++k)
        c[u][k] = in_mask<T>(x0[u][k], m0, p.thr32, p.thr64) ? contrast(x0[u][k], x1[u][k], p.mu_hi, p.mu_lo, ref0, ref1)
                                                             : -INFINITY;
    running_add<U, N>(rc, c, p.scale);
  }
  const double zc = running_total(rc);
  __syncthreads();
  publish_wave_stat(ws, 0, rc.o, zc);
  __syncthreads();
  int omax = kNoOffset;
  for (int w = 0; w < kWaves; ++w)
    if (ws[w].z > 0.0 && ws[w].o > omax) omax = ws[w].o;
  double z = 0.0;
  for (int w = 0; w < kWaves; ++w)
    if (ws[w].z > 0.0) z += ldexp(ws[w].z, ws[w].o - omax);
  return z > 0.0 ? (double)omax + log2(z) : -INFINITY;
}

template <typename T, bool ALIGNED>
__device__ __forceinline__ double slow_alpha(const Params& p, int b, int j, int pi, float m0, double lse_c,
                                             double lse_q, double* red) {
  constexpr int N = VecOf<T>::N;
  constexpr int U = 4;
  constexpr int kStep = kThreads * U;
  const T* row0 = row_ptr<T>(p, 0, b, j);
  const T* row1 = row_ptr<T>(p, 1, b, j);
  const float ref0 = row_reference<T>(row0), ref1 = row_reference<T>(row1);
  const double Kc = rint(lse_c), Kq = rint(lse_q);
  const float offc = (float)Kc, offq = (float)Kq;
  const float cr = (float)exp2(Kc - lse_c), cq = (float)exp2(Kq - lse_q);
  double acc = 0.0;
  for (int base = 0; base < p.nvec; base += kStep) {
    float x0[U][N], x1[U][N];
    load_group<T, ALIGNED, true, U>(row0, base, p.nvec, p.V, x0);
    load_group<T, ALIGNED, true, U>(row1, base, p.nvec, p.V, x1);
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int k = 0; k < N; ++k)
        if (in_mask<T>(x0[u][k], m0, p.thr32, p.thr64)) {  // r = 0 elsewhere, and so is min(q, r)
          const float cc = contrast(x0[u][k], x1[u][k], p.mu_hi, p.mu_lo, ref0, ref1);
          const float r = cr * fast_exp2(fmaf(cc, p.scale, -offc));
          const float q = cq * fast_exp2(fmaf((pi ? x1[u][k] - ref1 : x0[u][k] - ref0), p.scale, -offq));
          acc += (double)fminf(q, r);
        }
  }
  return block_sum(acc, red);
}

// Workgroup b: the masked statistics of every position of the window, Eq. (6), the first rejection,
// the outputs, the acceptance rates, and the draw.  The positions are worked on side by side -- a
// wavefront per position for what is per position, all threads for the candidates -- so that the
// kernel is a handful of dependent memory round trips, not one per position and chunk.
template <typename T, bool ALIGNED>
__global__ void __launch_bounds__(kThreads) contrastive_finish_kernel(Params p) {
  extern __shared__ double tile_sum[];  // general draw only: one double per tile
  __shared__ DecideShared sh;
  __shared__ FinishShared fs;
  __shared__ WaveStat ws[kWaves];
  __shared__ Refine<2> s_rf;

  const int b = blockIdx.x;
  const int tid = threadIdx.x;
  const int lane = lane_id();
  const int wave = tid >> 6;
  if (p.win > 0 && p.plans[b].jstar >= 0) return;  // decided by an earlier window
  const int g1 = p.gamma + 1;
  const int gb = drafts_of(p, b);
  const int Sb = splits_of(p, b);
  const int nj = p.nj;
  const int ndraft = max(min(p.j0 + nj, gb) - p.j0, 0);
  const double log2e = (double)p.scale;
  // The kernel is a chain of dependent memory round trips; everything that depends on nothing is asked
  // for at once: the side arrays of the drafts, the uniform of the draw, what the chunks left behind.
  DraftGather g;
  gather_drafts_side(p, b, ndraft, g);
  const double u_res = p.u_resample[b];

  // 1. per position (a wavefront each): the expert maximum, how many candidates the chunks left and
  //    whether they all fit, the rows' references.  The loads go out before the proposer rows'
  //    partials are combined (which waits for its own loads), the results are used after it.
  constexpr int kPos = (kWin + kWaves - 1) / kWaves;  // positions a wavefront can have
  constexpr int kSeg = kMaxSplits / 64;               // chunks a lane can have
  float ld_max[kPos][kSeg], ld_ref[kPos];
  int ld_cnt[kPos][kSeg];
#pragma unroll
  for (int q = 0; q < kPos; ++q) {
    const int jj = wave + q * kWaves;
    const int j = p.j0 + jj;
    const bool live = jj < nj && !position_unread(p, gb, j);
    const size_t slot0 = ((size_t)b * g1 + j) * p.S;
#pragma unroll
    for (int t = 0; t < kSeg; ++t) {
      const int s = lane + t * 64;
      ld_max[q][t] = (live && s < Sb) ? p.rowmax[slot0 + s] : -INFINITY;
      ld_cnt[q][t] = (live && s < Sb) ? p.cand_count[slot0 + s] : 0;
    }
    ld_ref[q] = (live && lane < 2) ? row_reference<T>(row_ptr<T>(p, lane, b, j)) : 0.0f;
  }
  combine_partials(p, b, sh);  // the proposer rows' statistics (statistic 2 is filled below)
  gather_drafts_logits<T, kCd>(p, b, ndraft, g);  // second round trip, together with the candidates below
#pragma unroll
  for (int q = 0; q < kPos; ++q) {
    const int jj = wave + q * kWaves;
    if (jj >= nj) continue;  // wave-uniform
    float lm = -INFINITY;
    int bad = 0, carry = 0;
#pragma unroll
    for (int t = 0; t < kSeg; ++t) {
      lm = fmaxf(lm, ld_max[q][t]);
      bad |= ld_cnt[q][t] < 0;
      // candidates of this position's chunks before chunk s (inclusive scan over the lanes, minus its own)
      const int c = max(ld_cnt[q][t], 0);
      int incl = c;
#pragma unroll
      for (int d = 1; d < 64; d <<= 1) {
        const int y = __shfl_up(incl, d, 64);
        if (lane >= d) incl += y;
      }
      const int s = lane + t * 64;
      if (s < Sb) fs.pre[jj * Sb + s] = carry + incl - c;
      carry += __shfl(incl, 63, 64);
    }
    lm = wave_max(lm);
    bad = __ballot(bad != 0) != 0;
    if (lane < 2) fs.ref[jj][lane] = ld_ref[q];
    if (lane == 0) {
      const bool unread = position_unread(p, gb, p.j0 + jj);
      fs.m0[jj] = unread ? 0.0f : lm;
      fs.total[jj] = (bad || unread) ? 0 : carry;
      fs.slow[jj] = bad ? 1 : 0;
      fs.n[jj] = 0;
    }
  }
  __syncthreads();
  // 2. a segment of the list for every position.  What the chunks left passes the test against their own
  //    maxima, the segments need only hold what passes against the position's: when the former do not fit
  //    (many chunks of a huge vocabulary, many positions), the sweep below first only counts.
  if (tid == 0) {
    int at = 0;
    for (int jj = 0; jj < nj; ++jj) {
      fs.toff[jj] = fs.off[jj] = at;
      at += fs.total[jj];
    }
    fs.toff[nj] = fs.off[nj] = at;
    fs.recount = at > kCandRow;
  }
  __syncthreads();
  // 3. every chunk's candidates, tested against the position's true maximum, into the segments: entry
  //    e of the window's candidates belongs to the position whose stretch of the totals holds e and to
  //    the chunk whose prefix holds the rest; four entries per thread at a time, their loads independent.
  auto sweep = [&](bool count_only) {
    const int all = fs.toff[nj];
    constexpr int R = 4;
    for (int e0 = tid; e0 < all; e0 += kThreads * R) {
      Cand c[R];
      int seg[R];
#pragma unroll
      for (int r = 0; r < R; ++r) {
        const int e = e0 + r * kThreads;
        seg[r] = -1;
        c[r].idx = 0;
        c[r].l0 = c[r].l1 = 0.0f;
        if (e < all) {
          int jj = 0;
          while (fs.toff[jj + 1] <= e) ++jj;  // (empty stretches are skipped: their end is not above e)
          const int within = e - fs.toff[jj];
          const int* pre = fs.pre + jj * Sb;
          int lo = 0, hi = Sb - 1;  // last chunk whose prefix is <= within
          while (lo < hi) {
            const int mid = (lo + hi + 1) >> 1;
            if (pre[mid] <= within) lo = mid; else hi = mid - 1;
          }
          const size_t slot = ((size_t)b * g1 + p.j0 + jj) * p.S + lo;
          c[r] = p.cand[slot * (size_t)p.cand_cap + (within - pre[lo])];
          seg[r] = jj;
        }
      }
#pragma unroll
      for (int r = 0; r < R; ++r)
        if (seg[r] >= 0 && !fs.slow[seg[r]] && in_mask<T>(c[r].l0, fs.m0[seg[r]], p.thr32, p.thr64)) {
          const int at = atomicAdd(&fs.n[seg[r]], 1);
          if (!count_only) fs.list[fs.off[seg[r]] + at] = c[r];
        }
    }
  };
  if (fs.recount) {  // uniform over the workgroup
    sweep(true);
    __syncthreads();
    if (tid == 0) {  // segments by the masked tokens; a position that still does not fit takes the slow route
      int at = 0;
      for (int jj = 0; jj < nj; ++jj) {
        fs.off[jj] = at;
        if (at + fs.n[jj] > kCandRow) fs.slow[jj] = 1; else at += fs.n[jj];
        fs.n[jj] = 0;
      }
      fs.off[nj] = at;
    }
    __syncthreads();
  }
  sweep(false);
  __syncthreads();
  // 4. per position (a wavefront each): the masked normaliser and the acceptance rate
  for (int jj = wave; jj < nj; jj += kWaves) {
    const int j = p.j0 + jj;
    if (position_unread(p, gb, j)) {
      if (lane == 0) {
        sh.rowmax[jj] = 0.0f;
        sh.lse2[jj * 3 + 2] = -INFINITY;
      }
      continue;
    }
    if (fs.slow[jj]) continue;
    const Cand* seg = fs.list + fs.off[jj];
    const int n = fs.n[jj];
    const double ref0 = (double)fs.ref[jj][0], ref1 = (double)fs.ref[jj][1];
    double cmax = -INFINITY;
    for (int i = lane; i < n; i += 64) cmax = fmax(cmax, cand_c(p, seg[i], ref0, ref1));
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) cmax = fmax(cmax, __shfl_xor(cmax, d, 64));
    // (float32 exponentials of float64 arguments: 1e-7 of each term, as in the streaming statistics)
    long long zf = 0;
    for (int i = lane; i < n; i += 64)
      zf += to_fix((double)fast_exp2((float)((cand_c(p, seg[i], ref0, ref1) - cmax) * log2e)));
    zf = wave_sum_ll(zf);
    const double z = (double)zf / kFix;
    const double lse_c = z > 0.0 ? cmax * log2e + log2(z) : -INFINITY;
    if (p.alpha && j < gb) {  // Eq. (7): min(q, r) vanishes outside the mask
      const int pi = p.proposer_pos ? p.proposer_pos[(size_t)b * p.gamma + j] : p.proposer[b];
      const double lse_q = sh.lse2[jj * 3 + pi];
      long long af = 0;
      for (int i = lane; i < n; i += 64) {
        const Cand c = seg[i];
        const double r = exp2(cand_c(p, c, ref0, ref1) * log2e - lse_c);
        const double q = exp2(cand_q(c, pi, ref0, ref1) * log2e - lse_q);
        af += to_fix(fmin(fmin(q, r), 1.0));
      }
      af = wave_sum_ll(af);
      if (lane == 0) p.alpha[(size_t)b * p.gamma + j] = (double)af / kFix;
    }
    if (lane == 0) {
      sh.rowmax[jj] = fs.m0[jj];
      sh.lse2[jj * 3 + 2] = lse_c;
    }
  }
  __syncthreads();
  // positions whose candidates did not fit: the whole workgroup reads their rows again (uniform)
  for (int jj = 0; jj < nj; ++jj) {
    if (!fs.slow[jj]) continue;
    const int j = p.j0 + jj;
    const float m0 = fs.m0[jj];
    const double lse_c = slow_masked_lse<T, ALIGNED>(p, b, j, m0, ws);
    double alpha = 0.0;
    const bool want = p.alpha && j < gb;
    if (want) {
      const int pi = p.proposer_pos ? p.proposer_pos[(size_t)b * p.gamma + j] : p.proposer[b];
      alpha = slow_alpha<T, ALIGNED>(p, b, j, pi, m0, lse_c, sh.lse2[jj * 3 + pi], fs.red);
    }
    if (tid == 0) {
      sh.rowmax[jj] = m0;
      sh.lse2[jj * 3 + 2] = lse_c;
      if (want) p.alpha[(size_t)b * p.gamma + j] = alpha;
    }
  }
  if (p.alpha)  // positions of the window without a draft have no acceptance rate
    for (int jj = tid; jj < nj; jj += kThreads)
      if (p.j0 + jj >= gb && p.j0 + jj < p.gamma) p.alpha[(size_t)b * p.gamma + p.j0 + jj] = NAN;
  __syncthreads();
  decide_outcome<T, kCd>(p, b, sh, g, ndraft);
  __syncthreads();
  const int jstar = sh.jstar;
  if (jstar < 0 || sh.skip) return;  // undecided (a later window continues), or nothing is drawn

  const int jj = jstar - p.j0;
  const bool residual = sh.residual != 0;
  const int pi = sh.pi;
  // a verifier's own bonus token is drawn from its whole softmax: the general route, as for a mask
  // that did not fit
  if (sh.bonus < 0 && !fs.slow[jj]) {
    Cand* seg = fs.list + fs.off[jj];
    const int n = fs.n[jj];
    sort_by_token(seg, n);
    // the weights norm(max(0, r - q)) or r of the masked tokens, float64, one thread per token ...
    const double ref0 = (double)fs.ref[jj][0], ref1 = (double)fs.ref[jj][1];
    const double lse_c = sh.lse2[jj * 3 + 2], lse_q = sh.lse2[jj * 3 + pi];
    // (The sparse mask holds nearly all of q's mass whenever r is close to q here, so this float64
    // evaluation on the masked tokens -- exact but for the 1e-7 of q's float32 normaliser -- is the best
    // there is also for residuals of little mass; a residual without any mass falls back to r.)
    for (int pass = 0; pass < 2; ++pass) {
      const bool res = residual && pass == 0;
      for (int i = tid; i < n; i += kThreads) {
        const Cand c = seg[i];
        const double r = exp2(cand_c(p, c, ref0, ref1) * log2e - lse_c);
        double f = r;
        if (res) {
          const double q = exp2(cand_q(c, pi, ref0, ref1) * log2e - lse_q);
          f = r - q > 0.0 ? r - q : 0.0;
        }
        fs.f[i] = f;
      }
      __syncthreads();
      // ... and the first wavefront scans them in ascending token order: a run of tokens per lane
      if (wave == 0) {
        const int per = (n + 63) / 64;
        const int i0 = min(lane * per, n), i1 = min(i0 + per, n);
        double run = 0.0;
        for (int i = i0; i < i1; ++i) run += fs.f[i];
        const double incl = wave_inclusive_scan(run);
        const double F = __shfl(incl, 63, 64);
        const bool fine = (F > 0.0 && F < INFINITY) || !res;
        if (fine) {
          const double up = __shfl_up(incl, 1, 64);
          const double target = u_res * F;
          // first token whose inclusive prefix exceeds the target; else the last token with mass
          double cum = lane ? up : 0.0, lo = 0.0, hi = 0.0, last_lo = 0.0, last_hi = 0.0;
          int hit = -1, last = -1;
          for (int i = i0; i < i1; ++i) {
            const double f = fs.f[i];
            const double nxt = cum + f;
            if (hit < 0 && nxt > target) {
              hit = i;
              lo = cum;
              hi = nxt;
            }
            if (f > 0.0) {
              last = i;
              last_lo = cum;
              last_hi = nxt;
            }
            cum = nxt;
          }
          const unsigned long long hits = __ballot(hit >= 0);
          const unsigned long long lasts = __ballot(last >= 0);
          int flags = (residual && !res) ? COS_FLAG_RESIDUAL_FALLBACK : 0;
          int src = 0, at = -1;
          if (hits) {
            src = __ffsll((long long)hits) - 1;
            at = hit;
          } else {  // rounding left no prefix above the target: the last token with mass
            flags |= COS_FLAG_TAIL_CLAMP;
            if (lasts) src = 63 - __clzll((long long)lasts);
            at = last;
            lo = last_lo;
            hi = last_hi;
          }
          if (lane == src) {
            const int token = at >= 0 ? seg[at].idx : 0;
            p.out_tokens[(size_t)b * g1 + jstar] = min(max(token, 0), p.V - 1);
            if (p.diag.sample_mass) p.diag.sample_mass[b] = F;
            if (p.diag.cdf_lo) p.diag.cdf_lo[b] = lo / F;
            if (p.diag.cdf_hi) p.diag.cdf_hi[b] = hi / F;
            if (p.diag.flags) p.diag.flags[b] = flags;
          }
        }
        if (lane == 0) fs.flag = fine ? 1 : 0;  // 0: no residual mass, once more from r itself
      }
      __syncthreads();
      if (fs.flag) break;
    }
    return;
  }

  if (p.whole_row_bonus && sh.bonus >= 0 && !residual) {
    // a verifier's own bonus token, large rows: left to refine_draw_kernel, which splits the marked
    // sequences' rows between a thousand workgroups (this one alone would take tens of microseconds)
    if (tid == 0) {
      p.plans[b].redo = kWholeRow;
      const int slot = __hip_atomic_fetch_add(p.refine_ctl, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      p.refine_list[slot] = b;
    }
    return;
  }
  // general draw: every tile sum of the sampled position by this one workgroup, then as the sampling kernel
  const SeqPlan plan = p.plans[b];  // written by this workgroup in decide_outcome (a barrier since)
  const T* rows[2];
  rows[0] = row_ptr<T>(p, 0, b, jstar);
  rows[1] = row_ptr<T>(p, 1, b, jstar);
  float coef[2], off[2], ref[2];
  plan_coefficients<2, kCd>(p, plan, residual, 2, coef, off);
  ref[0] = row_reference<T>(rows[0]);
  ref[1] = row_reference<T>(rows[1]);
  const Refine<2> no_refine = {};
  for (int t = wave; t < p.ntiles; t += kWaves) {
    float f[VecOf<T>::N];
    tile_weights<T, ALIGNED, 2, kCd>(p, rows, 2, t, plan.pi, plan.bonus, plan.m0, coef, off, ref, f, false, no_refine);
    const double ts = wave_sum(lane_mass<VecOf<T>::N>(f));
    if (lane == 0) tile_sum[t] = ts;
  }
  __syncthreads();
  finish_draw<T, ALIGNED, 2, kCd>(p, b, plan, rows, 2, coef, off, ref, tile_sum, fs.flag, s_rf);
}

}  // namespace
