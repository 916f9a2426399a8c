// cos_launch.h -- launches of one call, per storage format T.  Included by the
// translation units that instantiate the kernels for one format each
// (cos_kernels_f32.hip, cos_kernels_bf16.hip, cos_kernels_f16.hip), so that the
// formats compile in parallel.
#pragma once

#include "cos_device.h"
#include "cos_stats.h"
#include "cos_sample.h"
#include "cos_cand.h"

namespace {

// Kernels that hold the rows of all n models in registers are specialised for
// n = 1..4; more models take the generic instance.
template <typename T, bool ALIGNED, int NM, int MODE>
void launch_sampling_kernels(const Params& p, bool refine_kernels, dim3 grid, size_t lds, hipStream_t st) {
  const dim3 block(kThreads);
  if (!refine_kernels) {
    hipLaunchKernelGGL((sample_kernel<T, ALIGNED, NM, MODE, true>), grid, block, lds, st, p);
    return;
  }
  // The sampling kernel only marks a sequence whose residual has little or no mass; the two launches
  // after it split the marked sequences between their workgroups (which return at once when there is none).
  hipLaunchKernelGGL((sample_kernel<T, ALIGNED, NM, MODE, false>), grid, block, lds, st, p);
  const dim3 rgrid((unsigned)p.refine_grid);
  hipLaunchKernelGGL((refine_sums_kernel<T, ALIGNED, NM, MODE>), rgrid, block, 0, st, p);
  hipLaunchKernelGGL((refine_draw_kernel<T, ALIGNED, NM, MODE>), rgrid, block, lds, st, p);
}

template <typename T, bool ALIGNED, int MODE>
cos_status_t launch_sampling(const Params& p, bool refine_kernels, size_t lds, hipStream_t st) {
  const long blocks = (long)p.B * p.C;
  if (blocks <= 0 || blocks > 0x7fffffffL) return COS_ERR_SHAPE;
  const dim3 grid((unsigned)blocks);
  if constexpr (MODE == kCd) {
    launch_sampling_kernels<T, ALIGNED, 2, kCd>(p, refine_kernels, grid, lds, st);
  } else {
    switch (p.n) {
      case 1: launch_sampling_kernels<T, ALIGNED, 1, MODE>(p, refine_kernels, grid, lds, st); break;
      case 2: launch_sampling_kernels<T, ALIGNED, 2, MODE>(p, refine_kernels, grid, lds, st); break;
      case 3: launch_sampling_kernels<T, ALIGNED, 3, MODE>(p, refine_kernels, grid, lds, st); break;
      case 4: launch_sampling_kernels<T, ALIGNED, 4, MODE>(p, refine_kernels, grid, lds, st); break;
      default: launch_sampling_kernels<T, ALIGNED, 0, MODE>(p, refine_kernels, grid, lds, st); break;
    }
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
  } else {
    switch (p.n) {
      case 1: hipLaunchKernelGGL((acceptance_rate_kernel<T, ALIGNED, 1, MODE>), grid, block, 0, st, p); break;
      case 2: hipLaunchKernelGGL((acceptance_rate_kernel<T, ALIGNED, 2, MODE>), grid, block, 0, st, p); break;
      case 3: hipLaunchKernelGGL((acceptance_rate_kernel<T, ALIGNED, 3, MODE>), grid, block, 0, st, p); break;
      case 4: hipLaunchKernelGGL((acceptance_rate_kernel<T, ALIGNED, 4, MODE>), grid, block, 0, st, p); break;
      default: hipLaunchKernelGGL((acceptance_rate_kernel<T, ALIGNED, 0, MODE>), grid, block, 0, st, p); break;
    }
  }
  return hipGetLastError() == hipSuccess ? COS_OK : COS_ERR_LAUNCH;
}

template <typename T, bool ALIGNED>
void launch_mix_stats(const Params& p, dim3 grid, hipStream_t st) {
  const dim3 block(kThreads);
  switch (p.n) {
    case 1: hipLaunchKernelGGL((mix_stats_kernel<T, ALIGNED, 1>), grid, block, 0, st, p); break;
    case 2: hipLaunchKernelGGL((mix_stats_kernel<T, ALIGNED, 2>), grid, block, 0, st, p); break;
    case 3: hipLaunchKernelGGL((mix_stats_kernel<T, ALIGNED, 3>), grid, block, 0, st, p); break;
    case 4: hipLaunchKernelGGL((mix_stats_kernel<T, ALIGNED, 4>), grid, block, 0, st, p); break;
    default: hipLaunchKernelGGL((mix_stats_kernel<T, ALIGNED, 0>), grid, block, 0, st, p); break;
  }
}

// Workgroups of a streaming launch: rows_per_b rows per sequence, cut into Sh chunks for the
// sequences before b_tail and into St for the rest.
inline long stream_blocks(const Params& p, int rows_per_b) {
  return ((long)p.b_tail * p.Sh + (long)(p.B - p.b_tail) * p.St) * rows_per_b;
}

// All launches of one call after the fill kernel.  `window` positions are
// verified per streaming launch; sequences decided by an earlier window are
// skipped by every later one (their workgroups return at once).
template <typename T, bool ALIGNED>
cos_status_t launch_all(Params p, int mode, int window, bool refine_kernels, size_t lds, hipStream_t st,
                        hipEvent_t ev_start, hipEvent_t ev_stop) {
  const dim3 block(kThreads);
  const int g1 = p.gamma + 1;
  if (ev_start) (void)hipEventRecord(ev_start, st);
  p.win = 0;
  for (int j0 = 0; j0 < g1; j0 += window, ++p.win) {
    p.j0 = j0;
    p.nj = (j0 + window <= g1) ? window : g1 - j0;
    const long blocks = stream_blocks(p, p.nj * (mode == kEns ? p.n : 1));
    if (blocks <= 0 || blocks > 0x7fffffffL) return COS_ERR_SHAPE;
    const dim3 grid((unsigned)blocks);
    if (mode == kEns) {
      hipLaunchKernelGGL((ensemble_stats_kernel<T, ALIGNED>), grid, block, 0, st, p);
    } else if (mode == kMix) {
      launch_mix_stats<T, ALIGNED>(p, grid, st);
    } else {
      // alpha_cd = 0 is Eq. (5) as printed: no mask, so no pass for the expert maxima
      if (p.masked) hipLaunchKernelGGL((expert_rowmax_kernel<T, ALIGNED>), grid, block, 0, st, p);
      if (p.masked)
        hipLaunchKernelGGL((contrastive_stats_kernel<T, ALIGNED, true>), grid, block, 0, st, p);
      else
        hipLaunchKernelGGL((contrastive_stats_kernel<T, ALIGNED, false>), grid, block, 0, st, p);
    }
    if (hipGetLastError() != hipSuccess) return COS_ERR_LAUNCH;
  }
  if (ev_stop) (void)hipEventRecord(ev_stop, st);
  cos_status_t rc = mode == kEns   ? launch_sampling<T, ALIGNED, kEns>(p, refine_kernels, lds, st)
                    : mode == kMix ? launch_sampling<T, ALIGNED, kMix>(p, refine_kernels, lds, st)
                                   : launch_sampling<T, ALIGNED, kCd>(p, refine_kernels, lds, st);
  if (rc != COS_OK || !p.alpha) return rc;
  return mode == kEns   ? launch_acceptance_rate<T, ALIGNED, kEns>(p, st)
         : mode == kMix ? launch_acceptance_rate<T, ALIGNED, kMix>(p, st)
                        : launch_acceptance_rate<T, ALIGNED, kCd>(p, st);
}

// Masked contrastive mode in one read of the logits: per window the streaming kernel (statistics of the
// proposer rows, chunk maxima of the expert rows, candidates of the mask), then one finishing workgroup
// per sequence.  No arrival counters, no fill kernel, no sampling or acceptance-rate kernel.
template <typename T, bool ALIGNED>
cos_status_t launch_onepass(Params p, const LaunchPlan& lp) {
  const dim3 block(kThreads);
  const int g1 = p.gamma + 1;
  // Verifier bonus tokens of large rows are drawn by refine_draw_kernel, the only user of counters in this mode.
  if (p.whole_row_bonus && !lp.ready) {
    hipLaunchKernelGGL(fill_zero_kernel, dim3((lp.counters + kThreads - 1) / kThreads), block, 0, lp.stream,
                       p.counters, lp.counters, p.plans, 0);
    if (hipGetLastError() != hipSuccess) return COS_ERR_LAUNCH;
  }
  if (lp.ev_start) (void)hipEventRecord(lp.ev_start, lp.stream);
  p.win = 0;
  for (int j0 = 0; j0 < g1; j0 += lp.window, ++p.win) {
    p.j0 = j0;
    p.nj = (j0 + lp.window <= g1) ? lp.window : g1 - j0;
    const long blocks = stream_blocks(p, p.nj);
    if (blocks <= 0 || blocks > 0x7fffffffL) return COS_ERR_SHAPE;
    hipLaunchKernelGGL((contrastive_onepass_kernel<T, ALIGNED>), dim3((unsigned)blocks), block, 0, lp.stream, p);
    if (p.win == 0 && j0 + lp.window >= g1 && lp.ev_stop) (void)hipEventRecord(lp.ev_stop, lp.stream);
    hipLaunchKernelGGL((contrastive_finish_kernel<T, ALIGNED>), dim3((unsigned)p.B), block, lp.lds, lp.stream, p);
    if (hipGetLastError() != hipSuccess) return COS_ERR_LAUNCH;
  }
  if (p.win > 1 && lp.ev_stop) (void)hipEventRecord(lp.ev_stop, lp.stream);
  if (p.whole_row_bonus) {  // (a sequence is decided, hence marked, in one window only: one launch for all)
    hipLaunchKernelGGL((refine_draw_kernel<T, ALIGNED, 2, kCd>), dim3((unsigned)p.refine_grid), block, lp.lds,
                       lp.stream, p);
    if (hipGetLastError() != hipSuccess) return COS_ERR_LAUNCH;
  }
  return COS_OK;
}

// Temperature 0: the expert maxima (contrastive with a mask only), then one argmax kernel.
template <typename T, bool ALIGNED>
cos_status_t launch_greedy(Params p, const LaunchPlan& lp) {
  p.j0 = 0;
  p.nj = p.gamma + 1;
  p.win = 0;
  const long blocks = stream_blocks(p, (p.gamma + 1) * (lp.mode == kEns ? p.n : 1));
  if (blocks <= 0 || blocks > 0x7fffffffL) return COS_ERR_SHAPE;
  const dim3 grid((unsigned)blocks), block(kThreads);
  if (lp.ev_start) (void)hipEventRecord(lp.ev_start, lp.stream);
  if (lp.mode == kEns) {
    hipLaunchKernelGGL((greedy_ensemble_kernel<T, ALIGNED>), grid, block, 0, lp.stream, p);
  } else if (lp.mode == kMix) {
    switch (p.n) {
      case 1: hipLaunchKernelGGL((greedy_mix_kernel<T, ALIGNED, 1>), grid, block, 0, lp.stream, p); break;
      case 2: hipLaunchKernelGGL((greedy_mix_kernel<T, ALIGNED, 2>), grid, block, 0, lp.stream, p); break;
      case 3: hipLaunchKernelGGL((greedy_mix_kernel<T, ALIGNED, 3>), grid, block, 0, lp.stream, p); break;
      case 4: hipLaunchKernelGGL((greedy_mix_kernel<T, ALIGNED, 4>), grid, block, 0, lp.stream, p); break;
      default: hipLaunchKernelGGL((greedy_mix_kernel<T, ALIGNED, 0>), grid, block, 0, lp.stream, p); break;
    }
  } else {
    if (p.masked) hipLaunchKernelGGL((expert_rowmax_kernel<T, ALIGNED>), grid, block, 0, lp.stream, p);
    hipLaunchKernelGGL((greedy_contrastive_kernel<T, ALIGNED>), grid, block, 0, lp.stream, p);
  }
  if (lp.ev_stop) (void)hipEventRecord(lp.ev_stop, lp.stream);
  return hipGetLastError() == hipSuccess ? COS_OK : COS_ERR_LAUNCH;
}

// Everything one call enqueues: the fill kernel, then the kernels of the mode.
template <typename T>
cos_status_t run_kernels(Params p, const LaunchPlan& lp) {
  if (lp.onepass) return lp.aligned ? launch_onepass<T, true>(p, lp) : launch_onepass<T, false>(p, lp);
  // The masked contrastive mode starts with a kernel that uses neither counters nor plans (the expert
  // maxima): it clears them on its way, one launch less.
  p.fill_count = (lp.mode == kCd && p.masked && !lp.ready) ? lp.counters : 0;
  if (p.fill_count == 0 && !lp.ready) {
    hipLaunchKernelGGL(fill_zero_kernel, dim3((lp.counters + kThreads - 1) / kThreads), dim3(kThreads), 0,
                       lp.stream, p.counters, lp.counters, p.plans, p.B);
    if (hipGetLastError() != hipSuccess) return COS_ERR_LAUNCH;
  }
  if (lp.greedy) return lp.aligned ? launch_greedy<T, true>(p, lp) : launch_greedy<T, false>(p, lp);
  const bool rk = lp.refine_kernels != 0;
  return lp.aligned ? launch_all<T, true>(p, lp.mode, lp.window, rk, lp.lds, lp.stream, lp.ev_start, lp.ev_stop)
                    : launch_all<T, false>(p, lp.mode, lp.window, rk, lp.lds, lp.stream, lp.ev_start, lp.ev_stop);
}

}  // namespace
