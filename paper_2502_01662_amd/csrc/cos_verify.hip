// cos_verify.hip -- C ABI and host side of the CoS verification step for gfx950.
// The kernels live in the headers beside this file -- cos_device.h (structures,
// wavefront and hand-off primitives, loads), cos_stats.h (streaming kernels and
// the decision of a sequence), cos_sample.h (sampling and acceptance-rate
// kernels), cos_launch.h (their launches) -- and are instantiated once per logit
// format in cos_kernels_f32.hip, cos_kernels_bf16.hip and cos_kernels_f16.hip.
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
// maximum before anything can be masked, so a row-max kernel runs first.  The
// logit-level modes (contrastive, logit mix) stream the rows of all models of a
// position together, since their statistic is of a combination of the rows.
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
#include <mutex>

#include "cos_verify.h"

#include "cos_device.h"

// Built-in scratch of cos_verify_noalloc: one array per GPU the library runs on, held until the
// process ends.  In host code this name is only a handle for hipGetSymbolAddress; the device
// address it resolves to (per device) is what kernels, and every other use, are given.
static __device__ __align__(256) unsigned char scratch[COS_NOALLOC_SCRATCH_BYTES];

namespace {

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------

// Launch-shape overrides of one call (cos_options_t); all zero: the built-in heuristics.
struct Tune {
  int chunk_vectors = 0;   // 0 = heuristic
  int sample_blocks = 0;   // 0 = heuristic
  int tail_sequences = -1; // sequences at the end of the grid with shorter chunks (-1 = heuristic, 0 = none)
  int tail_factor = 4;     // how many times shorter
  int refine_kernels = 0;  // 0 = by the size of a row-set, > 0 = the two refinement launches, < 0 = never
};
Tune tune_of(const cos_options_t* o) {
  Tune t;
  if (!o) return t;
  t.chunk_vectors = o->chunk_vectors > 0 ? o->chunk_vectors : 0;
  t.sample_blocks = o->sample_blocks > 0 ? o->sample_blocks : 0;
  t.tail_sequences = o->tail_sequences == 0 ? -1 : (o->tail_sequences < 0 ? 0 : o->tail_sequences);
  t.tail_factor = o->tail_factor == 0 ? 4 : (o->tail_factor > 1 ? o->tail_factor : 1);
  t.refine_kernels = o->refine_kernels;
  return t;
}

struct Plan {
  int nvec, ntiles, nstat;
  size_t off_counters, off_partials, off_rowmax, off_plans, off_tiles, off_lse_all, off_rowmax_all,
      off_alpha_partials, off_cand, off_cand_count, off_refine_partials, off_refine_dlse, off_refine_list, bytes;
};

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Device address of `scratch` on the current device, resolved once per device (each GPU holds its
// own copy of the array at its own address).
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices];
cos_status_t scratch_on_current_device(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) return COS_ERR_LAUNCH;
  if (dev < 0 || dev >= kMaxDevices) return COS_ERR_UNSUPPORTED;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return COS_ERR_LAUNCH;
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return COS_OK;
}

bool shape_ok(int n, int B, int gamma, int V) {
  return n >= 1 && n <= COS_MAX_MODELS && B >= 0 && gamma >= 1 && gamma <= COS_MAX_GAMMA &&
         V >= 1 && V <= COS_MAX_VOCAB;
}

int alpha_blocks(int B, int gamma, int ntiles);

// Workspace layout for S chunks per row.
// Launch shape of the refinement kernels: a sequence is split over at most cmax workgroups (eight tiles
// each at least), the launch has about a thousand workgroups and never fewer than sequences.
void refine_shape(int B, int ntiles, int* grid, int* cmax) {
  const int cm = ntiles / 8 > 1 ? ntiles / 8 : 1;
  const long want = (long)(B > 0 ? B : 1) * cm;
  int g = (int)(want < 1024 ? want : 1024);
  if (g < B) g = B;
  *grid = g;
  *cmax = cm;
}

void plan_layout(int n, int B, int gamma, int V, cos_dtype_t dt, cos_combine_t mode, int S,
                 Plan* pl) {
  const int N = dt == COS_DTYPE_F32 ? 4 : 8;
  pl->nvec = (V + N - 1) / N;
  pl->ntiles = (pl->nvec + 63) / 64;
  pl->nstat = mode == COS_COMBINE_CONTRASTIVE ? 3 : (mode == COS_COMBINE_LOGIT_MIX ? 2 : n);
  const size_t g1 = (size_t)gamma + 1;
  size_t at = 0;
  pl->off_counters = at;
  at += align_up(((size_t)(gamma + 4) * B + 2 + (size_t)B * gamma) * kCtrStride * sizeof(int), 256);
  pl->off_plans = at;
  at += align_up((size_t)B * sizeof(SeqPlan), 256);
  pl->off_tiles = at;
  at += align_up((size_t)B * pl->ntiles * sizeof(double), 256);
  int rgrid, rcmax;
  refine_shape(B, pl->ntiles, &rgrid, &rcmax);
  pl->off_refine_partials = at;
  at += align_up((size_t)rgrid * (COS_MAX_MODELS + 1) * sizeof(double), 256);
  pl->off_refine_dlse = at;
  at += align_up((size_t)B * COS_MAX_MODELS * sizeof(float), 256);
  pl->off_refine_list = at;
  at += align_up((size_t)B * sizeof(int), 256);
  pl->off_lse_all = at;
  at += align_up((size_t)B * g1 * pl->nstat * sizeof(double), 256);
  pl->off_rowmax_all = at;
  at += align_up((size_t)B * g1 * sizeof(float), 256);
  pl->off_alpha_partials = at;
  at += align_up((size_t)B * gamma * alpha_blocks(B, gamma, pl->ntiles) * sizeof(double), 256);
  pl->off_rowmax = at;
  if (mode == COS_COMBINE_CONTRASTIVE) at += align_up((size_t)B * g1 * S * sizeof(float), 256);
  // masked contrastive mode in one pass: the candidates every chunk leaves behind
  pl->off_cand = at;
  if (mode == COS_COMBINE_CONTRASTIVE) at += align_up((size_t)B * g1 * S * kCandChunk * sizeof(Cand), 256);
  pl->off_cand_count = at;
  if (mode == COS_COMBINE_CONTRASTIVE) at += align_up((size_t)B * g1 * S * sizeof(int), 256);
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
void choose_split(const Tune& tn, int rows_total, int nvec, int* S_out, int* cv_out) {
  int cv;
  if (tn.chunk_vectors > 0) {
    cv = tn.chunk_vectors;
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

// The end of the grid.  While the GPU drains, the workgroups still running no longer share the
// memory system with a full machine, but one workgroup cannot use what is freed: it streams at the
// rate its own loads in flight allow, a few times its share of the full machine.  The last whole-row
// workgroups therefore run alone for tens of microseconds.  The rows of the last sequences -- about
// as many workgroups as are resident at once -- are cut into shorter chunks, so that the drain is
// short; everywhere else chunks stay long (a workgroup's start-up and hand-off are paid per chunk).
// Measured: half a generation of resident workgroups, cut four times finer, is about the optimum
// (0.6 % of the streaming kernel at 14336 rows of 512 KB, 3 % at 4608 rows of 256 KB, 5 % at 960 rows).
void choose_tail(const Tune& tn, int B, int rows_per_b, int nvec, int Sh, int cvh, int* b_tail, int* St, int* cvt) {
  *b_tail = B;
  *St = Sh;
  *cvt = cvh;
  constexpr long kResident = 1536;  // workgroups the streaming kernels keep resident (6 per CU)
  const long per_b = (long)rows_per_b * Sh;
  long K = tn.tail_sequences;
  if (K < 0) K = ((long)B * per_b >= 2 * kResident) ? (kResident / 2 + per_b - 1) / per_b : 0;
  if (K <= 0 || tn.tail_factor <= 1) return;
  if (K > B) K = B;
  const int smax = max_splits(nvec);
  long s_want = (long)Sh * tn.tail_factor;
  if (s_want > smax) s_want = smax;
  int cv = (int)((nvec + s_want - 1) / s_want);
  // one full group of loads per thread, as everywhere (unless the chunk length is dictated)
  const int cv_min = tn.chunk_vectors > 0 ? kThreads : kThreads * kUnroll;
  if (cv < cv_min) cv = cv_min;
  cv = (cv + kThreads - 1) / kThreads * kThreads;
  const int S = (nvec + cv - 1) / cv;
  if (S <= Sh) return;
  *b_tail = B - (int)K;
  *St = S;
  *cvt = cv;
}

// Chunking of one streaming launch over `window` positions.
struct Split {
  int Sh, cvh, St, cvt, b_tail, stride;
};
Split split_for(const Tune& tn, int n, int B, int window, int nvec, bool ensemble) {
  Split sp;
  const int rows_per_b = (ensemble ? n : 1) * window;
  choose_split(tn, rows_per_b * (B > 0 ? B : 1), nvec, &sp.Sh, &sp.cvh);
  choose_tail(tn, B, rows_per_b, nvec, sp.Sh, sp.cvh, &sp.b_tail, &sp.St, &sp.cvt);
  sp.stride = sp.St > sp.Sh ? sp.St : sp.Sh;
  return sp;
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

// Sampling workgroups per sequence: about 1024 in total -- one generation of resident workgroups; a
// sampling workgroup's fixed cost (the plan, the coefficients, the hand-off) is large beside its
// streaming, so few long ones beat many short ones (measured: 1024 against 2048 saves 1.5 us at
// B = 64 and B = 256, 10 us at B = 512) --, at least 4 tiles each.  (Finer workgroups at the end of
// this grid, as choose_tail makes them for the streaming kernels, were measured and do not pay.)
void choose_sampling(const Tune& tn, int B, int ntiles, int* C_out, int* tpc_out) {
  const int target = tn.sample_blocks > 0 ? tn.sample_blocks : 1024;
  if (B < 1) B = 1;  // an empty batch: sized like one sequence, nothing is launched
  int C = (target + B - 1) / B;
  const int cmax = (ntiles + 3) / 4;
  if (C > cmax) C = cmax;
  if (C < 1) C = 1;
  const int tpc = (ntiles + C - 1) / C;
  *C_out = (ntiles + tpc - 1) / tpc;
  *tpc_out = tpc;
}

__global__ void zero_int_kernel(int* dst) { *dst = 0; }

// Counts the entries of the side arrays that break the caller's contract (one thread per entry of
// the [B][gamma] arrays; the first B threads also look at the per-sequence arrays).
__global__ void check_inputs_kernel(int n, int B, int gamma, int V, const int* draft, const int* proposer,
                                    const int* proposer_pos, const int* bonus_idx, const int* num_drafts,
                                    const double* u_accept, const double* u_resample, int* bad) {
  const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  int wrong = 0;
  if (i < (long)B * gamma) {
    const int b = (int)(i / gamma), j = (int)(i - (long)b * gamma);
    int nd = num_drafts ? num_drafts[b] : gamma;
    if (nd < 0 || nd > gamma) nd = 0;  // counted below, once per sequence
    if (j < nd) {
      wrong += draft[i] < 0 || draft[i] >= V;
      wrong += !(u_accept[i] >= 0.0 && u_accept[i] < 1.0);
      if (proposer_pos) wrong += proposer_pos[i] < 0 || proposer_pos[i] >= n;
    }
  }
  if (i < B) {
    wrong += proposer[i] < 0 || proposer[i] >= n;
    wrong += !(u_resample[i] >= 0.0 && u_resample[i] < 1.0);
    if (bonus_idx) wrong += bonus_idx[i] < -1 || bonus_idx[i] >= n;
    if (num_drafts) wrong += num_drafts[i] < 0 || num_drafts[i] > gamma;
  }
  if (wrong) atomicAdd(bad, wrong);
}

}  // namespace

extern "C" {

size_t cos_verify_workspace_bytes(int n, int B, int gamma, int V, cos_dtype_t dt,
                                  cos_combine_t mode) {
  return cos_verify_workspace_bytes_ex(n, B, gamma, V, dt, mode, nullptr);
}

size_t cos_verify_workspace_bytes_ex(int n, int B, int gamma, int V, cos_dtype_t dt, cos_combine_t mode,
                                     const cos_options_t* options) {
  if (options && options->struct_bytes != sizeof(cos_options_t)) return 0;
  const Tune tn = tune_of(options);
  if (!shape_ok(n, B, gamma, V)) return 0;
  if (dt != COS_DTYPE_F32 && dt != COS_DTYPE_BF16 && dt != COS_DTYPE_F16) return 0;
  if (mode != COS_COMBINE_ENSEMBLE && mode != COS_COMBINE_CONTRASTIVE && mode != COS_COMBINE_LOGIT_MIX)
    return 0;
  // Sized for the window length that cuts rows into the most chunks (one position per launch, as a
  // rule; every length is tried, there are at most gamma + 1).
  Plan pl;
  const int N = dt == COS_DTYPE_F32 ? 4 : 8;
  int S = 1;
  for (int window = 1; window <= gamma + 1; ++window) {
    const Split sp = split_for(tn, n, B, window, (V + N - 1) / N, mode == COS_COMBINE_ENSEMBLE);
    if (sp.stride > S) S = sp.stride;
  }
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

}  // extern "C"

namespace {

// The step behind every entry point.  builtin_scratch: the workspace is the library's own array.
cos_status_t verify_impl(const void* logits, cos_dtype_t dt, int n, int B, int gamma, int V,
                         const int32_t* draft_tokens, const int32_t* proposer_idx,
                         cos_combine_t combine_mode, const double* weights,
                         const double* u_accept, const double* u_resample,
                         int32_t* accepted_len, int32_t* out_tokens, void* workspace,
                         size_t workspace_bytes, bool builtin_scratch, const cos_diag_t* diag,
                         const cos_options_t* options, void* hip_stream, cos_launch_info_t* info = nullptr) {
  // info: fill in what the call would enqueue and return before anything touches a device (the
  // device pointers and the workspace are then not looked at).
  // ---- host-side validation (no HIP call before it passes) ----
  double temperature = 1.0;
  if (options) {
    if (options->struct_bytes != sizeof(cos_options_t)) return COS_ERR_UNSUPPORTED;
    if (!(options->temperature >= 0.0) || !std::isfinite(options->temperature)) return COS_ERR_WEIGHTS;
    if (options->temperature > 0.0) temperature = options->temperature;
    if (options->stop_window < 0) return COS_ERR_SHAPE;
    if (options->greedy) {
      // temperature 0: the whole step in one launch; only the ensemble's step looks at the proposers
      if (options->alpha || (options->proposer_pos && combine_mode != COS_COMBINE_ENSEMBLE) ||
          (options->stop_window > 0 && options->stop_window <= gamma))
        return COS_ERR_UNSUPPORTED;
    }
    // acceptance rates of positions that were never read do not exist
    if (options->stop_window > 0 && options->stop_window <= gamma && options->alpha)
      return COS_ERR_UNSUPPORTED;
  }
  if (!shape_ok(n, B, gamma, V)) return COS_ERR_SHAPE;
  if (dt != COS_DTYPE_F32 && dt != COS_DTYPE_BF16 && dt != COS_DTYPE_F16) return COS_ERR_DTYPE;
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
  if (!info && (!logits || !draft_tokens || !proposer_idx || !u_accept || !u_resample || !accepted_len ||
                !out_tokens))
    return COS_ERR_NULL;
  const size_t esize = dt == COS_DTYPE_F32 ? 4 : 2;
  if (!info && reinterpret_cast<uintptr_t>(logits) % esize) return COS_ERR_ALIGN;
  const size_t need = cos_verify_workspace_bytes_ex(n, B, gamma, V, dt, combine_mode, options);
  if ((size_t)(gamma + 1) * (contrastive ? 3 : (mix ? 2 : n)) > kMaxStatsPerSeq) return COS_ERR_SHAPE;
  if (info) {
    workspace_bytes = need;  // planned as with a workspace of exactly the needed size
  } else if (builtin_scratch) {
    if (need > (size_t)COS_NOALLOC_SCRATCH_BYTES) return COS_ERR_SCRATCH;
    const cos_status_t rc = scratch_on_current_device(&workspace);
    if (rc != COS_OK) return rc;
    workspace_bytes = COS_NOALLOC_SCRATCH_BYTES;
  }
  if (!info && (!workspace || reinterpret_cast<uintptr_t>(workspace) % 256 || workspace_bytes < need))
    return COS_ERR_WORKSPACE;

  // ---- launch plan ----
  const int N = dt == COS_DTYPE_F32 ? 4 : 8;
  const int nvec = (V + N - 1) / N;
  int window = gamma + 1;  // positions per streaming launch
  if (options && options->stop_window > 0 && options->stop_window < window) window = options->stop_window;
  const Tune tn = tune_of(options);
  const Split sp = split_for(tn, n, B, window, nvec, mode == kEns);
  Plan pl;
  plan_layout(n, B, gamma, V, dt, combine_mode, sp.stride, &pl);
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
  p.cand = reinterpret_cast<Cand*>(wsb + pl.off_cand);
  p.cand_count = reinterpret_cast<int*>(wsb + pl.off_cand_count);
  p.cand_cap = kCandChunk;
  p.plans = reinterpret_cast<SeqPlan*>(wsb + pl.off_plans);
  p.tile_sums = reinterpret_cast<HandOff<double>*>(wsb + pl.off_tiles);
  p.refine_partials = reinterpret_cast<HandOff<double>*>(wsb + pl.off_refine_partials);
  p.refine_dlse = reinterpret_cast<float*>(wsb + pl.off_refine_dlse);
  p.refine_list = reinterpret_cast<int*>(wsb + pl.off_refine_list);
  refine_shape(B, pl.ntiles, &p.refine_grid, &p.refine_cmax);
  p.alpha = options ? options->alpha : nullptr;
  p.lse_all = reinterpret_cast<double*>(wsb + pl.off_lse_all);
  p.rowmax_all = reinterpret_cast<float*>(wsb + pl.off_rowmax_all);
  p.alpha_partials = reinterpret_cast<HandOff<double>*>(wsb + pl.off_alpha_partials);
  {
    const int ca = alpha_blocks(B, gamma, pl.ntiles);
    p.tpa = (pl.ntiles + ca - 1) / ca;
    p.CA = (pl.ntiles + p.tpa - 1) / p.tpa;  // <= ca
  }
  p.nwin = (gamma + 1 + window - 1) / window;
  p.refine_ctl = p.counters + (size_t)(p.nwin + 3) * B * kCtrStride;
  p.S = sp.stride;
  p.Sh = sp.Sh;
  p.cvh = sp.cvh;
  p.St = sp.St;
  p.cvt = sp.cvt;
  p.b_tail = sp.b_tail;
  p.nvec = pl.nvec;
  p.ntiles = pl.ntiles;
  p.nstat = pl.nstat;
  choose_sampling(tn, B, pl.ntiles, &p.C, &p.tpc);
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
  // one double per tile; the rare difference-form path also parks a few totals per wavefront there
  const size_t lds = (size_t)(pl.ntiles > kWaves * (COS_MAX_MODELS + 1) ? pl.ntiles : kWaves * (COS_MAX_MODELS + 1)) * sizeof(double);
  hipEvent_t ev_start = options ? static_cast<hipEvent_t>(options->event_start) : nullptr;
  hipEvent_t ev_stop = options ? static_cast<hipEvent_t>(options->event_stop) : nullptr;

  // counters in use: one set per streaming launch, the sampling set, and the acceptance-rate sets if wanted
  LaunchPlan lp;
  lp.mode = mode;
  lp.window = window;
  lp.greedy = (options && options->greedy) ? 1 : 0;
  lp.ready = (options && options->workspace_ready) ? 1 : 0;
  // Masked contrastive mode: one read with candidate lists while the mask can be expected to be sparse --
  // tokens within T ln(1/alpha_cd) <= ln 25 of the expert's maximum; the usual alpha_cd = 0.1 keeps a few
  // dozen -- else the two-pass route, whose cost does not depend on how many tokens pass (a position whose
  // candidates do not fit is read again by one workgroup alone in the one-read route; measured on Gaussian
  // logits the routes cross at alpha_cd = 0.03, some 80 tokens per position).
  const int route = options ? options->two_pass_mask : 0;
  const bool sparse_mask = p.thr64 >= -3.21888;  // ln 25, a hair wider so that alpha_cd = 0.04 is in
  lp.onepass = (mode == kCd && p.masked && !lp.greedy && (route < 0 || (route == 0 && sparse_mask))) ? 1 : 0;
  lp.aligned = aligned ? 1 : 0;
  // A residual of little mass is drawn from once more in its difference form -- two more passes over the
  // row-set.  One workgroup alone does that at the rate of one compute unit's arithmetic: fine for a small
  // row-set, but a stall of the whole call for a large one, and in a large batch some sequence needs it in most calls (a rejection where
  // the models nearly agree).  Above 256 KiB per row-set two more launches do it with many workgroups per
  // marked sequence; they cost a few microseconds when no sequence is marked.
  lp.refine_kernels = tn.refine_kernels > 0 || (tn.refine_kernels == 0 && (size_t)n * V * esize > ((size_t)256 << 10));
  lp.counters = ((p.nwin + 3 + (p.alpha ? gamma : 0)) * B + 2) * kCtrStride;
  p.whole_row_bonus = (lp.onepass && lp.refine_kernels && p.bonus_idx) ? 1 : 0;
  lp.lds = lds;
  lp.stream = st;
  lp.ev_start = ev_start;
  lp.ev_stop = ev_stop;
  if (info) {
    const bool samples = !lp.greedy && !lp.onepass;
    info->streaming_launches = lp.greedy ? 1 : p.nwin;
    info->chunks_per_row = p.Sh;
    info->chunk_vectors = p.cvh;
    info->tail_sequences = B - p.b_tail;
    info->tail_chunks_per_row = p.St;
    info->sample_workgroups = samples ? p.C : 0;
    info->refine_launches = (samples && lp.refine_kernels) ? 1 : 0;
    info->one_read_mask = lp.onepass;
    info->greedy = lp.greedy;
    info->workspace_bytes = need;
    return COS_OK;
  }
  return dt == COS_DTYPE_F32 ? run_f32(p, lp) : (dt == COS_DTYPE_F16 ? run_f16(p, lp) : run_bf16(p, lp));
}

}  // namespace

extern "C" {

cos_status_t cos_verify_ex(const void* logits, cos_dtype_t dt, int n, int B, int gamma, int V,
                           const int32_t* draft_tokens, const int32_t* proposer_idx,
                           cos_combine_t combine_mode, const double* weights,
                           const double* u_accept, const double* u_resample,
                           int32_t* accepted_len, int32_t* out_tokens, void* workspace,
                           size_t workspace_bytes, const cos_diag_t* diag,
                           const cos_options_t* options, void* hip_stream) {
  return verify_impl(logits, dt, n, B, gamma, V, draft_tokens, proposer_idx, combine_mode, weights, u_accept,
                     u_resample, accepted_len, out_tokens, workspace, workspace_bytes, false, diag, options,
                     hip_stream);
}

cos_status_t cos_verify_noalloc(const void* logits, cos_dtype_t dt, int n, int B, int gamma, int V,
                                const int32_t* draft_tokens, const int32_t* proposer_idx,
                                cos_combine_t combine_mode, const double* weights,
                                const double* u_accept, const double* u_resample,
                                int32_t* accepted_len, int32_t* out_tokens, const cos_diag_t* diag,
                                const cos_options_t* options, void* hip_stream) {
  return verify_impl(logits, dt, n, B, gamma, V, draft_tokens, proposer_idx, combine_mode, weights, u_accept,
                     u_resample, accepted_len, out_tokens, nullptr, 0, true, diag, options, hip_stream);
}

size_t cos_verify_noalloc_capacity(void) { return COS_NOALLOC_SCRATCH_BYTES; }

cos_status_t cos_verify_launch_info(int n, int B, int gamma, int V, cos_dtype_t dt, cos_combine_t combine_mode,
                                    const double* weights, const cos_options_t* options, cos_launch_info_t* info) {
  if (!info) return COS_ERR_NULL;
  if (info->struct_bytes != sizeof(cos_launch_info_t)) return COS_ERR_UNSUPPORTED;
  *info = cos_launch_info_t{};
  info->struct_bytes = sizeof(cos_launch_info_t);
  return verify_impl(nullptr, dt, n, B, gamma, V, nullptr, nullptr, combine_mode, weights, nullptr, nullptr, nullptr,
                     nullptr, nullptr, 0, false, nullptr, options, nullptr, info);
}

cos_status_t cos_verify_check_inputs(int n, int B, int gamma, int V, const int32_t* draft_tokens,
                                     const int32_t* proposer_idx, const double* u_accept,
                                     const double* u_resample, const cos_options_t* options,
                                     void* workspace, size_t workspace_bytes, int* bad_entries,
                                     void* hip_stream) {
  if (options && options->struct_bytes != sizeof(cos_options_t)) return COS_ERR_UNSUPPORTED;
  if (!shape_ok(n, B, gamma, V)) return COS_ERR_SHAPE;
  if (!bad_entries) return COS_ERR_NULL;
  *bad_entries = 0;
  if (B == 0) return COS_OK;
  if (!draft_tokens || !proposer_idx || !u_accept || !u_resample) return COS_ERR_NULL;
  if (!workspace || reinterpret_cast<uintptr_t>(workspace) % 256 || workspace_bytes < 256) return COS_ERR_WORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  int* bad = static_cast<int*>(workspace);
  hipLaunchKernelGGL(zero_int_kernel, dim3(1), dim3(1), 0, st, bad);
  const long entries = (long)B * gamma;
  hipLaunchKernelGGL(check_inputs_kernel, dim3((unsigned)((entries + 255) / 256)), dim3(256), 0, st, n, B, gamma, V,
                     draft_tokens, proposer_idx, options ? options->proposer_pos : nullptr,
                     options ? options->bonus_idx : nullptr, options ? options->num_drafts : nullptr, u_accept,
                     u_resample, bad);
  if (hipGetLastError() != hipSuccess) return COS_ERR_LAUNCH;
  if (hipMemcpyAsync(bad_entries, bad, sizeof(int), hipMemcpyDeviceToHost, st) != hipSuccess) return COS_ERR_LAUNCH;
  if (hipStreamSynchronize(st) != hipSuccess) return COS_ERR_LAUNCH;
  return *bad_entries == 0 ? COS_OK : COS_ERR_SHAPE;
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
    case COS_ERR_SCRATCH: return "this shape needs more scratch than the library's built-in array holds";
  }
  return "unknown status";
}

int cos_verify_version(void) { return 7; }

}  // extern "C"
