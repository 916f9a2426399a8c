/*
 * cos_verify.h -- C ABI of the MI355X (gfx950) batched verification step of
 * Collaborative decoding via Speculation (CoS).
 *
 * One call verifies, for B sequences at once, gamma draft tokens per sequence
 * against the combined distribution r of n collaborating models and emits the
 * accepted prefix plus one sampled token:
 *
 *   s_m   = softmax(l_m)                         Sec. 3.2 (temperature 1)
 *   r     = sum_m w_m s_m                        Eq. (4), n-model coefficients as
 *                                                in Sec. 4.1 / Alg. 2, or
 *   r     = Softmax(l_0 - mu l_1) on the mask    Eq. (5) plus a plausibility mask
 *           {x : s_0(x) >= alpha_cd max s_0}     (alpha_cd = 0: Eq. (5) exactly), or
 *   r     = Softmax(sum_m beta_m l_m)            Eq. (3) at the logit level, linear
 *   q     = s_{proposer_idx[b]}                  the row's current proposer
 *   accept draft d_j  iff  u_j < min(1, r(d_j)/q(d_j))        Eq. (2) / Eq. (6)
 *   first rejected position j*: token ~ norm(max(0, r - q))   Sec. 3.1-3.2, App. A.1
 *   no rejection: j* = gamma, bonus token ~ r at position gamma   Sec. 3.1
 *   draws are by inverse CDF in ascending token index: the smallest k with
 *   sum_{x<=k} f(x) > u_resample * sum_x f(x).
 *
 * All pointers are plain device or host pointers as stated per argument; the
 * caller owns every buffer.  Nothing here allocates device memory.  Calls are
 * asynchronous on the given HIP stream.
 */
#ifndef COS_VERIFY_H_
#define COS_VERIFY_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Storage format of the logits: float32, bfloat16, or IEEE binary16 (half). */
typedef enum { COS_DTYPE_F32 = 0, COS_DTYPE_BF16 = 1, COS_DTYPE_F16 = 2 } cos_dtype_t;

/* How the models' outputs become the target distribution r (Eq. (3)):
 *   ENSEMBLE     probability level, Eq. (4): r = sum_m w_m softmax(l_m)
 *   CONTRASTIVE  logit level, Eq. (5): r = softmax(l_0 - mu l_1) over the
 *                plausibility mask of the expert (n == 2)
 *   LOGIT_MIX    logit level, linear: r = softmax(sum_m beta_m l_m) -- the form
 *                of decoding-time realignment (Sec. 2), of logit-level ensembles
 *                (beta_m = 1/n) and of Eq. (5) without its mask (beta = (1, -mu)) */
typedef enum {
  COS_COMBINE_ENSEMBLE = 0,
  COS_COMBINE_CONTRASTIVE = 1,
  COS_COMBINE_LOGIT_MIX = 2
} cos_combine_t;

typedef enum {
  COS_OK = 0,
  COS_ERR_NULL = -1,        /* a required pointer is NULL */
  COS_ERR_SHAPE = -2,       /* n, B, gamma or V out of the supported range */
  COS_ERR_DTYPE = -3,
  COS_ERR_MODE = -4,        /* unknown combine mode, or contrastive with n != 2 */
  COS_ERR_WEIGHTS = -5,     /* ensemble: w < 0 or |sum w - 1| > 1e-9; contrastive: mu not finite or alpha_cd outside [0,1];
                               logit mix: a beta that is not finite */
  COS_ERR_WORKSPACE = -6,   /* workspace NULL, misaligned (256 B) or smaller than cos_verify_workspace_bytes() */
  COS_ERR_ALIGN = -7,       /* logits pointer not aligned to its element size */
  COS_ERR_LAUNCH = -8,      /* a HIP call failed (no usable GPU, launch error) */
  COS_ERR_UNSUPPORTED = -9,
  COS_ERR_SCRATCH = -10     /* cos_verify_noalloc: the shape needs more than COS_NOALLOC_SCRATCH_BYTES of scratch */
} cos_status_t;

/* Supported ranges: 1 <= n <= COS_MAX_MODELS, 1 <= gamma <= COS_MAX_GAMMA,
 * 1 <= V <= COS_MAX_VOCAB, B >= 0 (B == 0 is a no-op).                      */
#define COS_MAX_MODELS 8
#define COS_MAX_GAMMA 31
#define COS_MAX_VOCAB 1048576

/* Flags written to cos_diag_t.flags. */
#define COS_FLAG_RESIDUAL_FALLBACK 1 /* residual mass was <= 0 or not finite: token drawn from r instead */
#define COS_FLAG_TAIL_CLAMP 2        /* rounding left no prefix above u*F: last token with mass taken */
#define COS_FLAG_RESIDUAL_REFINED 4  /* the residual had little mass (below 1/32: r close to q, an acceptance
                                        rate above 97 %) and was evaluated in its difference form q (r/q - 1),
                                        whose rounding error is relative to r - q itself; not an error */

/* Optional per-row diagnostics; every member is a DEVICE pointer or NULL. */
typedef struct cos_diag_t {
  double *r_at_draft;  /* [B][gamma]  r(d_{b,j}) for every position (not only up to j*) */
  double *q_at_draft;  /* [B][gamma]  q(d_{b,j}) */
  double *sample_mass; /* [B]         F = sum_x f(x) of the sampled position */
  double *cdf_lo;      /* [B]         normalised CDF just below the drawn token */
  double *cdf_hi;      /* [B]         normalised CDF just above the drawn token */
  int32_t *flags;      /* [B]         COS_FLAG_* bits */
} cos_diag_t;

/* Bytes of device scratch cos_verify needs for this shape (0 on invalid
 * arguments).  Host-only computation; needs no GPU.                        */
size_t cos_verify_workspace_bytes(int n, int B, int gamma, int V, cos_dtype_t dt,
                                  cos_combine_t mode);

/*
 * The verification step (VERIFY of Alg. 1 / Alg. 2; Eq. (2)-(6), App. A.1).
 *
 * logits        DEVICE, [n][B][gamma+1][V] contiguous (V fastest), dtype dt.
 *               Position gamma is the bonus position.  -inf entries are legal
 *               (probability 0); NaN or +inf entries give undefined outputs
 *               but never an out-of-bounds access or a hang.
 * draft_tokens  DEVICE, [B][gamma] int32, each in [0, V) (caller's contract).
 * proposer_idx  DEVICE, [B] int32, each in [0, n): whose softmax is q.
 * combine_mode  ensemble, contrastive or logit mix (see cos_combine_t).
 * weights       HOST.  ensemble: w[0..n-1].  contrastive (n must be 2; model 0
 *               is the expert l^p, model 1 the amateur l^q): weights[0] = mu,
 *               weights[1] = alpha_cd in [0,1].  logit mix: beta[0..n-1], any
 *               finite values; a model with beta_m = 0 takes no part in r (its
 *               logits still give q when it proposes); a -inf logit under a
 *               positive beta_m gives probability 0, under a negative one the
 *               outputs are undefined.
 * u_accept      DEVICE, [B][gamma] float64 in [0,1).
 * u_resample    DEVICE, [B] float64 in [0,1): used for the one draw of the row
 *               (residual or bonus).
 * accepted_len  DEVICE out, [B] int32 in [0, gamma].
 * out_tokens    DEVICE out, [B][gamma+1] int32: accepted drafts, the drawn
 *               token at index accepted_len[b], then -1.
 * workspace     DEVICE scratch, 256-byte aligned, at least
 *               cos_verify_workspace_bytes() bytes, contents arbitrary on
 *               entry (but see options->workspace_ready); two calls that overlap in
 *               time need distinct ones.
 * diag          HOST pointer to a struct of device pointers, or NULL.
 * hip_stream    hipStream_t (NULL = the default stream).
 *
 * Host-side validation only; returns COS_OK once every kernel is enqueued.
 * Out-of-range tokens or proposer indices are undefined behaviour.
 */
cos_status_t cos_verify(const void *logits, cos_dtype_t dt, int n, int B, int gamma, int V,
                        const int32_t *draft_tokens, const int32_t *proposer_idx,
                        cos_combine_t combine_mode, const double *weights,
                        const double *u_accept, const double *u_resample,
                        int32_t *accepted_len, int32_t *out_tokens, void *workspace,
                        size_t workspace_bytes, const cos_diag_t *diag, void *hip_stream);

/*
 * Extensions of the step; every member is optional (0 / NULL = the base step).
 *
 * struct_bytes  sizeof(cos_options_t) of the caller (else COS_ERR_UNSUPPORTED).
 * temperature   T > 0 divides every logit before every softmax (Sec. 4.1 runs
 *               T = 1; how T enters Eq. (5) is not stated: it divides both l^p
 *               and l^q, so the mask reads s_0 >= alpha_cd max s_0 at that T).
 *               0 means 1.  Negative or non-finite: COS_ERR_WEIGHTS.  The ensemble
 *               keeps its accuracy (r(d), q(d) to 1e-7) at every T; the logit-level
 *               modes round their combination to float32 before it is divided by
 *               T, so their relative error is about 1e-6 / T: inside 1e-5 for
 *               T >= 0.15 (for T -> 0 there is `greedy`, which is exact).
 * bonus_idx     DEVICE [B] int32 or NULL.  bonus_idx[b] = v >= 0: when every
 *               draft of the row is accepted, the extra token is drawn from
 *               the verifier's own distribution s_v (Sec. 3.1, Sec. 3.3:
 *               the token the alternate proposal framework hands to the next
 *               cycle) instead of from r.  The other models' logits at
 *               position gamma are then ignored (ensemble mode does not even
 *               read them), so they need not be valid.  -1: drawn from r.
 * proposer_pos  DEVICE [B][gamma] int32 or NULL: the proposer of every draft
 *               position (Alg. 2: tokens of one window can come from different
 *               models); overrides proposer_idx, which must still be valid.
 * alpha         DEVICE out [B][gamma] float64 or NULL: the acceptance rate
 *               alpha = sum_x min(q(x), r(x)) = 1 - (1/2) sum_x |q(x) - r(x)|
 *               (Eq. (7), App. A.1) of every draft position.  Costs a second
 *               read of the draft positions' logits (one more kernel).
 * stop_window   0 (or > gamma): every position of every sequence is read, in
 *               one streaming launch.  w >= 1: the positions are verified w at
 *               a time, one streaming launch per window, and a sequence's
 *               logits after the window of its first rejection are never read
 *               (Sec. 3.1: they are discarded).  accepted_len and out_tokens
 *               are identical; diag.r_at_draft / q_at_draft are written only
 *               for positions that were read; alpha must be NULL
 *               (COS_ERR_UNSUPPORTED).  Fewer bytes, more launches.
 * greedy        non-zero: temperature 0 (the T = 0 runs of Sec. 4.1): every softmax
 *               is one-hot at its largest entry, ties to the lowest index.
 *               Logit-level modes: r of Eq. (5) is one-hot at a_j = argmax over
 *               the mask of l_0 - mu l_1 (the mask stays the temperature-1 one,
 *               l_0 - max l_0 >= ln alpha_cd), r of the logit mix at a_j = argmax
 *               of sum_m beta_m l_m: draft d_j is accepted iff d_j == a_j, the
 *               token at the first mismatch -- or the bonus token -- is a_j (with
 *               bonus_idx[b] = v >= 0: the argmax of l_v alone); u_accept,
 *               u_resample, proposer_idx and temperature are not used.
 *               Ensemble mode: r = sum_m w_m e_{a_m} over the models' own tokens
 *               a_m = argmax l_m and q = e_{a_pi}; Eq. (6), the residual and the
 *               draw are taken as always, on those at most n tokens, with
 *               u_accept and u_resample (a draft equal to the proposer's token
 *               is accepted with probability r(d); another model's token
 *               always; any other token never); proposer_pos may be given.
 *               diag is not written.  Bit-exact against a float64 reference.
 *               Not combinable with alpha or stop_window, nor (logit-level
 *               modes) with proposer_pos.
 * num_drafts    DEVICE [B] int32 or NULL.  Row b carries only num_drafts[b]
 *               drafts, in [0, gamma] (caller's contract): the rows of a batch,
 *               and the windows Alg. 2 verifies, differ in length.  Position
 *               num_drafts[b] takes the role of position gamma (bonus position);
 *               draft_tokens, u_accept, proposer_pos and logits beyond it are
 *               never read, accepted_len[b] is in [0, num_drafts[b]], alpha
 *               and diag.r_at_draft / q_at_draft of positions without a draft
 *               are NaN.  num_drafts[b] = 0 draws one token from r (or s_v) at
 *               position 0.
 * no_bonus      non-zero: when every draft of a row is accepted, nothing is
 *               drawn (Alg. 2's VERIFY only tests and resamples; Naive-CoS of
 *               Sec. 3.2 discards the extra token): out_tokens[b][num_drafts[b]]
 *               = -1 and the logits of that position are not read, so the
 *               tensor's last position may hold anything.  diag.sample_mass,
 *               cdf_lo, cdf_hi and flags of such a row are 0.
 * chunk_vectors, sample_blocks, tail_sequences, tail_factor
 *               Launch-shape overrides for experiments and tests; 0 everywhere is
 *               the built-in heuristic.  Outputs do not depend on them beyond the
 *               rounding order of float64 sums.  chunk_vectors: 16-byte vectors of
 *               one logit row that one workgroup of the streaming kernel reduces.
 *               sample_blocks: total workgroups the sampling kernel aims for.
 *               tail_sequences / tail_factor: the rows of the last tail_sequences
 *               sequences of a streaming launch are cut into tail_factor times more
 *               chunks than the others (they run while the GPU drains);
 *               tail_sequences < 0 turns that off, tail_factor 0 means 4.
 *               The workspace a call needs depends on chunk_vectors and the tail
 *               fields: size it with cos_verify_workspace_bytes_ex and the same
 *               options.
 * two_pass_mask the route of the masked contrastive mode (alpha_cd > 0).  0: chosen by
 *               the width of the mask -- a single read of the logits with candidate lists
 *               when T ln(1/alpha_cd) <= ln 25 (the usual alpha_cd = 0.1 keeps a few dozen
 *               tokens of a peaked expert row), else one pass for the expert maxima, one
 *               for the masked statistic and the sampling kernel, whose cost does not
 *               depend on how many tokens pass.  > 0: always the two passes; < 0: always
 *               the single read (a position whose candidates do not fit its lists -- a few
 *               hundred tokens in the mask -- is then read again by one workgroup alone).
 *               Same outputs up to near-ties.
 * workspace_ready  non-zero: the caller promises that every arrival counter in the
 *               workspace is zero, which is the case if the workspace was zero-filled,
 *               or if its last use was a completed call of this library with the same
 *               shape, mode and options (every call leaves its counters at zero).  The
 *               call then skips the kernel that clears them.  For loops that verify
 *               the same shape step after step; a promise that does not hold gives
 *               undefined outputs (never an out-of-bounds access).
 * refine_kernels  how a residual of little mass (the models nearly agree at the rejected
 *               position: Sec. 3.2's norm(max(0, r - q)) with r close to q) is drawn from once
 *               more in its difference form, which takes two more passes over that
 *               position's rows.  0: by the size of a row-set (n * V * element size) --
 *               up to 256 KiB the sequence's last sampling workgroup does it alone, above
 *               that two more launches do it with many workgroups per such sequence
 *               (a few microseconds when no sequence needs them, against a stall of the
 *               whole call on one workgroup's two passes over a large row-set).
 *               > 0: always the two launches; < 0: never.  Same outputs either way.  The
 *               workspace does not depend on it.
 * event_start, event_stop
 *               hipEvent_t handles created by the caller, or NULL.  The call records
 *               event_start on its stream just before its streaming kernel(s) -- the
 *               kernel(s) that read every logit -- and event_stop just after, so that
 *               a benchmark can time that part of the step alone.
 */
typedef struct cos_options_t {
  size_t struct_bytes;
  double temperature;
  const int32_t *bonus_idx;
  const int32_t *proposer_pos;
  double *alpha;
  int stop_window;
  int greedy;
  const int32_t *num_drafts;
  int no_bonus;
  int chunk_vectors;
  int sample_blocks;
  int tail_sequences;
  int tail_factor;
  int two_pass_mask;
  int workspace_ready;
  int refine_kernels;
  void *event_start;
  void *event_stop;
} cos_options_t;

/* cos_verify with extensions; options == NULL is exactly cos_verify. */
cos_status_t cos_verify_ex(const void *logits, cos_dtype_t dt, int n, int B, int gamma, int V,
                           const int32_t *draft_tokens, const int32_t *proposer_idx,
                           cos_combine_t combine_mode, const double *weights,
                           const double *u_accept, const double *u_resample,
                           int32_t *accepted_len, int32_t *out_tokens, void *workspace,
                           size_t workspace_bytes, const cos_diag_t *diag,
                           const cos_options_t *options, void *hip_stream);

/* cos_verify_workspace_bytes for a call with these options (NULL: the same value).  Only the
 * launch-shape overrides enter; 0 on invalid arguments.  Host-only computation. */
size_t cos_verify_workspace_bytes_ex(int n, int B, int gamma, int V, cos_dtype_t dt, cos_combine_t mode,
                                     const cos_options_t *options);

/*
 * cos_verify_ex for callers that cannot allocate device memory or hand over a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  The scratch the kernels need (arrival counters, partial
 * statistics, plans, tile sums) lives in an array of COS_NOALLOC_SCRATCH_BYTES
 * bytes built into the library, one copy per GPU, held until the process ends;
 * its device address is looked up once per device, on the first call made with
 * that device current.  Every other argument is as in cos_verify_ex, outputs
 * included: the caller still passes them.  The call allocates nothing (no
 * hipMalloc, no hipFree, no allocating library routine) and enqueues exactly
 * the kernels cos_verify_ex enqueues; the outputs are identical.
 *
 * A shape whose cos_verify_workspace_bytes() exceeds the array is rejected with
 * COS_ERR_SCRATCH before anything is enqueued (the largest listed workload,
 * n = 4, B = 512, gamma = 6, V = 256000, needs 5.0 MB).  All calls on one GPU
 * share that GPU's array: calls that overlap in time on one GPU (two streams,
 * two threads) race and give undefined outputs -- use cos_verify_ex with one
 * workspace per stream there.  The array keeps the last call's contents; each
 * call clears the counters it uses itself.
 */
#define COS_NOALLOC_SCRATCH_BYTES (8u << 20)
cos_status_t cos_verify_noalloc(const void *logits, cos_dtype_t dt, int n, int B, int gamma, int V,
                                const int32_t *draft_tokens, const int32_t *proposer_idx,
                                cos_combine_t combine_mode, const double *weights,
                                const double *u_accept, const double *u_resample,
                                int32_t *accepted_len, int32_t *out_tokens, const cos_diag_t *diag,
                                const cos_options_t *options, void *hip_stream);

/* COS_NOALLOC_SCRATCH_BYTES as the loaded library was built with. */
size_t cos_verify_noalloc_capacity(void);

/*
 * Debugging aid for the caller's side of the contract (cos_verify itself does not
 * look at these values before using them): counts, on the device, the entries
 * that are out of range -- draft tokens outside [0, V), proposer indices (and
 * options->proposer_pos) outside [0, n), options->bonus_idx outside [-1, n),
 * options->num_drafts outside [0, gamma], uniforms outside [0, 1) or NaN; with
 * num_drafts given, only the drafts, proposers and uniforms of positions that
 * carry a draft are looked at.  Waits for the stream, writes the count to
 * *bad_entries (HOST) and returns COS_OK if it is zero, COS_ERR_SHAPE otherwise.
 * Allocates nothing: the count lives in the first bytes of the workspace
 * (256-byte aligned, at least 256 bytes).  options may be NULL.
 */
cos_status_t cos_verify_check_inputs(int n, int B, int gamma, int V, const int32_t *draft_tokens,
                                     const int32_t *proposer_idx, const double *u_accept,
                                     const double *u_resample, const cos_options_t *options,
                                     void *workspace, size_t workspace_bytes, int *bad_entries,
                                     void *hip_stream);

/*
 * What a call with these arguments would enqueue (host-only; nothing is launched, no pointer
 * to device memory is needed): for tools, tests and whoever tunes the launch-shape options.
 * weights as in cos_verify (the contrastive mode's alpha_cd chooses its route); options may be
 * NULL.  Returns the status cos_verify_ex would return for these arguments, as far as it
 * depends on them alone.
 */
typedef struct cos_launch_info_t {
  size_t struct_bytes;          /* sizeof(cos_launch_info_t), set by the caller */
  int streaming_launches;       /* launches that read the logits (more than one: stop_window) */
  int chunks_per_row;           /* workgroups a row is cut into ... */
  int chunk_vectors;            /* ... of this many 16-byte vectors each */
  int tail_sequences;           /* sequences at the end of the grid cut finer ... */
  int tail_chunks_per_row;      /* ... into this many chunks per row */
  int sample_workgroups;        /* sampling workgroups per sequence (0: no sampling kernel) */
  int refine_launches;          /* 1: residuals of little mass go to the two refinement launches */
  int one_read_mask;            /* 1: masked contrastive mode in one read with candidate lists */
  int greedy;                   /* 1: temperature 0, one argmax kernel */
  size_t workspace_bytes;       /* cos_verify_workspace_bytes_ex for these options */
} cos_launch_info_t;
cos_status_t cos_verify_launch_info(int n, int B, int gamma, int V, cos_dtype_t dt, cos_combine_t combine_mode,
                                    const double *weights, const cos_options_t *options,
                                    cos_launch_info_t *info);

/* Static, NUL-terminated description of a status code. */
const char *cos_status_string(cos_status_t status);

/* Version of this library's interface: bumped whenever an entry point, an option or a mode is added
 * or changes meaning (7: refine_kernels option and the refinement launches, two_pass_mask with three values,
 * cos_verify_launch_info). */
int cos_verify_version(void);

#ifdef __cplusplus
}
#endif
#endif /* COS_VERIFY_H_ */
