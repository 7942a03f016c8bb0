/*
 * npd.h -- C ABI of libnpd, the packed knowledge-distillation loss of Near-Policy
 * Distillation (NPD) for AMD MI355X (gfx950).
 *
 * NPD precomputes student-generated responses and teacher logits so that
 * distillation runs as packed-sequence SFT (Alg. 1).  This library is the loss of
 * Alg. 1's "Student Optimization" phase and the arithmetic of its "Delta-IFD
 * Filtering" step, given logits that are already in device memory.
 *
 * Conventions for every entry point
 *   - All array pointers are DEVICE pointers unless marked "host".  The caller owns
 *     every buffer; the library allocates nothing, frees nothing, never synchronises
 *     and never copies to the host.  Work is enqueued on `stream` (a hipStream_t
 *     passed as void*; NULL is the default stream) and the call returns at once.
 *   - An output the caller does not want is passed as NULL where the comment allows.
 *   - The return value is an npd_status.  On any status other than NPD_OK nothing has
 *     been enqueued and no output was touched.  Argument checks run before any HIP
 *     call, so they work on a machine without a GPU.
 *   - bf16 = upper 16 bits of an IEEE binary32.  Logits must be finite (-inf is allowed as the
 *     mark of a vocabulary entry of probability 0: see npd_kd_loss_fwd_bwd).
 *   - Packed layout: the batch is flattened to T positions.  Position p is scored iff
 *     loss_mask[p] != 0.  labels[p] is the token position p predicts (already
 *     shifted).  Sample i owns positions [cu_seqlens[i], cu_seqlens[i+1]).
 *   - Kernels report data errors they meet (a label or top-k index outside [0, V), a
 *     decreasing cu_seqlens) by OR-ing NPD_DEV_* bits into *dev_status (one int32 the
 *     caller zeroes; may be NULL) and writing NaN for the position concerned.
 */
#ifndef NPD_H
#define NPD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  NPD_OK = 0,
  NPD_ERR_NULL = 1,        /* a required pointer is NULL                                  */
  NPD_ERR_SHAPE = 2,       /* a size, stride or count is out of range                     */
  NPD_ERR_VALUE = 3,       /* tau <= 0 or not finite, grad_scale not finite, lo > hi ...;
                              a pointer that is not a multiple of its element size        */
  NPD_ERR_ALIAS = 4,       /* an output (or the workspace) overlaps an input or another
                              output in a way the flags do not allow                      */
  NPD_ERR_UNSUPPORTED = 5, /* a combination this build does not implement                 */
  NPD_ERR_WORKSPACE = 6,   /* workspace smaller than npd_workspace_bytes() says           */
  NPD_ERR_HIP = 7          /* the HIP runtime refused the launch (hipGetLastError kept)   */
} npd_status;

/* what the teacher arguments hold */
enum {
  NPD_TEACHER_DENSE_BF16 = 0, /* full-vocabulary bf16 logits [T, teacher_stride]                  */
  NPD_TEACHER_TOPK = 1,       /* per position k vocabulary ids + k fp32 values (logits or log p)  */
  NPD_TEACHER_NONE = 2        /* no teacher: only nll_tok / lse_tok are produced (scoring pass)   */
};

/* npd_kd_desc.divergence: what kd_tok measures between p_T and p_S (Related Works names reverse KL and skew KL
 * beside the forward KL of Eq. 2; alpha = npd_kd_desc.skew_alpha).  All but FORWARD need a dense teacher. */
enum {
  NPD_DIV_FORWARD_KL = 0,      /* sum p_T log(p_T / p_S)                                  (Eq. 2)      */
  NPD_DIV_REVERSE_KL = 1,      /* sum p_S log(p_S / p_T)                                               */
  NPD_DIV_SKEW_KL = 2,         /* sum p_T log(p_T / m),  m = alpha p_T + (1 - alpha) p_S               */
  NPD_DIV_SKEW_REVERSE_KL = 3  /* sum p_S log(p_S / m),  m = (1 - alpha) p_T + alpha p_S               */
};

/* npd_kd_desc.flags */
enum {
  NPD_FLAG_FWD_ONLY = 1u,      /* no gradient: grad_out must be NULL                               */
  NPD_FLAG_INPLACE_GRAD = 2u,  /* grad_out == student_logits: each row is overwritten by its gradient */
  NPD_FLAG_NO_WORKSPACE = 4u   /* the caller brings no workspace: npd_workspace_bytes() is 0 and only kernels that
                                  need none run (for gradient calls on rows of 30,624 logits and more these are
                                  slower than the ones that exchange partial sums through a workspace)           */
};

/* bits OR-ed into *dev_status by kernels */
enum {
  NPD_DEV_BAD_LABEL = 1,      /* labels[p] outside [0, V) at a scored position        */
  NPD_DEV_BAD_TOPK_INDEX = 2, /* teacher_idx outside [0, V) at a scored position      */
  NPD_DEV_BAD_CU_SEQLENS = 4, /* cu_seqlens decreasing or outside [0, T]              */
  NPD_DEV_GANG_TIMEOUT = 8    /* workgroups that share a row gave up waiting for one another (never in a healthy
                                 run: every such wait is bounded so that a kernel cannot hang); the outputs of the
                                 rows concerned are NaN                                                        */
};

/* zone codes written by npd_delta_ifd_score (Sec. 3.2, "Differential Difficulty") */
enum {
  NPD_ZONE_DEGENERATE = 0, /* Delta < lo                                     */
  NPD_ZONE_PROXIMAL = 1,   /* lo <= Delta <= hi : the samples that are kept  */
  NPD_ZONE_DISCONNECT = 2, /* Delta > hi                                     */
  NPD_ZONE_INVALID = 3     /* empty sample, zero denominator or non-finite   */
};

/* npd_delta_ifd_score flags */
enum { NPD_IFD_REQUIRE_TEACHER_LE_1 = 1u };

/* Largest vocabulary and number of positions one call takes (beyond: NPD_ERR_UNSUPPORTED). */
#define NPD_MAX_VOCAB (1 << 26)
#define NPD_MAX_TOKENS 0x7fffffffLL

typedef struct {
  int64_t n_tokens;       /* T in [1, NPD_MAX_TOKENS]: flattened positions of the packed batch     */
  int32_t vocab;          /* V in [1, NPD_MAX_VOCAB]                                               */
  int32_t teacher_kind;   /* NPD_TEACHER_*                                                         */
  int64_t student_stride; /* elements between consecutive rows of student_logits (>= V); grad_out
                             uses the same stride                                                  */
  int64_t teacher_stride; /* dense: elements between rows (>= V); top-k / none: ignored            */
  int32_t topk;           /* k in [1, V] for NPD_TEACHER_TOPK, else ignored                        */
  uint32_t flags;         /* NPD_FLAG_*                                                            */
  float tau;              /* KD temperature, finite, > 0; divides student and teacher logits alike */
  float grad_scale;       /* finite; multiplies the KD gradient (the caller folds the loss weight
                             lambda of Eq. 1, a tau^2 factor or 1/N_tokens in here)                */
  float ce_grad_scale;    /* finite; weight of the hard-label CE gradient of Eq. 1 (the caller sets
                             (1 - lambda) / N_tokens); 0 = KD gradient only.  Non-zero needs labels
                             and a gradient buffer                                                 */
  int32_t divergence;     /* NPD_DIV_*; 0 = the forward KL of Eq. 2                                */
  float skew_alpha;       /* skew coefficient in [0, 1) of NPD_DIV_SKEW_*; ignored otherwise       */
} npd_kd_desc;

/* Library version (major * 100 + minor). */
int npd_version(void);

/* Static, never NULL. */
const char* npd_status_string(npd_status st);

/*
 * Name of the kernel family npd_kd_loss_fwd_bwd launches for `desc` when every row is 16-byte aligned and the
 * workspace npd_workspace_bytes() asks for is given ("kd_gang_kernel", "kd_cached_kernel", "kd_rows_kernel",
 * "div_rows_kernel"; "" for an invalid desc): lets a benchmark or profile say what it measured.  Static string.
 */
const char* npd_kd_kernel_name(const npd_kd_desc* desc);

/*
 * Testing aid: how many times a workgroup of the row-gang kernels polls for the other workgroups of its row before
 * it gives up (NPD_DEV_GANG_TIMEOUT).  polls <= 0 restores the default (about a second).  Returns the previous
 * value.  A tiny limit lets a test reach the give-up path while every kernel still ends normally.  Process-wide.
 */
int npd_debug_gang_spin_limit(int polls);

/*
 * Bytes of device workspace npd_kd_loss_fwd_bwd needs for `desc` (host call; 0 is a
 * legal answer and then `workspace` may be NULL).  Returns 0 for an invalid desc.
 */
size_t npd_workspace_bytes(const npd_kd_desc* desc);

/*
 * The fused KD loss of one packed batch: for every scored position p (Alg. 1,
 * "Compute Probs" / "Compute KD Loss"; Eq. 2; L_CE of Eq. 1):
 *
 *   p_S = Softmax(student[p, :] / tau)                 over the full vocabulary
 *   p_T = Softmax(teacher[p, :] / tau)                 dense: over the full vocabulary
 *                                                      top-k: over the k stored entries only
 *   kd_tok[p]  = sum_{c in support} p_T(c) * log(p_T(c) / p_S(c))        (Eq. 2; support = V or top-k)
 *   grad[p, c] = grad_scale / tau * (p_S(c) - p_T(c) * [c in support])   (d kd_tok / d student logit)
 *              + ce_grad_scale * (Softmax(student[p, :])(c) - [c == labels[p]])   (d nll_tok / d student logit;
 *                together the gradient of L_total = (1 - lambda) L_CE + lambda L_KD of Eq. 1)
 *   nll_tok[p]         = logsumexp(student[p, :]) - student[p, labels[p]]   (tau = 1 always)
 *   teacher_nll_tok[p] = logsumexp(teacher[p, :]) - teacher[p, labels[p]]   (dense teacher only)
 *   lse_tok[p]         = logsumexp(student[p, :])                           (tau = 1)
 *
 * With desc->divergence != NPD_DIV_FORWARD_KL (dense teacher only, else NPD_ERR_UNSUPPORTED) kd_tok[p] is that
 * divergence D of p_T and p_S and the first gradient term becomes grad_scale * dD / d student logit
 *   = grad_scale / tau * p_S(c) * (u_c - sum_c' p_S(c') u_c'),  u = dD / d p_S.
 *
 * At positions with loss_mask[p] == 0 the scalar outputs are 0 and the gradient row is
 * zero-filled (its logits are not read).  No tau^2 factor is applied.
 *
 * Logits are expected to be finite, with one exception: -inf marks a vocabulary entry of probability 0
 * (vocabulary padding, a banned token).  In the teacher (dense logits or a top-k value) such an entry
 * contributes nothing to kd_tok and the gradient there is the student term alone; in the student its
 * gradient is 0 where the teacher agrees, and kd_tok is +inf where the teacher does not.  NaN or +inf
 * make the outputs of their own position non-finite and touch no other position.
 *
 *   student_logits   bf16 [T, student_stride], required
 *   teacher_dense    bf16 [T, teacher_stride]; required iff teacher_kind == DENSE, else NULL
 *   teacher_idx      int32 [T, k], unique per row, in [0, V); required iff TOPK, else NULL
 *   teacher_val      fp32 [T, k] logits or log-probabilities at tau = 1 (a per-row additive
 *                    constant changes nothing); required iff TOPK, else NULL
 *   labels           int32 [T]; required iff nll_tok or teacher_nll_tok is given or ce_grad_scale != 0
 *   loss_mask        uint8 [T], required
 *   grad_out         bf16 [T, student_stride]; NULL iff NPD_FLAG_FWD_ONLY or teacher NONE; may equal
 *                    student_logits iff NPD_FLAG_INPLACE_GRAD (then the student logits are
 *                    destroyed); any other overlap with an input is NPD_ERR_ALIAS
 *   kd_tok           fp32 [T] or NULL (must be NULL for teacher NONE)
 *   nll_tok          fp32 [T] or NULL
 *   teacher_nll_tok  fp32 [T] or NULL (dense teacher only)
 *   lse_tok          fp32 [T] or NULL
 *   dev_status       int32 [1] or NULL
 *   workspace        device, >= npd_workspace_bytes(desc) bytes, 256-byte aligned (NULL if 0); scratch of the call
 *                    (contents meaningless before and after); must not overlap any other argument, and two
 *                    calls that may run at the same time need a workspace each
 *
 * Each gradient element is rounded to bf16 once (round to nearest even) from an fp32
 * value; all sums are accumulated in fp32.  A call's results are bitwise reproducible from
 * run to run (no floating-point atomics).  Two different calls on the same data (forward only
 * vs with gradient, other strides or alignment) may sum a row in another order: their scalar
 * outputs then agree to fp32 rounding, not bit for bit.  Rows that are 16-byte aligned with
 * strides that are multiples of 8 elements take the fast kernels; anything else is handled
 * element-wise, with the same results to rounding.
 */
npd_status npd_kd_loss_fwd_bwd(const npd_kd_desc* desc, const void* student_logits, const void* teacher_dense,
                               const int32_t* teacher_idx, const float* teacher_val, const int32_t* labels,
                               const uint8_t* loss_mask, void* grad_out, float* kd_tok, float* nll_tok,
                               float* teacher_nll_tok, float* lse_tok, int32_t* dev_status, void* workspace,
                               size_t workspace_bytes, void* stream);

/*
 * The same call for callers that cannot allocate or hold a workspace: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Arguments, results and errors are those of npd_kd_loss_fwd_bwd without
 * `workspace` / `workspace_bytes`; the scratch record comes from a fixed array of NPD_NOALLOC_WORKSPACE_BYTES bytes
 * of device memory that is part of the library's code object (each GPU the library runs on holds its own copy until
 * the process ends).  The call allocates and frees nothing.
 *
 *   - A call whose npd_workspace_bytes(desc) exceeds NPD_NOALLOC_WORKSPACE_BYTES returns NPD_ERR_WORKSPACE and
 *     enqueues nothing (at tau = 1 the array covers n_tokens * ceil(vocab / 20416) <= 524,288, e.g. 65,536 positions
 *     of a 151,936-entry vocabulary; with a dense teacher at tau != 1 half of that; the skew divergences count
 *     ceil(vocab / 12224)).  Pass NPD_FLAG_NO_WORKSPACE, or use
 *     npd_kd_loss_fwd_bwd with a workspace, for larger batches.
 *   - Every call on a GPU uses that GPU's one array (cleared by the call itself before use): calls that overlap in
 *     time on one GPU -- two streams, two host threads -- race on it and give wrong results.  Order them on one
 *     stream.
 *   - The first call on a device asks the runtime for the array's address (no allocation); make it outside stream
 *     capture.
 */
#define NPD_NOALLOC_WORKSPACE_BYTES (16u << 20)
npd_status npd_kd_loss_fwd_bwd_noalloc(const npd_kd_desc* desc, const void* student_logits,
                                       const void* teacher_dense, const int32_t* teacher_idx,
                                       const float* teacher_val, const int32_t* labels, const uint8_t* loss_mask,
                                       void* grad_out, float* kd_tok, float* nll_tok, float* teacher_nll_tok,
                                       float* lse_tok, int32_t* dev_status, void* stream);

/* npd_teacher_topk flags */
enum { NPD_TOPK_LOG_PROBS = 1u /* values = log-softmax of the k selected logits instead of the logits */ };

/*
 * Teacher-side top-k record (Sec. 3.1, "record only the top-k logits"; Alg. 1, Phase 2): for every
 * scored position p the k vocabulary ids with the largest teacher logits and their values, in the
 * format npd_kd_loss_fwd_bwd takes as NPD_TEACHER_TOPK.
 *
 *   topk_idx[p, 0..k)  ids, largest logit first; equal logits in order of increasing id (exact, deterministic)
 *   topk_val[p, 0..k)  the logits (as fp32), or with NPD_TOPK_LOG_PROBS their log-softmax over the k entries
 *                      (the renormalised teacher distribution of Eq. 2)
 *   positions with loss_mask[p] == 0 get ids 0..k-1 and values 0 (their logits are not read)
 *
 *   teacher_logits bf16 [T, teacher_stride] (finite), loss_mask uint8 [T] or NULL (all scored),
 *   topk_idx int32 [T, k], topk_val fp32 [T, k].  1 <= k <= min(V, 4096) (larger k: NPD_ERR_UNSUPPORTED);
 *   T and V within NPD_MAX_TOKENS and NPD_MAX_VOCAB.
 */
npd_status npd_teacher_topk(int64_t n_tokens, int32_t vocab, int64_t teacher_stride, int32_t k, uint32_t flags,
                            const void* teacher_logits, const uint8_t* loss_mask, int32_t* topk_idx,
                            float* topk_val, void* stream);

/*
 * Per-sample reduction of a per-position quantity over the packed layout (the
 * per-sample losses behind Eq. 1-3): for sample i in [0, S)
 *
 *   seg_count[i] = #{p in [cu[i], cu[i+1]) : loss_mask[p] != 0}
 *   seg_sum[i]   = sum of values[p] over those p     (fixed summation order: reproducible)
 *   seg_mean[i]  = seg_sum[i] / seg_count[i], or 0 when seg_count[i] == 0
 *   token_to_sample[p] = i for p in [cu[i], cu[i+1]), -1 for positions no sample owns
 *
 *   values fp32 [T], loss_mask uint8 [T], cu_seqlens int32 [S+1] (non-decreasing, inside [0, T]);
 *   seg_sum fp32 [S] / seg_count int32 [S] / seg_mean fp32 [S] / token_to_sample int32 [T]: each may
 *   be NULL.  n_tokens >= 0, n_segments >= 0 (0 is a no-op apart from token_to_sample = -1).
 *   A segment whose bounds are decreasing or outside [0, T] sets NPD_DEV_BAD_CU_SEQLENS, gets
 *   count 0 / sum NaN / mean NaN and owns no position.
 */
npd_status npd_segment_reduce(int64_t n_tokens, int32_t n_segments, const float* values, const uint8_t* loss_mask,
                              const int32_t* cu_seqlens, float* seg_sum, int32_t* seg_count, float* seg_mean,
                              int32_t* token_to_sample, int32_t* dev_status, void* stream);

/*
 * Delta-IFD selection score (Sec. 3.2): pair j names two packed samples, pair_cond[j]
 * = instruction + response (its mean response loss is L(A|Q)) and pair_uncond[j] = the
 * response alone (L(A)).  With the per-sample mean CE losses of student and teacher:
 *
 *   IFD_M   = mean_nll_M[pair_cond] / mean_nll_M[pair_uncond],  M in {student, teacher}   (Eq. 3)
 *   delta   = IFD_teacher - IFD_student                                                    (Eq. 4)
 *   zone    = DEGENERATE (delta < lo) | PROXIMAL (lo <= delta <= hi) | DISCONNECT (delta > hi)
 *             (the paper's lo is 0, hi its threshold tau, e.g. 0.8 or 1.0) | INVALID
 *   keep    = zone == PROXIMAL  [and IFD_teacher <= 1 if NPD_IFD_REQUIRE_TEACHER_LE_1]
 *   keep_count[0] = number of kept pairs (written, not accumulated)
 *
 * INVALID: a sample of the pair has seg_count == 0, a denominator is 0, one of the four mean
 * losses is not finite (also where plain division would give a finite ratio, 1 / inf = 0), or a
 * result is not finite; ifd_* and delta are then NaN and keep = 0.  All arithmetic in fp32.
 *
 *   mean_nll_student, mean_nll_teacher fp32 [S]; seg_count int32 [S]; pair_cond, pair_uncond
 *   int32 [P], entries in [0, S) (an entry outside marks the pair INVALID);
 *   ifd_student, ifd_teacher, delta fp32 [P], zone, keep uint8 [P], keep_count int32 [1]:
 *   each output may be NULL.  n_pairs >= 0; lo <= hi, both finite.
 */
npd_status npd_delta_ifd_score(int32_t n_pairs, int32_t n_segments, const float* mean_nll_student,
                               const float* mean_nll_teacher, const int32_t* seg_count, const int32_t* pair_cond,
                               const int32_t* pair_uncond, float lo, float hi, uint32_t flags, float* ifd_student,
                               float* ifd_teacher, float* delta, uint8_t* zone, uint8_t* keep, int32_t* keep_count,
                               void* stream);

/*
 * Policy-latency monitor (appendix, "Analysis of Policy Latency"): the paper tracks
 * D_KL(pi_learner || pi_generator) between the model being trained and the model that generated the
 * rollouts, calls training near-policy while D_KL <= epsilon (it reports epsilon ~ 0.10) and names a
 * refresh of the rollouts as due when the distance goes beyond.
 *
 * kl_tok is the per-position KL of the two next-token distributions: kd_tok of a forward-only
 * npd_kd_loss_fwd_bwd call with the generator's logits as student_logits and the learner's as
 * teacher_dense (Eq. 2's form puts the teacher slot's distribution first).  Over the packed layout:
 *
 *   seg_kl_mean[i], seg_count[i]  mean of kl_tok over the scored positions of sample i, and their number
 *                                 (as npd_segment_reduce; a bad segment: NaN / 0 and NPD_DEV_BAD_CU_SEQLENS)
 *   batch_count[0]                scored positions that a sample owns
 *   batch_kl_mean[0]              sum of kl_tok over those positions / batch_count: the step's D_KL, every
 *                                 scored position weighing the same (0 if there is none)
 *   lag_exceeded[0]               1 if batch_kl_mean > epsilon or is not a number, else 0 (the bound is closed)
 *
 *   kl_tok fp32 [T], loss_mask uint8 [T], cu_seqlens int32 [S+1]; every output may be NULL.
 *   epsilon finite, >= 0.  A cu_seqlens that decreases or leaves [0, T] gives batch_kl_mean NaN, count 0,
 *   lag_exceeded 1 and NPD_DEV_BAD_CU_SEQLENS.  Fixed summation order: reproducible.
 */
npd_status npd_policy_lag(int64_t n_tokens, int32_t n_segments, const float* kl_tok, const uint8_t* loss_mask,
                          const int32_t* cu_seqlens, float epsilon, float* seg_kl_mean, int32_t* seg_count,
                          float* batch_kl_mean, int32_t* batch_count, int32_t* lag_exceeded, int32_t* dev_status,
                          void* stream);

/*
 * Perplexity of every packed sample, PPL = exp(mean CE loss over its scored positions) -- the PPL filter that the
 * paper's data-filter ablation compares Delta-IFD with -- from the per-sample means and counts npd_segment_reduce
 * gives for nll_tok: seg_ppl[i] = exp(seg_mean_nll[i]), or 0 where seg_count[i] == 0.  All arrays [S], required.
 */
npd_status npd_segment_ppl(int32_t n_segments, const float* seg_mean_nll, const int32_t* seg_count, float* seg_ppl,
                           void* stream);

#ifdef __cplusplus
}
#endif
#endif /* NPD_H */
