// C ABI of libnpd (declared in include/npd.h): argument validation and kernel selection.
// Every check runs before the first HIP call, so error paths work on a machine without a GPU.
#include <math.h>
#include <stdint.h>

#include "../../include/npd.h"
#include "npd_internal.hpp"

namespace {

struct Range {
  uintptr_t b, e;
};

Range range_of(const void* p, size_t bytes) {
  const uintptr_t b = reinterpret_cast<uintptr_t>(p);
  return Range{b, b + bytes};
}

bool overlaps(const Range& x, const Range& y) { return x.b < y.e && y.b < x.e && x.b != x.e && y.b != y.e; }

size_t rows_bytes(int64_t T, int64_t stride, int64_t width, size_t elem) {
  return (size_t)(((T - 1) * stride + width) * (int64_t)elem);
}

// a row stride the byte extent of [T, stride] bf16 / fp32 arrays can be computed with in 64 bits
bool stride_fits(int64_t T, int64_t stride) { return stride <= (INT64_MAX / 8) / T; }

// a pointer that is not a multiple of its element size (NULL counts as aligned)
bool misaligned(const void* p, uintptr_t elem) { return (reinterpret_cast<uintptr_t>(p) & (elem - 1)) != 0; }

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

npd_status check_desc(const npd_kd_desc* d) {
  if (!d) return NPD_ERR_NULL;
  if (d->n_tokens <= 0 || d->vocab <= 0) return NPD_ERR_SHAPE;
  if (d->teacher_kind != NPD_TEACHER_DENSE_BF16 && d->teacher_kind != NPD_TEACHER_TOPK &&
      d->teacher_kind != NPD_TEACHER_NONE)
    return NPD_ERR_VALUE;
  if (d->student_stride < d->vocab) return NPD_ERR_SHAPE;
  if (d->teacher_kind == NPD_TEACHER_DENSE_BF16 && d->teacher_stride < d->vocab) return NPD_ERR_SHAPE;
  if (d->n_tokens > NPD_MAX_TOKENS) return NPD_ERR_UNSUPPORTED;  // one workgroup per position, 1-D grid
  if (d->vocab > NPD_MAX_VOCAB) return NPD_ERR_UNSUPPORTED;    // in-row offsets are 32-bit
  if (!stride_fits(d->n_tokens, d->student_stride)) return NPD_ERR_SHAPE;
  if (d->teacher_kind == NPD_TEACHER_DENSE_BF16 && !stride_fits(d->n_tokens, d->teacher_stride)) return NPD_ERR_SHAPE;
  if (d->teacher_kind == NPD_TEACHER_TOPK && (d->topk < 1 || d->topk > d->vocab)) return NPD_ERR_SHAPE;
  if (!(d->tau > 0.0f) || !isfinite(d->tau)) return NPD_ERR_VALUE;
  if (!isfinite(d->grad_scale) || !isfinite(d->ce_grad_scale)) return NPD_ERR_VALUE;
  if (d->ce_grad_scale != 0.0f && ((d->flags & NPD_FLAG_FWD_ONLY) || d->teacher_kind == NPD_TEACHER_NONE))
    return NPD_ERR_VALUE;  // a CE gradient needs a gradient buffer
  if (d->flags & ~(uint32_t)(NPD_FLAG_FWD_ONLY | NPD_FLAG_INPLACE_GRAD | NPD_FLAG_NO_WORKSPACE)) return NPD_ERR_VALUE;
  if ((d->flags & NPD_FLAG_FWD_ONLY) && (d->flags & NPD_FLAG_INPLACE_GRAD)) return NPD_ERR_VALUE;
  if (d->divergence < NPD_DIV_FORWARD_KL || d->divergence > NPD_DIV_SKEW_REVERSE_KL) return NPD_ERR_VALUE;
  if ((d->divergence == NPD_DIV_SKEW_KL || d->divergence == NPD_DIV_SKEW_REVERSE_KL) &&
      !(d->skew_alpha >= 0.0f && d->skew_alpha < 1.0f))
    return NPD_ERR_VALUE;
  if (d->divergence != NPD_DIV_FORWARD_KL && d->teacher_kind != NPD_TEACHER_DENSE_BF16)
    return NPD_ERR_UNSUPPORTED;  // off the top-k support p_T is 0: the other divergences need the full row
  if (d->teacher_kind == NPD_TEACHER_TOPK && d->topk > npd::kTopkMax) return NPD_ERR_UNSUPPORTED;
  return NPD_OK;
}

}  // namespace

extern "C" {

int npd_version(void) { return 105; }

const char* npd_status_string(npd_status st) {
  switch (st) {
    case NPD_OK: return "ok";
    case NPD_ERR_NULL: return "a required pointer is NULL";
    case NPD_ERR_SHAPE: return "a size, stride or count is out of range";
    case NPD_ERR_VALUE: return "a scalar argument or flag has an illegal value, or a pointer is misaligned";
    case NPD_ERR_ALIAS: return "an output overlaps an input in a way the flags do not allow";
    case NPD_ERR_UNSUPPORTED: return "combination not supported by this build";
    case NPD_ERR_WORKSPACE: return "workspace too small or misaligned";
    case NPD_ERR_HIP: return "the HIP runtime refused the launch";
  }
  return "unknown status";
}

int npd_debug_gang_spin_limit(int polls) { return npd::set_gang_spin_limit(polls); }

size_t npd_workspace_bytes(const npd_kd_desc* desc) {
  if (check_desc(desc) != NPD_OK) return 0;
  const npd_kd_desc& d = *desc;
  // only the row-gang kernels (long rows, dense teacher, gradient, forward or reverse KL) exchange partial sums
  // through device memory; every other kernel keeps them in registers and LDS
  if (d.flags & (NPD_FLAG_FWD_ONLY | NPD_FLAG_NO_WORKSPACE)) return 0;
  if (d.teacher_kind != NPD_TEACHER_DENSE_BF16) return 0;
  if (d.divergence != NPD_DIV_FORWARD_KL && d.divergence != NPD_DIV_REVERSE_KL) return 0;
  if (d.ce_grad_scale != 0.0f && d.tau != 1.0f) return 0;
  return npd::gang_workspace_bytes(d.n_tokens, d.vocab, d.tau != 1.0f);
}

npd_status npd_kd_loss_fwd_bwd(const npd_kd_desc* desc, const void* student_logits, const void* teacher_dense,
                               const int32_t* teacher_idx, const float* teacher_val, const int32_t* labels,
                               const uint8_t* loss_mask, void* grad_out, float* kd_tok, float* nll_tok,
                               float* teacher_nll_tok, float* lse_tok, int32_t* dev_status, void* workspace,
                               size_t workspace_bytes, void* stream) {
  npd_status st = check_desc(desc);
  if (st != NPD_OK) return st;
  const npd_kd_desc& d = *desc;
  const int64_t T = d.n_tokens;
  const int V = d.vocab;
  if (!student_logits || !loss_mask) return NPD_ERR_NULL;
  if (misaligned(student_logits, 2) || misaligned(teacher_dense, 2) || misaligned(grad_out, 2) ||
      misaligned(teacher_idx, 4) || misaligned(teacher_val, 4) || misaligned(labels, 4) || misaligned(kd_tok, 4) ||
      misaligned(nll_tok, 4) || misaligned(teacher_nll_tok, 4) || misaligned(lse_tok, 4) || misaligned(dev_status, 4))
    return NPD_ERR_VALUE;
  const bool fwd_only = (d.flags & NPD_FLAG_FWD_ONLY) != 0;
  const bool inplace = (d.flags & NPD_FLAG_INPLACE_GRAD) != 0;

  if (d.teacher_kind == NPD_TEACHER_DENSE_BF16) {
    if (!teacher_dense) return NPD_ERR_NULL;
    if (teacher_idx || teacher_val) return NPD_ERR_VALUE;
  } else if (d.teacher_kind == NPD_TEACHER_TOPK) {
    if (!teacher_idx || !teacher_val) return NPD_ERR_NULL;
    if (teacher_dense || teacher_nll_tok) return NPD_ERR_VALUE;
  } else {
    if (teacher_dense || teacher_idx || teacher_val || teacher_nll_tok || kd_tok) return NPD_ERR_VALUE;
    if (!fwd_only || grad_out) return NPD_ERR_VALUE;  // nothing to differentiate without a teacher
  }
  if ((nll_tok || teacher_nll_tok || d.ce_grad_scale != 0.0f) && !labels) return NPD_ERR_NULL;
  if (fwd_only) {
    if (grad_out) return NPD_ERR_VALUE;
  } else {
    if (!grad_out) return NPD_ERR_NULL;
    if (inplace != (grad_out == student_logits)) return NPD_ERR_ALIAS;
  }
  const size_t need = npd_workspace_bytes(desc);
  if (need > 0 && (!workspace || workspace_bytes < need || (reinterpret_cast<uintptr_t>(workspace) & 255u)))
    return NPD_ERR_WORKSPACE;

  // overlap of the gradient with any input (other than the declared in-place case) or scalar output
  const Range rs = range_of(student_logits, rows_bytes(T, d.student_stride, V, 2));
  if (grad_out) {
    const Range rg = range_of(grad_out, rows_bytes(T, d.student_stride, V, 2));
    if (!inplace && overlaps(rg, rs)) return NPD_ERR_ALIAS;
    if (teacher_dense && overlaps(rg, range_of(teacher_dense, rows_bytes(T, d.teacher_stride, V, 2)))) return NPD_ERR_ALIAS;
    if (teacher_idx && overlaps(rg, range_of(teacher_idx, (size_t)T * d.topk * 4))) return NPD_ERR_ALIAS;
    if (teacher_val && overlaps(rg, range_of(teacher_val, (size_t)T * d.topk * 4))) return NPD_ERR_ALIAS;
    if (labels && overlaps(rg, range_of(labels, (size_t)T * 4))) return NPD_ERR_ALIAS;
    if (overlaps(rg, range_of(loss_mask, (size_t)T))) return NPD_ERR_ALIAS;
    const float* outs[4] = {kd_tok, nll_tok, teacher_nll_tok, lse_tok};
    for (const float* o : outs)
      if (o && overlaps(rg, range_of(o, (size_t)T * 4))) return NPD_ERR_ALIAS;
  }

  npd::KdArgs a{};
  a.s = static_cast<const uint16_t*>(student_logits);
  a.t = static_cast<const uint16_t*>(teacher_dense);
  a.tidx = teacher_idx;
  a.tval = teacher_val;
  a.labels = labels;
  a.mask = loss_mask;
  a.g = static_cast<uint16_t*>(grad_out);
  a.kd = kd_tok;
  a.nll = nll_tok;
  a.tnll = teacher_nll_tok;
  a.lse = lse_tok;
  a.status = dev_status;
  a.T = T;
  a.s_stride = d.student_stride;
  a.t_stride = d.teacher_stride;
  a.V = V;
  a.k = d.teacher_kind == NPD_TEACHER_TOPK ? d.topk : 0;
  // 128-bit accesses need 16-byte aligned rows in every dense tensor the kernel touches
  bool vec = aligned16(student_logits) && d.student_stride % 8 == 0;
  if (grad_out) vec = vec && aligned16(grad_out);
  if (teacher_dense) vec = vec && aligned16(teacher_dense) && d.teacher_stride % 8 == 0;
  a.nvec_s = vec ? V / 8 : 0;
  a.c = (float)(1.4426950408889634 / (double)d.tau);
  a.inv_tau = 1.0f / d.tau;
  a.gscale = (float)((double)d.grad_scale / (double)d.tau);
  a.cscale = d.ce_grad_scale;
  a.divergence = d.divergence;
  a.alpha = d.skew_alpha;
  a.need_lse1 = (d.tau != 1.0f && (nll_tok || teacher_nll_tok || lse_tok || d.ce_grad_scale != 0.0f)) ? 1 : 0;
  a.ws = need > 0 ? static_cast<uint32_t*>(workspace) : nullptr;

  const hipError_t e = npd::launch_kd(a, d.teacher_kind, !fwd_only, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? NPD_OK : NPD_ERR_HIP;
}

npd_status npd_teacher_topk(int64_t n_tokens, int32_t vocab, int64_t teacher_stride, int32_t k, uint32_t flags,
                            const void* teacher_logits, const uint8_t* loss_mask, int32_t* topk_idx,
                            float* topk_val, void* stream) {
  if (n_tokens <= 0 || vocab <= 0 || teacher_stride < vocab || k < 1 || k > vocab) return NPD_ERR_SHAPE;
  if (flags & ~(uint32_t)NPD_TOPK_LOG_PROBS) return NPD_ERR_VALUE;
  if (!teacher_logits || !topk_idx || !topk_val) return NPD_ERR_NULL;
  if (k > npd::kTopkMax || n_tokens > NPD_MAX_TOKENS || vocab > NPD_MAX_VOCAB) return NPD_ERR_UNSUPPORTED;
  if (!stride_fits(n_tokens, teacher_stride)) return NPD_ERR_SHAPE;
  if (misaligned(teacher_logits, 2) || misaligned(topk_idx, 4) || misaligned(topk_val, 4)) return NPD_ERR_VALUE;
  const hipError_t e = npd::launch_teacher_topk(n_tokens, vocab, teacher_stride, k, (flags & NPD_TOPK_LOG_PROBS) != 0,
                                                static_cast<const uint16_t*>(teacher_logits), loss_mask, topk_idx,
                                                topk_val, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? NPD_OK : NPD_ERR_HIP;
}

npd_status npd_segment_reduce(int64_t n_tokens, int32_t n_segments, const float* values, const uint8_t* loss_mask,
                              const int32_t* cu_seqlens, float* seg_sum, int32_t* seg_count, float* seg_mean,
                              int32_t* token_to_sample, int32_t* dev_status, void* stream) {
  if (n_tokens < 0 || n_segments < 0) return NPD_ERR_SHAPE;
  if (n_tokens > NPD_MAX_TOKENS) return NPD_ERR_UNSUPPORTED;
  if (misaligned(values, 4) || misaligned(cu_seqlens, 4) || misaligned(seg_sum, 4) || misaligned(seg_count, 4) ||
      misaligned(seg_mean, 4) || misaligned(token_to_sample, 4) || misaligned(dev_status, 4))
    return NPD_ERR_VALUE;
  if (n_segments > 0 && (!loss_mask || !cu_seqlens)) return NPD_ERR_NULL;
  if (n_segments > 0 && (seg_sum || seg_mean) && !values) return NPD_ERR_NULL;
  const hipError_t e =
      npd::launch_segment_reduce(n_tokens, n_segments, values, loss_mask, cu_seqlens, seg_sum, seg_count, seg_mean,
                                 token_to_sample, dev_status, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? NPD_OK : NPD_ERR_HIP;
}

npd_status npd_delta_ifd_score(int32_t n_pairs, int32_t n_segments, const float* mean_nll_student,
                               const float* mean_nll_teacher, const int32_t* seg_count, const int32_t* pair_cond,
                               const int32_t* pair_uncond, float lo, float hi, uint32_t flags, float* ifd_student,
                               float* ifd_teacher, float* delta, uint8_t* zone, uint8_t* keep, int32_t* keep_count,
                               void* stream) {
  if (n_pairs < 0 || n_segments < 0) return NPD_ERR_SHAPE;
  if (!isfinite(lo) || !isfinite(hi) || lo > hi) return NPD_ERR_VALUE;
  if (flags & ~(uint32_t)NPD_IFD_REQUIRE_TEACHER_LE_1) return NPD_ERR_VALUE;
  if (misaligned(mean_nll_student, 4) || misaligned(mean_nll_teacher, 4) || misaligned(seg_count, 4) ||
      misaligned(pair_cond, 4) || misaligned(pair_uncond, 4) || misaligned(ifd_student, 4) ||
      misaligned(ifd_teacher, 4) || misaligned(delta, 4) || misaligned(keep_count, 4))
    return NPD_ERR_VALUE;
  if (n_pairs > 0 && (!mean_nll_student || !mean_nll_teacher || !seg_count || !pair_cond || !pair_uncond))
    return NPD_ERR_NULL;
  const hipError_t e = npd::launch_delta_ifd(n_pairs, n_segments, mean_nll_student, mean_nll_teacher, seg_count,
                                             pair_cond, pair_uncond, lo, hi, flags, ifd_student, ifd_teacher, delta,
                                             zone, keep, keep_count, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? NPD_OK : NPD_ERR_HIP;
}

}  // extern "C"
