// C ABI of libnpd (declared in include/npd.h): argument validation and kernel selection.
// Every check runs before the first HIP call, so error paths work on a machine without a GPU.
#include <math.h>
#include <stdint.h>

#include <atomic>

#include "../../include/npd.h"
#include "npd_internal.hpp"

// Scratch of npd_kd_loss_fwd_bwd_noalloc: one copy per GPU, held from the time the library is loaded on that GPU
// until the process ends.  In host code the array's name is only a handle; its device address is asked for once per
// device (hipGetSymbolAddress) and that pointer is what kernels get.
static __device__ __align__(256) unsigned char scratch[NPD_NOALLOC_WORKSPACE_BYTES];

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

// true if an output range overlaps an input range or another output range
bool any_alias(const Range* in, int n_in, const Range* out, int n_out) {
  for (int o = 0; o < n_out; ++o) {
    for (int i = 0; i < n_in; ++i)
      if (overlaps(out[o], in[i])) return true;
    for (int o2 = o + 1; o2 < n_out; ++o2)
      if (overlaps(out[o], out[o2])) return true;
  }
  return false;
}

Range opt_range(const void* p, size_t bytes) { return p ? range_of(p, bytes) : Range{0, 0}; }


constexpr int kMaxDevices = 64;
std::atomic<void*> noalloc_scratch_ptr[kMaxDevices];  // zero-initialised

// device address of the current device's scratch array (nullptr and *err set on failure)
void* noalloc_scratch_address(hipError_t* err) {
  int dev = 0;
  *err = hipGetDevice(&dev);
  if (*err != hipSuccess) return nullptr;
  if (dev < 0 || dev >= kMaxDevices) {
    *err = hipErrorInvalidDevice;
    return nullptr;
  }
  void* p = noalloc_scratch_ptr[dev].load(std::memory_order_acquire);
  if (!p) {
    *err = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (*err != hipSuccess) return nullptr;
    noalloc_scratch_ptr[dev].store(p, std::memory_order_release);  // racing host threads store the same address
  }
  return p;
}

// workspace bytes of a call with a valid descriptor
size_t workspace_bytes_of(const npd_kd_desc& d) {
  // only the row-gang kernels (gradient calls on long rows) exchange partial sums through device memory; every other
  // kernel keeps them in registers and LDS
  if (d.flags & (NPD_FLAG_FWD_ONLY | NPD_FLAG_NO_WORKSPACE)) return 0;
  if (d.ce_grad_scale != 0.0f && d.tau != 1.0f) return 0;
  if (d.teacher_kind == NPD_TEACHER_TOPK)  // (forward KL only: checked with the descriptor)
    return npd::gang_workspace_bytes(d.n_tokens, d.vocab, npd::kTopk, npd::kForwardKl, false);
  if (d.teacher_kind != NPD_TEACHER_DENSE_BF16) return 0;
  return npd::gang_workspace_bytes(d.n_tokens, d.vocab, npd::kDense, d.divergence, d.tau != 1.0f);
}

// Every input and output buffer of a KD call as a byte range (empty for arguments that are absent).
struct KdBuffers {
  Range in[6];   // student logits, dense teacher, top-k ids, top-k values, labels, loss mask
  Range out[6];  // gradient, kd_tok, nll_tok, teacher_nll_tok, lse_tok, dev_status
  bool overlaps_any(const Range& r) const {
    for (const Range& x : in)
      if (overlaps(r, x)) return true;
    for (const Range& x : out)
      if (overlaps(r, x)) return true;
    return false;
  }
};

KdBuffers kd_buffers(const npd_kd_desc& d, const void* student_logits, const void* teacher_dense,
                     const int32_t* teacher_idx, const float* teacher_val, const int32_t* labels,
                     const uint8_t* loss_mask, void* grad_out, float* kd_tok, float* nll_tok, float* teacher_nll_tok,
                     float* lse_tok, int32_t* dev_status) {
  const int64_t T = d.n_tokens;
  const size_t kbytes = d.teacher_kind == NPD_TEACHER_TOPK ? (size_t)T * d.topk * 4 : 0;
  auto opt = [](const void* p, size_t bytes) { return p ? range_of(p, bytes) : Range{0, 0}; };
  KdBuffers b;
  b.in[0] = range_of(student_logits, rows_bytes(T, d.student_stride, d.vocab, 2));
  b.in[1] = opt(teacher_dense, d.teacher_kind == NPD_TEACHER_DENSE_BF16 ? rows_bytes(T, d.teacher_stride, d.vocab, 2) : 0);
  b.in[2] = opt(teacher_idx, kbytes);
  b.in[3] = opt(teacher_val, kbytes);
  b.in[4] = opt(labels, (size_t)T * 4);
  b.in[5] = range_of(loss_mask, (size_t)T);
  b.out[0] = opt(grad_out, rows_bytes(T, d.student_stride, d.vocab, 2));
  b.out[1] = opt(kd_tok, (size_t)T * 4);
  b.out[2] = opt(nll_tok, (size_t)T * 4);
  b.out[3] = opt(teacher_nll_tok, (size_t)T * 4);
  b.out[4] = opt(lse_tok, (size_t)T * 4);
  b.out[5] = opt(dev_status, 4);
  return b;
}

// All argument checks of a KD call except those of the workspace; fills the kernel arguments (without workspace) and
// the number of workspace bytes the call needs.  Runs before any HIP call.
npd_status check_kd_call(const npd_kd_desc* desc, const void* student_logits, const void* teacher_dense,
                         const int32_t* teacher_idx, const float* teacher_val, const int32_t* labels,
                         const uint8_t* loss_mask, void* grad_out, float* kd_tok, float* nll_tok,
                         float* teacher_nll_tok, float* lse_tok, int32_t* dev_status, npd::KdArgs* args,
                         size_t* workspace_need) {
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

  // No output may overlap an input (other than the declared in-place gradient) or another output: a row's workgroup
  // would read what another workgroup has already overwritten.
  const KdBuffers b = kd_buffers(d, student_logits, teacher_dense, teacher_idx, teacher_val, labels, loss_mask, grad_out,
                                 kd_tok, nll_tok, teacher_nll_tok, lse_tok, dev_status);
  for (int o = 0; o < 6; ++o) {
    for (int i = 0; i < 6; ++i) {
      if (o == 0 && i == 0 && inplace) continue;
      if (overlaps(b.out[o], b.in[i])) return NPD_ERR_ALIAS;
    }
    for (int o2 = o + 1; o2 < 6; ++o2)
      if (overlaps(b.out[o], b.out[o2])) return NPD_ERR_ALIAS;
  }

  npd::KdArgs& a = *args;
  a = npd::KdArgs{};
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
  a.ws = nullptr;
  *workspace_need = workspace_bytes_of(d);
  return NPD_OK;
}

}  // namespace

extern "C" {

int npd_version(void) { return 116; }

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

const char* npd_kd_kernel_name(const npd_kd_desc* desc) {
  if (check_desc(desc) != NPD_OK) return "";
  const npd_kd_desc& d = *desc;
  npd::KdArgs a{};
  a.T = d.n_tokens;
  a.V = d.vocab;
  a.nvec_s = (d.student_stride % 8 == 0 && (d.teacher_kind != NPD_TEACHER_DENSE_BF16 || d.teacher_stride % 8 == 0))
                 ? d.vocab / 8
                 : 0;
  a.cscale = d.ce_grad_scale;
  a.divergence = d.divergence;
  a.need_lse1 = d.tau != 1.0f;
  uint32_t some_workspace = 0;
  a.ws = workspace_bytes_of(d) > 0 ? &some_workspace : nullptr;  // only tested against null
  return npd::kd_kernel_name(a, d.teacher_kind, !(d.flags & NPD_FLAG_FWD_ONLY));
}

size_t npd_workspace_bytes(const npd_kd_desc* desc) {
  if (check_desc(desc) != NPD_OK) return 0;
  return workspace_bytes_of(*desc);
}

npd_status npd_kd_loss_fwd_bwd(const npd_kd_desc* desc, const void* student_logits, const void* teacher_dense,
                               const int32_t* teacher_idx, const float* teacher_val, const int32_t* labels,
                               const uint8_t* loss_mask, void* grad_out, float* kd_tok, float* nll_tok,
                               float* teacher_nll_tok, float* lse_tok, int32_t* dev_status, void* workspace,
                               size_t workspace_bytes, void* stream) {
  npd::KdArgs a{};
  size_t need = 0;
  const npd_status st = check_kd_call(desc, student_logits, teacher_dense, teacher_idx, teacher_val, labels, loss_mask,
                                      grad_out, kd_tok, nll_tok, teacher_nll_tok, lse_tok, dev_status, &a, &need);
  if (st != NPD_OK) return st;
  if (need > 0) {
    if (!workspace || workspace_bytes < need || (reinterpret_cast<uintptr_t>(workspace) & 255u))
      return NPD_ERR_WORKSPACE;
    const KdBuffers b = kd_buffers(*desc, student_logits, teacher_dense, teacher_idx, teacher_val, labels, loss_mask,
                                   grad_out, kd_tok, nll_tok, teacher_nll_tok, lse_tok, dev_status);
    if (b.overlaps_any(range_of(workspace, need))) return NPD_ERR_ALIAS;
    a.ws = static_cast<uint32_t*>(workspace);
  }
  const bool want_grad = !(desc->flags & NPD_FLAG_FWD_ONLY);
  const hipError_t e = npd::launch_kd(a, desc->teacher_kind, want_grad, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? NPD_OK : NPD_ERR_HIP;
}

npd_status npd_kd_loss_fwd_bwd_noalloc(const npd_kd_desc* desc, const void* student_logits,
                                       const void* teacher_dense, const int32_t* teacher_idx,
                                       const float* teacher_val, const int32_t* labels, const uint8_t* loss_mask,
                                       void* grad_out, float* kd_tok, float* nll_tok, float* teacher_nll_tok,
                                       float* lse_tok, int32_t* dev_status, void* stream) {
  npd::KdArgs a{};
  size_t need = 0;
  const npd_status st = check_kd_call(desc, student_logits, teacher_dense, teacher_idx, teacher_val, labels, loss_mask,
                                      grad_out, kd_tok, nll_tok, teacher_nll_tok, lse_tok, dev_status, &a, &need);
  if (st != NPD_OK) return st;
  if (need > (size_t)NPD_NOALLOC_WORKSPACE_BYTES) return NPD_ERR_WORKSPACE;  // the built-in scratch is too small
  if (need > 0) {
    hipError_t e = hipSuccess;
    void* scratch = noalloc_scratch_address(&e);
    if (!scratch) return NPD_ERR_HIP;
    a.ws = static_cast<uint32_t*>(scratch);
  }
  const bool want_grad = !(desc->flags & NPD_FLAG_FWD_ONLY);
  const hipError_t e = npd::launch_kd(a, desc->teacher_kind, want_grad, static_cast<hipStream_t>(stream));
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
  {
    const Range in[2] = {range_of(teacher_logits, rows_bytes(n_tokens, teacher_stride, vocab, 2)),
                         opt_range(loss_mask, (size_t)n_tokens)};
    const Range out[2] = {range_of(topk_idx, (size_t)n_tokens * k * 4), range_of(topk_val, (size_t)n_tokens * k * 4)};
    if (any_alias(in, 2, out, 2)) return NPD_ERR_ALIAS;
  }
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
  {
    const size_t T = (size_t)n_tokens, S = (size_t)n_segments;
    const Range in[3] = {opt_range(values, T * 4), opt_range(loss_mask, T), opt_range(cu_seqlens, (S + 1) * 4)};
    const Range out[5] = {opt_range(seg_sum, S * 4), opt_range(seg_count, S * 4), opt_range(seg_mean, S * 4),
                          opt_range(token_to_sample, T * 4), opt_range(dev_status, 4)};
    if (any_alias(in, 3, out, 5)) return NPD_ERR_ALIAS;
  }
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
  {
    const size_t P = (size_t)n_pairs, S = (size_t)n_segments;
    const Range in[5] = {opt_range(mean_nll_student, S * 4), opt_range(mean_nll_teacher, S * 4),
                         opt_range(seg_count, S * 4), opt_range(pair_cond, P * 4), opt_range(pair_uncond, P * 4)};
    const Range out[6] = {opt_range(ifd_student, P * 4), opt_range(ifd_teacher, P * 4), opt_range(delta, P * 4),
                          opt_range(zone, P), opt_range(keep, P), opt_range(keep_count, 4)};
    if (any_alias(in, 5, out, 6)) return NPD_ERR_ALIAS;
  }
  const hipError_t e = npd::launch_delta_ifd(n_pairs, n_segments, mean_nll_student, mean_nll_teacher, seg_count,
                                             pair_cond, pair_uncond, lo, hi, flags, ifd_student, ifd_teacher, delta,
                                             zone, keep, keep_count, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? NPD_OK : NPD_ERR_HIP;
}

npd_status npd_policy_lag(int64_t n_tokens, int32_t n_segments, const float* kl_tok, const uint8_t* loss_mask,
                          const int32_t* cu_seqlens, float epsilon, float* seg_kl_mean, int32_t* seg_count,
                          float* batch_kl_mean, int32_t* batch_count, int32_t* lag_exceeded, int32_t* dev_status,
                          void* stream) {
  if (n_tokens < 0 || n_segments < 0) return NPD_ERR_SHAPE;
  if (n_tokens > NPD_MAX_TOKENS) return NPD_ERR_UNSUPPORTED;
  if (!(epsilon >= 0.0f) || !isfinite(epsilon)) return NPD_ERR_VALUE;
  if (misaligned(kl_tok, 4) || misaligned(cu_seqlens, 4) || misaligned(seg_kl_mean, 4) || misaligned(seg_count, 4) ||
      misaligned(batch_kl_mean, 4) || misaligned(batch_count, 4) || misaligned(lag_exceeded, 4) ||
      misaligned(dev_status, 4))
    return NPD_ERR_VALUE;
  if (n_segments > 0 && (!kl_tok || !loss_mask || !cu_seqlens)) return NPD_ERR_NULL;
  {
    const size_t T = (size_t)n_tokens, S = (size_t)n_segments;
    const Range in[3] = {opt_range(kl_tok, T * 4), opt_range(loss_mask, T), opt_range(cu_seqlens, (S + 1) * 4)};
    const Range out[6] = {opt_range(seg_kl_mean, S * 4), opt_range(seg_count, S * 4), opt_range(batch_kl_mean, 4),
                          opt_range(batch_count, 4),      opt_range(lag_exceeded, 4),  opt_range(dev_status, 4)};
    if (any_alias(in, 3, out, 6)) return NPD_ERR_ALIAS;
  }
  const hipError_t e =
      npd::launch_policy_lag(n_tokens, n_segments, kl_tok, loss_mask, cu_seqlens, epsilon, seg_kl_mean, seg_count,
                             batch_kl_mean, batch_count, lag_exceeded, dev_status, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? NPD_OK : NPD_ERR_HIP;
}

npd_status npd_segment_ppl(int32_t n_segments, const float* seg_mean_nll, const int32_t* seg_count, float* seg_ppl,
                           void* stream) {
  if (n_segments < 0) return NPD_ERR_SHAPE;
  if (misaligned(seg_mean_nll, 4) || misaligned(seg_count, 4) || misaligned(seg_ppl, 4)) return NPD_ERR_VALUE;
  if (n_segments > 0 && (!seg_mean_nll || !seg_count || !seg_ppl)) return NPD_ERR_NULL;
  {
    const size_t S = (size_t)n_segments;
    const Range in[2] = {opt_range(seg_mean_nll, S * 4), opt_range(seg_count, S * 4)};
    const Range out[1] = {opt_range(seg_ppl, S * 4)};
    if (any_alias(in, 2, out, 1)) return NPD_ERR_ALIAS;
  }
  const hipError_t e =
      npd::launch_segment_ppl(n_segments, seg_mean_nll, seg_count, seg_ppl, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? NPD_OK : NPD_ERR_HIP;
}

}  // extern "C"
