// Host-side launch interface between the C ABI (npd_api.hip) and the kernel files.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace npd {

enum TeacherKind { kDense = 0, kTopk = 1, kNone = 2 };
enum Divergence { kForwardKl = 0, kReverseKl = 1, kSkewKl = 2, kSkewReverseKl = 3 };

constexpr int kTopkMax = 4096;  // largest k the top-k kernels stage per row

struct KdArgs {
  const uint16_t* s;      // student logits, bf16 [T, s_stride]
  const uint16_t* t;      // dense teacher logits, bf16 [T, t_stride]
  const int32_t* tidx;    // top-k ids [T, k]
  const float* tval;      // top-k values [T, k]
  const int32_t* labels;  // [T] or null
  const uint8_t* mask;    // [T]
  uint16_t* g;            // gradient, bf16 [T, s_stride] or null
  float* kd;
  float* nll;
  float* tnll;
  float* lse;
  int32_t* status;
  int64_t T;
  int64_t s_stride, t_stride;
  int32_t V, k;
  int32_t nvec_s;      // 8-element groups of a row that are moved with 128-bit accesses (0: unaligned)
  float c;             // log2(e) / tau
  float inv_tau;
  float gscale;        // grad_scale / tau
  float cscale;        // ce_grad_scale (weight of the hard-label CE gradient; 0 = none)
  int32_t need_lse1;   // tau != 1 and a tau = 1 quantity (nll, teacher nll, lse) is wanted
  int32_t divergence;  // Divergence
  float alpha;         // skew coefficient
  // row-gang kernels (npd_kd_gang.hpp)
  uint32_t* ws;          // scratch record, gang_workspace_bytes() bytes
  int32_t gang;          // slices (workgroups) per row
  int32_t gang_groups;   // 128-bit groups per slice
  int32_t gang_pow2;     // gang rounded up to a power of two
  int32_t spin_limit;    // polls before a waiting workgroup gives up
};

// Enqueues `kernel` and returns this launch's own status: the thread's pending HIP error (something an earlier call
// of the application left behind) is neither reported as ours nor cleared.  Arguments are converted to the kernel's
// parameter types.
template <class T>
struct launch_param {
  using type = T;
};
template <class... Params>
inline hipError_t launch_kernel(void (*kernel)(Params...), dim3 grid, dim3 block, size_t lds_bytes, hipStream_t stream,
                                typename launch_param<Params>::type... params) {
  void* argv[] = {const_cast<void*>(static_cast<const void*>(&params))...};
  return hipLaunchKernel(reinterpret_cast<const void*>(kernel), grid, block, argv, lds_bytes, stream);
}

hipError_t launch_kd(const KdArgs& a, int teacher_kind, bool want_grad, hipStream_t stream);
const char* kd_kernel_name(const KdArgs& a, int teacher_kind, bool want_grad);

// divergences other than the forward KL, dense teacher (npd_div_kernels.hip)
hipError_t launch_div(const KdArgs& a, bool want_grad, hipStream_t stream);

// row-resident kernels for large vocabularies (npd_kd_cached.hip)
bool cached_path_applies(const KdArgs& a, int teacher_kind, bool want_grad);
hipError_t launch_kd_cached(const KdArgs& a, int teacher_kind, bool want_grad, hipStream_t stream);

// row-gang kernels for long rows with a dense teacher (npd_kd_gang.hip); `lse1`: tau != 1 and a tau = 1 quantity wanted
bool gang_path_applies(const KdArgs& a, int teacher_kind, bool want_grad);
size_t gang_workspace_bytes(int64_t T, int32_t V, int teacher_kind, int divergence, bool lse1);
hipError_t launch_kd_gang(const KdArgs& a, int teacher_kind, hipStream_t stream);
int set_gang_spin_limit(int polls);  // returns the previous limit; <= 0 restores the default

// compute units of the current device (cached per device)
int compute_units();

// the instantiations of the row-resident kernel, one translation unit each (npd_kd_cached_*.hip)
hipError_t launch_cached_forward_1024(const KdArgs& a, int cs, int teacher_kind, hipStream_t stream);
hipError_t launch_cached_divergence_1024(const KdArgs& a, int cs, hipStream_t stream);
hipError_t launch_cached_divergence_512(const KdArgs& a, int cs, hipStream_t stream);
hipError_t launch_cached_divergence_256(const KdArgs& a, int cs, hipStream_t stream);
hipError_t launch_cached_short_512(const KdArgs& a, int cs, int teacher_kind, hipStream_t stream);
hipError_t launch_cached_short_256(const KdArgs& a, int cs, int teacher_kind, hipStream_t stream);
hipError_t launch_cached_forward_only(const KdArgs& a, int threads, int teacher_kind, hipStream_t stream);

// arguments of the top-k kernels (npd_topk_impl.hpp)
struct TopkArgs {
  const uint16_t* t;
  const uint8_t* mask;
  int32_t* idx;
  float* val;
  int64_t stride;
  int64_t T;
  int32_t V, k, nvec, log_probs;
};

hipError_t launch_teacher_topk(int64_t T, int32_t V, int64_t stride, int32_t k, int log_probs, const uint16_t* t,
                               const uint8_t* mask, int32_t* idx, float* val, hipStream_t stream);

hipError_t launch_segment_reduce(int64_t T, int32_t S, const float* values, const uint8_t* mask, const int32_t* cu,
                                 float* seg_sum, int32_t* seg_count, float* seg_mean, int32_t* token_to_sample,
                                 int32_t* status, hipStream_t stream);

hipError_t launch_delta_ifd(int32_t P, int32_t S, const float* ms, const float* mt, const int32_t* cnt,
                            const int32_t* pc, const int32_t* pu, float lo, float hi, uint32_t flags, float* ifd_s,
                            float* ifd_t, float* delta, uint8_t* zone, uint8_t* keep, int32_t* keep_count,
                            hipStream_t stream);

hipError_t launch_policy_lag(int64_t T, int32_t S, const float* kl, const uint8_t* mask, const int32_t* cu,
                             float epsilon, float* seg_mean, int32_t* seg_count, float* batch_mean,
                             int32_t* batch_count, int32_t* exceeded, int32_t* status, hipStream_t stream);

hipError_t launch_segment_ppl(int32_t S, const float* mean_nll, const int32_t* cnt, float* ppl, hipStream_t stream);

}  // namespace npd
