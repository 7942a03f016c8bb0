// Per-sample reduction over the packed layout, the Delta-IFD score (Sec. 3.2, Eq. 3 and Eq. 4), the policy-latency
// monitor of the appendix and the perplexity of a sample.
// Both are tiny next to the loss kernel; what matters here is exact bookkeeping and a fixed
// summation order (no floating-point atomics), so results are bitwise reproducible.
#include "npd_device.hpp"
#include "npd_internal.hpp"

namespace npd {

constexpr int kSegBlock = 256;

__global__ __launch_bounds__(kSegBlock) void fill_i32_kernel(int32_t* p, int64_t n, int32_t v) {
  for (int64_t i = blockIdx.x * (int64_t)kSegBlock + threadIdx.x; i < n; i += (int64_t)gridDim.x * kSegBlock) p[i] = v;
}

// One workgroup per sample.  Thread t adds positions begin + t, begin + t + 256, ... in order; the 256
// partials are then folded by the fixed shuffle tree and the four wave totals in wave order.
__global__ __launch_bounds__(kSegBlock) void segment_reduce_kernel(int64_t T, const float* __restrict__ x,
                                                                   const uint8_t* __restrict__ mask,
                                                                   const int32_t* __restrict__ cu, float* seg_sum,
                                                                   int32_t* seg_count, float* seg_mean,
                                                                   int32_t* token_to_sample, int32_t* status) {
  __shared__ float fred[kSegBlock / kWave];
  __shared__ int ired[kSegBlock / kWave];
  const int seg = blockIdx.x;
  const int64_t b = cu[seg], e = cu[seg + 1];
  if (b < 0 || e < b || e > T) {  // uniform: the whole workgroup leaves together
    if (threadIdx.x == 0) {
      if (seg_sum) seg_sum[seg] = __builtin_nanf("");
      if (seg_mean) seg_mean[seg] = __builtin_nanf("");
      if (seg_count) seg_count[seg] = 0;
      if (status) atomicOr(status, 4);  // NPD_DEV_BAD_CU_SEQLENS
    }
    return;
  }
  float acc = 0.0f;
  int n = 0;
  for (int64_t p = b + threadIdx.x; p < e; p += kSegBlock) {
    if (token_to_sample) token_to_sample[p] = seg;
    if (mask[p]) {
      if (x) acc += x[p];
      n += 1;
    }
  }
  acc = block_sum<kSegBlock>(acc, fred);
  n = block_sum_int<kSegBlock>(n, ired);
  if (threadIdx.x == 0) {
    if (seg_sum) seg_sum[seg] = acc;
    if (seg_count) seg_count[seg] = n;
    if (seg_mean) seg_mean[seg] = n > 0 ? acc / (float)n : 0.0f;
  }
}

hipError_t launch_segment_reduce(int64_t T, int32_t S, const float* values, const uint8_t* mask, const int32_t* cu,
                                 float* seg_sum, int32_t* seg_count, float* seg_mean, int32_t* token_to_sample,
                                 int32_t* status, hipStream_t stream) {
  if (token_to_sample && T > 0) {
    const int64_t want = (T + kSegBlock - 1) / kSegBlock;
    const unsigned blocks = (unsigned)(want < 4096 ? want : 4096);
    const hipError_t e = launch_kernel(fill_i32_kernel, dim3(blocks), dim3(kSegBlock), 0, stream, token_to_sample, T, -1);
    if (e != hipSuccess) return e;
  }
  if (S > 0) {
    return launch_kernel(segment_reduce_kernel, dim3((unsigned)S), dim3(kSegBlock), 0, stream, T, values, mask, cu,
                         seg_sum, seg_count, seg_mean, token_to_sample, status);
  }
  return hipSuccess;
}

// One thread per pair.  The number of kept pairs is an integer sum: exact in any order.
__global__ __launch_bounds__(kSegBlock) void delta_ifd_kernel(int32_t P, int32_t S, const float* __restrict__ ms,
                                                              const float* __restrict__ mt,
                                                              const int32_t* __restrict__ cnt,
                                                              const int32_t* __restrict__ pc,
                                                              const int32_t* __restrict__ pu, float lo, float hi,
                                                              uint32_t flags, float* ifd_s, float* ifd_t, float* delta,
                                                              uint8_t* zone, uint8_t* keep, int32_t* keep_count) {
  __shared__ int ired[kSegBlock / kWave];
  int kept = 0;
  for (int64_t j = blockIdx.x * (int64_t)kSegBlock + threadIdx.x; j < P; j += (int64_t)gridDim.x * kSegBlock) {
    const int ic = pc[j], iu = pu[j];
    const float nanv = __builtin_nanf("");
    float fs = nanv, ft = nanv, d = nanv;
    uint8_t z = 3, kp = 0;  // NPD_ZONE_INVALID
    // a pair with an empty sample, a zero denominator or a mean loss that is not finite has no score (also where
    // plain division would give a finite ratio: 1 / inf = 0)
    if ((unsigned)ic < (unsigned)S && (unsigned)iu < (unsigned)S && cnt[ic] > 0 && cnt[iu] > 0 && ms[iu] != 0.0f &&
        mt[iu] != 0.0f && isfinite(ms[ic]) && isfinite(ms[iu]) && isfinite(mt[ic]) && isfinite(mt[iu])) {
      fs = ms[ic] / ms[iu];  // IEEE division
      ft = mt[ic] / mt[iu];
      d = ft - fs;
    }
    if (isfinite(fs) && isfinite(ft) && isfinite(d)) {
      z = d < lo ? 0 : (d > hi ? 2 : 1);
      kp = z == 1;
      if ((flags & 1u) && !(ft <= 1.0f)) kp = 0;
    } else {
      fs = ft = d = nanv;
    }
    if (ifd_s) ifd_s[j] = fs;
    if (ifd_t) ifd_t[j] = ft;
    if (delta) delta[j] = d;
    if (zone) zone[j] = z;
    if (keep) keep[j] = kp;
    kept += kp;
  }
  kept = block_sum_int<kSegBlock>(kept, ired);
  if (threadIdx.x == 0 && keep_count && kept) atomicAdd(keep_count, kept);
}

hipError_t launch_delta_ifd(int32_t P, int32_t S, const float* ms, const float* mt, const int32_t* cnt,
                            const int32_t* pc, const int32_t* pu, float lo, float hi, uint32_t flags, float* ifd_s,
                            float* ifd_t, float* delta, uint8_t* zone, uint8_t* keep, int32_t* keep_count,
                            hipStream_t stream) {
  if (keep_count) {
    const hipError_t e = launch_kernel(fill_i32_kernel, dim3(1), dim3(kSegBlock), 0, stream, keep_count, (int64_t)1, 0);
    if (e != hipSuccess) return e;
  }
  if (P > 0) {
    const int want = (P + kSegBlock - 1) / kSegBlock;
    const unsigned blocks = (unsigned)(want < 1024 ? want : 1024);
    return launch_kernel(delta_ifd_kernel, dim3(blocks), dim3(kSegBlock), 0, stream, P, S, ms, mt, cnt, pc, pu, lo, hi,
                         flags, ifd_s, ifd_t, delta, zone, keep, keep_count);
  }
  return hipSuccess;
}

// ---- policy-latency monitor (appendix, "Analysis of Policy Latency") and perplexity

constexpr int kLagBlock = 1024;

// The step's D_KL(learner || generator): mean of kl_tok over the scored positions that a sample owns -- with a valid
// cu_seqlens those are the scored positions of [cu[0], cu[S]) -- against the near-policy bound epsilon.  One workgroup;
// thread t adds positions begin + t, begin + t + 1024, ... in order, then one fixed tree: reproducible.
__global__ __launch_bounds__(kLagBlock) void policy_lag_batch_kernel(int64_t T, int32_t S, const float* __restrict__ kl,
                                                                    const uint8_t* __restrict__ mask,
                                                                    const int32_t* __restrict__ cu, float epsilon,
                                                                    float* batch_mean, int32_t* batch_count,
                                                                    int32_t* exceeded, int32_t* status) {
  __shared__ float fred[kLagBlock / kWave];
  __shared__ int ired[kLagBlock / kWave];
  int bad = 0;
  for (int i = threadIdx.x; i < S; i += kLagBlock)
    if (cu[i] > cu[i + 1]) bad = 1;
  if (S > 0 && threadIdx.x == 0 && (cu[0] < 0 || cu[S] > T)) bad = 1;
  bad = __syncthreads_or(bad);
  float acc = 0.0f;
  int n = 0;
  if (!bad && S > 0) {
    const int64_t b = cu[0], e = cu[S];
    for (int64_t p = b + threadIdx.x; p < e; p += kLagBlock) {
      if (mask[p]) {
        acc += kl[p];
        n += 1;
      }
    }
  }
  acc = block_sum<kLagBlock>(acc, fred);
  n = block_sum_int<kLagBlock>(n, ired);
  if (threadIdx.x == 0) {
    const float mean = bad ? __builtin_nanf("") : (n > 0 ? acc / (float)n : 0.0f);
    if (batch_mean) *batch_mean = mean;
    if (batch_count) *batch_count = bad ? 0 : n;
    if (exceeded) *exceeded = !(mean <= epsilon);  // near-policy: D_KL <= epsilon; NaN counts as beyond
    if (bad && status) atomicOr(status, 4);        // NPD_DEV_BAD_CU_SEQLENS
  }
}

hipError_t launch_policy_lag(int64_t T, int32_t S, const float* kl, const uint8_t* mask, const int32_t* cu,
                             float epsilon, float* seg_mean, int32_t* seg_count, float* batch_mean,
                             int32_t* batch_count, int32_t* exceeded, int32_t* status, hipStream_t stream) {
  if (S > 0 && (seg_mean || seg_count)) {
    const hipError_t e = launch_kernel(segment_reduce_kernel, dim3((unsigned)S), dim3(kSegBlock), 0, stream, T, kl, mask,
                                       cu, static_cast<float*>(nullptr), seg_count, seg_mean,
                                       static_cast<int32_t*>(nullptr), status);
    if (e != hipSuccess) return e;
  }
  return launch_kernel(policy_lag_batch_kernel, dim3(1), dim3(kLagBlock), 0, stream, T, S, kl, mask, cu, epsilon,
                       batch_mean, batch_count, exceeded, status);
}

// PPL = exp(mean CE loss) of every sample; 0 for samples without a scored position
__global__ __launch_bounds__(kSegBlock) void segment_ppl_kernel(int32_t S, const float* __restrict__ mean_nll,
                                                                const int32_t* __restrict__ cnt, float* ppl) {
  for (int64_t i = blockIdx.x * (int64_t)kSegBlock + threadIdx.x; i < S; i += (int64_t)gridDim.x * kSegBlock)
    ppl[i] = cnt[i] > 0 ? expf(mean_nll[i]) : 0.0f;
}

hipError_t launch_segment_ppl(int32_t S, const float* mean_nll, const int32_t* cnt, float* ppl, hipStream_t stream) {
  if (S <= 0) return hipSuccess;
  const int want = (S + kSegBlock - 1) / kSegBlock;
  return launch_kernel(segment_ppl_kernel, dim3((unsigned)(want < 1024 ? want : 1024)), dim3(kSegBlock), 0, stream, S,
                       mean_nll, cnt, ppl);
}

}  // namespace npd
