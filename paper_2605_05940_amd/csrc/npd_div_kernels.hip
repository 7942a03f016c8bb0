// Token-level divergences other than the forward KL of Eq. 2 -- the ones the Related Works section names beside it
// (reverse KL; skew KL and skew reverse KL with coefficient alpha), dense teacher, any row shape.  Same boundary,
// scalars and composite-loss term as the forward kernels; one workgroup streams one token row.
//
//   reverse       D = sum_c p_S log(p_S / p_T)
//   skew          D = sum_c p_T log(p_T / m),  m = alpha p_T + (1 - alpha) p_S
//   skew reverse  D = sum_c p_S log(p_S / m),  m = (1 - alpha) p_T + alpha p_S
//   dD / d s_j = (1 / tau) p_S(j) (u_j - ubar),  u = dD / d p_S,  ubar = sum_c p_S(c) u_c.
//
// Sweep 1 is the forward kernels' (base-2 partial log-sum-exps per lane, merged in a fixed order); for the reverse
// KL the cross term rides on the student stream, so that D = (a / z)_S / tau - lse_S + lse_T and
//   u_j - ubar = (s_j - t_j) / tau - (lse_S - lse_T) - D
// need nothing else: two sweeps, one v_exp_f32 per element in the second.  The skew forms are not linear in the
// normalisers, so D and ubar take a sweep of their own over normalised probabilities (block-wide sum of two floats)
// before the gradient sweep: three sweeps.
#include "npd_device.hpp"
#include "npd_internal.hpp"

namespace npd {

static_assert(kDivReverseKl == kReverseKl && kDivSkewKl == kSkewKl && kDivSkewReverseKl == kSkewReverseKl, "");

template <int BLOCK, int DIV, bool GRAD>
__global__ __launch_bounds__(BLOCK) void div_rows_kernel(const KdArgs a) {
  __shared__ float red[4 * 3 * (BLOCK / kWave)];
  const int tid = threadIdx.x;
  const int64_t row = blockIdx.x;
  const int V = a.V, nvec = a.nvec_s;
  uint16_t* grow = GRAD ? a.g + row * a.s_stride : nullptr;

  if (!a.mask[row]) {  // not scored: scalars 0, gradient row zero-filled, logits never read
    if (tid == 0) {
      if (a.kd) a.kd[row] = 0.0f;
      if (a.nll) a.nll[row] = 0.0f;
      if (a.tnll) a.tnll[row] = 0.0f;
      if (a.lse) a.lse[row] = 0.0f;
    }
    if constexpr (GRAD) {
      const uint4 z = make_uint4(0, 0, 0, 0);
      for (int i = tid; i < nvec; i += BLOCK) reinterpret_cast<uint4*>(grow)[i] = z;
      for (int e = nvec * 8 + tid; e < V; e += BLOCK) grow[e] = 0;
    }
    return;
  }

  const uint16_t* srow = a.s + row * a.s_stride;
  const uint16_t* trow = a.t + row * a.t_stride;
  const uint4* svec = reinterpret_cast<const uint4*>(srow);
  const uint4* tvec = reinterpret_cast<const uint4*>(trow);
  const float c = a.c;
  const bool lse1 = a.need_lse1 != 0;  // uniform
  const bool lse1_t = lse1 && a.tnll != nullptr;

  int y = -1;
  float s_y = 0.0f, t_y = 0.0f;
  if (a.labels) {  // label logits are fetched before an in-place gradient can overwrite them
    y = a.labels[row];
    if ((unsigned)y < (unsigned)V) {
      s_y = bf16_one(srow[y]);
      t_y = bf16_one(trow[y]);
    }
  }

  Lse acc[4];  // 0 student / tau (+ cross term), 1 teacher / tau, 2 student tau = 1, 3 teacher tau = 1
#pragma unroll
  for (int i = 0; i < 4; ++i) acc[i].init();

  // ---- sweep 1: normalisers (the same code path for both streams keeps them bitwise symmetric)
  for (int i = tid; i < nvec; i += BLOCK) {
    float xs[8], xt[8];
    unpack8(svec[i], xs);
    unpack8(tvec[i], xt);
    acc[0].add8_cross(xs, xt, c);
    acc[1].add8(xt, c);
    if (lse1) acc[2].add8(xs, kLog2e);
    if (lse1_t) acc[3].add8(xt, kLog2e);
  }
  for (int e = nvec * 8 + tid; e < V; e += BLOCK) {
    const float xs = bf16_one(srow[e]), xt = bf16_one(trow[e]);
    acc[0].add1_cross(xs, xs - xt, c);
    acc[1].add1(xt, c);
    if (lse1) acc[2].add1(xs, kLog2e);
    if (lse1_t) acc[3].add1(xt, kLog2e);
  }
  block_merge<BLOCK, 4>(acc, red);

  DivCoef k;
  k.c = c;
  k.Ls = acc[0].log2_sum();
  k.Lt = acc[1].log2_sum();
  k.inv_tau = a.inv_tau;
  k.alpha = a.alpha;
  k.gscale = a.gscale;
  k.cscale = a.cscale;
  k.ce = GRAD && a.cscale != 0.0f;
  k.ce_shared = !lse1;
  k.L1 = lse1 ? acc[2].log2_sum() : k.Ls;
  k.K = 0.0f;
  k.ubar = 0.0f;
  const float lse1_s = __fmul_rn(lse1 ? acc[2].log2_sum() : k.Ls, kLn2);

  float kd;
  if constexpr (DIV == kReverseKl) {
    // differences of like terms first: the references can be in the hundreds, their difference is small
    const float dl = ((acc[0].r - acc[1].r) + (acc[0].log2_z() - acc[1].log2_z())) * kLn2;  // lse_S - lse_T
    kd = (acc[0].a / acc[0].z) * a.inv_tau - dl;
    kd = kd < 0.0f ? 0.0f : kd;  // a KL divergence is >= 0; NaN passes through
    k.K = dl + kd;
  } else {
    // ---- sweep 2 of the skew forms: D and ubar over normalised probabilities
    float dsum = 0.0f, usum = 0.0f;
    for (int i = tid; i < nvec; i += BLOCK) {
      float xs[8], xt[8];
      unpack8(svec[i], xs);
      unpack8(tvec[i], xt);
#pragma unroll
      for (int j = 0; j < 8; ++j)
        skew_elem<DIV>(__builtin_fmaf(xs[j], c, -k.Ls), __builtin_fmaf(xt[j], c, -k.Lt), k.alpha, dsum, usum);
    }
    for (int e = nvec * 8 + tid; e < V; e += BLOCK)
      skew_elem<DIV>(__builtin_fmaf(bf16_one(srow[e]), c, -k.Ls), __builtin_fmaf(bf16_one(trow[e]), c, -k.Lt),
                     k.alpha, dsum, usum);
    kd = block_sum<BLOCK>(dsum, red);
    kd = kd < 0.0f ? 0.0f : kd;
    k.ubar = block_sum<BLOCK>(usum, red);
  }

  const bool bad_label = a.labels && (unsigned)y >= (unsigned)V;  // uniform
  if (tid == 0) {
    if (a.kd) a.kd[row] = kd;
    if (a.nll) a.nll[row] = bad_label ? __builtin_nanf("") : __fsub_rn(lse1_s, s_y);
    if (a.tnll) {
      const float lse1_tt = __fmul_rn(lse1 ? acc[3].log2_sum() : k.Lt, kLn2);
      a.tnll[row] = bad_label ? __builtin_nanf("") : __fsub_rn(lse1_tt, t_y);
    }
    if (a.lse) a.lse[row] = lse1_s;
    if (bad_label && (a.nll || a.tnll || k.ce) && a.status) atomicOr(a.status, 1);  // NPD_DEV_BAD_LABEL
  }

  // ---- gradient sweep, last group first (every thread rewrites only what it has just read: in place is safe)
  if constexpr (GRAD) {
    if (k.ce && bad_label) {  // uniform: the row cannot be differentiated
      const uint16_t qnan = 0x7fc0;
      for (int e = tid; e < V; e += BLOCK) grow[e] = qnan;
      return;
    }
    for (int e = nvec * 8 + tid; e < V; e += BLOCK)
      grow[e] = one_bf16(div_grad_elem<DIV>(bf16_one(srow[e]), bf16_one(trow[e]), k));
    for (int i = nvec - 1 - tid; i >= 0; i -= BLOCK) {
      float xs[8], xt[8], gv[8];
      unpack8(svec[i], xs);
      unpack8(tvec[i], xt);
#pragma unroll
      for (int j = 0; j < 8; ++j) gv[j] = div_grad_elem<DIV>(xs[j], xt[j], k);
      uint4 o;
      o.x = pack_bf16(gv[0], gv[1]);
      o.y = pack_bf16(gv[2], gv[3]);
      o.z = pack_bf16(gv[4], gv[5]);
      o.w = pack_bf16(gv[6], gv[7]);
      reinterpret_cast<uint4*>(grow)[i] = o;
    }
    if (k.ce) {  // uniform
      // the label position gets its final value once the dense stores of the whole workgroup are ordered before it
      __syncthreads();
      if (tid == 0) grow[y] = one_bf16(div_grad_elem<DIV>(s_y, t_y, k) - a.cscale);
    }
  }
}

template <int BLOCK, int DIV>
static hipError_t launch_block(const KdArgs& a, bool want_grad, hipStream_t stream) {
  const dim3 grid((unsigned)a.T), block(BLOCK);
  if (want_grad) return launch_kernel(div_rows_kernel<BLOCK, DIV, true>, grid, block, 0, stream, a);
  return launch_kernel(div_rows_kernel<BLOCK, DIV, false>, grid, block, 0, stream, a);
}

template <int DIV>
static hipError_t launch_div_kind(const KdArgs& a, bool want_grad, hipStream_t stream) {
  if (a.V >= 32768) return launch_block<1024, DIV>(a, want_grad, stream);
  if (a.V >= 4096) return launch_block<256, DIV>(a, want_grad, stream);
  return launch_block<64, DIV>(a, want_grad, stream);
}

hipError_t launch_div(const KdArgs& a, bool want_grad, hipStream_t stream) {
  switch (a.divergence) {
    case kReverseKl: return launch_div_kind<kReverseKl>(a, want_grad, stream);
    case kSkewKl: return launch_div_kind<kSkewKl>(a, want_grad, stream);
    case kSkewReverseKl: return launch_div_kind<kSkewReverseKl>(a, want_grad, stream);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace npd
