// Fused per-position KD loss and gradient (Alg. 1 "Compute Probs" / "Compute KD Loss"; Eq. 2;
// L_CE of Eq. 1) for gfx950: one workgroup streams one token row.
//
// Sweep 1 reads the student row (and the dense teacher row) once with 128-bit loads and keeps, per
// lane, partial log-sum-exps in registers (see npd_device.hpp); with a dense teacher the KL follows
// from the same sweep:
//     KL = sum_c p_T(c) (t_c - s_c) / tau  - lse(t / tau) + lse(s / tau)
// whose first term is the cross accumulator a / z of the teacher stream.  Wave totals are merged with
// cross-lane shuffles and wave totals through LDS.  Sweep 2 walks the row backwards (the lines read
// last are the ones still in cache), recomputes e = 2^(x c - r) against the row's merged reference
// exponent r and stores the bf16 gradient
//     grad_scale / tau * (p_S - p_T) = (e_S - e_T z_S / z_T) w,   w = grad_scale / (tau z_S),
// with one rounding to bf16 (the form gives an exact 0 when teacher and student coincide).  Subtracting only r inside the exponent keeps the argument small where p
// matters, so logits in the hundreds do not cost precision.
#include "npd_device.hpp"
#include "npd_internal.hpp"

namespace npd {

template <int BLOCK>
__device__ __forceinline__ void zero_row(uint16_t* grow, int nvec, int V) {
  const uint4 z = make_uint4(0, 0, 0, 0);
  for (int i = threadIdx.x; i < nvec; i += BLOCK) reinterpret_cast<uint4*>(grow)[i] = z;
  for (int e = nvec * 8 + threadIdx.x; e < V; e += BLOCK) grow[e] = 0;
}

template <int BLOCK, int TEACHER, bool GRAD>
__global__ __launch_bounds__(BLOCK) void kd_rows_kernel(const KdArgs a) {
  __shared__ float red[4 * 3 * (BLOCK / kWave)];
  __shared__ uint16_t patch[TEACHER == kTopk && GRAD ? kTopkMax : 1];
  __shared__ int y_in_support;  // top-k teacher: the label is one of the k support positions of this row
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
    if constexpr (GRAD) zero_row<BLOCK>(grow, nvec, V);
    return;
  }

  const uint16_t* srow = a.s + row * a.s_stride;
  const uint16_t* trow = TEACHER == kDense ? a.t + row * a.t_stride : nullptr;
  const float c = a.c;
  const bool lse1 = a.need_lse1 != 0;       // uniform
  const bool lse1_t = lse1 && a.tnll != nullptr;

  // label logits are fetched before anything can overwrite the row (in-place gradient)
  int y = -1;
  float s_y = 0.0f, t_y = 0.0f;
  if (a.labels) {
    y = a.labels[row];
    if ((unsigned)y < (unsigned)V) {
      s_y = bf16_one(srow[y]);
      if (TEACHER == kDense) t_y = bf16_one(trow[y]);
    }
  }

  Lse acc[4];  // 0 student / tau, 1 teacher / tau (+ cross term), 2 student tau = 1, 3 teacher tau = 1
#pragma unroll
  for (int i = 0; i < 4; ++i) acc[i].init();

  // ---- sweep 1
  for (int i = tid; i < nvec; i += BLOCK) {
    float xs[8];
    unpack8(reinterpret_cast<const uint4*>(srow)[i], xs);
    if constexpr (TEACHER == kDense) {
      float xt[8];
      unpack8(reinterpret_cast<const uint4*>(trow)[i], xt);
      acc[1].add8_cross(xt, xs, c);
      if (lse1_t) acc[3].add8(xt, kLog2e);
    }
    acc[0].add8(xs, c);
    if (lse1) acc[2].add8(xs, kLog2e);
  }
  for (int e = nvec * 8 + tid; e < V; e += BLOCK) {
    const float xs = bf16_one(srow[e]);
    if constexpr (TEACHER == kDense) {
      const float xt = bf16_one(trow[e]);
      acc[1].add1_cross(xt, xt - xs, c);
      if (lse1_t) acc[3].add1(xt, kLog2e);
    }
    acc[0].add1(xs, c);
    if (lse1) acc[2].add1(xs, kLog2e);
  }
  int bad_index = 0;
  if constexpr (TEACHER == kTopk) {
    const int32_t* irow = a.tidx + row * (int64_t)a.k;
    const float* vrow = a.tval + row * (int64_t)a.k;
    for (int j = tid; j < a.k; j += BLOCK) {
      if ((unsigned)irow[j] >= (unsigned)V) bad_index = 1;
      acc[1].add1(vrow[j], c);
    }
  }

  block_merge<BLOCK, 4>(acc, red);

  const float Ls = acc[0].log2_sum();                                   // log2 sum 2^(s c)
  const float Lt = TEACHER == kNone ? 0.0f : acc[1].log2_sum();
  // natural log-sum-exp of the raw logits; explicit roundings so student and teacher go the same way
  const float lse1_s = __fmul_rn(lse1 ? acc[2].log2_sum() : Ls, kLn2);
  float kd = 0.0f;

  if constexpr (TEACHER == kDense) {
    // differences of like terms first: the references can be in the hundreds, their difference is small
    kd = (acc[1].a / acc[1].z) * a.inv_tau + ((acc[0].r - acc[1].r) + (acc[0].log2_z() - acc[1].log2_z())) * kLn2;
    kd = kd < 0.0f ? 0.0f : kd;  // a KL divergence is >= 0; NaN passes through
  }

  const bool ce = GRAD && a.cscale != 0.0f;                           // uniform: hard-label CE gradient wanted
  const bool bad_label = a.labels && (unsigned)y >= (unsigned)V;      // uniform
  const GradCoef gk = make_grad_coef(acc[0], acc[1], acc[2], c, a.gscale, a.cscale, TEACHER != kNone, lse1);

  if constexpr (TEACHER == kTopk) {
    bad_index = __syncthreads_or(bad_index);
    if (tid == 0) y_in_support = 0;
    __syncthreads();
    const int32_t* irow = a.tidx + row * (int64_t)a.k;
    const float* vrow = a.tval + row * (int64_t)a.k;
    float part = 0.0f;
    if (!bad_index) {
      for (int j = tid; j < a.k; j += BLOCK) {
        const float b = vrow[j] * c;
        const float sj = bf16_one(srow[irow[j]]);
        const float lpt = b - Lt;                         // log2 p_T
        const float lps = __builtin_fmaf(sj, c, -Ls);     // log2 p_S
        part = __builtin_fmaf(exp2_fast(lpt), __builtin_fmaxf(lpt - lps, -3.4028234663852886e38f) * kLn2, part);  // a -inf entry: 0
        if constexpr (GRAD) {
          // the value this position finally holds, from fp32, rounded once
          float gj = grad_pair_elem(sj, b, gk);
          if (ce && irow[j] == y) {
            gj -= a.cscale;
            y_in_support = 1;
          }
          patch[j] = one_bf16(gj);
        }
      }
    }
    kd = block_sum<BLOCK>(part, red);
    kd = kd < 0.0f ? 0.0f : kd;
    if (bad_index) kd = __builtin_nanf("");
  }

  if (tid == 0) {
    int flags = 0;
    if (bad_index) flags |= 2;  // NPD_DEV_BAD_TOPK_INDEX
    if (bad_label && (a.nll || a.tnll || ce)) flags |= 1;  // NPD_DEV_BAD_LABEL
    if (a.kd) a.kd[row] = kd;
    if (a.nll) a.nll[row] = bad_label ? __builtin_nanf("") : __fsub_rn(lse1_s, s_y);
    if (TEACHER == kDense && a.tnll) {
      const float lse1_tt = __fmul_rn(lse1 ? acc[3].log2_sum() : Lt, kLn2);
      a.tnll[row] = bad_label ? __builtin_nanf("") : __fsub_rn(lse1_tt, t_y);
    }
    if (a.lse) a.lse[row] = lse1_s;
    if (flags && a.status) atomicOr(a.status, flags);
  }

  // ---- sweep 2: gradient, last group first
  if constexpr (GRAD) {
    if ((TEACHER == kTopk && bad_index) || (ce && bad_label)) {  // uniform: the row cannot be differentiated
      const uint16_t qnan = 0x7fc0;
      for (int e = tid; e < V; e += BLOCK) grow[e] = qnan;
      return;
    }
    for (int e = nvec * 8 + tid; e < V; e += BLOCK) {
      const float xs = bf16_one(srow[e]);
      grow[e] = one_bf16(TEACHER == kDense ? grad_dense_elem(xs, bf16_one(trow[e]), gk) : grad_student_elem(xs, gk));
    }
    for (int i = nvec - 1 - tid; i >= 0; i -= BLOCK) {
      float xs[8], gv[8];
      unpack8(reinterpret_cast<const uint4*>(srow)[i], xs);
      if constexpr (TEACHER == kDense) {
        float xt[8];
        unpack8(reinterpret_cast<const uint4*>(trow)[i], xt);
#pragma unroll
        for (int j = 0; j < 8; ++j) gv[j] = grad_dense_elem(xs[j], xt[j], gk);
      } else {
#pragma unroll
        for (int j = 0; j < 8; ++j) gv[j] = grad_student_elem(xs[j], gk);
      }
      uint4 o;
      o.x = pack_bf16(gv[0], gv[1]);
      o.y = pack_bf16(gv[2], gv[3]);
      o.z = pack_bf16(gv[4], gv[5]);
      o.w = pack_bf16(gv[6], gv[7]);
      reinterpret_cast<uint4*>(grow)[i] = o;
    }
    if (TEACHER == kTopk || ce) {  // uniform
      // the k support positions and the label position are overwritten with their final values once the dense
      // stores of the whole workgroup are ordered before them
      __syncthreads();
      if constexpr (TEACHER == kTopk) {
        const int32_t* irow = a.tidx + row * (int64_t)a.k;
        for (int j = tid; j < a.k; j += BLOCK) grow[irow[j]] = patch[j];
      }
      if (ce && tid == 0 && !(TEACHER == kTopk && y_in_support)) {
        const float gy = TEACHER == kDense ? grad_dense_elem(s_y, t_y, gk) : grad_student_elem(s_y, gk);
        grow[y] = one_bf16(gy - a.cscale);
      }
    }
  }
}

template <int BLOCK, int TEACHER>
static hipError_t launch_block(const KdArgs& a, bool want_grad, hipStream_t stream) {
  const dim3 grid((unsigned)a.T), block(BLOCK);
  if (want_grad) return launch_kernel(kd_rows_kernel<BLOCK, TEACHER, true>, grid, block, 0, stream, a);
  return launch_kernel(kd_rows_kernel<BLOCK, TEACHER, false>, grid, block, 0, stream, a);
}

template <int TEACHER>
static hipError_t launch_teacher(const KdArgs& a, bool want_grad, hipStream_t stream) {
  if (a.V >= 32768) return launch_block<1024, TEACHER>(a, want_grad, stream);
  if (a.V >= 4096) return launch_block<256, TEACHER>(a, want_grad, stream);
  return launch_block<64, TEACHER>(a, want_grad, stream);
}

// the kernel family launch_kd picks for these arguments
const char* kd_kernel_name(const KdArgs& a, int teacher_kind, bool want_grad) {
  if (a.ws && gang_path_applies(a, teacher_kind, want_grad)) return "kd_gang_kernel";
  if (cached_path_applies(a, teacher_kind, want_grad)) return "kd_cached_kernel";
  if (a.divergence != kForwardKl) return "div_rows_kernel";
  return "kd_rows_kernel";
}

hipError_t launch_kd(const KdArgs& a, int teacher_kind, bool want_grad, hipStream_t stream) {
  if (a.ws && gang_path_applies(a, teacher_kind, want_grad)) return launch_kd_gang(a, teacher_kind, stream);
  if (cached_path_applies(a, teacher_kind, want_grad)) return launch_kd_cached(a, teacher_kind, want_grad, stream);
  if (a.divergence != kForwardKl) return launch_div(a, want_grad, stream);  // dense teacher (checked by the API)
  switch (teacher_kind) {
    case kDense: return launch_teacher<kDense>(a, want_grad, stream);
    case kTopk: return launch_teacher<kTopk>(a, want_grad, stream);
    default: return launch_teacher<kNone>(a, false, stream);
  }
}

}  // namespace npd
