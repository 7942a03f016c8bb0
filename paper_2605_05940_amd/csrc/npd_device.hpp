// Device-side building blocks shared by the libnpd kernels (gfx950, wave64).
//
// Numerics.  All soft-max work is done in the base-2 domain: with c = log2(e) / tau,
// exp(x / tau) = 2^(x * c).  A partial log-sum-exp is a pair (r, z) meaning
// sum = z * 2^r; a partial cross term `a` carries the same implicit 2^r.  r is a lane's
// private reference exponent.  It only moves when an incoming value exceeds it by more
// than 2^32, so the common case costs one fused multiply-add and one v_exp_f32 per
// element and no rescaling; terms stay below 2^32 relative to r, far from fp32 overflow.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace npd {

constexpr int kWave = 64;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kRefSlack = 32.0f;  // a lane's reference exponent may lag its largest term by 2^32

__device__ __forceinline__ float exp2_fast(float x) { return __builtin_amdgcn_exp2f(x); }  // v_exp_f32

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __builtin_bit_cast(float, w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __builtin_bit_cast(float, w & 0xffff0000u); }
__device__ __forceinline__ float bf16_one(uint16_t h) { return __builtin_bit_cast(float, (uint32_t)h << 16); }

typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

// two fp32 -> packed bf16, round to nearest even (v_cvt_pk_bf16_f32); `lo` lands in bits 0..15
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  f32x2 v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}
__device__ __forceinline__ uint16_t one_bf16(float x) { return (uint16_t)(pack_bf16(x, 0.0f) & 0xffffu); }

__device__ __forceinline__ void unpack8(const uint4& v, float x[8]) {
  x[0] = bf16_lo(v.x); x[1] = bf16_hi(v.x);
  x[2] = bf16_lo(v.y); x[3] = bf16_hi(v.y);
  x[4] = bf16_lo(v.z); x[5] = bf16_hi(v.z);
  x[6] = bf16_lo(v.w); x[7] = bf16_hi(v.w);
}

// v_max3_f32 without the input canonicalisation the compiler adds around fmaxf (the values come straight
// from bf16 bit patterns; a NaN among them simply propagates into the sums)
__device__ __forceinline__ float max3(float a, float b, float c) {
  float d;
  asm("v_max3_f32 %0, %1, %2, %3" : "=v"(d) : "v"(a), "v"(b), "v"(c));
  return d;
}
__device__ __forceinline__ float max8(const float x[8]) {
  float m = max3(x[0], x[1], x[2]);
  m = max3(m, x[3], x[4]);
  m = max3(m, x[5], x[6]);
  return max3(m, x[7], x[7]);
}

// Partial log-sum-exp with an optional cross term.
struct Lse {
  float r, z, a;
  // the reference starts far below every finite logit but finite, so that a first element of -inf (a masked
  // vocabulary entry) gives 2^(-inf - r) = 0 rather than 2^(-inf + inf)
  __device__ __forceinline__ void init() { r = -1.0e30f; z = 0.0f; a = 0.0f; }
  // raise the reference to `u` if it lags by more than the slack (also the first touch).
  // The outer test is wave-uniform, so the common case is one compare and a scalar branch not taken.
  __device__ __forceinline__ void raise(float u) {
    const bool lag = u > r + kRefSlack;
    if (__builtin_amdgcn_ballot_w64(lag) != 0) {
      asm volatile("");  // not speculatable: keeps this rare path behind a real branch
      if (lag) {
        const float f = exp2_fast(r - u);  // the initial reference gives 0
        z *= f;
        a *= f;
        r = u;
      }
    }
  }
  __device__ __forceinline__ void add8(const float x[8], float c) {
    raise(max8(x) * c);
#pragma unroll
    for (int i = 0; i < 8; ++i) z += exp2_fast(__builtin_fmaf(x[i], c, -r));
  }
  // also accumulates a += 2^(x*c - r) * (x - y).  The difference is kept above -FLT_MAX: a logit of -inf on the
  // x side (a masked vocabulary entry: probability 0) then contributes 0 * finite = 0 rather than 0 * -inf.
  __device__ __forceinline__ void add8_cross(const float x[8], const float y[8], float c) {
    raise(max8(x) * c);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const float e = exp2_fast(__builtin_fmaf(x[i], c, -r));
      z += e;
      a = __builtin_fmaf(e, __builtin_fmaxf(x[i] - y[i], -3.4028234663852886e38f), a);
    }
  }
  __device__ __forceinline__ void add1(float x, float c) {
    raise(x * c);
    z += exp2_fast(__builtin_fmaf(x, c, -r));
  }
  __device__ __forceinline__ void add1_cross(float x, float d, float c) {
    raise(x * c);
    const float e = exp2_fast(__builtin_fmaf(x, c, -r));
    z += e;
    a = __builtin_fmaf(e, __builtin_fmaxf(d, -3.4028234663852886e38f), a);
  }
  // merge another partial into this one (same code for every stream, so that two streams fed
  // identical data stay bitwise identical)
  __device__ __forceinline__ void merge(float r2, float z2, float a2) {
    const float R = fmaxf(r, r2);
    const float f1 = (r == R) ? 1.0f : exp2_fast(r - R);
    const float f2 = (r2 == R) ? 1.0f : exp2_fast(r2 - R);
    // explicit products and fused adds: the contraction must not depend on the call site
    z = __builtin_fmaf(z, f1, __fmul_rn(z2, f2));
    a = __builtin_fmaf(a, f1, __fmul_rn(a2, f2));
    r = R;
  }
  __device__ __forceinline__ float log2_z() const { return __log2f(z); }
  __device__ __forceinline__ float log2_sum() const { return r + __log2f(z); }
};

// Coefficients of the gradient write (sweep 2), precise form:
//   grad_scale / tau * (p_S - p_T) = (e_S - e_T z_S / z_T) w_S,   e = 2^(x c - r),  w_S = grad_scale / (tau z_S)
// (exactly 0 when teacher and student coincide), plus, for the composite loss of Eq. 1, the hard-label CE term
//   ce_grad_scale * Softmax(s)(c) = 2^(x log2(e) - r1) w_C,   w_C = ce_grad_scale / z1,
// whose softmax has no temperature; at tau = 1 it shares e_S with the KD term.
struct GradCoef {
  float c, rs, rt, ratio, ws;
  float r1, wc;
  bool ce;         // uniform: CE term present
  bool ce_shared;  // tau = 1
};

__device__ __forceinline__ GradCoef make_grad_coef(const Lse& S, const Lse& Tt, const Lse& S1, float c, float gscale,
                                                   float cscale, bool has_teacher_stream, bool lse1) {
  GradCoef k;
  k.c = c;
  k.rs = S.r;
  k.rt = Tt.r;
  k.ws = gscale / S.z;
  k.ratio = has_teacher_stream ? S.z / Tt.z : 0.0f;
  k.ce = cscale != 0.0f;
  k.ce_shared = !lse1;
  k.r1 = lse1 ? S1.r : S.r;
  k.wc = k.ce ? cscale / (lse1 ? S1.z : S.z) : 0.0f;
  return k;
}

// e_S-only part (no teacher term): the dense part of a top-k row
__device__ __forceinline__ float grad_student_elem(float xs, const GradCoef& k) {
  const float es = exp2_fast(__builtin_fmaf(xs, k.c, -k.rs));
  float g = es * k.ws;
  if (k.ce) g = __builtin_fmaf(k.ce_shared ? es : exp2_fast(__builtin_fmaf(xs, kLog2e, -k.r1)), k.wc, g);
  return g;
}
// with a teacher term e_T = 2^(bt - rt) given by its scaled exponent argument bt = (teacher value) * c
__device__ __forceinline__ float grad_pair_elem(float xs, float bt, const GradCoef& k) {
  const float es = exp2_fast(__builtin_fmaf(xs, k.c, -k.rs));
  float g = __builtin_fmaf(-exp2_fast(bt - k.rt), k.ratio, es) * k.ws;
  if (k.ce) g = __builtin_fmaf(k.ce_shared ? es : exp2_fast(__builtin_fmaf(xs, kLog2e, -k.r1)), k.wc, g);
  return g;
}
__device__ __forceinline__ float grad_dense_elem(float xs, float xt, const GradCoef& k) {
  const float es = exp2_fast(__builtin_fmaf(xs, k.c, -k.rs));
  float g = __builtin_fmaf(-exp2_fast(__builtin_fmaf(xt, k.c, -k.rt)), k.ratio, es) * k.ws;
  if (k.ce) g = __builtin_fmaf(k.ce_shared ? es : exp2_fast(__builtin_fmaf(xs, kLog2e, -k.r1)), k.wc, g);
  return g;
}

// ---- divergences other than the forward KL (dense teacher): reverse KL, skew KL, skew reverse KL
constexpr int kDivReverseKl = 1, kDivSkewKl = 2, kDivSkewReverseKl = 3;  // the values of npd::Divergence

// per-element terms of the skew forms from log2-probabilities; returns u_c, adds this element's share of D
// (in nats) to `dsum` and of ubar to `usum`
// The mixture m is kept away from 0 (both probabilities underflowed), so that neither the logarithm nor the
// reciprocal needs a guard: such an element contributes 0 * finite = 0 everywhere.
template <int DIV>
__device__ __forceinline__ float skew_elem(float lps, float lpt, float alpha, float& dsum, float& usum) {
  const float ps = exp2_fast(lps), pt = exp2_fast(lpt);
  constexpr float kTiny = 1.0e-37f;
  float u;
  if constexpr (DIV == kDivSkewKl) {
    const float m = __builtin_fmaxf(__builtin_fmaf(alpha, pt, (1.0f - alpha) * ps), kTiny);
    dsum = __builtin_fmaf(pt, __builtin_fmaxf(lpt - __log2f(m), -3.0e38f) * kLn2, dsum);  // p_T = 0: no term
    u = (alpha - 1.0f) * pt * __builtin_amdgcn_rcpf(m);
  } else {
    const float m = __builtin_fmaxf(__builtin_fmaf(1.0f - alpha, pt, alpha * ps), kTiny);
    const float l = __builtin_fmaxf(lps - __log2f(m), -3.0e38f) * kLn2;  // p_S = 0: no term, no gradient
    u = __builtin_fmaf(-alpha * ps, __builtin_amdgcn_rcpf(m), l + 1.0f);
    dsum = __builtin_fmaf(ps, l, dsum);
  }
  usum = __builtin_fmaf(ps, u, usum);
  return u;
}

struct DivCoef {
  float c, Ls, Lt;      // log2 normalisers at temperature tau
  float inv_tau, K;     // reverse: u - ubar = (s - t) inv_tau - K
  float alpha, ubar;    // skew forms
  float gscale, cscale;
  float L1;             // log2 normaliser of the student at tau = 1 (CE term when tau != 1)
  bool ce, ce_shared;
};

template <int DIV>
__device__ __forceinline__ float div_grad_elem(float xs, float xt, const DivCoef& k) {
  const float lps = __builtin_fmaf(xs, k.c, -k.Ls);
  const float ps = exp2_fast(lps);
  float w;
  if constexpr (DIV == kDivReverseKl) {
    w = __builtin_fmaf(__builtin_fmaxf(xs - xt, -1.0e30f), k.inv_tau, -k.K);  // p_S = 0: finite times 0
  } else {
    float d = 0.0f, us = 0.0f;
    w = skew_elem<DIV>(lps, __builtin_fmaf(xt, k.c, -k.Lt), k.alpha, d, us) - k.ubar;
  }
  float g = ps * (w * k.gscale);
  if (k.ce) g = __builtin_fmaf(k.ce_shared ? ps : exp2_fast(__builtin_fmaf(xs, kLog2e, -k.L1)), k.cscale, g);
  return g;
}

__device__ __forceinline__ void wave_merge(Lse& v) {
#pragma unroll
  for (int off = kWave / 2; off > 0; off >>= 1) {
    const float r2 = __shfl_xor(v.r, off, kWave);
    const float z2 = __shfl_xor(v.z, off, kWave);
    const float a2 = __shfl_xor(v.a, off, kWave);
    v.merge(r2, z2, a2);
  }
}

__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
  for (int off = kWave / 2; off > 0; off >>= 1) x += __shfl_xor(x, off, kWave);
  return x;
}

__device__ __forceinline__ int wave_sum_int(int x) {
#pragma unroll
  for (int off = kWave / 2; off > 0; off >>= 1) x += __shfl_xor(x, off, kWave);
  return x;
}

// Block-wide merge of N partials; every thread returns with the block totals.
// smem: at least N * 3 * (BLOCK / 64) floats.  Contains two barriers.
template <int BLOCK, int N>
__device__ __forceinline__ void block_merge(Lse (&v)[N], float* smem) {
  constexpr int NW = BLOCK / kWave;
  const int lane = threadIdx.x & (kWave - 1), wid = threadIdx.x / kWave;
#pragma unroll
  for (int i = 0; i < N; ++i) wave_merge(v[i]);
  if constexpr (NW > 1) {
    if (lane == 0) {
#pragma unroll
      for (int i = 0; i < N; ++i) {
        smem[(i * 3 + 0) * NW + wid] = v[i].r;
        smem[(i * 3 + 1) * NW + wid] = v[i].z;
        smem[(i * 3 + 2) * NW + wid] = v[i].a;
      }
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < N; ++i) {
      // every wave folds the NW partials in the same tree: lane l starts from partial l mod NW, a butterfly over
      // log2(NW) steps merges them, and lane 0's result (one fixed order of operations) is what every lane keeps --
      // identical totals everywhere, three LDS reads per lane instead of 3 NW
      Lse t;
      t.r = smem[(i * 3 + 0) * NW + (lane & (NW - 1))];
      t.z = smem[(i * 3 + 1) * NW + (lane & (NW - 1))];
      t.a = smem[(i * 3 + 2) * NW + (lane & (NW - 1))];
#pragma unroll
      for (int off = NW / 2; off > 0; off >>= 1) {
        const float r2 = __shfl_xor(t.r, off, kWave);
        const float z2 = __shfl_xor(t.z, off, kWave);
        const float a2 = __shfl_xor(t.a, off, kWave);
        t.merge(r2, z2, a2);
      }
      v[i].r = __shfl(t.r, 0, kWave);
      v[i].z = __shfl(t.z, 0, kWave);
      v[i].a = __shfl(t.a, 0, kWave);
    }
    __syncthreads();
  } else {
#pragma unroll
    for (int i = 0; i < N; ++i) {  // one wave: every lane takes lane 0's totals
      v[i].r = __shfl(v[i].r, 0, kWave);
      v[i].z = __shfl(v[i].z, 0, kWave);
      v[i].a = __shfl(v[i].a, 0, kWave);
    }
  }
}

template <int BLOCK>
__device__ __forceinline__ float block_sum(float x, float* smem) {
  constexpr int NW = BLOCK / kWave;
  const int lane = threadIdx.x & (kWave - 1), wid = threadIdx.x / kWave;
  x = wave_sum(x);
  if constexpr (NW > 1) {
    if (lane == 0) smem[wid] = x;
    __syncthreads();
    float t = smem[0];
#pragma unroll
    for (int w = 1; w < NW; ++w) t += smem[w];
    __syncthreads();
    x = t;
  }
  return x;
}

template <int BLOCK>
__device__ __forceinline__ int block_sum_int(int x, int* smem) {
  constexpr int NW = BLOCK / kWave;
  const int lane = threadIdx.x & (kWave - 1), wid = threadIdx.x / kWave;
  x = wave_sum_int(x);
  if constexpr (NW > 1) {
    if (lane == 0) smem[wid] = x;
    __syncthreads();
    int t = smem[0];
#pragma unroll
    for (int w = 1; w < NW; ++w) t += smem[w];
    __syncthreads();
    x = t;
  }
  return x;
}

}  // namespace npd
