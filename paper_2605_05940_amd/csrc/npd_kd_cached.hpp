// Row-resident variant of the fused KD loss + gradient kernel (gfx950), for rows of 8,192 entries and more, 16-byte
// aligned: the kernel template and its launcher.  The instantiations are spread over several translation units
// (npd_kd_cached_*.hip) so that they compile in parallel.
//
// One workgroup per token row.  A row of ~150k bf16 logits (student + teacher = 608 KB) does not fit one CU, but most
// of it does: CB threads x CSR 128-bit groups of the student row stay in VGPRs (packed bf16, as loaded), CT groups
// per thread of the teacher row are parked in LDS, and only the remaining groups are read a second time --
// last-read-first, so that many of them still sit in the XCD's L2.  The gradient goes out with non-temporal 128-bit
// stores; loads of groups that stay on chip, and every second read, carry the non-temporal hint so that they do not
// displace what is still to be read again.
//
// Rows of more than 131,072 entries take a CU's whole register file (1024 threads, 128 VGPRs each); shorter rows run
// with 512 or 256 threads, so that a thread still owns 10 .. 19 groups while two or four rows are in flight per CU
// and one row's reductions overlap another row's streaming.
//
// Loads are software-pipelined by hand: group it + D is requested before group it is consumed.  The first CS groups
// per thread are straight-line code (CS is a template parameter), so the compiler can keep several loads in flight;
// groups beyond CS (longer rows) are streamed in sweep 1 and read again in sweep 2.  The arithmetic is the one of
// npd_kd_kernels.hip (same helpers, same merge tree).  The same kernel carries the reverse KL (two sweeps) and the
// skew forms (three sweeps) of the dense-teacher divergences.
#pragma once
#include <atomic>

#include "npd_device.hpp"
#include "npd_internal.hpp"

namespace npd {

constexpr int kCB = 1024;  // threads per workgroup: one workgroup owns a CU's whole register file
constexpr int kGroupBytes = kCB * 16;  // one 128-bit group per thread

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Rows are addressed through buffer resources: the row base and its length live in scalar registers, a
// thread contributes the same tid * 16 for every group and the group offset is a scalar constant, so
// no per-group address registers or 64-bit vector adds are needed.  The hardware drops accesses past the
// end of the row (loads return 0, stores do nothing), but its range check sees only the vector part of
// the offset: the one group that can be ragged (the last of the CS) therefore carries its group offset in
// the vector part (`checked`), all others -- always inside the row -- in the scalar part.
// The resource spans the whole 128-bit groups of a row only: a lane of the ragged group that has no whole
// group left is out of range as a whole (the sub-group tail is handled element-wise).
__device__ __forceinline__ __amdgpu_buffer_rsrc_t row_rsrc(const uint16_t* row, int nvec) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(row), 0, nvec * 16, 0x00020000);
}
// Cache-policy bits of the loads (2 = non-temporal).  Measured on 32,768 x 151,936 (one workgroup per row): the hint
// on loads of groups that stay on chip and on second reads, 4.59 ms against 4.69 ms without; on the first read of a
// group that will be read again it costs 2 % (the second read then misses L2 more often).
constexpr int kNtResident = 2;  // loads of groups that stay on chip (registers or LDS) and are not read again
constexpr int kNtReread = 2;    // the second, last read of a group
// `once`: the group stays on chip after this load (registers or LDS) and is not read again
template <int GB = kGroupBytes>
__device__ __forceinline__ uint4 ld_group(__amdgpu_buffer_rsrc_t r, int voff, int it, bool checked,
                                          bool once = false, bool last = false) {
  u32x4 v;
  if (once && kNtResident)
    v = checked ? __builtin_amdgcn_raw_buffer_load_b128(r, voff + it * GB, 0, kNtResident)
                : __builtin_amdgcn_raw_buffer_load_b128(r, voff, it * GB, kNtResident);
  else if (last && kNtReread)
    v = checked ? __builtin_amdgcn_raw_buffer_load_b128(r, voff + it * GB, 0, kNtReread)
                : __builtin_amdgcn_raw_buffer_load_b128(r, voff, it * GB, kNtReread);
  else
    v = checked ? __builtin_amdgcn_raw_buffer_load_b128(r, voff + it * GB, 0, 0)
                : __builtin_amdgcn_raw_buffer_load_b128(r, voff, it * GB, 0);
  return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ uint4 ld16(const uint16_t* row, int group) {
  return reinterpret_cast<const uint4*>(row)[group];
}
// second (last) read of a group of the streamed part of a row longer than the cache: with the non-temporal hint
// (65,536 x 262,144 in place: 17.1 ms against 17.5 ms without)
__device__ __forceinline__ uint4 ld16_last(const uint16_t* row, int group) {
  const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(row) + group);
  return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void st16_stream(uint16_t* row, int group, const uint4& v) {
  u32x4 w = {v.x, v.y, v.z, v.w};
  __builtin_nontemporal_store(w, reinterpret_cast<u32x4*>(row) + group);
}

// Hides where a value came from: without it the compiler keeps sweep 1's unpacked fp32 copies of the
// cached row alive for sweep 2 (and spills them) instead of unpacking the packed registers again.
__device__ __forceinline__ void opaque(uint4& v) {
  asm volatile("" : "+v"(v.x), "+v"(v.y), "+v"(v.z), "+v"(v.w));
}

// Sweep-2 coefficients.  Precise form: see GradCoef.  Folded form: the weights go into the exponents,
//   grad = +-(2^(x c - fs) - 2^(x c - ft)),   fs = r_S + log2(z_S / |A|),  ft = r_T + log2(z_T / |B|),
// with A = grad_scale / tau + ce_grad_scale (weight of p_S; the CE softmax shares e_S, so tau = 1 whenever
// ce_grad_scale != 0 here) and B = grad_scale / tau (weight of p_T): one instruction less per element.  It is used
// only while A and B do not differ in sign and |fs|, |ft| < 1024, where rounding fs, ft to fp32 moves a probability
// by less than 2.2e-5 of itself (rows with logits in the thousands take the precise form).
struct Sweep2Coef {
  GradCoef p;     // precise form
  float c, fs, ft;
  uint32_t sign;  // 0x80008000 when the weights are negative (folded form)
  bool folded;    // uniform
  // reverse KL (and its CE term at tau = 1): grad = 2^(x_s c - r_S) ((x_s - x_t) ra + rb),
  //   ra = grad_scale / (tau^2 z_S),  rb = (ce_grad_scale - grad_scale / tau (lse_S - lse_T + D)) / z_S
  float ra, rb;
  DivCoef dv;  // skew forms
};

// An entry of probability 0 in the student (-inf, with the teacher at -inf or finite) has no gradient: the
// difference is kept finite so that the product with e_S = 0 is 0 and not NaN.
__device__ __forceinline__ float grad_reverse_elem(float xs, float xt, const Sweep2Coef& k) {
  return exp2_fast(__builtin_fmaf(xs, k.c, -k.p.rs)) * __builtin_fmaf(__builtin_fmaxf(xs - xt, -1.0e30f), k.ra, k.rb);
}

__device__ __forceinline__ Sweep2Coef sweep2_coef(const Lse& S, const Lse& Tt, float c, float gscale, float cscale,
                                                  bool has_teacher_stream, bool dense) {
  Sweep2Coef k;
  k.p = make_grad_coef(S, Tt, S, c, gscale, cscale, has_teacher_stream, false);
  k.c = c;
  const float A = gscale + cscale, B = dense ? gscale : 0.0f;
  // log2(0) = -inf: the term becomes 2^-inf = 0
  k.fs = S.r + (S.log2_z() - __log2f(fabsf(A)));
  k.ft = dense ? Tt.r + (Tt.log2_z() - __log2f(fabsf(B))) : 0.0f;
  k.sign = (A < 0.0f || B < 0.0f) ? 0x80008000u : 0u;
  const bool same_sign = (A >= 0.0f && B >= 0.0f) || (A <= 0.0f && B <= 0.0f);
  const bool small_s = A == 0.0f || fabsf(k.fs) < 1024.0f;
  const bool small_t = !dense || B == 0.0f || fabsf(k.ft) < 1024.0f;
  k.folded = same_sign && small_s && small_t;
  k.ra = k.rb = 0.0f;
  return k;
}

// gradient of 8 elements
template <int TEACHER, bool FOLDED, int DIVK = kForwardKl>
__device__ __forceinline__ uint4 grad8(const uint4& vs, const uint4& vt, const Sweep2Coef& k) {
  float xs[8], gv[8];
  unpack8(vs, xs);
  if constexpr (DIVK == kReverseKl) {
    float xt[8];
    unpack8(vt, xt);
#pragma unroll
    for (int j = 0; j < 8; ++j) gv[j] = grad_reverse_elem(xs[j], xt[j], k);
  } else if constexpr (DIVK != kForwardKl) {
    float xt[8];
    unpack8(vt, xt);
#pragma unroll
    for (int j = 0; j < 8; ++j) gv[j] = div_grad_elem<DIVK>(xs[j], xt[j], k.dv);
  } else if constexpr (TEACHER == kDense) {
    float xt[8];
    unpack8(vt, xt);
    if constexpr (FOLDED) {
#pragma unroll
      for (int j = 0; j < 8; ++j)
        gv[j] = exp2_fast(__builtin_fmaf(xs[j], k.c, -k.fs)) - exp2_fast(__builtin_fmaf(xt[j], k.c, -k.ft));
    } else {
#pragma unroll
      for (int j = 0; j < 8; ++j) gv[j] = grad_dense_elem(xs[j], xt[j], k.p);
    }
  } else {
    if constexpr (FOLDED) {
#pragma unroll
      for (int j = 0; j < 8; ++j) gv[j] = exp2_fast(__builtin_fmaf(xs[j], k.c, -k.fs));
    } else {
#pragma unroll
      for (int j = 0; j < 8; ++j) gv[j] = grad_student_elem(xs[j], k.p);
    }
  }
  uint4 o;
  o.x = pack_bf16(gv[0], gv[1]);
  o.y = pack_bf16(gv[2], gv[3]);
  o.z = pack_bf16(gv[4], gv[5]);
  o.w = pack_bf16(gv[6], gv[7]);
  if constexpr (FOLDED && DIVK == kForwardKl) {
    o.x ^= k.sign;
    o.y ^= k.sign;
    o.z ^= k.sign;
    o.w ^= k.sign;
  }
  return o;
}

// sweep-1 contribution of 8 elements
template <int TEACHER, bool LSE1, bool REV = false>
__device__ __forceinline__ void accum8(const uint4& vs, const uint4& vt, float c, bool lse1_t,
                                       Lse (&acc)[LSE1 ? 4 : 2]) {
  float xs[8];
  unpack8(vs, xs);
  if constexpr (TEACHER == kDense) {
    float xt[8];
    unpack8(vt, xt);
    if constexpr (REV) {  // reverse KL: the cross term sum e_S (s - t) rides on the student stream
      acc[1].add8(xt, c);
      acc[0].add8_cross(xs, xt, c);
    } else {
      acc[1].add8_cross(xt, xs, c);
    }
    if constexpr (LSE1)
      if (lse1_t) acc[3].add8(xt, kLog2e);
  }
  if constexpr (!REV) acc[0].add8(xs, c);
  if constexpr (LSE1) acc[2].add8(xs, kLog2e);
}

// CB = threads per workgroup (1024, or 512 / 256 for shorter rows, so that a thread still holds 10 .. 19 groups and
// several rows are in flight per CU).  SHORT: the row may have fewer than CS groups per thread; every group is then
// range-checked by the buffer hardware and by a per-thread bound on its use.
template <int CS, int CSR, int CT, int D, int TEACHER, bool GRAD, bool LSE1, int DIVK = kForwardKl, int CB = kCB,
          bool SHORT = false>
__global__ __launch_bounds__(CB, 4) void kd_cached_kernel(const KdArgs a) {
  constexpr int GB = CB * 16;
  static_assert(DIVK == kForwardKl || (TEACHER == kDense && GRAD), "the other divergences need the full teacher row");
  constexpr bool REV = DIVK == kReverseKl;
  constexpr bool SKEW = DIVK == kSkewKl || DIVK == kSkewReverseKl;  // three sweeps: normalisers, D and ubar, gradient
  // groups parked for sweep 2, [CB][LS]: a thread's groups are contiguous, so one base register plus an immediate
  // offset addresses them all
  extern __shared__ uint4 lds_t[];
  __shared__ float red[4 * 3 * (CB / kWave)];
  __shared__ uint16_t patch[TEACHER == kTopk && GRAD ? kTopkMax : 1];
  __shared__ int y_in_support;  // top-k teacher: the label is one of the k support positions of this row
  static_assert(CT <= CS && CSR <= CS && D >= 1 && D <= CS, "bad cache shape");
  // a thread's parked groups are LS * 16 bytes apart from its neighbour's: an odd LS keeps 128-bit accesses
  // conflict-free
  constexpr int LS = CT | 1;
  // without a dense teacher the LDS parks student groups instead: groups CSR .. CSR + SL - 1
  constexpr int SL = TEACHER == kDense ? 0 : (CT < CS - CSR ? CT : CS - CSR);
  const int tid = threadIdx.x;
  const int voff = tid * 16;
  const int V = a.V, nvec = a.nvec_s;  // only launched with 16-byte aligned rows: nvec = V / 8
  const float c = a.c;
  const bool lse1_t = LSE1 && a.tnll != nullptr;
  // without SHORT: launched only for rows of more than (CS - 1) * CB groups, so every one of the first CS groups
  // per thread is full except, when the row has at most CS * CB groups, the last one
  const int nit = (nvec + CB - 1) / CB;  // 128-bit groups per thread

  // One workgroup per row.  A row that is not scored: scalars 0, gradient row zero-filled, logits never read.
  const int64_t row = blockIdx.x;
  if (!a.mask[row]) {
    if (tid == 0) {
      if (a.kd) a.kd[row] = 0.0f;
      if (a.nll) a.nll[row] = 0.0f;
      if (a.tnll) a.tnll[row] = 0.0f;
      if (a.lse) a.lse[row] = 0.0f;
    }
    if constexpr (GRAD) {
      uint16_t* grow0 = a.g + row * a.s_stride;
      const uint4 z = make_uint4(0, 0, 0, 0);
      for (int i = tid; i < nvec; i += CB) st16_stream(grow0, i, z);
      for (int e = nvec * 8 + tid; e < V; e += CB) grow0[e] = 0;
    }
    return;
  }

  uint4 sreg[CSR > 0 ? CSR : 1];  // the first CSR groups of the student row, as loaded (packed bf16)
  uint4 sst[D], tst[D];           // student groups beyond CSR / teacher groups in flight
  auto request_student = [&](__amdgpu_buffer_rsrc_t rs) {
#pragma unroll
    for (int it = 0; it < CSR; ++it) sreg[it] = ld_group<GB>(rs, voff, it, SHORT || (it) == CS - 1, true);
  };

  {
    const uint16_t* srow = a.s + row * a.s_stride;
    const uint16_t* trow = TEACHER == kDense ? a.t + row * a.t_stride : nullptr;
    uint16_t* grow = GRAD ? a.g + row * a.s_stride : nullptr;
    const __amdgpu_buffer_rsrc_t rs = row_rsrc(srow, nvec);
    const __amdgpu_buffer_rsrc_t rt = row_rsrc(TEACHER == kDense ? trow : srow, nvec);

    int y = -1;
    float s_y = 0.0f, t_y = 0.0f;
    if (a.labels) {  // label logits are fetched before an in-place gradient can overwrite them
      y = a.labels[row];
      if ((unsigned)y < (unsigned)V) {
        s_y = bf16_one(srow[y]);
        if (TEACHER == kDense) t_y = bf16_one(trow[y]);
      }
    }

    constexpr int NS = LSE1 ? 4 : 2;  // 0 student / tau, 1 teacher / tau (+ cross), 2 student tau = 1, 3 teacher tau = 1
    Lse acc[NS];
#pragma unroll
    for (int i = 0; i < NS; ++i) acc[i].init();

    // ---- sweep 1, first CS groups per thread: the register-resident student groups are requested first; the
    // other student groups and the teacher groups are requested D ahead of their use
    request_student(rs);
#pragma unroll
    for (int d = 0; d < D; ++d) {
      if constexpr (TEACHER == kDense) tst[d] = ld_group<GB>(rt, voff, d, SHORT || (d) == CS - 1, GRAD ? d < CT : true);
      if (d >= CSR) sst[d] = ld_group<GB>(rs, voff, d, SHORT || (d) == CS - 1, !GRAD || d < CSR + SL);
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int it = 0; it < CS; ++it) {
      const uint4 vs = it < CSR ? sreg[it < CSR ? it : 0] : sst[it % D];
      const uint4 vt = TEACHER == kDense ? tst[it % D] : make_uint4(0, 0, 0, 0);
      if (it + D < CS) {
        if constexpr (TEACHER == kDense)
          tst[it % D] = ld_group<GB>(rt, voff, it + D, SHORT || (it + D) == CS - 1, GRAD ? it + D < CT : true);
        if (it + D >= CSR) sst[it % D] = ld_group<GB>(rs, voff, it + D, SHORT || (it + D) == CS - 1, !GRAD || it + D < CSR + SL);
      }
      if ((!SHORT && it < CS - 1) || it * CB + tid < nvec) accum8<TEACHER, LSE1, REV>(vs, vt, c, lse1_t, acc);
      if constexpr (TEACHER == kDense)
        if (it < CT) lds_t[tid * LS + it] = vt;
      if constexpr (SL > 0)
        if (it >= CSR && it < CSR + SL) lds_t[tid * LS + (it - CSR)] = vs;
      __builtin_amdgcn_sched_barrier(0);  // keep the instruction scheduler from piling all loads up front
    }
    // ---- sweep 1, streamed part (rows longer than the cache) and the sub-group tail
    for (int i = CS * CB + tid; i < nvec; i += CB) {
      const uint4 vs = ld16(srow, i);
      const uint4 vt = TEACHER == kDense ? ld16(trow, i) : make_uint4(0, 0, 0, 0);
      accum8<TEACHER, LSE1, REV>(vs, vt, c, lse1_t, acc);
    }
    for (int e = nvec * 8 + tid; e < V; e += CB) {
      const float xs = bf16_one(srow[e]);
      if constexpr (TEACHER == kDense) {
        const float xt = bf16_one(trow[e]);
        if constexpr (REV) {
          acc[1].add1(xt, c);
          acc[0].add1_cross(xs, xs - xt, c);
        } else {
          acc[1].add1_cross(xt, xt - xs, c);
        }
        if constexpr (LSE1)
          if (lse1_t) acc[3].add1(xt, kLog2e);
      }
      if constexpr (!REV) acc[0].add1(xs, c);
      if constexpr (LSE1) acc[2].add1(xs, kLog2e);
    }
    int bad_index = 0;
    if constexpr (TEACHER == kTopk) {
      const int32_t* irow = a.tidx + row * (int64_t)a.k;
      const float* vrow = a.tval + row * (int64_t)a.k;
      for (int j = tid; j < a.k; j += CB) {
        if ((unsigned)irow[j] >= (unsigned)V) bad_index = 1;
        acc[1].add1(vrow[j], c);
      }
    }

    // groups that are neither in registers nor in LDS are requested a second time, newest first (they are
    // still in cache); the first D of them travel while the partial sums are merged
    auto request_again = [&](bool last) {
#pragma unroll
      for (int d = 0; d < D; ++d) {
        const int it = CS - 1 - d;
        if (TEACHER == kDense && it >= CT) tst[d] = ld_group<GB>(rt, voff, it, SHORT || (it) == CS - 1, false, last);
        if (it >= CSR + SL) sst[d] = ld_group<GB>(rs, voff, it, SHORT || (it) == CS - 1, false, last);
      }
    };
    // one backward walk over the first CS groups per thread: on-chip groups from where they are, the others from
    // the D-deep ring that request_again() primed; f(it, vs, vt) consumes a group
    auto walk_back = [&](auto&& f, bool last) {
      // a second walk must fetch the parked groups from LDS again rather than keep the first walk's copies (and
      // everything derived from them) alive in registers
      if constexpr (SKEW) asm volatile("" ::: "memory");
#pragma unroll
      for (int q = 0; q < CS; ++q) {
        const int it = CS - 1 - q;
        uint4 vs, vt = make_uint4(0, 0, 0, 0);
        if (it < CSR) {
          opaque(sreg[it < CSR ? it : 0]);
          vs = sreg[it < CSR ? it : 0];
        } else if (it < CSR + SL) {
          vs = lds_t[tid * LS + (it - CSR)];
        } else {
          vs = sst[q % D];  // requested D visits ago
          if (it - D >= CSR + SL) sst[q % D] = ld_group<GB>(rs, voff, it - D, SHORT || (it - D) == CS - 1, false, last);
        }
        if constexpr (TEACHER == kDense) {
          if (it < CT) {
            vt = lds_t[tid * LS + it];
          } else {
            vt = tst[q % D];
            if (it - D >= CT) tst[q % D] = ld_group<GB>(rt, voff, it - D, SHORT || (it - D) == CS - 1, false, last);
          }
        }
        f(it, vs, vt);
        __builtin_amdgcn_sched_barrier(0);
      }
    };
    if constexpr (GRAD) request_again(!SKEW);

    block_merge<CB, NS>(acc, red);

    const float Ls = acc[0].log2_sum();
    const float Lt = TEACHER == kNone ? 0.0f : acc[1].log2_sum();
    const float lse1_s = __fmul_rn(LSE1 ? acc[NS - 2].log2_sum() : Ls, kLn2);
    float kd = 0.0f;
    float lse_diff = 0.0f;  // lse_S - lse_T at temperature tau
    if constexpr (TEACHER == kDense) {
      lse_diff = ((acc[0].r - acc[1].r) + (acc[0].log2_z() - acc[1].log2_z())) * kLn2;
      kd = REV ? (acc[0].a / acc[0].z) * a.inv_tau - lse_diff : (acc[1].a / acc[1].z) * a.inv_tau + lse_diff;
      kd = kd < 0.0f ? 0.0f : kd;  // (the skew forms replace it below)
    }
    const bool ce = GRAD && a.cscale != 0.0f;                       // uniform (tau = 1 here whenever it is set)
    const bool bad_label = a.labels && (unsigned)y >= (unsigned)V;  // uniform
    Sweep2Coef k = sweep2_coef(acc[0], acc[1], c, a.gscale, a.cscale, TEACHER != kNone, TEACHER == kDense);
    if constexpr (REV) {
      const float inv_z = 1.0f / acc[0].z;
      k.ra = a.gscale * a.inv_tau * inv_z;
      k.rb = (a.cscale - a.gscale * (lse_diff + kd)) * inv_z;
      k.folded = true;  // one form for all rows: the exponent is taken against the row's reference as in sweep 1
    }
    if constexpr (SKEW) {
      k.dv.c = c;
      k.dv.Ls = Ls;
      k.dv.Lt = Lt;
      k.dv.inv_tau = a.inv_tau;
      k.dv.K = 0.0f;
      k.dv.alpha = a.alpha;
      k.dv.gscale = a.gscale;
      k.dv.cscale = a.cscale;
      k.dv.L1 = Ls;
      k.dv.ce = ce;
      k.dv.ce_shared = true;  // tau = 1 whenever the CE term is present on this path
      k.folded = true;
      // ---- sweep 2 of the skew forms: D and ubar over normalised probabilities; same walk as the gradient sweep
      float dsum = 0.0f, usum = 0.0f;
      auto accum = [&](const uint4& vs, const uint4& vt) {
        float xs[8], xt[8];
        unpack8(vs, xs);
        unpack8(vt, xt);
#pragma unroll
        for (int j = 0; j < 8; ++j)
          skew_elem<DIVK>(__builtin_fmaf(xs[j], c, -Ls), __builtin_fmaf(xt[j], c, -Lt), a.alpha, dsum, usum);
        // both running sums are due here: otherwise the compiler sinks one chain below the whole walk and keeps
        // every element's probabilities alive for it (in scratch memory)
        asm volatile("" : "+v"(dsum), "+v"(usum));
      };
      for (int e = nvec * 8 + tid; e < V; e += CB)
        skew_elem<DIVK>(__builtin_fmaf(bf16_one(srow[e]), c, -Ls), __builtin_fmaf(bf16_one(trow[e]), c, -Lt), a.alpha,
                        dsum, usum);
      for (int i = (nit - 1) * CB + tid; i >= CS * CB; i -= CB)
        if (i < nvec) accum(ld16(srow, i), ld16(trow, i));
      walk_back([&](int it, const uint4& vs, const uint4& vt) {
        if ((!SHORT && it < CS - 1) || it * CB + tid < nvec) accum(vs, vt);
      }, false);
      request_again(true);  // travels while the two sums are merged
      kd = block_sum<CB>(dsum, red);
      kd = kd < 0.0f ? 0.0f : kd;
      k.dv.ubar = block_sum<CB>(usum, red);
    }
    if constexpr (TEACHER == kTopk) {
      bad_index = __syncthreads_or(bad_index);
      if (tid == 0) y_in_support = 0;
      __syncthreads();
      const int32_t* irow = a.tidx + row * (int64_t)a.k;
      const float* vrow = a.tval + row * (int64_t)a.k;
      float part = 0.0f;
      if (!bad_index) {
        for (int j = tid; j < a.k; j += CB) {
          const float b = vrow[j] * c;
          const float sj = bf16_one(srow[irow[j]]);
          const float lpt = b - Lt;
          const float lps = __builtin_fmaf(sj, c, -Ls);
          part = __builtin_fmaf(exp2_fast(lpt), __builtin_fmaxf(lpt - lps, -3.4028234663852886e38f) * kLn2, part);  // a -inf entry: 0
          if constexpr (GRAD) {
            float gj = grad_pair_elem(sj, b, k.p);
            if (ce && irow[j] == y) {
              gj -= a.cscale;
              y_in_support = 1;
            }
            patch[j] = one_bf16(gj);
          }
        }
      }
      kd = block_sum<CB>(part, red);
      kd = kd < 0.0f ? 0.0f : kd;
      if (bad_index) kd = __builtin_nanf("");
    }

    if (tid == 0) {
      int flags = 0;
      if (bad_index) flags |= 2;
      if (bad_label && (a.nll || a.tnll || ce)) flags |= 1;
      if (a.kd) a.kd[row] = kd;
      if (a.nll) a.nll[row] = bad_label ? __builtin_nanf("") : __fsub_rn(lse1_s, s_y);
      if (TEACHER == kDense && a.tnll) {
        const float lse1_tt = __fmul_rn(LSE1 ? acc[NS - 1].log2_sum() : Lt, kLn2);
        a.tnll[row] = bad_label ? __builtin_nanf("") : __fsub_rn(lse1_tt, t_y);
      }
      if (a.lse) a.lse[row] = lse1_s;
      if (flags && a.status) atomicOr(a.status, flags);
    }

    // ---- sweep 2
    if constexpr (GRAD) {
      if ((TEACHER == kTopk && bad_index) || (ce && bad_label)) {  // uniform: the row cannot be differentiated
        const uint16_t qnan = 0x7fc0;
        for (int e = tid; e < V; e += CB) grow[e] = qnan;
      } else {
        // sub-group tail and streamed part first (read most recently), then the first CS groups backwards
        for (int e = nvec * 8 + tid; e < V; e += CB) {
          const float xs = bf16_one(srow[e]);
          if constexpr (REV)
            grow[e] = one_bf16(grad_reverse_elem(xs, bf16_one(trow[e]), k));
          else if constexpr (SKEW)
            grow[e] = one_bf16(div_grad_elem<DIVK>(xs, bf16_one(trow[e]), k.dv));
          else
            grow[e] = one_bf16(TEACHER == kDense ? grad_dense_elem(xs, bf16_one(trow[e]), k.p)
                                                 : grad_student_elem(xs, k.p));
        }
        for (int i = (nit - 1) * CB + tid; i >= CS * CB; i -= CB) {
          if (i < nvec) {
            const uint4 vs = ld16_last(srow, i);
            const uint4 vt = TEACHER == kDense ? ld16_last(trow, i) : make_uint4(0, 0, 0, 0);
            st16_stream(grow, i, grad8<TEACHER, false, DIVK>(vs, vt, k));
          }
        }
        if (k.folded) {  // uniform
          if constexpr (SKEW) asm volatile("" ::: "memory");  // see walk_back
#pragma unroll
          for (int q = 0; q < CS; ++q) {  // the same walk as walk_back, spelled out (register allocation differs)
            const int it = CS - 1 - q;
            uint4 vs, vt = make_uint4(0, 0, 0, 0);
            if (it < CSR) {
              opaque(sreg[it < CSR ? it : 0]);
              vs = sreg[it < CSR ? it : 0];
            } else if (it < CSR + SL) {
              vs = lds_t[tid * LS + (it - CSR)];
            } else {
              vs = sst[q % D];  // requested D visits ago
              if (it - D >= CSR + SL) sst[q % D] = ld_group<GB>(rs, voff, it - D, SHORT || (it - D) == CS - 1, false, true);
            }
            if constexpr (TEACHER == kDense) {
              if (it < CT) {
                vt = lds_t[tid * LS + it];
              } else {
                vt = tst[q % D];
                if (it - D >= CT) tst[q % D] = ld_group<GB>(rt, voff, it - D, SHORT || (it - D) == CS - 1, false, true);
              }
            }
            {
              const uint4 gq = grad8<TEACHER, true, DIVK>(vs, vt, k);
              if ((!SHORT && it < CS - 1) || it * CB + tid < nvec) st16_stream(grow, it * CB + tid, gq);
            }
            __builtin_amdgcn_sched_barrier(0);
          }
        } else {
          // rows whose reference exponents are in the thousands: precise form, plain loop over the row
          for (int i = (nit < CS ? nit : CS) * CB - CB + tid; i >= 0; i -= CB) {
            if (i < nvec) {
              const uint4 vs = ld16(srow, i);
              const uint4 vt = TEACHER == kDense ? ld16(trow, i) : make_uint4(0, 0, 0, 0);
              st16_stream(grow, i, grad8<TEACHER, false, DIVK>(vs, vt, k));
            }
          }
        }
        if (TEACHER == kTopk || ce) {  // uniform
          // the k support positions and the label position get their final values once the dense stores of the
          // whole workgroup are ordered before them
          __syncthreads();
          if constexpr (TEACHER == kTopk) {
            const int32_t* irow = a.tidx + row * (int64_t)a.k;
            for (int j = tid; j < a.k; j += CB) grow[irow[j]] = patch[j];
          }
          if (ce && tid == 0 && !(TEACHER == kTopk && y_in_support)) {
            float gy;
            if constexpr (REV)
              gy = grad_reverse_elem(s_y, t_y, k);
            else if constexpr (SKEW)
              gy = div_grad_elem<DIVK>(s_y, t_y, k.dv);
            else
              gy = TEACHER == kDense ? grad_dense_elem(s_y, t_y, k.p) : grad_student_elem(s_y, k.p);
            grow[y] = one_bf16(gy - a.cscale);
          }
        }
      }
    }
  }
}

template <int CS, int CSR, int CT, int D, int TEACHER, bool GRAD, int DIVK = kForwardKl, int CB = kCB, bool SHORT = false>
static hipError_t launch_cached_lse1(const KdArgs& a, hipStream_t stream) {
  constexpr size_t lds_bytes = CT > 0 ? (size_t)(CT | 1) * CB * sizeof(uint4) : 0;
  auto launch = [&](auto kernel) -> hipError_t {
    if (lds_bytes > 0) {
      // more than the default 64 KB of dynamic LDS has to be asked for, once per kernel and device
      static std::atomic<uint64_t> asked[1];  // bit d: done on device d (devices beyond 63 ask every time)
      int dev = 0;
      if (hipGetDevice(&dev) != hipSuccess) dev = 64;
      if (dev < 0 || dev >= 64 || !((asked[0].load(std::memory_order_acquire) >> dev) & 1u)) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (e != hipSuccess) return e;
        if (dev >= 0 && dev < 64) asked[0].fetch_or(uint64_t(1) << dev, std::memory_order_release);
      }
    }
    return launch_kernel(kernel, dim3((unsigned)a.T), dim3(CB), lds_bytes, stream, a);
  };
  if (a.need_lse1) return launch(kd_cached_kernel<CS, CSR, CT, D, TEACHER, GRAD, true, DIVK, CB, SHORT>);
  return launch(kd_cached_kernel<CS, CSR, CT, D, TEACHER, GRAD, false, DIVK, CB, SHORT>);
}

// Shape of the dense-teacher gradient kernels (measured on MI355X, 32,768 x 151,936): how many student groups per
// thread stay in registers and how far ahead teacher / non-resident student groups are requested.  Times are flat
// (+-2 %) for 8..16 resident groups; 12 leaves the register allocator enough room to avoid spills, whose reloads
// would stall the load pipeline.
constexpr int kResidentGroups = 12;
constexpr int kResidentGroupsForward = 16;  // forward KL with 1024 threads: 4.53 ms with 12 resident groups, 4.48 ms with 16
constexpr int kResidentGroupsTopk = 12;
constexpr int kAhead = 2;
}  // namespace npd
