// Row-gang variant of the fused KD loss + gradient kernel (gfx950): a token row is shared by G short-lived
// workgroups of 256 threads, each of which owns one contiguous slice of the row (up to K 128-bit groups per thread
// and tensor) and keeps it in registers from the first sweep to the gradient write -- nothing is read twice, whatever
// the vocabulary.  The G partial log-sum-exps of a row meet through a small scratch record in device memory:
//
//   sweep 1 over the slice -> workgroup partials (r, z, a) -> posted to scratch[row][slice]
//   wait until all G slices of the row have posted -> merge them in one fixed tree (every workgroup of the row
//   computes bit-identical row totals) -> gradient of the slice from the registers -> written once
//
// Why: the memory system of this GPU gives a mix of two reads and one write 6.7 TB/s when the chip sweeps memory
// front to back, every row is read completely before it is written and no cache line is shared by two workgroups,
// against 5.7 TB/s when each compute unit works on a row of its own.  Consecutive workgroups are consecutive slices
// (which begin on 128-byte boundaries of the row), four workgroups run per compute unit (one row's wait and arithmetic
// overlap three other slices' memory traffic), and the workgroups of rows that are not scored zero-fill their slices
// in the same address order.
//
// The exchange needs no fence: every posted word is a 32-bit atomic store that carries its own validity (the
// scratch record is cleared to a pattern no posted word takes, by a fill kernel enqueued in front of each launch),
// and consumers poll those words with atomic loads at device scope.  Forward progress: a workgroup waits only for
// workgroups of smaller or neighbouring index (the other slices of its own row), a workgroup never waits before it
// has posted, and workgroups start in index order, so the lowest unfinished row always has all its workgroups
// resident or next to start.  Every wait is bounded all the same: a workgroup that gives up marks its row NaN, sets
// NPD_DEV_GANG_TIMEOUT and raises a launch-wide flag that ends every other wait of the launch early, so a kernel can
// never hang, nor spend one limit per row.
#pragma once
#include "npd_kd_cached.hpp"

namespace npd {

constexpr int kGangThreads = 256;
constexpr int kGangMax = 32;                      // slices per row at most
constexpr uint32_t kGangEmpty = 0xffffffffu;      // scratch word not posted yet (a NaN pattern no partial is stored as)
constexpr int kGangSpinLimitDefault = 1 << 20;    // polls before a workgroup gives up (seconds; never reached in a healthy run)

// ---- merging partial log-sum-exps: largest reference first, every partial rescaled to it once, then plain sums.
// Cross-lane steps are DPP operands of the adds and maxima (no LDS traffic, no address arithmetic); the order of operations is
// fixed, so results are bitwise reproducible and two streams fed the same data stay bitwise identical.
__device__ __forceinline__ float lane63(float x) {
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x), 63));
}
// Sum / maximum over the 64 lanes, every lane gets the result: pairs, quads, half rows, rows of 16, then lane 15 of
// rows 0 / 2 into rows 1 / 3 and lane 31 into rows 2 and 3, so that lane 63 holds everything.  Each step is one
// instruction whose first operand is read through DPP (lanes that a row mask leaves out keep their value); written out
// because the compiler spends four instructions per step on the maximum.  A DPP operand must not be read within two
// wait states of the instruction that wrote it: hence the s_nop in front of every step.
#define NPD_DPP_REDUCE(op)                                                  \
  "s_nop 4\n" op " %0, %0, %0 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n" \
  "s_nop 1\n" op " %0, %0, %0 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n" \
  "s_nop 1\n" op " %0, %0, %0 row_half_mirror row_mask:0xf bank_mask:0xf\n"     \
  "s_nop 1\n" op " %0, %0, %0 row_mirror row_mask:0xf bank_mask:0xf\n"          \
  "s_nop 1\n" op " %0, %0, %0 row_bcast:15 row_mask:0xa bank_mask:0xf\n"        \
  "s_nop 1\n" op " %0, %0, %0 row_bcast:31 row_mask:0xc bank_mask:0xf\n"        \
  "s_nop 1\n"
__device__ __forceinline__ float wave_sum_dpp(float x) {
  asm volatile(NPD_DPP_REDUCE("v_add_f32_dpp") : "+v"(x));
  return lane63(x);
}
__device__ __forceinline__ float wave_max_dpp(float x) {
  asm volatile(NPD_DPP_REDUCE("v_max_f32_dpp") : "+v"(x));
  return lane63(x);
}
// merges the 64 lanes' partials (sum = z 2^r, cross term a 2^r); every lane returns with the total
template <bool CROSS>
__device__ __forceinline__ void wave_merge_rescaled(Lse& v) {
  const float R = wave_max_dpp(v.r);
  const float f = exp2_fast(v.r - R);  // exactly 1 where r == R; 0 for empty partials far below
  v.z = wave_sum_dpp(__fmul_rn(v.z, f));
  if constexpr (CROSS) v.a = wave_sum_dpp(__fmul_rn(v.a, f));
  v.r = R;
}
// a lane's partial with its sum brought into [1, 2): r takes up the exponent of z, so that later rescaling to a
// larger reference can only shrink values (z may be anywhere below 2^100 when the reference was a guess)
__device__ __forceinline__ void normalise(Lse& v) {
  const int e = (int)((__builtin_bit_cast(uint32_t, v.z) >> 23) & 0xffu) - 127;
  if (v.z > 0.0f && e > -127 && e < 128) {  // normal, positive (zero, NaN and infinity stay as they are)
    const float down = __builtin_bit_cast(float, (uint32_t)(127 - e) << 23);  // 2^-e
    v.z = __fmul_rn(v.z, down);
    v.a = __fmul_rn(v.a, down);
    v.r += (float)e;
  }
}

// Largest of the eight bf16 values packed in a group, as a float -- by packed 16-bit integer maxima on the bit
// patterns, which order non-negative values correctly and put every negative value below them.  Among negative
// values alone the integer order is the reverse of the value order, so for a group whose logits are all negative the
// result is its smallest logit: still a usable reference exponent (lower by the spread of the group), and the
// caller's check of the sums catches the case where that is not enough.
typedef short s16x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pk_max_i16(uint32_t a, uint32_t b) {
  return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(s16x2, a), __builtin_bit_cast(s16x2, b)));
}
__device__ __forceinline__ uint32_t pk_max_group(const uint4& v) { return pk_max_i16(pk_max_i16(v.x, v.y), pk_max_i16(v.z, v.w)); }
__device__ __forceinline__ float pk_max_value(uint32_t m) {
  const int lo = (int)(short)(m & 0xffffu), hi = (int)(short)(m >> 16);
  return bf16_one((uint16_t)(lo > hi ? lo : hi));
}

__device__ __forceinline__ void gang_post(uint32_t* p, float v) {
  uint32_t w = __builtin_bit_cast(uint32_t, v);
  if (w == kGangEmpty) w = 0x7fc00000u;  // another NaN
  __hip_atomic_store(p, w, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Waits for a posted word.  Gives up after `spin_limit` polls, or -- looked at every 256th poll -- as soon as any
// workgroup of the launch has given up (the word *abandon, cleared with the record): once one wait has run out, no
// other workgroup spends its own limit, so a launch whose workgroups cannot see each other ends within seconds
// however many rows it has.  Returns the word, or kGangEmpty with *gave_up set.
constexpr int kGangTailWords = 64;  // words behind the record; word 0: a workgroup has given up
__device__ __forceinline__ uint32_t gang_wait(const uint32_t* p, uint32_t* abandon, int spin_limit, int* gave_up) {
  int spins = 0;
  while (true) {
    const uint32_t v = __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (v != kGangEmpty) return v;
    ++spins;
    if (spins > spin_limit) {
      __hip_atomic_store(abandon, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      *gave_up = 1;
      return v;
    }
    if ((spins & 255) == 0 && __hip_atomic_load(abandon, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 1u) {
      *gave_up = 1;
      return v;
    }
    __builtin_amdgcn_s_sleep(8);
  }
}

// words of scratch per slice: 3 per partial log-sum-exp, rounded up to a power of two
__host__ __device__ constexpr int gang_words(int ns) { return ns == 2 ? 8 : 16; }

// Runs in front of every launch of a row-gang kernel: clears the scratch record (and the words behind it) to the
// pattern no posted word takes.
__global__ __launch_bounds__(256) void gang_clear_kernel(uint32_t* ws, size_t words) {
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < words; i += (size_t)gridDim.x * 256) ws[i] = kGangEmpty;
}

// Zero-fills the groups [g0, g0 + ng) of a gradient row, ng <= K * 256: what the workgroup of a slice does when its
// row is not scored.  With slices that begin on 128-byte boundaries these short-lived workgroups, started in address
// order among those of the scored rows, fill as fast as a separate fill pass (and save that pass).
template <int K>
__device__ __forceinline__ void gang_zero_slice(uint16_t* grow, int g0, int ng, int tid) {
  const u32x4 z = {0, 0, 0, 0};
  u32x4* p = reinterpret_cast<u32x4*>(grow) + g0;
#pragma unroll
  for (int k = 0; k < K; ++k)
    if (k * kGangThreads + tid < ng) __builtin_nontemporal_store(z, p + k * kGangThreads + tid);
}

// ---- the skew divergences (three sweeps): sums and gradient on normalised log2-probabilities.
//   skew KL          D = KL(p_T || m),  m = alpha p_T + (1 - alpha) p_S,  u = (alpha - 1) p_T / m
//   skew reverse KL  D = KL(p_S || m),  m = (1 - alpha) p_T + alpha p_S,  u = ln(p_S / m) + 1 - alpha p_S / m
// gradient = grad_scale / tau * p_S (u - ubar) with ubar = sum p_S u (+ ce_grad_scale p_S from the CE term at tau = 1).
// Entries of probability 0 (logits of -inf, underflow) contribute nothing: m has a floor, log ratios are kept finite.
struct SkewCoef {
  float c, Rs, Rt, izs, izt;  // p = 2^(x c - R) / z with the row's merged reference and sum (the reference is not
                              // folded into one logarithm: at logits in the thousands that would cost 2e-4 of p)
  float alpha, beta;          // beta = 1 - alpha
  float Av, B;                // gradient = Av v + B p_S, see skew_terms
};
constexpr float kSkewTiny = 1.0e-37f;

// Sweep 2 of an element, whose gradient is then finished from two fp32 values, p = p_S and v (g = grad_scale / tau,
// ce = ce_grad_scale):
//   skew KL          v = p_S p_T / m,                                       gradient = (alpha - 1) g v + (ce - g ubar) p
//   skew reverse KL  v = p_S (ln(p_S / m) - alpha p_S / m) = p_S (u - 1),   gradient = g v + (g (1 - ubar) + ce) p
// dsum: D in log2 units; usum = sum v.
template <int DIVK>
__device__ __forceinline__ void skew_terms(float ps, float pt, const SkewCoef& k, float& dsum, float& usum, float& p,
                                           float& v) {
  p = ps;
  // The floors are additive here (one fused operation each instead of a maximum): kSkewTiny changes nothing above
  // 2e-30, and below that the element's terms are far under one rounding step of the sums.  The log ratio is taken of
  // the quotient itself, which sweep 2 needs anyway.
  if constexpr (DIVK == kSkewKl) {
    const float m = __builtin_fmaf(k.alpha, pt, __builtin_fmaf(k.beta, ps, kSkewTiny));
    const float w = __builtin_fmaf(pt, __builtin_amdgcn_rcpf(m), kSkewTiny);  // p_T / m
    dsum = __builtin_fmaf(pt, __log2f(w), dsum);
    v = ps * w;
  } else {
    const float m = __builtin_fmaf(k.beta, pt, __builtin_fmaf(k.alpha, ps, kSkewTiny));
    const float t = __builtin_fmaf(ps, __builtin_amdgcn_rcpf(m), kSkewTiny);  // p_S / m
    const float l = __log2f(t);
    dsum = __builtin_fmaf(ps, l, dsum);
    v = ps * __builtin_fmaf(l, kLn2, t * -k.alpha);
  }
  usum += v;
}
// the same from logits (elements outside the cached slice: the sub-group tail of a row)
template <int DIVK>
__device__ __forceinline__ void skew_cache(float xs, float xt, const SkewCoef& k, float& dsum, float& usum, float& p,
                                           float& v) {
  skew_terms<DIVK>(exp2_fast(__builtin_fmaf(xs, k.c, -k.Rs)) * k.izs, exp2_fast(__builtin_fmaf(xt, k.c, -k.Rt)) * k.izt, k, dsum,
                   usum, p, v);
}
template <int DIVK>
__device__ __forceinline__ float skew_grad(float xs, float xt, const SkewCoef& k) {
  float d = 0.0f, u = 0.0f, p, v;
  skew_cache<DIVK>(xs, xt, k, d, u, p, v);
  return __builtin_fmaf(v, k.Av, k.B * p);
}

// K: groups per thread and tensor a workgroup holds (a slice has at most a.gang_groups + 7 <= K * 256 - 1 groups).
template <int K, int TEACHER, bool LSE1, int DIVK = kForwardKl>
__global__ __launch_bounds__(kGangThreads, 4) void kd_gang_kernel(const KdArgs a) {
  static_assert(TEACHER == kDense, "dense teacher");
  constexpr int TH = kGangThreads;
  constexpr int GB = TH * 16;
  constexpr int NS = LSE1 ? 4 : 2;  // 0 student / tau, 1 teacher / tau (+ cross), 2 student tau = 1, 3 teacher tau = 1
  constexpr int NW3 = NS * 3;
  constexpr int W = gang_words(NS);
  constexpr bool REV = DIVK == kReverseKl;
  // the skew forms take three sweeps over the registers and a second exchange: normalisers; D and ubar; gradient
  constexpr bool SKEW = DIVK == kSkewKl || DIVK == kSkewReverseKl;
  static_assert(NW3 + 2 <= W, "the second exchange of the skew forms uses two spare words of a slice's record");
  __shared__ float red[4 * 3 * (TH / kWave)];
  __shared__ uint32_t xch[kGangMax * W];
  __shared__ uint32_t xch2[SKEW ? kGangMax * 2 : 1];
  __shared__ int gave_up;

  const int G = a.gang;
  const int64_t row = blockIdx.x / (unsigned)G;
  const int slice = (int)(blockIdx.x - (unsigned)(row * G));
  const int tid = threadIdx.x;
  const int V = a.V, nvec = a.nvec_s;
  uint16_t* grow = a.g + row * a.s_stride;
  // This workgroup owns groups [g0, g1) -- the last slice also the sub-group tail of the row.  Boundaries inside the row
  // are moved down to the next 128-byte boundary of the gradient row's address (by `shift` groups), so that no cache
  // line is shared by two workgroups of a row; a slice is at most 7 groups longer than a.gang_groups for it.
  const bool last = slice == G - 1;
  const int shift = (int)((reinterpret_cast<uintptr_t>(grow) >> 4) & 7u);
  const int b0 = slice * a.gang_groups - shift, b1 = b0 + a.gang_groups;
  const int g0 = slice == 0 ? 0 : (b0 < nvec ? b0 : nvec);
  const int g1 = last ? nvec : (b1 < nvec ? b1 : nvec);
  const int ng = g1 > g0 ? g1 - g0 : 0;

  if (!a.mask[row]) {  // not scored: scalars 0, the slice of the gradient row zero-filled, logits never read
    if (slice == 0 && tid == 0) {
      if (a.kd) a.kd[row] = 0.0f;
      if (a.nll) a.nll[row] = 0.0f;
      if (a.tnll) a.tnll[row] = 0.0f;
      if (a.lse) a.lse[row] = 0.0f;
    }
    gang_zero_slice<K>(grow, g0, ng, tid);
    if (last)
      for (int e = nvec * 8 + tid; e < V; e += TH) grow[e] = 0;
    return;
  }

  const uint16_t* srow = a.s + row * a.s_stride;
  const uint16_t* trow = a.t + row * a.t_stride;
  const float c = a.c;
  const bool lse1_t = LSE1 && a.tnll != nullptr;
  if (tid == 0) gave_up = 0;  // ordered before its use by the barriers of block_merge

  // The slice as a buffer: all of a thread's groups are requested at once, unconditionally (a predicate around a load
  // makes the compiler wait for it on the spot); groups past the slice's end read as zero and are never used.  Groups
  // k < q are whole for every thread, group q belongs to the first `part` threads.
  const __amdgpu_buffer_rsrc_t rs = row_rsrc(srow + (size_t)g0 * 8, ng);
  const __amdgpu_buffer_rsrc_t rt = row_rsrc(trow + (size_t)g0 * 8, ng);
  const int voff = tid * 16;
  const int q = ng / TH, part = ng - q * TH;  // uniform
  uint4 sreg[K], treg[K];
#pragma unroll
  for (int k = 0; k < K; ++k) {
    sreg[k] = ld_group<GB>(rs, voff, k, true, true);
    treg[k] = ld_group<GB>(rt, voff, k, true, true);
  }

  // the label logits belong to the slice that holds them (it reads them before it can overwrite them in place)
  int y = -1;
  bool own_y = false;
  float s_y = 0.0f, t_y = 0.0f;
  if (a.labels) {
    y = a.labels[row];
    if ((unsigned)y < (unsigned)V) {
      const int gy = y >> 3;
      own_y = (gy >= g0 && gy < g1) || (last && gy >= nvec);
      if (own_y) {
        s_y = bf16_one(srow[y]);
        t_y = bf16_one(trow[y]);
      }
    }
  }
  const bool bad_label = a.labels && (unsigned)y >= (unsigned)V;  // uniform

  Lse acc[NS];
#pragma unroll
  for (int i = 0; i < NS; ++i) acc[i].init();
  __builtin_amdgcn_sched_barrier(0);

  // ---- sweep 1 over the slice.  Fast form: a thread's reference exponents are fixed by its first group -- the
  // largest of its eight logits (integer maxima on the packed bit patterns, see pk_max_i16) plus kRefBias bits of
  // head room -- before the other groups have arrived, and no element is inspected again.  Terms are then 2^-100 and
  // below, sums stay far inside the fp32 range while no later logit exceeds the first group's by 2^200 (139 nats at
  // tau = 1), and a term that matters (within 2^-24 of the row's largest) cannot underflow.  What this form cannot take
  // -- a wider excursion, a logit of -inf (a masked vocabulary entry: 0 * -inf in the cross term) -- shows in the sums;
  // a wave that sees such a sum takes the careful form below (references that follow the data, guarded differences)
  // over the same registers.
  // The skew forms keep the exponentials of sweep 1 (two fp32 values per element pair, in place of the packed logits,
  // which are dead from here on -- hence the smaller K of these instances): sweep 2 scales them to probabilities with
  // one multiplication each instead of unpacking and exponentiating again, and leaves p_S and p_S (u - const) in the
  // same registers, so that the gradient sweep is one multiply-add per element.  Their references get 64 bits of head
  // room: an element's exponential is kept down to 2^-62 of the thread's first group's largest.
  constexpr float kRefBias = SKEW ? 64.0f : 100.0f;
  float cp[SKEW ? K : 1][8], cv[SKEW ? K : 1][8];
  if (ng > tid) {  // (threads without a group keep their empty partials)
    const float fs = pk_max_value(pk_max_group(sreg[0])), ft = pk_max_value(pk_max_group(treg[0]));
    acc[0].r = __builtin_fmaxf(__builtin_fmaf(fs, c, kRefBias), -1.0e30f);
    acc[1].r = __builtin_fmaxf(__builtin_fmaf(ft, c, kRefBias), -1.0e30f);
    if constexpr (LSE1) {
      acc[2].r = __builtin_fmaxf(__builtin_fmaf(fs, kLog2e, kRefBias), -1.0e30f);
      acc[3].r = __builtin_fmaxf(__builtin_fmaf(ft, kLog2e, kRefBias), -1.0e30f);
    }
  }
#pragma unroll
  for (int k = 0; k < K; ++k) {
    if (k < q || (k == q && tid < part)) {
      float xs[8], xt[8];
      unpack8(sreg[k], xs);
      unpack8(treg[k], xt);
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const float es = exp2_fast(__builtin_fmaf(xs[j], c, -acc[0].r));
        const float et = exp2_fast(__builtin_fmaf(xt[j], c, -acc[1].r));
        acc[0].z += es;
        acc[1].z += et;
        if constexpr (REV)
          acc[0].a = __builtin_fmaf(es, xs[j] - xt[j], acc[0].a);
        else if constexpr (!SKEW)
          acc[1].a = __builtin_fmaf(et, xt[j] - xs[j], acc[1].a);
        if constexpr (SKEW) {
          cp[k][j] = es;
          cv[k][j] = et;
        }
        if constexpr (LSE1) {
          acc[2].z += exp2_fast(__builtin_fmaf(xs[j], kLog2e, -acc[2].r));
          if (lse1_t) acc[3].z += exp2_fast(__builtin_fmaf(xt[j], kLog2e, -acc[3].r));
        }
      }
    }
    __builtin_amdgcn_sched_barrier(0);
  }
  {
    constexpr float kBig = 1.2676506e30f;  // 2^100
    bool odd = false;
#pragma unroll
    for (int i = 0; i < NS; ++i) odd = odd || !(acc[i].z < kBig) || !(fabsf(acc[i].a) < kBig);
    if (__builtin_amdgcn_ballot_w64(odd) != 0) {  // wave-uniform
#pragma unroll
      for (int i = 0; i < NS; ++i) acc[i].init();
      if constexpr (SKEW) {  // the packed logits are gone: fetched again (rare; they are still in a cache)
#pragma unroll
        for (int k = 0; k < K; ++k) {
          sreg[k] = ld_group<GB>(rs, voff, k, true, true);
          treg[k] = ld_group<GB>(rt, voff, k, true, true);
        }
      }
#pragma unroll
      for (int k = 0; k < K; ++k) {
        if (k < q || (k == q && tid < part)) accum8<kDense, LSE1, REV>(sreg[k], treg[k], c, lse1_t, acc);
        __builtin_amdgcn_sched_barrier(0);
      }
      if constexpr (SKEW) {  // the exponentials again, against the references the careful form ended with
#pragma unroll
        for (int k = 0; k < K; ++k) {  // (every group, also those past the slice's end: all of the cache is rewritten)
          float xs[8], xt[8];
          unpack8(sreg[k], xs);
          unpack8(treg[k], xt);
#pragma unroll
          for (int j = 0; j < 8; ++j) {
            cp[k][j] = exp2_fast(__builtin_fmaf(xs[j], c, -acc[0].r));
            cv[k][j] = exp2_fast(__builtin_fmaf(xt[j], c, -acc[1].r));
          }
          __builtin_amdgcn_sched_barrier(0);
        }
      }
    }
  }
  const float r_s_thread = acc[0].r, r_t_thread = acc[1].r;  // what this thread's cached exponentials refer to
  if (last) {
    for (int e = nvec * 8 + tid; e < V; e += TH) {
      const float xs = bf16_one(srow[e]);
      const float xt = bf16_one(trow[e]);
      if constexpr (REV) {
        acc[1].add1(xt, c);
        acc[0].add1_cross(xs, xs - xt, c);
      } else {
        acc[1].add1_cross(xt, xt - xs, c);
        acc[0].add1(xs, c);
      }
      if constexpr (LSE1) {
        if (lse1_t) acc[3].add1(xt, kLog2e);
        acc[2].add1(xs, kLog2e);
      }
    }
  }

  // ---- wave totals, workgroup totals (through LDS), post, wait for the row's, row totals: the same merge each time
  const int lane = tid & (kWave - 1), wid = tid / kWave;
  constexpr int NWV = TH / kWave;
#pragma unroll
  for (int i = 0; i < NS; ++i) {
    normalise(acc[i]);
    if (i == (REV ? 0 : 1) && !SKEW)  // the stream that carries the cross term
      wave_merge_rescaled<true>(acc[i]);
    else
      wave_merge_rescaled<false>(acc[i]);
  }
  if (lane == 0) {
#pragma unroll
    for (int i = 0; i < NS; ++i) {
      red[(i * 3 + 0) * NWV + wid] = acc[i].r;
      red[(i * 3 + 1) * NWV + wid] = acc[i].z;
      red[(i * 3 + 2) * NWV + wid] = acc[i].a;
    }
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < NS; ++i) {
    acc[i].init();
    if (lane < NWV) {
      acc[i].r = red[(i * 3 + 0) * NWV + lane];
      acc[i].z = red[(i * 3 + 1) * NWV + lane];
      acc[i].a = red[(i * 3 + 2) * NWV + lane];
    }
    if (i == (REV ? 0 : 1) && !SKEW)  // the stream that carries the cross term
      wave_merge_rescaled<true>(acc[i]);
    else
      wave_merge_rescaled<false>(acc[i]);
  }

  uint32_t* rec = a.ws + (size_t)blockIdx.x * W;  // scratch[row][slice]
  uint32_t* abandon = a.ws + (size_t)gridDim.x * W;  // behind the record
  if (tid < NW3) {
    float v = acc[0].r;
#pragma unroll
    for (int i = 0; i < NS; ++i) {
      if (tid == i * 3 + 0) v = acc[i].r;
      if (tid == i * 3 + 1) v = acc[i].z;
      if (tid == i * 3 + 2) v = acc[i].a;
    }
    gang_post(rec + tid, v);
  }
  {
    const uint32_t* rrow = a.ws + (size_t)row * G * W;
    const int nw = G * NW3;
    for (int w = tid; w < nw; w += TH) {
      const int s = w / NW3, f = w - s * NW3;
      xch[s * W + f] = gang_wait(rrow + s * W + f, abandon, a.spin_limit, &gave_up);
    }
  }
  __syncthreads();
  bool timeout = gave_up != 0;  // uniform
#pragma unroll
  for (int i = 0; i < NS; ++i) {  // lane s < G takes slice s: every wave of every workgroup of the row computes the
    acc[i].init();                // same totals in the same order
    if (lane < G) {
      acc[i].r = __builtin_bit_cast(float, xch[lane * W + i * 3 + 0]);
      acc[i].z = __builtin_bit_cast(float, xch[lane * W + i * 3 + 1]);
      acc[i].a = __builtin_bit_cast(float, xch[lane * W + i * 3 + 2]);
    }
    if (i == (REV ? 0 : 1) && !SKEW)  // the stream that carries the cross term
      wave_merge_rescaled<true>(acc[i]);
    else
      wave_merge_rescaled<false>(acc[i]);
  }

  const float Ls = acc[0].log2_sum();
  const float Lt = acc[1].log2_sum();
  const float lse1_s = __fmul_rn(LSE1 ? acc[NS - 2].log2_sum() : Ls, kLn2);
  const float lse_diff = ((acc[0].r - acc[1].r) + (acc[0].log2_z() - acc[1].log2_z())) * kLn2;  // lse_S - lse_T at tau
  float kd = REV ? (acc[0].a / acc[0].z) * a.inv_tau - lse_diff : (acc[1].a / acc[1].z) * a.inv_tau + lse_diff;
  kd = kd < 0.0f ? 0.0f : kd;  // (the skew forms replace it below)
  const bool ce = a.cscale != 0.0f;  // uniform (tau = 1 here whenever it is set)
  Sweep2Coef kf = sweep2_coef(acc[0], acc[1], c, a.gscale, a.cscale, true, true);
  SkewCoef ks;
  if constexpr (SKEW) {
    // ---- sweep 2 of the skew forms over the registers: D and ubar need the row's normalisers in every term
    ks.c = c;
    ks.Rs = acc[0].r;
    ks.Rt = acc[1].r;
    ks.izs = 1.0f / acc[0].z;
    ks.izt = 1.0f / acc[1].z;
    ks.alpha = a.alpha;
    ks.beta = 1.0f - a.alpha;
    float dsum = 0.0f, usum = 0.0f;
    // cached exponential -> probability
    const float fs = exp2_fast(r_s_thread - ks.Rs) * ks.izs, ft = exp2_fast(r_t_thread - ks.Rt) * ks.izt;
#pragma unroll
    for (int k = 0; k < K; ++k) {
      if (k < q || (k == q && tid < part)) {
#pragma unroll
        for (int j = 0; j < 8; ++j) skew_terms<DIVK>(cp[k][j] * fs, cv[k][j] * ft, ks, dsum, usum, cp[k][j], cv[k][j]);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    if (last)
      for (int e = nvec * 8 + tid; e < V; e += TH) {
        float p, v;
        skew_cache<DIVK>(bf16_one(srow[e]), bf16_one(trow[e]), ks, dsum, usum, p, v);
      }
    // workgroup totals, second post / wait, row totals -- plain sums in a fixed order
    dsum = wave_sum_dpp(dsum);
    usum = wave_sum_dpp(usum);
    if (lane == 0) {
      red[wid] = dsum;
      red[NWV + wid] = usum;
    }
    __syncthreads();
    dsum = wave_sum_dpp(lane < NWV ? red[lane] : 0.0f);
    usum = wave_sum_dpp(lane < NWV ? red[NWV + lane] : 0.0f);
    if (tid < 2) gang_post(rec + NW3 + tid, tid == 0 ? dsum : usum);
    {
      const uint32_t* rrow = a.ws + (size_t)row * G * W;
      for (int w = tid; w < 2 * G; w += TH) {
        const int s = w >> 1, f = w & 1;
        xch2[w] = gang_wait(rrow + s * W + NW3 + f, abandon, a.spin_limit, &gave_up);
      }
    }
    __syncthreads();
    timeout = gave_up != 0;
    dsum = wave_sum_dpp(lane < G ? __builtin_bit_cast(float, xch2[2 * lane]) : 0.0f);
    usum = wave_sum_dpp(lane < G ? __builtin_bit_cast(float, xch2[2 * lane + 1]) : 0.0f);
    kd = dsum * kLn2;
    kd = kd < 0.0f ? 0.0f : kd;
    const float g = a.gscale;  // (grad_scale / tau)
    if constexpr (DIVK == kSkewKl) {
      const float ubar = (a.alpha - 1.0f) * usum;
      ks.Av = (a.alpha - 1.0f) * g;
      ks.B = a.cscale - g * ubar;
    } else {
      const float ubar = usum + 1.0f;
      ks.B = __builtin_fmaf(g, 1.0f - ubar, a.cscale);
      ks.Av = g;
    }
  }
  if constexpr (REV) {
    const float inv_z = 1.0f / acc[0].z;
    kf.ra = a.gscale * a.inv_tau * inv_z;
    kf.rb = (a.cscale - a.gscale * (lse_diff + kd)) * inv_z;
    kf.folded = true;
  }

  if (tid == 0) {
    const float nanv = __builtin_nanf("");
    int flags = 0;
    if (slice == 0) {
      if (timeout) flags |= 8;
      if (bad_label && (a.nll || a.tnll || ce)) flags |= 1;
      if (a.kd) a.kd[row] = timeout ? nanv : kd;
      if (a.lse) a.lse[row] = timeout ? nanv : lse1_s;
      if (bad_label) {
        if (a.nll) a.nll[row] = nanv;
        if (a.tnll) a.tnll[row] = nanv;
      }
    } else if (timeout) {
      flags |= 8;
    }
    if (own_y) {
      if (a.nll) a.nll[row] = timeout ? nanv : __fsub_rn(lse1_s, s_y);
      if (a.tnll) {
        const float lse1_tt = __fmul_rn(LSE1 ? acc[NS - 1].log2_sum() : Lt, kLn2);
        a.tnll[row] = timeout ? nanv : __fsub_rn(lse1_tt, t_y);
      }
    }
    if (flags && a.status) atomicOr(a.status, flags);
  }

  // ---- sweep 2: the gradient of the slice, from the registers, last group first
  uint8_t* gslice = reinterpret_cast<uint8_t*>(grow) + (size_t)g0 * 16;
  auto store = [&](int k, const uint4& o) {  // the group's base is uniform, the thread adds tid * 16
    const u32x4 w = {o.x, o.y, o.z, o.w};
    __builtin_nontemporal_store(w, reinterpret_cast<u32x4*>(gslice + (size_t)k * GB) + tid);
  };
  if (timeout || (ce && bad_label)) {  // uniform: the row cannot be differentiated
    const uint4 qnan = make_uint4(0x7fc07fc0u, 0x7fc07fc0u, 0x7fc07fc0u, 0x7fc07fc0u);
#pragma unroll
    for (int k = 0; k < K; ++k)
      if (k < q || (k == q && tid < part)) store(k, qnan);
    if (last)
      for (int e = nvec * 8 + tid; e < V; e += TH) grow[e] = 0x7fc0;
    return;
  }
  // The label position of the composite loss (Eq. 1) gets its final value from fp32, rounded once: the group that
  // holds it is the same for every thread (k_y, uniform), the thread that owns it keeps a mask and the bits.
  int k_y = -1;
  uint4 y_keep = make_uint4(~0u, ~0u, ~0u, ~0u), y_bits = make_uint4(0, 0, 0, 0);
  uint16_t y_tail = 0;
  if (ce && own_y) {  // uniform
    float gy;
    if constexpr (REV)
      gy = grad_reverse_elem(s_y, t_y, kf);
    else if constexpr (SKEW)
      gy = skew_grad<DIVK>(s_y, t_y, ks);
    else
      gy = grad_dense_elem(s_y, t_y, kf.p);
    const uint32_t b16 = one_bf16(gy - a.cscale);
    y_tail = (uint16_t)b16;
    if ((y >> 3) < nvec) {
      const int yg = (y >> 3) - g0;  // group of the slice
      k_y = yg / TH;
      if (yg - k_y * TH == tid) {
        const int j = y & 7;
        const uint32_t keep = (j & 1) ? 0x0000ffffu : 0xffff0000u, bits = (j & 1) ? b16 << 16 : b16;
        if ((j >> 1) == 0) { y_keep.x = keep; y_bits.x = bits; }
        if ((j >> 1) == 1) { y_keep.y = keep; y_bits.y = bits; }
        if ((j >> 1) == 2) { y_keep.z = keep; y_bits.z = bits; }
        if ((j >> 1) == 3) { y_keep.w = keep; y_bits.w = bits; }
      }
    }
  }
  auto patch_label = [&](uint4& o) {  // a no-op in every thread but the one that owns the label
    o.x = (o.x & y_keep.x) | y_bits.x;
    o.y = (o.y & y_keep.y) | y_bits.y;
    o.z = (o.z & y_keep.z) | y_bits.z;
    o.w = (o.w & y_keep.w) | y_bits.w;
  };
  if (last) {
    for (int e = nvec * 8 + tid; e < V; e += TH) {
      const float xs = bf16_one(srow[e]), xt = bf16_one(trow[e]);
      uint16_t o;
      if constexpr (SKEW)
        o = one_bf16(skew_grad<DIVK>(xs, xt, ks));
      else
        o = one_bf16(REV ? grad_reverse_elem(xs, xt, kf) : grad_dense_elem(xs, xt, kf.p));
      if (ce && own_y && e == y) o = y_tail;
      grow[e] = o;
    }
  }
  if constexpr (SKEW) {
#pragma unroll
    for (int k = K - 1; k >= 0; --k) {
      float gv[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) gv[j] = __builtin_fmaf(cv[k][j], ks.Av, ks.B * cp[k][j]);
      uint4 o = make_uint4(pack_bf16(gv[0], gv[1]), pack_bf16(gv[2], gv[3]), pack_bf16(gv[4], gv[5]), pack_bf16(gv[6], gv[7]));
      if (k == k_y) patch_label(o);  // uniform
      if (k < q || (k == q && tid < part)) store(k, o);
      __builtin_amdgcn_sched_barrier(0);
    }
  } else if (kf.folded) {  // uniform
#pragma unroll
    for (int k = K - 1; k >= 0; --k) {
      opaque(sreg[k]);  // sweep 2 unpacks the registers again instead of keeping sweep 1's floats alive
      opaque(treg[k]);
      uint4 o = grad8<kDense, true, DIVK>(sreg[k], treg[k], kf);
      if (k == k_y) patch_label(o);  // uniform
      if (k < q || (k == q && tid < part)) store(k, o);
      __builtin_amdgcn_sched_barrier(0);
    }
  } else {  // rows whose reference exponents are in the thousands: precise form
#pragma unroll
    for (int k = K - 1; k >= 0; --k) {
      opaque(sreg[k]);
      opaque(treg[k]);
      uint4 o = grad8<kDense, false, DIVK>(sreg[k], treg[k], kf);
      if (k == k_y) patch_label(o);  // uniform
      if (k < q || (k == q && tid < part)) store(k, o);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
}

}  // namespace npd
