// Row-gang variant of the fused KD loss + gradient kernel (gfx950): a token row is shared by G short-lived
// workgroups of 256 threads, each of which owns one contiguous slice of the row (up to K 128-bit groups per thread
// and tensor) and keeps it in registers from the first sweep to the gradient write -- nothing is read twice, whatever
// the vocabulary.  The G partial log-sum-exps of a row meet through a small scratch record in device memory:
//
//   sweep 1 over the slice -> workgroup partials (r, z, a) -> posted to scratch[row][slice]
//   wait until all G slices of the row have posted -> merge them in one fixed tree (every workgroup of the row
//   computes bit-identical row totals) -> gradient of the slice from the registers -> written once
//
// Why: the memory system of this GPU gives a mix of two reads and one write 6.3 TB/s when the chip sweeps memory
// front to back and every row is read completely before it is written, against 5.7 TB/s when each compute unit
// works on a row of its own.  Consecutive workgroups are consecutive slices, four workgroups run per compute unit
// (one row's wait and arithmetic overlap three other slices' memory traffic), and masked rows are zero-filled in the
// same address order.
//
// The exchange needs no fence: every posted word is a 32-bit atomic store that carries its own validity (the
// scratch record is cleared to a pattern no posted word takes, by a fill kernel enqueued in front of each launch),
// and consumers poll those words with atomic loads at device scope.  Forward progress: a workgroup waits only for
// workgroups of smaller or neighbouring index (the other slices of its own row), a workgroup never waits before it
// has posted, and workgroups start in index order, so the lowest unfinished row always has all its workgroups
// resident or next to start.  Every wait is bounded all the same: a workgroup that gives up marks its row NaN and
// sets NPD_DEV_GANG_TIMEOUT, so a kernel can never hang.
#pragma once
#include "npd_kd_cached.hpp"

namespace npd {

constexpr int kGangThreads = 256;
constexpr int kGangMax = 32;                      // slices per row at most
constexpr uint32_t kGangEmpty = 0xffffffffu;      // scratch word not posted yet (a NaN pattern no partial is stored as)
constexpr int kGangSpinLimitDefault = 1 << 20;    // polls before a workgroup gives up (seconds; never reached in a healthy run)

__device__ __forceinline__ void gang_post(uint32_t* p, float v) {
  uint32_t w = __builtin_bit_cast(uint32_t, v);
  if (w == kGangEmpty) w = 0x7fc00000u;  // another NaN
  __hip_atomic_store(p, w, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// words of scratch per slice: 3 per partial log-sum-exp, rounded up to a power of two
__host__ __device__ constexpr int gang_words(int ns) { return ns == 2 ? 8 : 16; }

__global__ __launch_bounds__(256) void gang_clear_kernel(uint32_t* p, size_t n) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) p[i] = kGangEmpty;
}

// K: groups per thread and tensor a slice may have (the slice of a launch has a.gang_groups <= K * 256 groups).
template <int K, int TEACHER, bool LSE1, int DIVK = kForwardKl>
__global__ __launch_bounds__(kGangThreads, 4) void kd_gang_kernel(const KdArgs a) {
  static_assert(TEACHER == kDense, "dense teacher");
  static_assert(DIVK == kForwardKl || DIVK == kReverseKl, "two-sweep divergences");
  constexpr int TH = kGangThreads;
  constexpr int GB = TH * 16;
  constexpr int NS = LSE1 ? 4 : 2;  // 0 student / tau, 1 teacher / tau (+ cross), 2 student tau = 1, 3 teacher tau = 1
  constexpr int NW3 = NS * 3;
  constexpr int W = gang_words(NS);
  constexpr bool REV = DIVK == kReverseKl;
  __shared__ float red[4 * 3 * (TH / kWave)];
  __shared__ uint32_t xch[kGangMax * W];
  __shared__ int gave_up;

  const int G = a.gang;
  const int64_t row = blockIdx.x / (unsigned)G;
  const int slice = (int)(blockIdx.x - (unsigned)(row * G));
  const int tid = threadIdx.x;
  const int V = a.V, nvec = a.nvec_s;
  const int g0 = slice * a.gang_groups;
  const int g1 = g0 + a.gang_groups < nvec ? g0 + a.gang_groups : nvec;  // this workgroup owns groups [g0, g1)
  const bool last = slice == G - 1;                                      // ... and the sub-group tail of the row
  const int ng = g1 > g0 ? g1 - g0 : 0;
  uint16_t* grow = a.g + row * a.s_stride;

  if (!a.mask[row]) {  // not scored: scalars 0, gradient slice zero-filled, logits never read
    if (slice == 0 && tid == 0) {
      if (a.kd) a.kd[row] = 0.0f;
      if (a.nll) a.nll[row] = 0.0f;
      if (a.tnll) a.tnll[row] = 0.0f;
      if (a.lse) a.lse[row] = 0.0f;
    }
    const uint4 z = make_uint4(0, 0, 0, 0);
#pragma unroll
    for (int k = 0; k < K; ++k)
      if (k * TH + tid < ng) st16_stream(grow, g0 + k * TH + tid, z);
    if (last)
      for (int e = nvec * 8 + tid; e < V; e += TH) grow[e] = 0;
    return;
  }

  const uint16_t* srow = a.s + row * a.s_stride;
  const uint16_t* trow = a.t + row * a.t_stride;
  const float c = a.c;
  const bool lse1_t = LSE1 && a.tnll != nullptr;
  if (tid == 0) gave_up = 0;  // ordered before its use by the barriers of block_merge

  // the slice as a buffer: groups past its end read as zero and are never used
  const __amdgpu_buffer_rsrc_t rs = row_rsrc(srow + (size_t)g0 * 8, ng);
  const __amdgpu_buffer_rsrc_t rt = row_rsrc(trow + (size_t)g0 * 8, ng);
  const int voff = tid * 16;
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

  // ---- sweep 1 over the slice
#pragma unroll
  for (int k = 0; k < K; ++k) {
    if (k * TH + tid < ng) accum8<kDense, LSE1, REV>(sreg[k], treg[k], c, lse1_t, acc);
    __builtin_amdgcn_sched_barrier(0);
  }
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
  block_merge<TH, NS>(acc, red);

  // ---- post this slice's partials, wait for the row's, merge them in one fixed tree
  uint32_t* rec = a.ws + (size_t)blockIdx.x * W;  // scratch[row][slice]
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
      uint32_t v;
      int spins = 0;
      while (true) {
        v = __hip_atomic_load(rrow + s * W + f, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (v != kGangEmpty) break;
        if (++spins > a.spin_limit) {
          gave_up = 1;
          break;
        }
        __builtin_amdgcn_s_sleep(8);
      }
      xch[s * W + f] = v;
    }
  }
  __syncthreads();
  const bool timeout = gave_up != 0;  // uniform
  {
    // lane l starts from slice l mod NG (NG = G rounded up to a power of two; slices past G are empty partials), a
    // butterfly over log2(NG) steps merges them, and lane 0's result is what every lane of every workgroup of the row
    // keeps: one fixed order of operations
    const int NG = a.gang_pow2;
    const int lane = tid & (kWave - 1);
    const int s = lane & (NG - 1);
#pragma unroll
    for (int i = 0; i < NS; ++i) {
      Lse t;
      t.init();
      if (s < G) {
        t.r = __builtin_bit_cast(float, xch[s * W + i * 3 + 0]);
        t.z = __builtin_bit_cast(float, xch[s * W + i * 3 + 1]);
        t.a = __builtin_bit_cast(float, xch[s * W + i * 3 + 2]);
      }
      for (int off = NG >> 1; off > 0; off >>= 1) {
        const float r2 = __shfl_xor(t.r, off, kWave);
        const float z2 = __shfl_xor(t.z, off, kWave);
        const float a2 = __shfl_xor(t.a, off, kWave);
        t.merge(r2, z2, a2);
      }
      acc[i].r = __shfl(t.r, 0, kWave);
      acc[i].z = __shfl(t.z, 0, kWave);
      acc[i].a = __shfl(t.a, 0, kWave);
    }
  }

  const float Ls = acc[0].log2_sum();
  const float Lt = acc[1].log2_sum();
  const float lse1_s = __fmul_rn(LSE1 ? acc[NS - 2].log2_sum() : Ls, kLn2);
  const float lse_diff = ((acc[0].r - acc[1].r) + (acc[0].log2_z() - acc[1].log2_z())) * kLn2;  // lse_S - lse_T at tau
  float kd = REV ? (acc[0].a / acc[0].z) * a.inv_tau - lse_diff : (acc[1].a / acc[1].z) * a.inv_tau + lse_diff;
  kd = kd < 0.0f ? 0.0f : kd;
  const bool ce = a.cscale != 0.0f;  // uniform (tau = 1 here whenever it is set)
  Sweep2Coef kf = sweep2_coef(acc[0], acc[1], c, a.gscale, a.cscale, true, true);
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
  if (timeout || (ce && bad_label)) {  // uniform: the row cannot be differentiated
    const uint4 q = make_uint4(0x7fc07fc0u, 0x7fc07fc0u, 0x7fc07fc0u, 0x7fc07fc0u);
#pragma unroll
    for (int k = 0; k < K; ++k)
      if (k * TH + tid < ng) st16_stream(grow, g0 + k * TH + tid, q);
    if (last)
      for (int e = nvec * 8 + tid; e < V; e += TH) grow[e] = 0x7fc0;
    return;
  }
  // the label position of the composite loss (Eq. 1): its final value, from fp32, rounded once
  uint32_t y_bits = 0;
  const int y_group = (ce && own_y) ? (y >> 3) - g0 : -1;  // group of the slice that holds the label (this thread's if
  const bool y_mine = y_group >= 0 && (y >> 3) < nvec && (y_group % TH) == tid;  // y_group = k * TH + tid)
  if (ce && own_y) {
    float gy;
    if constexpr (REV)
      gy = grad_reverse_elem(s_y, t_y, kf);
    else
      gy = grad_dense_elem(s_y, t_y, kf.p);
    y_bits = one_bf16(gy - a.cscale);
  }
  auto patch_label = [&](uint4& o) {
    const int j = y & 7;
    const uint32_t m = (j & 1) ? 0x0000ffffu : 0xffff0000u, b = (j & 1) ? y_bits << 16 : y_bits;
    if ((j >> 1) == 0) o.x = (o.x & m) | b;
    if ((j >> 1) == 1) o.y = (o.y & m) | b;
    if ((j >> 1) == 2) o.z = (o.z & m) | b;
    if ((j >> 1) == 3) o.w = (o.w & m) | b;
  };
  if (last) {
    for (int e = nvec * 8 + tid; e < V; e += TH) {
      const float xs = bf16_one(srow[e]), xt = bf16_one(trow[e]);
      uint16_t o = one_bf16(REV ? grad_reverse_elem(xs, xt, kf) : grad_dense_elem(xs, xt, kf.p));
      if (ce && own_y && e == y) o = (uint16_t)y_bits;
      grow[e] = o;
    }
  }
  if (kf.folded) {  // uniform
#pragma unroll
    for (int k = K - 1; k >= 0; --k) {
      opaque(sreg[k]);
      uint4 o = grad8<kDense, true, DIVK>(sreg[k], treg[k], kf);
      if (y_mine && y_group == k * TH + tid) patch_label(o);
      if (k * TH + tid < ng) st16_stream(grow, g0 + k * TH + tid, o);
      __builtin_amdgcn_sched_barrier(0);
    }
  } else {  // rows whose reference exponents are in the thousands: precise form
#pragma unroll
    for (int k = K - 1; k >= 0; --k) {
      opaque(sreg[k]);
      uint4 o = grad8<kDense, false, DIVK>(sreg[k], treg[k], kf);
      if (y_mine && y_group == k * TH + tid) patch_label(o);
      if (k * TH + tid < ng) st16_stream(grow, g0 + k * TH + tid, o);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
}

}  // namespace npd
