// Row-resident variant of the fused KD loss + gradient kernel for large vocabularies (gfx950).
//
// A token row of ~150k bf16 logits (student + teacher = 608 KB) does not fit one CU, but most of it
// does: 1024 threads x CS 128-bit groups of the student row stay in VGPRs (packed bf16, as loaded),
// the first CT groups-per-thread of the teacher row are parked in LDS, and only the remaining teacher
// groups are read a second time -- last-read-first, so they come from the XCD's L2, not from HBM.
// HBM then sees each logit once and each gradient element once.  The gradient goes out with
// non-temporal 128-bit stores after all of the row's loads: reads and writes reach HBM in separate
// bursts, which it serves faster than an interleaved mix.
//
// Loads are software-pipelined by hand: group it + D is requested before group it is consumed.  The
// cached part is straight-line code (CS is a template parameter and every cached group but the last is
// full), so the compiler can keep several loads in flight.  Groups beyond the cached CS (vocabularies
// above CS * 8192 tokens) are streamed in sweep 1 and read again in sweep 2.  The arithmetic is the one of npd_kd_kernels.hip (same helpers, same merge tree).
#include "npd_device.hpp"
#include "npd_internal.hpp"

namespace npd {

constexpr int kCB = 1024;  // threads per workgroup: one workgroup owns a CU's whole register file

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ uint4 ld16(const uint16_t* row, int group) {
  return reinterpret_cast<const uint4*>(row)[group];
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

struct Sweep2Coef {
  float c, rs, rt, ratio, ws;
};

// gradient of 8 elements: (e_S - e_T z_S / z_T) w
template <int TEACHER>
__device__ __forceinline__ uint4 grad8(const uint4& vs, const uint4& vt, const Sweep2Coef& k) {
  float xs[8], gv[8];
  unpack8(vs, xs);
  if constexpr (TEACHER == kDense) {
    float xt[8];
    unpack8(vt, xt);
#pragma unroll
    for (int j = 0; j < 8; ++j)
      gv[j] = __builtin_fmaf(-exp2_fast(__builtin_fmaf(xt[j], k.c, -k.rt)), k.ratio,
                             exp2_fast(__builtin_fmaf(xs[j], k.c, -k.rs))) * k.ws;
  } else {
#pragma unroll
    for (int j = 0; j < 8; ++j) gv[j] = exp2_fast(__builtin_fmaf(xs[j], k.c, -k.rs)) * k.ws;
  }
  uint4 o;
  o.x = pack_bf16(gv[0], gv[1]);
  o.y = pack_bf16(gv[2], gv[3]);
  o.z = pack_bf16(gv[4], gv[5]);
  o.w = pack_bf16(gv[6], gv[7]);
  return o;
}

// sweep-1 contribution of 8 elements
template <int TEACHER, bool LSE1>
__device__ __forceinline__ void accum8(const uint4& vs, const uint4& vt, float c, bool lse1_t,
                                       Lse (&acc)[LSE1 ? 4 : 2]) {
  float xs[8];
  unpack8(vs, xs);
  if constexpr (TEACHER == kDense) {
    float xt[8];
    unpack8(vt, xt);
    acc[1].add8_cross(xt, xs, c);
    if constexpr (LSE1)
      if (lse1_t) acc[3].add8(xt, kLog2e);
  }
  acc[0].add8(xs, c);
  if constexpr (LSE1) acc[2].add8(xs, kLog2e);
}

template <int CS, int CT, int D, int TEACHER, bool GRAD, bool LSE1>
__global__ __launch_bounds__(kCB) void kd_cached_kernel(const KdArgs a) {
  extern __shared__ uint4 lds_t[];  // [CT][1024] teacher groups (dense teacher)
  __shared__ float red[4 * 3 * (kCB / kWave)];
  __shared__ uint16_t patch[TEACHER == kTopk && GRAD ? kTopkMax : 1];
  static_assert(CT <= CS && D >= 1 && D <= CS, "bad cache shape");
  const int tid = threadIdx.x;
  const int64_t row = blockIdx.x;
  const int V = a.V, nvec = a.nvec_s;  // this kernel is only launched with 16-byte aligned rows: nvec = V / 8
  uint16_t* grow = GRAD ? a.g + row * a.s_stride : nullptr;

  if (!a.mask[row]) {
    if (tid == 0) {
      if (a.kd) a.kd[row] = 0.0f;
      if (a.nll) a.nll[row] = 0.0f;
      if (a.tnll) a.tnll[row] = 0.0f;
      if (a.lse) a.lse[row] = 0.0f;
    }
    if constexpr (GRAD) {
      const uint4 z = make_uint4(0, 0, 0, 0);
      for (int i = tid; i < nvec; i += kCB) st16_stream(grow, i, z);
      for (int e = nvec * 8 + tid; e < V; e += kCB) grow[e] = 0;
    }
    return;
  }

  const uint16_t* srow = a.s + row * a.s_stride;
  const uint16_t* trow = TEACHER == kDense ? a.t + row * a.t_stride : nullptr;
  const float c = a.c;
  const bool lse1_t = LSE1 && a.tnll != nullptr;
  // launched only for rows of more than (CS - 1) * 1024 groups: every cached group is full except,
  // when the row has at most CS * 1024 groups, the last one
  const int nit = (nvec + kCB - 1) / kCB;  // 128-bit groups per thread

  int y = -1;
  float s_y = 0.0f, t_y = 0.0f;
  if (a.labels) {
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

  uint4 sreg[CS];  // the student row, as loaded
  uint4 tst[D];    // teacher groups in flight
  const int last = nvec - 1;
  // out-of-row lanes of the ragged group load the row's last group (in bounds) and are skipped in compute

  // ---- sweep 1, cached part: request D groups ahead
#pragma unroll
  for (int d = 0; d < D; ++d) {
    const int i = min(d * kCB + tid, last);
    sreg[d] = ld16(srow, i);
    if constexpr (TEACHER == kDense) tst[d] = ld16(trow, i);
  }
#pragma unroll
  for (int it = 0; it < CS; ++it) {
    const uint4 vt = TEACHER == kDense ? tst[it % D] : make_uint4(0, 0, 0, 0);
    if (it + D < CS) {
      const int nx = it + D < CS ? it + D : 0;  // constant once the loop is unrolled
      const int i = min(nx * kCB + tid, last);
      sreg[nx] = ld16(srow, i);
      if constexpr (TEACHER == kDense) tst[it % D] = ld16(trow, i);
    }
    if (it < CS - 1 || it * kCB + tid < nvec) accum8<TEACHER, LSE1>(sreg[it], vt, c, lse1_t, acc);
    if constexpr (TEACHER == kDense)
      if (it < CT) lds_t[it * kCB + tid] = vt;
    __builtin_amdgcn_sched_barrier(0);  // keep the instruction scheduler from piling all loads up front
  }
  // ---- sweep 1, streamed part (rows longer than the cache) and the sub-group tail
  for (int i = CS * kCB + tid; i < nvec; i += kCB) {
    const uint4 vs = ld16(srow, i);
    const uint4 vt = TEACHER == kDense ? ld16(trow, i) : make_uint4(0, 0, 0, 0);
    accum8<TEACHER, LSE1>(vs, vt, c, lse1_t, acc);
  }
  for (int e = nvec * 8 + tid; e < V; e += kCB) {
    const float xs = bf16_one(srow[e]);
    if constexpr (TEACHER == kDense) {
      const float xt = bf16_one(trow[e]);
      acc[1].add1_cross(xt, xt - xs, c);
      if constexpr (LSE1)
        if (lse1_t) acc[3].add1(xt, kLog2e);
    }
    acc[0].add1(xs, c);
    if constexpr (LSE1) acc[2].add1(xs, kLog2e);
  }
  int bad_index = 0;
  if constexpr (TEACHER == kTopk) {
    const int32_t* irow = a.tidx + row * (int64_t)a.k;
    const float* vrow = a.tval + row * (int64_t)a.k;
    for (int j = tid; j < a.k; j += kCB) {
      if ((unsigned)irow[j] >= (unsigned)V) bad_index = 1;
      acc[1].add1(vrow[j], c);
    }
  }

  // teacher groups that were not parked in LDS are requested again now, newest first; the first D of
  // them travel while the partial sums are merged
  constexpr int NRE = (TEACHER == kDense && GRAD) ? CS - CT : 0;  // re-read groups per thread (at most)
  if constexpr (NRE > 0) {
#pragma unroll
    for (int d = 0; d < D && d < NRE; ++d) tst[d] = ld16(trow, min((CS - 1 - d) * kCB + tid, last));
  }

  block_merge<kCB, NS>(acc, red);

  const float Ls = acc[0].log2_sum();
  const float Lt = TEACHER == kNone ? 0.0f : acc[1].log2_sum();
  const float lse1_s = __fmul_rn(LSE1 ? acc[NS - 2].log2_sum() : Ls, kLn2);
  float kd = 0.0f;
  if constexpr (TEACHER == kDense) {
    kd = (acc[1].a / acc[1].z) * a.inv_tau + ((acc[0].r - acc[1].r) + (acc[0].log2_z() - acc[1].log2_z())) * kLn2;
    kd = kd < 0.0f ? 0.0f : kd;
  }
  if constexpr (TEACHER == kTopk) {
    bad_index = __syncthreads_or(bad_index);
    const int32_t* irow = a.tidx + row * (int64_t)a.k;
    const float* vrow = a.tval + row * (int64_t)a.k;
    const float ws = a.gscale / acc[0].z, ratio = acc[0].z / acc[1].z;
    float part = 0.0f;
    if (!bad_index) {
      for (int j = tid; j < a.k; j += kCB) {
        const float b = vrow[j] * c;
        const float sj = bf16_one(srow[irow[j]]);
        const float lpt = b - Lt;
        const float lps = __builtin_fmaf(sj, c, -Ls);
        part = __builtin_fmaf(exp2_fast(lpt), (lpt - lps) * kLn2, part);
        if constexpr (GRAD) {
          const float gj =
              __builtin_fmaf(-exp2_fast(b - acc[1].r), ratio, exp2_fast(__builtin_fmaf(sj, c, -acc[0].r))) * ws;
          patch[j] = one_bf16(gj);
        }
      }
    }
    kd = block_sum<kCB>(part, red);
    kd = kd < 0.0f ? 0.0f : kd;
    if (bad_index) kd = __builtin_nanf("");
  }

  if (tid == 0) {
    int flags = 0;
    if (bad_index) flags |= 2;
    const bool bad_label = a.labels && (unsigned)y >= (unsigned)V;
    if (bad_label && (a.nll || a.tnll)) flags |= 1;
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
    Sweep2Coef k;
    k.c = c;
    k.rs = acc[0].r;
    k.rt = acc[1].r;
    k.ws = a.gscale / acc[0].z;
    k.ratio = TEACHER == kDense ? acc[0].z / acc[1].z : 0.0f;
    if (TEACHER == kTopk && bad_index) {
      const uint16_t qnan = 0x7fc0;
      for (int e = tid; e < V; e += kCB) grow[e] = qnan;
      return;
    }
    // sub-group tail and streamed part first (most recently read), then the cached groups backwards
    for (int e = nvec * 8 + tid; e < V; e += kCB) {
      float gv = exp2_fast(__builtin_fmaf(bf16_one(srow[e]), c, -k.rs));
      if constexpr (TEACHER == kDense)
        gv = __builtin_fmaf(-exp2_fast(__builtin_fmaf(bf16_one(trow[e]), c, -k.rt)), k.ratio, gv);
      grow[e] = one_bf16(gv * k.ws);
    }
    for (int i = (nit - 1) * kCB + tid; i >= CS * kCB; i -= kCB) {
      if (i < nvec) {
        const uint4 vs = ld16(srow, i);
        const uint4 vt = TEACHER == kDense ? ld16(trow, i) : make_uint4(0, 0, 0, 0);
        st16_stream(grow, i, grad8<TEACHER>(vs, vt, k));
      }
    }
#pragma unroll
    for (int q = 0; q < CS; ++q) {
      const int it = CS - 1 - q;
      uint4 vt = make_uint4(0, 0, 0, 0);
      if constexpr (TEACHER == kDense) {
        if (it < CT) {
          vt = lds_t[it * kCB + tid];
        } else {
          vt = tst[q % D];  // requested D visits ago
          if (it - D >= CT) tst[q % D] = ld16(trow, (it - D) * kCB + tid);
        }
      }
      const int i = it * kCB + tid;
      opaque(sreg[it]);
      if (it < CS - 1 || i < nvec) st16_stream(grow, i, grad8<TEACHER>(sreg[it], vt, k));
      __builtin_amdgcn_sched_barrier(0);
    }
    if constexpr (TEACHER == kTopk) {
      __syncthreads();
      const int32_t* irow = a.tidx + row * (int64_t)a.k;
      for (int j = tid; j < a.k; j += kCB) grow[irow[j]] = patch[j];
    }
  }
}

template <int CS, int CT, int D, int TEACHER, bool GRAD>
static hipError_t launch_cached_lse1(const KdArgs& a, hipStream_t stream) {
  const size_t lds_bytes = (size_t)CT * kCB * sizeof(uint4);
  auto launch = [&](auto kernel) -> hipError_t {
    if (lds_bytes > 0) {
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
      if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(kernel, dim3((unsigned)a.T), dim3(kCB), lds_bytes, stream, a);
    return hipGetLastError();
  };
  if (a.need_lse1) return launch(kd_cached_kernel<CS, CT, D, TEACHER, GRAD, true>);
  return launch(kd_cached_kernel<CS, CT, D, TEACHER, GRAD, false>);
}

constexpr int kCachedGroups = 19;  // covers vocabularies of 147,464 .. 155,648 tokens entirely, larger ones partly

// Row-resident path: 16-byte aligned rows of more than (kCachedGroups - 1) * 1024 groups.
bool cached_path_applies(const KdArgs& a) { return a.nvec_s > (kCachedGroups - 1) * kCB; }

hipError_t launch_kd_cached(const KdArgs& a, int teacher_kind, bool want_grad, hipStream_t stream) {
  switch (teacher_kind) {
    case kDense:
      return want_grad ? launch_cached_lse1<kCachedGroups, 9, 2, kDense, true>(a, stream)
                       : launch_cached_lse1<kCachedGroups, 0, 3, kDense, false>(a, stream);
    case kTopk:
      return want_grad ? launch_cached_lse1<kCachedGroups, 0, 3, kTopk, true>(a, stream)
                       : launch_cached_lse1<kCachedGroups, 0, 3, kTopk, false>(a, stream);
    default:
      return launch_cached_lse1<kCachedGroups, 0, 3, kNone, false>(a, stream);
  }
}

}  // namespace npd
