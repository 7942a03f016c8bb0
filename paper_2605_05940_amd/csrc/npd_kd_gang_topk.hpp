// Row-gang kernel for a top-k teacher (Sec. 3.1: the teacher is stored as k vocabulary ids + k values per position;
// Eq. 2 with p_T renormalised over the k stored entries and p_S over the full vocabulary).  Same scheme as
// npd_kd_gang.hpp -- a row shared by G short-lived workgroups of 256 threads, the student slice in registers, partial
// log-sum-exps exchanged through the scratch record -- with these differences:
//   - only the student row is dense: one read and one write per logit;
//   - every workgroup of a row reads the row's whole top-k record (k ids + k values, a few hundred bytes): the teacher's
//     normaliser over the k values is computed by each of them, the support positions that fall into its own slice
//     are patched after its dense stores (final values from fp32, rounded once), and slice 0 also gathers the student
//     logits of all k support positions for kd_tok;
//   - every student logit a workgroup needs from outside its registers (support positions, the label) is fetched
//     before the workgroup posts its partial sum, i.e. before any workgroup of the row can overwrite the row in place.
#pragma once
#include "npd_kd_gang.hpp"

namespace npd {

template <int K, bool LSE1>
__global__ __launch_bounds__(kGangThreads, 6) void kd_gang_topk_kernel(const KdArgs a) {
  constexpr int TH = kGangThreads;
  constexpr int GB = TH * 16;
  constexpr int NS = LSE1 ? 2 : 1;  // student / tau, student at tau = 1
  constexpr int NW3 = NS * 3;
  constexpr int W = 8;              // words of scratch per slice
  constexpr int NWV = TH / kWave;
  __shared__ float red[2 * 3 * NWV + NWV];
  __shared__ uint32_t xch[kGangMax * W];
  __shared__ uint16_t sup_s[kTopkMax];  // student logits at the support positions (bf16 bits); later their patches
  __shared__ int gave_up, y_in_support;

  const int G = a.gang;
  const int64_t row = blockIdx.x / (unsigned)G;
  const int slice = (int)(blockIdx.x - (unsigned)(row * G));
  const int tid = threadIdx.x;
  const int V = a.V, nvec = a.nvec_s, k_top = a.k;
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
      if (a.lse) a.lse[row] = 0.0f;
    }
    gang_zero_slice<K>(grow, g0, ng, tid);
    if (last)
      for (int e = nvec * 8 + tid; e < V; e += TH) grow[e] = 0;
    return;
  }

  const uint16_t* srow = a.s + row * a.s_stride;
  const float c = a.c;
  if (tid == 0) gave_up = y_in_support = 0;  // ordered before their use by the barrier below

  const __amdgpu_buffer_rsrc_t rs = row_rsrc(srow + (size_t)g0 * 8, ng);
  const int voff = tid * 16;
  const int q = ng / TH, part = ng - q * TH;  // uniform
  uint4 sreg[K];
#pragma unroll
  for (int k = 0; k < K; ++k) sreg[k] = ld_group<GB>(rs, voff, k, true, true);

  // elements [e0, e1) are this workgroup's (the last slice also owns the sub-group tail)
  const int e0 = g0 * 8, e1 = last ? V : g1 * 8;
  int y = -1;
  bool own_y = false;
  float s_y = 0.0f;
  if (a.labels) {
    y = a.labels[row];
    own_y = y >= e0 && y < e1 && (unsigned)y < (unsigned)V;
    if (own_y) s_y = bf16_one(srow[y]);
  }
  const bool bad_label = a.labels && (unsigned)y >= (unsigned)V;  // uniform

  // ---- the row's top-k record: the teacher's normaliser over the k values, the range check of the ids, and the
  // student logits at the support positions this workgroup will need (its own; all of them in slice 0)
  const int32_t* irow = a.tidx + row * (int64_t)k_top;
  const float* vrow = a.tval + row * (int64_t)k_top;
  Lse tt;
  tt.init();
  int bad_index = 0;
  for (int j = tid; j < k_top; j += TH) {
    const int id = irow[j];
    tt.add1(vrow[j], c);
    if ((unsigned)id >= (unsigned)V) {
      bad_index = 1;
    } else if (slice == 0 || (id >= e0 && id < e1)) {
      sup_s[j] = srow[id];
    }
  }

  // ---- sweep 1 over the student slice (see npd_kd_gang.hpp: fixed reference from the first group, careful re-run
  // of a wave whose sums show an anomaly)
  Lse acc[4];  // 0 student / tau, 2 student at tau = 1 (the indices accum8 uses; 1 and 3 stay empty)
#pragma unroll
  for (int i = 0; i < 4; ++i) acc[i].init();
  constexpr float kRefBias = 100.0f;
  if (ng > tid) {
    const float fs = pk_max_value(pk_max_group(sreg[0]));
    acc[0].r = __builtin_fmaxf(__builtin_fmaf(fs, c, kRefBias), -1.0e30f);
    if constexpr (LSE1) acc[2].r = __builtin_fmaxf(__builtin_fmaf(fs, kLog2e, kRefBias), -1.0e30f);
  }
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int k = 0; k < K; ++k) {
    if (k < q || (k == q && tid < part)) {
      float xs[8];
      unpack8(sreg[k], xs);
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        acc[0].z += exp2_fast(__builtin_fmaf(xs[j], c, -acc[0].r));
        if constexpr (LSE1) acc[2].z += exp2_fast(__builtin_fmaf(xs[j], kLog2e, -acc[2].r));
      }
    }
    __builtin_amdgcn_sched_barrier(0);
  }
  {
    constexpr float kBig = 1.2676506e30f;  // 2^100
    bool odd = !(acc[0].z < kBig);
    if constexpr (LSE1) odd = odd || !(acc[2].z < kBig);
    if (__builtin_amdgcn_ballot_w64(odd) != 0) {  // wave-uniform
      acc[0].init();
      acc[2].init();
#pragma unroll
      for (int k = 0; k < K; ++k) {
        if (k < q || (k == q && tid < part)) {
          float xs[8];
          unpack8(sreg[k], xs);
          acc[0].add8(xs, c);
          if constexpr (LSE1) acc[2].add8(xs, kLog2e);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  }
  if (last) {
    for (int e = nvec * 8 + tid; e < V; e += TH) {
      const float xs = bf16_one(srow[e]);
      acc[0].add1(xs, c);
      if constexpr (LSE1) acc[2].add1(xs, kLog2e);
    }
  }

  // ---- wave totals, workgroup totals, post, wait, row totals (student); workgroup totals of the teacher's k values
  const int lane = tid & (kWave - 1), wid = tid / kWave;
  Lse st[2] = {acc[0], acc[2]};
#pragma unroll
  for (int i = 0; i < NS; ++i) {
    normalise(st[i]);
    wave_merge_rescaled<false>(st[i]);
  }
  normalise(tt);
  wave_merge_rescaled<false>(tt);
  bad_index = __builtin_amdgcn_ballot_w64(bad_index != 0) != 0;
  if (lane == 0) {
#pragma unroll
    for (int i = 0; i < NS; ++i) {
      red[(i * 2 + 0) * NWV + wid] = st[i].r;
      red[(i * 2 + 1) * NWV + wid] = st[i].z;
    }
    red[4 * NWV + wid] = tt.r;
    red[5 * NWV + wid] = tt.z;
    red[6 * NWV + wid] = bad_index ? 1.0f : 0.0f;
  }
  __syncthreads();  // also orders the gathered support logits in sup_s before their readers
#pragma unroll
  for (int i = 0; i < NS; ++i) {
    st[i].init();
    if (lane < NWV) {
      st[i].r = red[(i * 2 + 0) * NWV + lane];
      st[i].z = red[(i * 2 + 1) * NWV + lane];
    }
    wave_merge_rescaled<false>(st[i]);
  }
  tt.init();
  if (lane < NWV) {
    tt.r = red[4 * NWV + lane];
    tt.z = red[5 * NWV + lane];
  }
  wave_merge_rescaled<false>(tt);
  bad_index = (red[6 * NWV + 0] + red[6 * NWV + 1] + red[6 * NWV + 2] + red[6 * NWV + 3]) != 0.0f;  // uniform

  uint32_t* rec = a.ws + (size_t)blockIdx.x * W;
  uint32_t* abandon = a.ws + (size_t)gridDim.x * W;  // behind the record
  if (tid < NW3) {
    float v = st[0].r;
#pragma unroll
    for (int i = 0; i < NS; ++i) {
      if (tid == i * 3 + 0) v = st[i].r;
      if (tid == i * 3 + 1) v = st[i].z;
      if (tid == i * 3 + 2) v = 0.0f;
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
  const bool timeout = gave_up != 0;  // uniform
#pragma unroll
  for (int i = 0; i < NS; ++i) {
    st[i].init();
    if (lane < G) {
      st[i].r = __builtin_bit_cast(float, xch[lane * W + i * 3 + 0]);
      st[i].z = __builtin_bit_cast(float, xch[lane * W + i * 3 + 1]);
    }
    wave_merge_rescaled<false>(st[i]);
  }

  const float Ls = st[0].log2_sum();
  const float Lt = tt.log2_sum();
  const float lse1_s = __fmul_rn(LSE1 ? st[1].log2_sum() : Ls, kLn2);
  const bool ce = a.cscale != 0.0f;  // uniform (tau = 1 here whenever it is set)
  Sweep2Coef kf = sweep2_coef(st[0], tt, c, a.gscale, a.cscale, true, false);

  // ---- kd_tok (slice 0) and the final values of the support positions of this slice
  float part_kd = 0.0f;
  int y_hit = 0;
  if (!bad_index) {
    for (int j = tid; j < k_top; j += TH) {
      const int id = irow[j];
      const bool mine = id >= e0 && id < e1;
      if (slice == 0 || mine) {
        const float b = vrow[j] * c;
        const float sj = bf16_one(sup_s[j]);
        if (slice == 0) {
          const float lpt = b - Lt;
          const float lps = __builtin_fmaf(sj, c, -Ls);
          part_kd = __builtin_fmaf(exp2_fast(lpt), __builtin_fmaxf(lpt - lps, -3.4028234663852886e38f) * kLn2, part_kd);
        }
        if (mine) {
          float gj = grad_pair_elem(sj, b, kf.p);
          if (ce && id == y) {
            gj -= a.cscale;
            y_hit = 1;
          }
          sup_s[j] = one_bf16(gj);  // this thread read sup_s[j] above: no other thread touches entry j
        }
      }
    }
  }
  float kd = wave_sum_dpp(part_kd);
  y_hit = __builtin_amdgcn_ballot_w64(y_hit != 0) != 0;
  if (lane == 0) {
    red[wid] = kd;
    if (y_hit) y_in_support = 1;
  }
  __syncthreads();
  kd = (red[0] + red[1]) + (red[2] + red[3]);
  kd = kd < 0.0f ? 0.0f : kd;
  if (bad_index) kd = __builtin_nanf("");

  if (tid == 0) {
    const float nanv = __builtin_nanf("");
    int flags = 0;
    if (slice == 0) {
      if (timeout) flags |= 8;
      if (bad_index) flags |= 2;
      if (bad_label && (a.nll || ce)) flags |= 1;
      if (a.kd) a.kd[row] = timeout ? nanv : kd;
      if (a.lse) a.lse[row] = timeout ? nanv : lse1_s;
      if (bad_label && a.nll) a.nll[row] = nanv;
    } else if (timeout) {
      flags |= 8;
    }
    if (own_y && a.nll) a.nll[row] = timeout ? nanv : __fsub_rn(lse1_s, s_y);
    if (flags && a.status) atomicOr(a.status, flags);
  }

  // ---- sweep 2: dense part p_S * weights from the registers, then the support positions of this slice
  uint8_t* gslice = reinterpret_cast<uint8_t*>(grow) + (size_t)g0 * 16;
  auto store = [&](int k, const uint4& o) {
    const u32x4 w = {o.x, o.y, o.z, o.w};
    __builtin_nontemporal_store(w, reinterpret_cast<u32x4*>(gslice + (size_t)k * GB) + tid);
  };
  if (timeout || bad_index || (ce && bad_label)) {  // uniform: the row cannot be differentiated
    const uint4 qnan = make_uint4(0x7fc07fc0u, 0x7fc07fc0u, 0x7fc07fc0u, 0x7fc07fc0u);
#pragma unroll
    for (int k = 0; k < K; ++k)
      if (k < q || (k == q && tid < part)) store(k, qnan);
    if (last)
      for (int e = nvec * 8 + tid; e < V; e += TH) grow[e] = 0x7fc0;
    return;
  }
  // the label position of the composite loss, unless it is one of the support positions (patched with them)
  int k_y = -1;
  uint4 y_keep = make_uint4(~0u, ~0u, ~0u, ~0u), y_bits = make_uint4(0, 0, 0, 0);
  uint16_t y_tail = 0;
  const bool patch_y = ce && own_y && !y_in_support;  // uniform
  if (patch_y) {
    const uint32_t b16 = one_bf16(grad_student_elem(s_y, kf.p) - a.cscale);
    y_tail = (uint16_t)b16;
    if ((y >> 3) < nvec) {
      const int yg = (y >> 3) - g0;
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
  auto patch_label = [&](uint4& o) {
    o.x = (o.x & y_keep.x) | y_bits.x;
    o.y = (o.y & y_keep.y) | y_bits.y;
    o.z = (o.z & y_keep.z) | y_bits.z;
    o.w = (o.w & y_keep.w) | y_bits.w;
  };
  if (last) {
    for (int e = nvec * 8 + tid; e < V; e += TH) {
      uint16_t o = one_bf16(grad_student_elem(bf16_one(srow[e]), kf.p));
      if (patch_y && e == y) o = y_tail;
      grow[e] = o;
    }
  }
  if (kf.folded) {  // uniform
#pragma unroll
    for (int k = K - 1; k >= 0; --k) {
      opaque(sreg[k]);
      uint4 o = grad8<kTopk, true>(sreg[k], sreg[k], kf);
      if (k == k_y) patch_label(o);  // uniform
      if (k < q || (k == q && tid < part)) store(k, o);
      __builtin_amdgcn_sched_barrier(0);
    }
  } else {
#pragma unroll
    for (int k = K - 1; k >= 0; --k) {
      opaque(sreg[k]);
      uint4 o = grad8<kTopk, false>(sreg[k], sreg[k], kf);
      if (k == k_y) patch_label(o);  // uniform
      if (k < q || (k == q && tid < part)) store(k, o);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  // the support positions get their final values once the dense stores of the whole workgroup are ordered before them
  __syncthreads();
  for (int j = tid; j < k_top; j += TH) {
    const int id = irow[j];
    if (id >= e0 && id < e1) grow[id] = sup_s[j];
  }
}

}  // namespace npd
