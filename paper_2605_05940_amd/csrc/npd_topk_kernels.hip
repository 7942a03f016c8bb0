// Teacher-side top-k record (Sec. 3.1, "record only the top-k logits"; Alg. 1, Phase 2): for every scored
// position the k vocabulary ids with the largest teacher logits, largest first, equal logits by increasing id,
// and their values (the logits, or their log-softmax over the k).  Exact selection, integer bookkeeping only.
//
// One 1024-thread workgroup per token row, two workgroups per CU.  bf16 bit patterns map to 16-bit keys that
// order like the values.  Pass A streams the row and keeps one maximum per thread; the k-th largest of those
// 1024 maxima (bitonic sort in LDS) is a lower bound L of the k-th largest logit, because k threads hold a value
// >= L.  Pass B reads the row again (from cache) and appends every element >= L -- typically ~100 of 150k -- as a
// 64-bit (key, ~id) word to an LDS list, which is sorted and cut at k.  Rows where more than 4096 elements pass
// the bound (massive ties, constant rows) take an exact slow path: binary search of the k-th key by counting
// passes, then the ties of lowest id are collected in id order with block-wide scans.
#include "npd_device.hpp"
#include "npd_internal.hpp"

namespace npd {

constexpr int kTB = 1024;
constexpr int kCandCap = kTopkMax;  // 4096 candidates = 32 KB of LDS

// order-preserving key of a bf16 bit pattern (-0 is filed under +0: equal values must tie)
__device__ __forceinline__ uint32_t key_of(uint32_t b) {
  b &= 0xffffu;
  if (b == 0x8000u) b = 0;
  return (b & 0x8000u) ? (~b & 0xffffu) : (b | 0x8000u);
}
__device__ __forceinline__ float value_of_key(uint32_t key) {
  const uint32_t b = (key & 0x8000u) ? (key & 0x7fffu) : (~key & 0xffffu);
  return __builtin_bit_cast(float, b << 16);
}
__device__ __forceinline__ unsigned long long cand_word(uint32_t key, uint32_t id) {
  return ((unsigned long long)key << 32) | (unsigned long long)(0xffffffffu - id);  // larger = better
}

__device__ __forceinline__ void keys8(const uint4& v, uint32_t k[8]) {
  k[0] = key_of(v.x); k[1] = key_of(v.x >> 16);
  k[2] = key_of(v.y); k[3] = key_of(v.y >> 16);
  k[4] = key_of(v.z); k[5] = key_of(v.z >> 16);
  k[6] = key_of(v.w); k[7] = key_of(v.w >> 16);
}

// descending bitonic sort of n (a power of two) LDS words by all kTB threads; ends with a barrier
template <typename W>
__device__ __forceinline__ void bitonic_desc(W* x, int n) {
  for (int size = 2; size <= n; size <<= 1) {
    for (int stride = size >> 1; stride > 0; stride >>= 1) {
      __syncthreads();
      for (int i = threadIdx.x; i < (n >> 1); i += kTB) {
        const int lo = 2 * i - (i & (stride - 1));
        const int hi = lo + stride;
        const bool first_half = (lo & size) == 0;  // this run is sorted descending, its sibling ascending
        const W a = x[lo], b = x[hi];
        if ((a < b) == first_half) {
          x[lo] = b;
          x[hi] = a;
        }
      }
    }
  }
  __syncthreads();
}

__device__ __forceinline__ int block_sum_i(int v, int* red) {
  v = wave_sum_int(v);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  int t = 0;
#pragma unroll
  for (int w = 0; w < kTB / kWave; ++w) t += red[w];
  __syncthreads();
  return t;
}

// exclusive prefix over threads (in thread order) of a per-thread count, plus the block total
__device__ __forceinline__ int block_excl_scan(int v, int* red, int& total) {
  const int lane = threadIdx.x & 63, wid = threadIdx.x >> 6;
  int incl = v;
#pragma unroll
  for (int off = 1; off < kWave; off <<= 1) {
    const int o = __shfl_up(incl, off, kWave);
    if (lane >= off) incl += o;
  }
  if (lane == kWave - 1) red[wid] = incl;
  __syncthreads();
  int base = 0, tot = 0;
#pragma unroll
  for (int w = 0; w < kTB / kWave; ++w) {
    if (w < wid) base += red[w];
    tot += red[w];
  }
  __syncthreads();
  total = tot;
  return base + incl - v;
}

struct TopkArgs {
  const uint16_t* t;
  const uint8_t* mask;
  int32_t* idx;
  float* val;
  int64_t stride;
  int32_t V, k, nvec, log_probs;
};

// two workgroups per CU (8 waves per SIMD): one streams while the other sorts
__global__ __launch_bounds__(kTB, 8) void teacher_topk_kernel(const TopkArgs a) {
  __shared__ unsigned long long cand[kCandCap];
  __shared__ uint32_t mx[kTB];
  __shared__ int red[kTB / kWave];
  __shared__ float fred[kTB / kWave];
  __shared__ int ncand;
  const int tid = threadIdx.x;
  const int64_t row = blockIdx.x;
  const int V = a.V, k = a.k, nvec = a.nvec;
  int32_t* irow = a.idx + row * (int64_t)k;
  float* vrow = a.val + row * (int64_t)k;

  if (a.mask && !a.mask[row]) {  // not scored: a harmless record (valid ids, zero values)
    for (int j = tid; j < k; j += kTB) {
      irow[j] = j;
      vrow[j] = 0.0f;
    }
    return;
  }
  const uint16_t* trow = a.t + row * a.stride;
  const uint4* tvec = reinterpret_cast<const uint4*>(trow);

  // ---- pass A: one maximum per thread
  uint32_t best = 0;  // below every key of a finite value
#pragma unroll 4
  for (int i = tid; i < nvec; i += kTB) {
    uint32_t kk[8];
    keys8(tvec[i], kk);
#pragma unroll
    for (int j = 0; j < 8; ++j) best = kk[j] > best ? kk[j] : best;
  }
  for (int e = nvec * 8 + tid; e < V; e += kTB) {
    const uint32_t kk = key_of(trow[e]);
    best = kk > best ? kk : best;
  }
  mx[tid] = best;
  if (tid == 0) ncand = 0;
  bitonic_desc(mx, kTB);
  // at least k elements are >= L (k threads hold one each); every larger bound could miss one
  const uint32_t L = k <= kTB ? mx[k - 1] : 0u;

  // ---- pass B: everything >= L becomes a candidate
  bool slow = k > kTB;  // uniform
  if (!slow) {
#pragma unroll 4
    for (int i = tid; i < nvec; i += kTB) {
      uint32_t kk[8];
      keys8(tvec[i], kk);
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        if (kk[j] >= L) {
          const int pos = atomicAdd(&ncand, 1);
          if (pos < kCandCap) cand[pos] = cand_word(kk[j], (uint32_t)(i * 8 + j));
        }
      }
    }
    for (int e = nvec * 8 + tid; e < V; e += kTB) {
      const uint32_t kk = key_of(trow[e]);
      if (kk >= L) {
        const int pos = atomicAdd(&ncand, 1);
        if (pos < kCandCap) cand[pos] = cand_word(kk, (uint32_t)e);
      }
    }
    __syncthreads();
    slow = ncand > kCandCap;
  }
  int n = ncand;
  __syncthreads();

  if (slow) {
    // ---- exact slow path.  Tk = the largest key with count(key >= Tk) >= k, by bisection over 16 bits.
    uint32_t lo = 0, hi = 0x10000u;  // invariant: count(>= lo) >= k, count(>= hi) < k
    while (hi - lo > 1) {
      const uint32_t mid = (lo + hi) >> 1;
      int c = 0;
      for (int i = tid; i < nvec; i += kTB) {
        uint32_t kk[8];
        keys8(tvec[i], kk);
#pragma unroll
        for (int j = 0; j < 8; ++j) c += kk[j] >= mid;
      }
      for (int e = nvec * 8 + tid; e < V; e += kTB) c += key_of(trow[e]) >= mid;
      c = block_sum_i(c, red);
      if (c >= k)
        lo = mid;
      else
        hi = mid;
    }
    const uint32_t Tk = lo;
    if (tid == 0) ncand = 0;
    __syncthreads();
    // every element above Tk is in (fewer than k of them); count them on the way
    int above = 0;
    for (int i = tid; i < nvec; i += kTB) {
      uint32_t kk[8];
      keys8(tvec[i], kk);
#pragma unroll
      for (int j = 0; j < 8; ++j)
        if (kk[j] > Tk) {
          ++above;
          const int pos = atomicAdd(&ncand, 1);  // fewer than k <= 4096 by the choice of Tk
          if (pos < kCandCap) cand[pos] = cand_word(kk[j], (uint32_t)(i * 8 + j));
        }
    }
    for (int e = nvec * 8 + tid; e < V; e += kTB) {
      const uint32_t kk = key_of(trow[e]);
      if (kk > Tk) {
        ++above;
        const int pos = atomicAdd(&ncand, 1);
        if (pos < kCandCap) cand[pos] = cand_word(kk, (uint32_t)e);
      }
    }
    above = block_sum_i(above, red);
    const int need = k - above;  // ties at Tk to take, lowest ids first (>= 1)
    // ties in id order: chunk after chunk, each thread owning consecutive ids inside a chunk
    int taken = 0;  // uniform
    for (int c0 = 0; c0 < nvec && taken < need; c0 += kTB) {
      const int i = c0 + tid;
      uint32_t kk[8];
      int mine = 0;
      if (i < nvec) {
        keys8(tvec[i], kk);
#pragma unroll
        for (int j = 0; j < 8; ++j) mine += kk[j] == Tk;
      }
      int total;
      int rank = taken + block_excl_scan(mine, red, total);
      if (i < nvec) {
#pragma unroll
        for (int j = 0; j < 8; ++j)
          if (kk[j] == Tk) {
            if (rank < need) cand[above + rank] = cand_word(Tk, (uint32_t)(i * 8 + j));
            ++rank;
          }
      }
      taken += total;
    }
    for (int e0 = nvec * 8; e0 < V && taken < need; e0 += kTB) {
      const int e = e0 + tid;
      const int mine = e < V && key_of(trow[e]) == Tk;
      int total;
      const int rank = taken + block_excl_scan(mine, red, total);
      if (mine && rank < need) cand[above + rank] = cand_word(Tk, (uint32_t)e);
      taken += total;
    }
    __syncthreads();
    n = k;
  }

  // ---- order the candidates and cut at k
  int P = 1;
  while (P < n) P <<= 1;
  for (int i = n + tid; i < P; i += kTB) cand[i] = 0ull;  // below every real candidate
  bitonic_desc(cand, P);

  float lse = 0.0f;
  if (a.log_probs) {  // log-softmax over the k selected logits; the first one is the largest
    const float v0 = value_of_key((uint32_t)(cand[0] >> 32));
    float part = 0.0f;
    for (int j = tid; j < k; j += kTB) part += __expf(value_of_key((uint32_t)(cand[j] >> 32)) - v0);
    part = block_sum<kTB>(part, fred);
    lse = v0 + __logf(part);
  }
  for (int j = tid; j < k; j += kTB) {
    const unsigned long long w = cand[j];
    irow[j] = (int32_t)(0xffffffffu - (uint32_t)w);
    vrow[j] = value_of_key((uint32_t)(w >> 32)) - lse;
  }
}

hipError_t launch_teacher_topk(int64_t T, int32_t V, int64_t stride, int32_t k, int log_probs, const uint16_t* t,
                               const uint8_t* mask, int32_t* idx, float* val, hipStream_t stream) {
  TopkArgs a;
  a.t = t;
  a.mask = mask;
  a.idx = idx;
  a.val = val;
  a.stride = stride;
  a.V = V;
  a.k = k;
  a.nvec = ((reinterpret_cast<uintptr_t>(t) & 15u) == 0 && stride % 8 == 0) ? V / 8 : 0;
  a.log_probs = log_probs;
  hipLaunchKernelGGL(teacher_topk_kernel, dim3((unsigned)T), dim3(kTB), 0, stream, a);
  return hipGetLastError();
}

}  // namespace npd
