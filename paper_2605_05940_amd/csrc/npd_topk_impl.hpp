// Implementation of the teacher-side top-k kernels, compiled once per configuration: the including translation unit
// defines NPD_TOPK_NS (namespace of this configuration), NPD_TOPK_TB (threads per workgroup, 512 or 1024),
// NPD_TOPK_CAND (candidate capacity per row), NPD_TOPK_WINDOW / NPD_TOPK_SAMPLE (register window of the one-read
// kernel and the part of it that gives the bound) and NPD_TOPK_ANY_SHAPE (1: also the kernel for unaligned or short
// rows).  See npd_topk_kernels.hip for the method.
#include "npd_device.hpp"
#include "npd_internal.hpp"

namespace npd {
namespace NPD_TOPK_NS {

constexpr int kTB = NPD_TOPK_TB;          // threads per workgroup
constexpr int kCandCap = NPD_TOPK_CAND;   // candidates staged per row (8 bytes each)
static_assert(kTB == 512 || kTB == 1024, "workgroups of 8 or 16 waves");
static_assert((kCandCap & (kCandCap - 1)) == 0 && kCandCap >= 2 * kTB, "the bitonic fallback pads the list to a power of two");

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


struct TopkShared {
  unsigned long long cand[kCandCap];
  unsigned long long shortlist[kTB];  // the candidates at or above the k-th key, when cand is long
  unsigned long long sorted[kTB];     // rank-sorted short lists
  int rank[kTB];
  int hist[2][256];
  int nshort;
#if NPD_TOPK_ANY_SHAPE
  uint32_t mx[kTB];
#endif
  int red[kTB / kWave];
  float fred[kTB / kWave];
  int wave_bound[kTB / kWave];
  int ncand;
};

// not scored: a harmless record (valid ids, zero values)
__device__ __forceinline__ void write_unscored(const TopkArgs& a, int64_t row, int tid) {
  int32_t* irow = a.idx + row * (int64_t)a.k;
  float* vrow = a.val + row * (int64_t)a.k;
  for (int j = tid; j < a.k; j += kTB) {
    irow[j] = j;
    vrow[j] = 0.0f;
  }
}

// Exact selection for any row, by counting passes over global memory.  Called by all threads; leaves the k
// selected words in sh.cand[0..k) (unordered) behind a barrier.
__device__ __forceinline__ void slow_select(const uint16_t* trow, int nvec, int V, int k, TopkShared& sh,
                                            int tid) {
  const uint4* tvec = reinterpret_cast<const uint4*>(trow);
  unsigned long long* cand = sh.cand;
  // Tk = the largest key with count(key >= Tk) >= k, by bisection over 16 bits.
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
    c = block_sum_i(c, sh.red);
    if (c >= k)
      lo = mid;
    else
      hi = mid;
  }
  const uint32_t Tk = lo;
  if (tid == 0) sh.ncand = 0;
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
        const int pos = atomicAdd(&sh.ncand, 1);  // fewer than k <= 4096 by the choice of Tk
        if (pos < kCandCap) cand[pos] = cand_word(kk[j], (uint32_t)(i * 8 + j));
      }
  }
  for (int e = nvec * 8 + tid; e < V; e += kTB) {
    const uint32_t kk = key_of(trow[e]);
    if (kk > Tk) {
      ++above;
      const int pos = atomicAdd(&sh.ncand, 1);
      if (pos < kCandCap) cand[pos] = cand_word(kk, (uint32_t)e);
    }
  }
  above = block_sum_i(above, sh.red);
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
    int rank = taken + block_excl_scan(mine, sh.red, total);
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
    const int rank = taken + block_excl_scan(mine, sh.red, total);
    if (mine && rank < need) cand[above + rank] = cand_word(Tk, (uint32_t)e);
    taken += total;
  }
  __syncthreads();
}

// The bin (counted from the top) in which the running count of a 256-bin histogram reaches k: returns the bin and,
// in `above`, the total of the bins above it.  Every wave computes it for itself from LDS; no barrier inside.
__device__ __forceinline__ int crossing_bin(const int* hist, int k, int& above) {
  const int lane = threadIdx.x & 63;
  const int h0 = hist[4 * lane], h1 = hist[4 * lane + 1], h2 = hist[4 * lane + 2], h3 = hist[4 * lane + 3];
  const int tot = h0 + h1 + h2 + h3;
  int sfx = tot;  // inclusive suffix sum over lanes: bins 4 lane .. 255
#pragma unroll
  for (int off = 1; off < kWave; off <<= 1) {
    const int o = __shfl_down(sfx, off, kWave);
    if (lane + off < kWave) sfx += o;
  }
  const unsigned long long reach = __ballot(sfx >= k);  // never empty: the whole histogram holds at least k
  const int ls = 63 - __builtin_clzll(reach | 1ull);
  int run = __shfl(sfx, ls, kWave) - __shfl(tot, ls, kWave);  // bins above lane ls
  const int b3 = __shfl(h3, ls, kWave), b2 = __shfl(h2, ls, kWave), b1 = __shfl(h1, ls, kWave);
  int bin = 4 * ls + 3;
  if (run + b3 < k) {
    run += b3;
    bin = 4 * ls + 2;
    if (run + b2 < k) {
      run += b2;
      bin = 4 * ls + 1;
      if (run + b1 < k) {
        run += b1;
        bin = 4 * ls;
      }
    }
  }
  above = run;
  return bin;
}

// rank sort of n <= 1024 distinct words from src into sh.sorted (only ranks below k are kept): the rank of a word
// is the number of larger words.  1024 threads split the n x n comparisons: thread (i, s) compares word i with
// segment s of the list; lanes of a wave read the same word (broadcast).
__device__ __forceinline__ void rank_sort(TopkShared& sh, const unsigned long long* src, int n, int k, int tid) {
  int lg = 0;
  while ((1 << lg) < n) ++lg;
  const int i = tid & ((1 << lg) - 1), seg = tid >> lg, nseg = kTB >> lg;
  const int chunk = (n + nseg - 1) / nseg;
  sh.rank[tid] = 0;
  __syncthreads();
  if (i < n) {
    const unsigned long long w = src[i];
    const int j1 = min(n, (seg + 1) * chunk);
    int c = 0;
    for (int j = seg * chunk; j < j1; ++j) c += src[j] > w;
    if (c) atomicAdd(&sh.rank[i], c);
  }
  __syncthreads();
  if (tid < n) {
    const int r = sh.rank[tid];
    if (r < k) sh.sorted[r] = src[tid];
  }
  __syncthreads();
}

constexpr int kDirectRankMax = 192;  // lists up to this length are rank-sorted as they are

// Orders the n >= k candidate words in sh.cand (all distinct: the ids differ) and writes the first k as the row's
// record.  Called by all threads after a barrier that made the candidates visible; ends with a barrier.
__device__ __forceinline__ void order_and_emit(TopkShared& sh, int n, int k, int log_probs, int32_t* irow,
                                               float* vrow, int tid) {
  const unsigned long long* out = nullptr;
  if (n <= kDirectRankMax) {
    rank_sort(sh, sh.cand, n, k, tid);
    out = sh.sorted;
  } else {
    // the k-th largest key Tk of the list by two 8-bit counting levels, then only the words >= Tk are ordered
    if (tid < 256) {
      sh.hist[0][tid] = 0;
      sh.hist[1][tid] = 0;
    }
    if (tid == 0) sh.nshort = 0;
    __syncthreads();
    for (int c = tid; c < n; c += kTB) atomicAdd(&sh.hist[0][(uint32_t)(sh.cand[c] >> 40) & 255u], 1);
    __syncthreads();
    int above_hi;
    const int hi = crossing_bin(sh.hist[0], k, above_hi);
    for (int c = tid; c < n; c += kTB) {
      const uint32_t key = (uint32_t)(sh.cand[c] >> 32);
      if ((int)(key >> 8) == hi) atomicAdd(&sh.hist[1][key & 255u], 1);
    }
    __syncthreads();
    int above_lo;
    const int lo = crossing_bin(sh.hist[1], k - above_hi, above_lo);
    const uint32_t Tk = ((uint32_t)hi << 8) | (uint32_t)lo;
    for (int c = tid; c < n; c += kTB) {
      const unsigned long long w = sh.cand[c];
      if ((uint32_t)(w >> 32) >= Tk) {
        const int pos = atomicAdd(&sh.nshort, 1);
        if (pos < kTB) sh.shortlist[pos] = w;
      }
    }
    __syncthreads();
    const int n2 = sh.nshort;  // >= k
    if (n2 <= kTB) {
      rank_sort(sh, sh.shortlist, n2, k, tid);
      out = sh.sorted;
    } else {  // a long run of equal keys at the cut: order the whole list
      int P = 1;
      while (P < n) P <<= 1;
      for (int i = n + tid; i < P; i += kTB) sh.cand[i] = 0ull;  // below every real candidate
      bitonic_desc(sh.cand, P);
      out = sh.cand;
    }
  }
  float lse = 0.0f;
  if (log_probs) {  // log-softmax over the k selected logits; the first one is the largest
    const float v0 = value_of_key((uint32_t)(out[0] >> 32));
    float part = 0.0f;
    for (int j = tid; j < k; j += kTB) part += __expf(value_of_key((uint32_t)(out[j] >> 32)) - v0);
    part = block_sum<kTB>(part, sh.fred);
    lse = v0 + __logf(part);
  }
  for (int j = tid; j < k; j += kTB) {
    const unsigned long long w = out[j];
    irow[j] = (int32_t)(0xffffffffu - (uint32_t)w);
    vrow[j] = value_of_key((uint32_t)(w >> 32)) - lse;
  }
  __syncthreads();
}

#if NPD_TOPK_ANY_SHAPE
// ------------------------------------------------------------------------------------------------ any shape
// two workgroups per CU (8 waves per SIMD): one streams while the other sorts
__global__ __launch_bounds__(kTB, 8) void teacher_topk_kernel(const TopkArgs a) {
  __shared__ TopkShared sh;
  const int tid = threadIdx.x;
  const int64_t row = blockIdx.x;
  const int V = a.V, k = a.k, nvec = a.nvec;
  if (a.mask && !a.mask[row]) {
    write_unscored(a, row, tid);
    return;
  }
  const uint16_t* trow = a.t + row * a.stride;
  const uint4* tvec = reinterpret_cast<const uint4*>(trow);

  // ---- one maximum per thread
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
  sh.mx[tid] = best;
  if (tid == 0) sh.ncand = 0;
  bitonic_desc(sh.mx, kTB);
  // at least k elements are >= L (k threads hold one each); every larger bound could miss one
  const uint32_t L = k <= kTB ? sh.mx[k - 1] : 0u;

  // ---- everything >= L becomes a candidate
  bool slow = k > kTB;  // uniform
  if (!slow) {
#pragma unroll 4
    for (int i = tid; i < nvec; i += kTB) {
      uint32_t kk[8];
      keys8(tvec[i], kk);
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        if (kk[j] >= L) {
          const int pos = atomicAdd(&sh.ncand, 1);
          if (pos < kCandCap) sh.cand[pos] = cand_word(kk[j], (uint32_t)(i * 8 + j));
        }
      }
    }
    for (int e = nvec * 8 + tid; e < V; e += kTB) {
      const uint32_t kk = key_of(trow[e]);
      if (kk >= L) {
        const int pos = atomicAdd(&sh.ncand, 1);
        if (pos < kCandCap) sh.cand[pos] = cand_word(kk, (uint32_t)e);
      }
    }
    __syncthreads();
    slow = sh.ncand > kCandCap;
  }
  int n = sh.ncand;
  __syncthreads();
  if (slow) {
    slow_select(trow, nvec, V, k, sh, tid);
    n = k;
  }
  order_and_emit(sh, n, k, a.log_probs, a.idx + row * (int64_t)k, a.val + row * (int64_t)k, tid);
}

#endif  // NPD_TOPK_ANY_SHAPE

// ------------------------------------------------------------------------------------------------ one read
typedef short short2v __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ short2v as_s2(uint32_t x) { return __builtin_bit_cast(short2v, x); }
__device__ __forceinline__ short2v pk_max(short2v a, short2v b) { return __builtin_elementwise_max(a, b); }
__device__ __forceinline__ short2v pk_min(short2v a, short2v b) { return __builtin_elementwise_min(a, b); }
// bf16 bit patterns (sign-magnitude) -> 16-bit two's complement integers in value order (an involution);
// -0 becomes -1, directly below +0
__device__ __forceinline__ uint32_t pk_ordered(uint32_t x) {
  const uint32_t sign = __builtin_bit_cast(uint32_t, as_s2(x) >> (short)15);
  return x ^ (sign & 0x7fff7fffu);
}
__device__ __forceinline__ int ordered_of(uint32_t b) {  // one pattern
  const int x = (int)(short)(uint16_t)b;
  return x < 0 ? (x ^ 0x7fff) : x;
}
// the 16-bit sort key of an ordered integer (the same keys as key_of: -0 is filed under +0)
__device__ __forceinline__ uint32_t key_of_ordered(int o) {
  const uint32_t key = ((uint32_t)o ^ 0x8000u) & 0xffffu;
  return key == 0x7fffu ? 0x8000u : key;
}

constexpr uint32_t kFillPair = 0xff80ff80u;  // two bf16 -inf: below every element, and never a candidate (id >= V)

// one 16-byte group of a row; 32-bit byte offsets keep the address in one VGPR next to the scalar row base
__device__ __forceinline__ u32x4 load_group(const uint16_t* trow, int i, int nvec) {
  u32x4 v = u32x4{kFillPair, kFillPair, kFillPair, kFillPair};
  const uint32_t off = (uint32_t)i * 16u;
  if (i < nvec) v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(reinterpret_cast<const char*>(trow) + off));
  return v;
}

__device__ __forceinline__ void append(TopkShared& sh, int o, int id) {
  const int pos = atomicAdd(&sh.ncand, 1);
  if (pos < kCandCap) sh.cand[pos] = cand_word(key_of_ordered(o), (uint32_t)id);
}

// candidates of one register group: elements whose ordered value is >= Lp.  With ORDERED = false the patterns are
// compared as they are, which is the same thing for Lp >= 1 (patterns of positive values are ordered integers,
// those of negative values are negative integers).
template <bool ORDERED>
__device__ __forceinline__ void collect_group(const u32x4& v, int i, int Lp, int nvec, TopkShared& sh) {
  uint32_t d[4] = {v.x, v.y, v.z, v.w};
  if (ORDERED) {
#pragma unroll
    for (int q = 0; q < 4; ++q) d[q] = pk_ordered(d[q]);
  }
  const short2v gm = pk_max(pk_max(as_s2(d[0]), as_s2(d[1])), pk_max(as_s2(d[2]), as_s2(d[3])));
  if (max((int)gm.x, (int)gm.y) >= Lp && i < nvec) {
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const short2v pr = as_s2(d[j >> 1]);
      const int o = (j & 1) ? (int)pr.y : (int)pr.x;
      if (o >= Lp) append(sh, o, i * 8 + j);
    }
  }
}

// W = register window (groups in flight per thread), S <= W = groups of the sample that gives the bound.
// ngroups = ceil(nvec / 1024) >= 1 groups are visited in the order (g * step) mod ngroups, step coprime to ngroups.
template <int W, int S>
__global__ __launch_bounds__(kTB, 8) void teacher_topk_stream_kernel(const TopkArgs a, int ngroups, int step) {
  __shared__ TopkShared sh;
  const int tid = threadIdx.x, lane = tid & 63, wid = tid >> 6;
  const int64_t row = blockIdx.x;
  const int V = a.V, k = a.k, nvec = a.nvec;
  if (a.mask && !a.mask[row]) {
    write_unscored(a, row, tid);
    return;
  }
  const uint16_t* trow = a.t + row * a.stride;
  auto vec_index = [&](int g) { return ((g * step) % ngroups) * kTB + tid; };

  u32x4 w[W];
#pragma unroll
  for (int j = 0; j < W; ++j) w[j] = load_group(trow, vec_index(j), j < ngroups ? nvec : 0);

  // ---- one maximum per thread over the sample, in value order: the largest non-negative pattern if there is one,
  // else the smallest negative pattern (sign-magnitude: the one closest to zero).  Group 0 is full (nvec >= 1024),
  // so every thread's maximum is an element of the row.
  short2v mx2 = as_s2(0x80008000u), mn2 = as_s2(0x7fff7fffu);
#pragma unroll
  for (int j = 0; j < S; ++j) {
    const uint32_t d[4] = {w[j].x, w[j].y, w[j].z, w[j].w};
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      mx2 = pk_max(mx2, as_s2(d[q]));
      mn2 = pk_min(mn2, as_s2(d[q]));
    }
  }
  const int hi = max((int)mx2.x, (int)mx2.y), lo = min((int)mn2.x, (int)mn2.y);
  const int best = hi >= 0 ? hi : (lo ^ 0x7fff);  // ordered integer of the thread's largest sample element

  bool slow = k > kTB;  // uniform
  if (!slow) {
    // each wave reports its m-th largest thread maximum (bisection on ballots); 16 m >= k elements of the row
    // are >= the smallest report
    const int m = (k + kTB / kWave - 1) / (kTB / kWave);
    int blo = -32768, bhi = 32768;  // count(best >= blo) >= m, count(best >= bhi) < m
    while (bhi - blo > 1) {
      const int mid = (blo + bhi) >> 1;
      if (__popcll(__ballot(best >= mid)) >= m)
        blo = mid;
      else
        bhi = mid;
    }
    if (lane == 0) sh.wave_bound[wid] = blo;
  }
  if (tid == 0) sh.ncand = 0;
  __syncthreads();

  if (!slow) {
    int L = sh.wave_bound[0];
#pragma unroll
    for (int q = 1; q < kTB / kWave; ++q) L = min(L, sh.wave_bound[q]);
    const int Lp = L == 0 ? -1 : L;  // +0 and -0 are one value
    // ---- the row streams through the window; every group is tested as it arrives and replaced by a later one
    for (int base = 0; base < ngroups; base += W) {
#pragma unroll
      for (int j = 0; j < W; ++j) {
        const int g = base + j;
        if (g < ngroups) {
          if (Lp >= 1)
            collect_group<false>(w[j], vec_index(g), Lp, nvec, sh);
          else
            collect_group<true>(w[j], vec_index(g), Lp, nvec, sh);
        }
        if (g + W < ngroups) w[j] = load_group(trow, vec_index(g + W), nvec);
      }
    }
    const int e = nvec * 8 + tid;  // the last V mod 8 elements
    if (e < V) {
      const int o = ordered_of(trow[e]);
      if (o >= Lp) append(sh, o, e);
    }
    __syncthreads();
    slow = sh.ncand > kCandCap;
  }
  int n = sh.ncand;
  __syncthreads();
  if (slow) {
    slow_select(trow, nvec, V, k, sh, tid);
    n = k;
  }
  order_and_emit(sh, n, k, a.log_probs, a.idx + row * (int64_t)k, a.val + row * (int64_t)k, tid);
}

static int gcd_int(int x, int y) {
  while (y) {
    const int r = x % y;
    x = y;
    y = r;
  }
  return x;
}

// one-read kernel of this configuration; a.nvec >= kTB (16-byte aligned rows)
hipError_t launch_stream(const TopkArgs& a, hipStream_t stream) {
  constexpr int kWindow = NPD_TOPK_WINDOW, kSample = NPD_TOPK_SAMPLE;
  const int ngroups = (a.nvec + kTB - 1) / kTB;
  // visiting order: the first kSample groups spread over the row
  int step = ngroups > kSample ? (ngroups + kSample - 1) / kSample : 1;
  while (gcd_int(step, ngroups) != 1) ++step;
  return launch_kernel(teacher_topk_stream_kernel<kWindow, kSample>, dim3((unsigned)a.T), dim3(kTB), 0, stream, a,
                       ngroups, step % ngroups == 0 ? 1 : step % ngroups);
}

#if NPD_TOPK_ANY_SHAPE
hipError_t launch_any(const TopkArgs& a, hipStream_t stream) {
  return launch_kernel(teacher_topk_kernel, dim3((unsigned)a.T), dim3(kTB), 0, stream, a);
}
#endif

}  // namespace NPD_TOPK_NS
}  // namespace npd
