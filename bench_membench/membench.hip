// Streaming kernels that do no arithmetic: what this GPU's memory system delivers to the access mixes of the KD
// kernels (read only; write only; one read + one write; two reads + one write), in two orders: the one those kernels
// use -- one workgroup per row of 16-byte groups, a thread owns every THREADS-th group, several loads in flight per
// thread -- and, for comparison, plain address order (one short-lived workgroup per THREADS consecutive groups), which
// a kernel that must reduce over a row before it can write cannot produce -- unless several workgroups share a row: the
// row-gang pattern (npd_membench_gang) is the order of the row-gang KD kernels.  Their rates are what the KD kernels'
// roofline fractions are read against; they are a measurement aid, not part of the loss path, and live in a library
// of their own (libnpd_membench.so).
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

enum Pattern { kRead1 = 0, kRead2 = 1, kWrite = 2, kCopy = 3, kRead2Write1 = 4, kRowRead2ThenWrite1 = 5, kPatterns = 6 };
constexpr int kRowGroupsPerThread = 19;  // the row-at-a-time pattern holds a row of up to 19 groups per thread in registers

template <bool NT>
__device__ __forceinline__ u32x4 ld(const u32x4* p) {
  return NT ? __builtin_nontemporal_load(p) : *p;
}
template <bool NT>
__device__ __forceinline__ void st(u32x4* p, u32x4 v) {
  if (NT)
    __builtin_nontemporal_store(v, p);
  else
    *p = v;
}

// UNROLL groups per thread are requested before the first is used.  Read-only patterns fold what they read into
// one word and store it only if it has a value the inputs cannot produce, so the loads cannot be dropped.
template <int PATTERN, int THREADS, int UNROLL, bool NT>
__global__ __launch_bounds__(THREADS) void stream_rows_kernel(const u32x4* __restrict__ a,
                                                              const u32x4* __restrict__ b, u32x4* __restrict__ o,
                                                              int row_groups, uint32_t never) {
  const size_t base = (size_t)blockIdx.x * (size_t)row_groups;
  const int tid = threadIdx.x;
  u32x4 fold = {0, 0, 0, 0};
  for (int g0 = tid; g0 < row_groups; g0 += THREADS * UNROLL) {
    u32x4 va[UNROLL], vb[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
      const int g = g0 + u * THREADS;
      va[u] = vb[u] = u32x4{0, 0, 0, 0};
      if (g < row_groups) {
        if (PATTERN != kWrite) va[u] = ld<NT>(a + base + g);
        if (PATTERN == kRead2 || PATTERN == kRead2Write1) vb[u] = ld<NT>(b + base + g);
      }
    }
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
      const int g = g0 + u * THREADS;
      const u32x4 v = va[u] ^ vb[u];
      if (PATTERN == kRead1 || PATTERN == kRead2)
        fold ^= v;
      else if (g < row_groups)
        st<NT>(o + base + g, v);
    }
  }
  if (PATTERN == kRead1 || PATTERN == kRead2)
    if ((fold.x ^ fold.y ^ fold.z ^ fold.w) == never) o[base + tid % row_groups] = fold;
}

// Address order: workgroup i handles groups [i * THREADS, (i + 1) * THREADS), one per thread, and ends.
template <int PATTERN, int THREADS, bool NT>
__global__ __launch_bounds__(THREADS) void stream_flat_kernel(const u32x4* __restrict__ a, const u32x4* __restrict__ b,
                                                              u32x4* __restrict__ o, size_t n, uint32_t never) {
  const size_t i = (size_t)blockIdx.x * THREADS + threadIdx.x;
  if (i >= n) return;
  u32x4 v = {0, 0, 0, 0};
  if (PATTERN != kWrite) v = ld<NT>(a + i);
  if (PATTERN == kRead2 || PATTERN == kRead2Write1) v ^= ld<NT>(b + i);
  if (PATTERN == kRead1 || PATTERN == kRead2) {
    if ((v.x ^ v.y ^ v.z ^ v.w) == never) o[i] = v;
  } else {
    st<NT>(o + i, v);
  }
}

// Two reads + one write, a row at a time: a workgroup first requests its whole row from both arrays (up to 19 groups
// per thread, combined in registers), then writes the whole row, last group first -- the read burst / write burst
// shape of a kernel that keeps a row on chip between its two sweeps.
template <int THREADS, bool NT>
__global__ __launch_bounds__(THREADS) void row_then_write_kernel(const u32x4* __restrict__ a,
                                                                 const u32x4* __restrict__ b, u32x4* __restrict__ o,
                                                                 int row_groups) {
  const size_t base = (size_t)blockIdx.x * (size_t)row_groups;
  const int tid = threadIdx.x;
  u32x4 r[kRowGroupsPerThread];
#pragma unroll
  for (int it = 0; it < kRowGroupsPerThread; ++it) {
    const int g = it * THREADS + tid;
    r[it] = u32x4{0, 0, 0, 0};
    if (g < row_groups) r[it] = ld<NT>(a + base + g) ^ ld<NT>(b + base + g);
  }
#pragma unroll
  for (int it = kRowGroupsPerThread - 1; it >= 0; --it) {
    const int g = it * THREADS + tid;
    if (g < row_groups) st<NT>(o + base + g, r[it]);
  }
}

// Two reads + one write by row gangs: a row is shared by `gang` short-lived workgroups of 256 threads, consecutive
// workgroups are consecutive slices of a row; each reads its slice of both inputs into registers (K groups per thread
// and array, kept apart as a kernel that needs both values would), posts six words to a scratch record, waits (a
// bounded number of polls) until all slices of its row have posted, and then writes its slice -- the access order of
// the row-gang KD kernels without their arithmetic.  Posted words carry their own validity: the record is cleared to
// kGangEmpty by gang_clear_kernel before each pass.
constexpr uint32_t kGangEmpty = 0xffffffffu;
constexpr int kGangWords = 8, kGangUsed = 6, kGangMax = 32, kGangK = 10;

__global__ __launch_bounds__(256) void gang_clear_kernel(uint32_t* p, size_t n) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) p[i] = kGangEmpty;
}

// READS = 1: one read + one write (the order of the row-gang kernel for a top-k teacher: array b is not touched, and
// with half the registers six workgroups run per compute unit instead of four).
template <int K, int READS>
__global__ __launch_bounds__(256, READS == 2 ? 4 : 6) void gang_rows_kernel(const u32x4* __restrict__ a, const u32x4* __restrict__ b,
                                                           u32x4* __restrict__ o, int row_groups, int slice_groups,
                                                           int gang, uint32_t* scratch, int spin_limit) {
  __shared__ uint32_t xch[kGangMax * kGangWords];
  __shared__ uint32_t red[4];
  const int row = blockIdx.x / gang, slice = blockIdx.x % gang, tid = threadIdx.x;
  const size_t base = (size_t)row * row_groups;
  const int g0 = slice * slice_groups;
  const int g1 = g0 + slice_groups < row_groups ? g0 + slice_groups : row_groups;
  u32x4 ra[K], rb[READS == 2 ? K : 1];
#pragma unroll
  for (int k = 0; k < K; ++k) {
    const int g = g0 + k * 256 + tid;
    ra[k] = u32x4{0, 0, 0, 0};
    if constexpr (READS == 2) rb[k] = u32x4{0, 0, 0, 0};
    if (g < g1) {
      ra[k] = __builtin_nontemporal_load(a + base + g);
      if constexpr (READS == 2) rb[k] = __builtin_nontemporal_load(b + base + g);
    }
  }
  uint32_t f = 0;  // something that depends on every load of the thread
#pragma unroll
  for (int k = 0; k < K; ++k) f ^= READS == 2 ? ra[k].x ^ rb[k].y : ra[k].x;
  for (int off = 32; off > 0; off >>= 1) f ^= __shfl_xor(f, off, 64);
  if ((tid & 63) == 0) red[tid >> 6] = f;
  __syncthreads();
  f = red[0] ^ red[1] ^ red[2] ^ red[3];
  if (tid < kGangUsed) {
    uint32_t w = f + tid;
    if (w == kGangEmpty) w = 0;
    __hip_atomic_store(scratch + ((size_t)blockIdx.x) * kGangWords + tid, w, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  for (int w = tid; w < gang * kGangUsed; w += 256) {
    const int s = w / kGangUsed, j = w - s * kGangUsed;
    const uint32_t* p = scratch + ((size_t)row * gang + s) * kGangWords + j;
    uint32_t v;
    int spins = 0;
    while ((v = __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) == kGangEmpty && ++spins <= spin_limit)
      __builtin_amdgcn_s_sleep(8);
    xch[s * kGangWords + j] = v;
  }
  __syncthreads();
  uint32_t mix = 0;
  for (int s = 0; s < gang; ++s) mix |= xch[s * kGangWords] & 0u;  // the stores depend on the exchange; adds nothing
#pragma unroll
  for (int k = K - 1; k >= 0; --k) {
    const int g = g0 + k * 256 + tid;
    u32x4 v = ra[k];
    if constexpr (READS == 2) v ^= rb[k];
    v.x ^= mix;
    if (g < g1) __builtin_nontemporal_store(v, o + base + g);
  }
}

template <int PATTERN, int THREADS, bool NT>
hipError_t launch(int order, const void* a, const void* b, void* o, int64_t rows, int row_groups,
                  hipStream_t stream) {
  if (order == 1) {
    const size_t n = (size_t)rows * (size_t)row_groups;
    const size_t blocks = (n + THREADS - 1) / THREADS;
    if (PATTERN == kRowRead2ThenWrite1 || blocks > 0x7fffffffu) return hipErrorInvalidValue;
    hipLaunchKernelGGL((stream_flat_kernel<PATTERN, THREADS, NT>), dim3((unsigned)blocks), dim3(THREADS), 0, stream,
                       static_cast<const u32x4*>(a), static_cast<const u32x4*>(b), static_cast<u32x4*>(o), n,
                       0x9e3779b9u);
    return hipGetLastError();
  }
  if (PATTERN == kRowRead2ThenWrite1) {
    if (row_groups > kRowGroupsPerThread * THREADS) return hipErrorInvalidValue;  // the row must fit the registers
    hipLaunchKernelGGL((row_then_write_kernel<THREADS, NT>), dim3((unsigned)rows), dim3(THREADS), 0, stream,
                       static_cast<const u32x4*>(a), static_cast<const u32x4*>(b), static_cast<u32x4*>(o), row_groups);
    return hipGetLastError();
  }
  hipLaunchKernelGGL((stream_rows_kernel<PATTERN, THREADS, 4, NT>), dim3((unsigned)rows), dim3(THREADS), 0, stream,
                     static_cast<const u32x4*>(a), static_cast<const u32x4*>(b), static_cast<u32x4*>(o), row_groups,
                     0x9e3779b9u);
  return hipGetLastError();
}

template <int PATTERN, int THREADS>
hipError_t launch_nt(int order, bool nt, const void* a, const void* b, void* o, int64_t rows, int row_groups,
                     hipStream_t stream) {
  return nt ? launch<PATTERN, THREADS, true>(order, a, b, o, rows, row_groups, stream)
            : launch<PATTERN, THREADS, false>(order, a, b, o, rows, row_groups, stream);
}

template <int PATTERN>
hipError_t launch_threads(int order, int threads, bool nt, const void* a, const void* b, void* o, int64_t rows,
                          int row_groups, hipStream_t stream) {
  switch (threads) {
    case 256: return launch_nt<PATTERN, 256>(order, nt, a, b, o, rows, row_groups, stream);
    case 512: return launch_nt<PATTERN, 512>(order, nt, a, b, o, rows, row_groups, stream);
    case 1024: return launch_nt<PATTERN, 1024>(order, nt, a, b, o, rows, row_groups, stream);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace

extern "C" {

// Number of access patterns: 0 read one array, 1 read two, 2 write one, 3 copy (1 read + 1 write), 4 two reads + one
// write (streaming), 5 two reads + one write a row at a time (whole row read, then whole row written; rows of at most
// 19 * threads groups).
int npd_membench_patterns(void) { return kPatterns; }

// Enqueues one pass of `pattern` over `rows` rows of `row_groups` 16-byte groups each (device arrays a, b, o of
// rows * row_groups * 16 bytes, 16-byte aligned; a pattern ignores the arrays it does not use, but all three must be
// valid) with `threads` in {256, 512, 1024} per workgroup; `order` 0 = one workgroup per row, 1 = address order (one
// workgroup per `threads` consecutive groups; not for pattern 5); `nontemporal` != 0 puts the non-temporal hint on
// every access.  Returns 0, or a hipError_t value (invalid arguments: nothing enqueued).
int npd_membench_run(int pattern, int order, int threads, int nontemporal, const void* a, const void* b, void* o,
                     int64_t rows, int32_t row_groups, void* stream) {
  if (!a || !b || !o || rows <= 0 || rows > 0x7fffffffLL || row_groups <= 0) return (int)hipErrorInvalidValue;
  if (order != 0 && order != 1) return (int)hipErrorInvalidValue;
  if (((uintptr_t)a | (uintptr_t)b | (uintptr_t)o) & 15u) return (int)hipErrorInvalidValue;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const bool nt = nontemporal != 0;
  switch (pattern) {
    case kRead1: return (int)launch_threads<kRead1>(order, threads, nt, a, b, o, rows, row_groups, s);
    case kRead2: return (int)launch_threads<kRead2>(order, threads, nt, a, b, o, rows, row_groups, s);
    case kWrite: return (int)launch_threads<kWrite>(order, threads, nt, a, b, o, rows, row_groups, s);
    case kCopy: return (int)launch_threads<kCopy>(order, threads, nt, a, b, o, rows, row_groups, s);
    case kRead2Write1: return (int)launch_threads<kRead2Write1>(order, threads, nt, a, b, o, rows, row_groups, s);
    case kRowRead2ThenWrite1: return (int)launch_threads<kRowRead2ThenWrite1>(order, threads, nt, a, b, o, rows, row_groups, s);
    default: return (int)hipErrorInvalidValue;
  }
}

// Bytes of scratch npd_membench_gang needs for `rows` rows of `row_groups` groups (0: the shape is not supported).
size_t npd_membench_gang_scratch_bytes(int64_t rows, int32_t row_groups) {
  if (rows <= 0 || row_groups <= 0) return 0;
  const int gang = (row_groups + kGangK * 256 - 1) / (kGangK * 256);
  if (gang > kGangMax || rows * gang > 0x7fffffffLL) return 0;
  return (size_t)rows * gang * kGangWords * sizeof(uint32_t);
}

// Enqueues one pass of the row-gang pattern (`reads` = 2: two reads + one write; 1: one read + one write, b is not
// touched; see gang_rows_kernel) over `rows` rows of `row_groups` 16-byte groups: device arrays a, b, o as in
// npd_membench_run, `scratch` a device buffer of npd_membench_gang_scratch_bytes() bytes.  Returns 0 or a hipError_t
// value (invalid arguments: nothing enqueued).
int npd_membench_gang(const void* a, const void* b, void* o, int64_t rows, int32_t row_groups, void* scratch,
                      int32_t reads, void* stream) {
  const size_t bytes = npd_membench_gang_scratch_bytes(rows, row_groups);
  if (!a || !b || !o || !scratch || bytes == 0 || (reads != 1 && reads != 2)) return (int)hipErrorInvalidValue;
  if (((uintptr_t)a | (uintptr_t)b | (uintptr_t)o | (uintptr_t)scratch) & 15u) return (int)hipErrorInvalidValue;
  const int gang = (row_groups + kGangK * 256 - 1) / (kGangK * 256);
  const int slice_groups = ((row_groups + gang - 1) / gang + 7) / 8 * 8;  // slices begin on 128-byte multiples of the row
  hipStream_t s = static_cast<hipStream_t>(stream);
  const size_t words = bytes / sizeof(uint32_t);
  hipLaunchKernelGGL(gang_clear_kernel, dim3((unsigned)((words + 255) / 256)), dim3(256), 0, s,
                     static_cast<uint32_t*>(scratch), words);
  if (reads == 2)
    hipLaunchKernelGGL((gang_rows_kernel<kGangK, 2>), dim3((unsigned)(rows * gang)), dim3(256), 0, s,
                       static_cast<const u32x4*>(a), static_cast<const u32x4*>(b), static_cast<u32x4*>(o), row_groups,
                       slice_groups, gang, static_cast<uint32_t*>(scratch), 1 << 20);
  else
    hipLaunchKernelGGL((gang_rows_kernel<kGangK, 1>), dim3((unsigned)(rows * gang)), dim3(256), 0, s,
                       static_cast<const u32x4*>(a), static_cast<const u32x4*>(b), static_cast<u32x4*>(o), row_groups,
                       slice_groups, gang, static_cast<uint32_t*>(scratch), 1 << 20);
  return (int)hipGetLastError();
}

}  // extern "C"
