// Streaming kernels that do no arithmetic: what this GPU's memory system delivers to the access mixes of the KD
// kernels (read only; write only; one read + one write; two reads + one write), in two orders: the one those kernels
// use -- one workgroup per row of 16-byte groups, a thread owns every THREADS-th group, several loads in flight per
// thread -- and, for comparison, plain address order (one short-lived workgroup per THREADS consecutive groups), which
// a kernel that must reduce over a row before it can write cannot produce.  Their rates are what the KD kernels'
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

}  // extern "C"
