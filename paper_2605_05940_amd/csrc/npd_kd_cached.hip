// Row-resident KD kernels: which shape runs a call (threads per workgroup, unrolled length), and the dispatch to the
// translation units that hold the instantiations.
#include <atomic>

#include "npd_kd_cached.hpp"

namespace npd {

// compute units of the current device (queried once per device, no allocation)
int compute_units() {
  static std::atomic<int> cached[64];  // zero-initialised; callers on several host threads may race to fill a slot
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
  int n = cached[dev].load(std::memory_order_relaxed);
  if (n == 0) {
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
    cached[dev].store(n, std::memory_order_relaxed);
  }
  return n;
}

// Groups per thread that the unrolled part of the kernel covers.  19 fits vocabularies of 147,464 .. 155,648
// tokens entirely (larger ones stream the remainder twice); 16 and 13 do the same for the gradient kernels at
// ~131k and ~104k tokens.  A row must have more than (CS - 1) * 1024 groups for the CS variant.
static int unrolled_groups(const KdArgs& a, bool want_grad) {
  const int nit = (a.nvec_s + kCB - 1) / kCB;
  if (nit >= 19) return 19;
  if (want_grad && nit >= 16) return 16;
  if (want_grad && nit >= 13) return 13;
  return 0;
}

// Workgroup size and unrolled length of the gradient kernels (measured with the forward KL).  Measured on MI355X (32,768 unmasked rows,
// % of 8 TB/s, 1024 / 512 / 256 threads per workgroup): dense teacher V = 81,920: 59 / 71 / 64, 100,352: 59 / 69 /
// 63, 128,256: 64 / 67 / 61, 151,936: 64 / 64 / 57, 200,000: 64 / 63 / 50, 262,144: 58 / 57 / 51; top-k teacher
// 128,256: 54 / 68 / 61, 151,936: 56 / 62 / 59, 262,144: 54 / 65 / 59.  Two 512-thread workgroups per CU overlap
// one row's reductions and sweep turn-around with the other row's streaming, at the price of half the on-chip
// share per row; rows above 131,072 entries are better off with the whole CU (with a top-k teacher only on the
// packed batch with contiguous masked spans and tau = 2 that the benchmark times: 3.36 against 3.48 ms).  Rows of
// 8,192 .. 40,959 entries run with 256 threads (four workgroups per CU).
struct RowShape {
  int cb, cs;
};
static RowShape forward_grad_shape(const KdArgs& a, int teacher_kind) {
  const int nvec = a.nvec_s;
  if (nvec < 1024) return {0, 0};
  int cb = 256;
  if (nvec > 16384)
    cb = 1024;
  else if (nvec >= 5120)
    cb = 512;
  const int nit = (nvec + cb - 1) / cb;
  return {cb, nit <= 13 ? 13 : (nit <= 16 ? 16 : 19)};
}

// Forward-only calls (scoring passes, monitors) stream a row once through the same software pipeline, nothing is
// kept: threads per workgroup by row length.  Measured (32,768 rows, dense forward-only, % of 8 TB/s, 1024 / 512 /
// 256 threads): V = 32,000: 50 / 75 / 84, 65,536: 79 / 88 / 85, 100,352: 87 / 87 / 85, 128,256: 88 / 87 / 85,
// 151,936: 87 / 87 / 84, 262,144: 84 / 86 / 81.
constexpr int kForwardGroups256 = 5120;   // up to this many 128-bit groups per row: 256 threads
constexpr int kForwardGroups512 = 13000;  // up to this many: 512 threads; beyond: 1024
static int forward_only_threads(const KdArgs& a) {
  const int nvec = a.nvec_s;
  if (nvec < 1024) return 0;
  if (nvec <= kForwardGroups256) return 256;
  if (nvec <= kForwardGroups512) return 512;
  return 1024;
}

// Row-resident path: 16-byte aligned rows that are long enough.  (The CE softmax of the composite loss has no
// temperature; this path covers it at tau = 1, where it shares the student's exponentials.)
bool cached_path_applies(const KdArgs& a, int teacher_kind, bool want_grad) {
  const bool grad = want_grad && teacher_kind != kNone;
  if (a.divergence != kForwardKl && !grad) return false;  // the other divergences: gradient runs only
  if (a.cscale != 0.0f && a.need_lse1) return false;
  if (grad) return forward_grad_shape(a, teacher_kind).cb > 0;
  return forward_only_threads(a) > 0;
}

hipError_t launch_kd_cached(const KdArgs& a, int teacher_kind, bool want_grad, hipStream_t stream) {
  const bool grad = want_grad && teacher_kind != kNone;
  if (grad) {
    const RowShape sh = forward_grad_shape(a, teacher_kind);  // the same shapes for every divergence
    if (a.divergence == kForwardKl) {
      if (sh.cb == 512) return launch_cached_short_512(a, sh.cs, teacher_kind, stream);
      if (sh.cb == 256) return launch_cached_short_256(a, sh.cs, teacher_kind, stream);
      return launch_cached_forward_1024(a, unrolled_groups(a, true), teacher_kind, stream);  // 17 or more groups
    }
    if (sh.cb == 512) return launch_cached_divergence_512(a, sh.cs, stream);
    if (sh.cb == 256) return launch_cached_divergence_256(a, sh.cs, stream);
    return launch_cached_divergence_1024(a, unrolled_groups(a, true), stream);
  }
  return launch_cached_forward_only(a, forward_only_threads(a), teacher_kind, stream);
}

}  // namespace npd
