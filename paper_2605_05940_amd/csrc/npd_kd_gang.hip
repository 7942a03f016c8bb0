// Row-gang KD kernels (npd_kd_gang.hpp): which calls they take, the scratch record they need, and the launch.
#include <atomic>

#include "npd_kd_gang.hpp"
#include "npd_kd_gang_topk.hpp"

namespace npd {

static std::atomic<int> g_spin_limit{kGangSpinLimitDefault};

int set_gang_spin_limit(int polls) {
  return g_spin_limit.exchange(polls > 0 ? polls : kGangSpinLimitDefault, std::memory_order_relaxed);
}

constexpr int kGangK = 10;      // 128-bit groups per thread and tensor: 80 of a thread's 128 registers hold its slice
constexpr int kGangTopkK = 10;  // top-k teacher: groups per thread of the student row alone
constexpr int kGangSkewK = 6;   // skew forms: the slice is kept as two fp32 values per element from sweep 2 on

static int gang_k(int teacher_kind, int divergence) {
  if (teacher_kind == kTopk) return kGangTopkK;
  return divergence == kSkewKl || divergence == kSkewReverseKl ? kGangSkewK : kGangK;
}

// Slices per row.  A workgroup holds up to k * 256 groups; slices are sized to 8 groups less, because a slice is moved
// by up to 7 groups so that it begins on a 128-byte boundary of memory (see launch_kd_gang).
// Rows of less than one and a half slices stay with one workgroup per row (1 is returned): two half-filled slices
// cost more in exchanges than the access order gains (dense teacher, % of the HBM peak, row gangs / one workgroup per
// row: V = 20,480 50 / 72, 24,576 67 / 74, 32,000 73 / 69, 50,304 77 / 69, 100,352 81 / 67).
// `on_lines`: every row of the launch begins on a 128-byte boundary, no boundary is ever moved and a slice may be as
// long as a workgroup holds (V = 102,400: 5 full slices instead of 6).
static int gang_size(int nvec, int k, bool on_lines) {
  const int cap = k * kGangThreads - 8;
  if (2 * nvec < 3 * cap) return 1;
  return on_lines ? (nvec + cap + 7) / (cap + 8) : (nvec + cap - 1) / cap;
}
static bool rows_on_lines(const KdArgs& a) {
  return a.g != nullptr && (reinterpret_cast<uintptr_t>(a.g) & 127u) == 0 && a.s_stride % 64 == 0;
}

// Gradient calls with a dense teacher (forward or reverse KL) or a top-k teacher (forward KL), 16-byte aligned rows
// that span at least two slices.  (The CE
// softmax of the composite loss has no temperature; this path covers it at tau = 1, where it shares the student's
// exponentials.)
bool gang_path_applies(const KdArgs& a, int teacher_kind, bool want_grad) {
  if ((teacher_kind != kDense && teacher_kind != kTopk) || !want_grad) return false;
  if (a.divergence != kForwardKl && teacher_kind != kDense) return false;
  if (a.cscale != 0.0f && a.need_lse1) return false;
  const int g = gang_size(a.nvec_s, gang_k(teacher_kind, a.divergence), rows_on_lines(a));
  if (g < 2 || g > kGangMax) return false;
  return a.T * (int64_t)g <= 0x7fffffffLL;  // one workgroup per slice, 1-D grid
}

size_t gang_workspace_bytes(int64_t T, int32_t V, int teacher_kind, int divergence, bool lse1) {
  const int g = gang_size(V / 8, gang_k(teacher_kind, divergence), false);  // (the larger of the two counts)
  if (g < 2 || T * (int64_t)g > 0x7fffffffLL) return 0;
  if (g > kGangMax && gang_size(V / 8, gang_k(teacher_kind, divergence), true) > kGangMax) return 0;
  return ((size_t)T * g * gang_words(lse1 ? 4 : 2) + kGangTailWords) * sizeof(uint32_t);
}

template <class Kernel>
static hipError_t launch_gang_kernel(const KdArgs& a, int words_per_slice, Kernel kernel, hipStream_t stream) {
  const size_t words = (size_t)a.T * a.gang * words_per_slice + kGangTailWords;
  const int64_t want = (int64_t)((words + 1023) / 1024);  // four words per thread
  const int64_t clear_grid = want < 8 * (int64_t)compute_units() ? want : 8 * (int64_t)compute_units();
  const hipError_t e = launch_kernel(gang_clear_kernel, dim3((unsigned)clear_grid), dim3(256), 0, stream, a.ws, words);
  if (e != hipSuccess) return e;
  return launch_kernel(kernel, dim3((unsigned)(a.T * a.gang)), dim3(kGangThreads), 0, stream, a);
}

template <bool LSE1, int DIVK>
static hipError_t launch_gang(const KdArgs& a, hipStream_t stream) {
  constexpr int K = DIVK == kSkewKl || DIVK == kSkewReverseKl ? kGangSkewK : kGangK;
  return launch_gang_kernel(a, gang_words(LSE1 ? 4 : 2), kd_gang_kernel<K, kDense, LSE1, DIVK>, stream);
}

hipError_t launch_kd_gang(const KdArgs& a0, int teacher_kind, hipStream_t stream) {
  KdArgs a = a0;
  a.gang = gang_size(a.nvec_s, gang_k(teacher_kind, a.divergence), rows_on_lines(a));
  // Slices are multiples of 8 groups = 128 bytes long, and the kernels move every boundary inside a row down to the
  // next 128-byte boundary of the gradient row's address (by 0 .. 7 groups: a row whose pitch is not a multiple of 128
  // bytes begins anywhere): no cache line is then shared by two workgroups of a row -- measured +2.4 points of the HBM
  // peak on config 1, +2.5 on config 4, +3.6 on config 2; a row pitch of 16 bytes more than config 1's: +4.
  a.gang_groups = ((a.nvec_s + a.gang - 1) / a.gang + 7) / 8 * 8;
  a.gang_pow2 = 1;
  while (a.gang_pow2 < a.gang) a.gang_pow2 *= 2;
  a.spin_limit = g_spin_limit.load(std::memory_order_relaxed);
  if (teacher_kind == kTopk) {
    if (a.need_lse1) return launch_gang_kernel(a, 8, kd_gang_topk_kernel<kGangTopkK, true>, stream);
    return launch_gang_kernel(a, 8, kd_gang_topk_kernel<kGangTopkK, false>, stream);
  }
  if (a.divergence == kReverseKl)
    return a.need_lse1 ? launch_gang<true, kReverseKl>(a, stream) : launch_gang<false, kReverseKl>(a, stream);
  if (a.divergence == kSkewKl)
    return a.need_lse1 ? launch_gang<true, kSkewKl>(a, stream) : launch_gang<false, kSkewKl>(a, stream);
  if (a.divergence == kSkewReverseKl)
    return a.need_lse1 ? launch_gang<true, kSkewReverseKl>(a, stream) : launch_gang<false, kSkewReverseKl>(a, stream);
  return a.need_lse1 ? launch_gang<true, kForwardKl>(a, stream) : launch_gang<false, kForwardKl>(a, stream);
}

}  // namespace npd
