// Teacher-side top-k record (Sec. 3.1, "record only the top-k logits"; Alg. 1, Phase 2): for every scored
// position the k vocabulary ids with the largest teacher logits, largest first, equal logits by increasing id,
// and their values (the logits, or their log-softmax over the k).  Exact selection, integer bookkeeping only.
//
// One workgroup per token row, several per CU so that one row's ordering phase overlaps the others' streaming
// (1024 threads, two per CU; for small k 512 threads, four per CU: npd_topk_kernels_512.hip).  Both kernels derive
// a lower bound L of the k-th largest logit from per-thread maxima, append every element >= L as a 64-bit
// (key, ~id) word to an LDS list, cut the list down to the k-th key with a two-level radix count when it is long,
// and order what is left by rank sort (bitonic sort for long tie lists).  Rows where more elements pass the bound
// than the list holds (massive ties, constant rows) and k beyond the workgroup size take an exact slow path: binary
// search of the k-th key by counting passes over the row, then the ties of lowest id are collected in id order with
// block-wide scans.
//
// teacher_topk_stream_kernel (16-byte aligned rows of at least 8192 elements) reads each row from HBM once: the
// 16-byte groups of a row are visited in a strided order, so that the first window of groups a thread loads (12 of
// the 19 groups of a 151,936-entry row with 1024 threads) samples the whole vocabulary range; the bound comes from
// that sample alone (the k-th largest of a subset never exceeds the k-th largest of the row), and the rest of the
// row streams through the same register window, compared as packed 16-bit integers.  teacher_topk_kernel (any
// shape) takes the bound from the whole row and reads it twice.
#define NPD_TOPK_NS topk1024
#define NPD_TOPK_TB 1024
#define NPD_TOPK_CAND kTopkMax  // 4096 candidates = 32 KB of LDS: also what the exact slow path leaves behind for any k
// Measured on MI355X, 32,768 x 151,936, k = 10 / 64 / 256: window 8 with a 4-group sample 1.72 / 2.04 / 2.77 ms,
// 8 with 8 1.62 / 1.80 / 2.48, 12 with 12 1.57 / 1.69 / 2.29 (a larger sample gives a tighter bound, hence fewer
// candidates to cut and order); 12 groups are what fits 64 VGPRs, i.e. two workgroups per CU.
#define NPD_TOPK_WINDOW 12
#define NPD_TOPK_SAMPLE 12
#define NPD_TOPK_ANY_SHAPE 1
#include "npd_topk_impl.hpp"

namespace npd {

namespace topk512 {
hipError_t launch_stream(const TopkArgs& a, hipStream_t stream);  // npd_topk_kernels_512.hip
}

// Small k (the paper's 5 .. 20, the benchmark's 64) runs with four 512-thread workgroups per CU: three rows stream
// while a fourth is in its ordering phase.  Measured on config 1's teacher logits (k = 10 / 64 / 256): 1024 threads
// 1.11 / 1.23 / 1.65 ms, 512 threads with an 8-group window 1.07 / 1.16 / 1.94 ms (with more candidates per row the
// smaller list capacity and the narrower sample cost more than the overlap brings).
constexpr int kSmallK = 128;

hipError_t launch_teacher_topk(int64_t T, int32_t V, int64_t stride, int32_t k, int log_probs, const uint16_t* t,
                               const uint8_t* mask, int32_t* idx, float* val, hipStream_t stream) {
  TopkArgs a;
  a.t = t;
  a.mask = mask;
  a.idx = idx;
  a.val = val;
  a.stride = stride;
  a.T = T;
  a.V = V;
  a.k = k;
  const bool aligned = (reinterpret_cast<uintptr_t>(t) & 15u) == 0 && stride % 8 == 0;
  a.nvec = aligned ? V / 8 : 0;
  a.log_probs = log_probs;
  if (a.nvec >= 1024) return k <= kSmallK ? topk512::launch_stream(a, stream) : topk1024::launch_stream(a, stream);
  return topk1024::launch_any(a, stream);
}

}  // namespace npd
