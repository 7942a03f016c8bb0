// Forward-only calls (scoring passes, monitors): the pipelined kernel with nothing kept on chip, 256 / 512 / 1024
// threads per workgroup.
#include "npd_kd_cached.hpp"

namespace npd {

template <int CB>
static hipError_t launch_forward_only(const KdArgs& a, int teacher_kind, hipStream_t stream) {
  switch (teacher_kind) {
    case kDense: return launch_cached_lse1<19, 0, 0, 4, kDense, false, kForwardKl, CB, true>(a, stream);
    case kTopk: return launch_cached_lse1<19, 0, 0, 4, kTopk, false, kForwardKl, CB, true>(a, stream);
    default: return launch_cached_lse1<19, 0, 0, 4, kNone, false, kForwardKl, CB, true>(a, stream);
  }
}

hipError_t launch_cached_forward_only(const KdArgs& a, int threads, int teacher_kind, hipStream_t stream) {
  switch (threads) {
    case 256: return launch_forward_only<256>(a, teacher_kind, stream);
    case 512: return launch_forward_only<512>(a, teacher_kind, stream);
    default: return launch_forward_only<1024>(a, teacher_kind, stream);
  }
}

}  // namespace npd
