// Row-resident KD kernels, forward KL with gradient, 256 threads per workgroup (see forward_grad_shape for the rows).
#include "npd_kd_cached.hpp"

namespace npd {

template <int CS>
static hipError_t launch_short(const KdArgs& a, int teacher_kind, hipStream_t stream) {
  constexpr int CB = 256;
  constexpr int CSR = kResidentGroups < CS ? kResidentGroups : CS;
  if (teacher_kind == kDense)
    return launch_cached_lse1<CS, CSR, 9, kAhead, kDense, true, kForwardKl, CB, true>(a, stream);
  constexpr int TCL = CS - CSR < 9 ? CS - CSR : 9;  // top-k teacher: the LDS parks student groups
  return launch_cached_lse1<CS, CSR, TCL, 3, kTopk, true, kForwardKl, CB, true>(a, stream);
}

hipError_t launch_cached_short_256(const KdArgs& a, int cs, int teacher_kind, hipStream_t stream) {
  if (cs == 13) return launch_short<13>(a, teacher_kind, stream);
  if (cs == 16) return launch_short<16>(a, teacher_kind, stream);
  return launch_short<19>(a, teacher_kind, stream);
}

}  // namespace npd
