// Row-resident KD kernels, forward KL with gradient, 1024 threads per workgroup (rows above 131,072 entries).
#include "npd_kd_cached.hpp"

namespace npd {

template <int CS>
static hipError_t launch_forward(const KdArgs& a, int teacher_kind, hipStream_t stream) {
  constexpr int CSRF = kResidentGroupsForward < CS ? kResidentGroupsForward : CS;
  if (teacher_kind == kDense) return launch_cached_lse1<CS, CSRF, 9, kAhead, kDense, true>(a, stream);
  // top-k teacher: only the student row is dense; what does not fit the registers is parked in LDS, so the whole
  // row is on chip for the gradient sweep
  constexpr int TCSR = CS < kResidentGroupsTopk ? CS : kResidentGroupsTopk;
  constexpr int TCL = CS - TCSR < 9 ? CS - TCSR : 9;
  return launch_cached_lse1<CS, TCSR, TCL, 3, kTopk, true>(a, stream);
}

hipError_t launch_cached_forward_1024(const KdArgs& a, int cs, int teacher_kind, hipStream_t stream) {
  if (cs == 19) return launch_forward<19>(a, teacher_kind, stream);
  if (cs == 16) return launch_forward<16>(a, teacher_kind, stream);
  return hipErrorInvalidValue;  // shorter rows run with smaller workgroups
}

}  // namespace npd
