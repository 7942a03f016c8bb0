// Row-resident KD kernels for the reverse KL and the skew forms (dense teacher, gradient), 512 threads per workgroup.
#include "npd_kd_cached.hpp"

namespace npd {

template <int CS>
static hipError_t launch_divergence(const KdArgs& a, hipStream_t stream) {
  constexpr int CB = 512;
  constexpr int CSR = kResidentGroups < CS ? kResidentGroups : CS;
  if (a.divergence == kReverseKl)
    return launch_cached_lse1<CS, CSR, 9, kAhead, kDense, true, kReverseKl, CB, true>(a, stream);
  if (a.divergence == kSkewKl)
    return launch_cached_lse1<CS, CSR, 9, kAhead, kDense, true, kSkewKl, CB, true>(a, stream);
  return launch_cached_lse1<CS, CSR, 9, kAhead, kDense, true, kSkewReverseKl, CB, true>(a, stream);
}

hipError_t launch_cached_divergence_512(const KdArgs& a, int cs, hipStream_t stream) {
  if (cs == 13) return launch_divergence<13>(a, stream);
  if (cs == 16) return launch_divergence<16>(a, stream);
  return launch_divergence<19>(a, stream);
}

}  // namespace npd
