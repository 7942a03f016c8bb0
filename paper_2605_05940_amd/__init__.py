"""MI355X-native packed KD loss of Near-Policy Distillation: HIP kernels behind a C ABI (``libnpd.so``).

``binding`` holds the ctypes wrappers (same names as the C entry points); ``synth`` the seeded input
generators; ``build`` compiles the library.  Nothing here computes on the CPU.
"""
from .binding import (NpdError, npd_delta_ifd_score, npd_kd_loss_fwd_bwd, npd_policy_lag,  # noqa: F401
                      npd_segment_ppl, npd_segment_reduce, npd_teacher_topk, npd_workspace_bytes, version)
