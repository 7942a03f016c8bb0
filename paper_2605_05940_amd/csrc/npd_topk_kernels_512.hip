// The one-read top-k kernel with 512-thread workgroups, four per CU, for small k (see npd_topk_kernels.hip).
// 2048 candidates per row keep a workgroup's LDS at 30 KB; rows that pass more take the exact slow path.
#define NPD_TOPK_NS topk512
#define NPD_TOPK_TB 512
#define NPD_TOPK_CAND 2048
#define NPD_TOPK_WINDOW 8
#define NPD_TOPK_SAMPLE 8
#define NPD_TOPK_ANY_SHAPE 0
#include "npd_topk_impl.hpp"
