// Instantiation of the projection kernel for workgroups of 6 waves (192 rows of W).
#include "gemm_mfma_kernel.h"
namespace firp {
FIRP_GEMM_INSTANTIATE(6)
}  // namespace firp
