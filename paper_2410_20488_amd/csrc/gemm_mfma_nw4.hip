// Instantiation of the projection kernel for workgroups of 4 waves (128 rows of W).
#include "gemm_mfma_kernel.h"
namespace firp {
FIRP_GEMM_INSTANTIATE(4)
}  // namespace firp
