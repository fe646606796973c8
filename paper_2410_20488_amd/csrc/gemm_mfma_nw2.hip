// Instantiation of the projection kernel for workgroups of 2 waves (64 rows of W).
#include "gemm_mfma_kernel.h"
namespace firp {
FIRP_GEMM_INSTANTIATE(2)
}  // namespace firp
