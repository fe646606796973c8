// Instantiation of the projection kernel for workgroups of 8 waves (256 rows of W).
#include "gemm_mfma_kernel.h"
namespace firp {
FIRP_GEMM_INSTANTIATE(8)
}  // namespace firp
