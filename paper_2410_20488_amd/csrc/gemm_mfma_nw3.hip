// Instantiation of the projection kernel for workgroups of 3 waves (96 rows of W).
#include "gemm_mfma_kernel.h"
namespace firp {
FIRP_GEMM_INSTANTIATE(3)
}  // namespace firp
