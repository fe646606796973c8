// Instantiation of the projection kernel for workgroups of 5 waves (160 rows of W).
#include "gemm_mfma_kernel.h"
namespace firp {
FIRP_GEMM_INSTANTIATE(5)
}  // namespace firp
