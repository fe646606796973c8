// Instantiation of the projection kernel for workgroups of 7 waves (224 rows of W).
#include "gemm_mfma_kernel.h"
namespace firp {
FIRP_GEMM_INSTANTIATE(7)
}  // namespace firp
