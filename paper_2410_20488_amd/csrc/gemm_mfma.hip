// MFMA weight-streaming projection (placeholder until the kernel lands).
#include "kernels.h"
namespace firp {
bool gemm_mfma_supported(int, int, int) { return false; }
GemmPlan gemm_mfma_plan(int, int, int, int) { return GemmPlan{1, 0, 0, 0}; }
void launch_gemm_mfma(const Act&, const bf16*, float*, int, size_t, int, int, int, const GemmPlan&, hipStream_t) {}
}  // namespace firp
