// Plain LDS-tiled projection y[rows][n] = x[rows][K] . W[n][K]^T in fp32 arithmetic.
// It serves fp32 models (the small correctness configuration) and is the selectable plain
// path for bf16 models; the weight-streaming MFMA kernel is in gemm_mfma.hip.
#include "kernels.h"

namespace firp {

template <typename WT>
__global__ __launch_bounds__(256) void k_gemm_simple(const float* __restrict__ x, int ldx,
                                                     const WT* __restrict__ w, float* __restrict__ y,
                                                     int ldy, int rows, int n, int K) {
  constexpr int BM = 64, BN = 64, BK = 16;
  __shared__ float xs[BK][BM + 4];
  __shared__ float ws[BK][BN + 4];
  int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
  int r0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < K; k0 += BK) {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      int idx = tid + e * 256;  // 0..1023
      int m = idx >> 4, kk = idx & 15;
      int r = r0 + m, c = n0 + m, k = k0 + kk;
      xs[kk][m] = (r < rows && k < K) ? x[(size_t)r * ldx + k] : 0.f;
      ws[kk][m] = (c < n && k < K) ? to_f32(w[(size_t)c * K + k]) : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < BK; ++kk) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = xs[kk][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) b[j] = ws[kk][tx * 4 + j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] += a[i] * b[j];
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    int r = r0 + ty * 4 + i;
    if (r >= rows) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int c = n0 + tx * 4 + j;
      if (c < n) y[(size_t)r * ldy + c] = acc[i][j];
    }
  }
}

void launch_gemm_simple(const float* x, int ldx, const void* w, int dtype, float* y, int ldy,
                        int rows, int n, int K, hipStream_t s) {
  dim3 g((n + 63) / 64, (rows + 63) / 64), b(256);
  if (dtype == DT_BF16)
    hipLaunchKernelGGL(k_gemm_simple<bf16>, g, b, 0, s, x, ldx, (const bf16*)w, y, ldy, rows, n, K);
  else
    hipLaunchKernelGGL(k_gemm_simple<float>, g, b, 0, s, x, ldx, (const float*)w, y, ldy, rows, n, K);
}

}  // namespace firp
