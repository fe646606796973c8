// Plain projections y[rows][n] = x[rows][K] . W[n][K]^T in fp32 arithmetic: an LDS-tiled kernel
// for any row count and, for the up to 16 rows of a small decoding step, one wave per output
// column.  They serve fp32 models (the small correctness configuration) and are the selectable
// plain path for bf16 models; the weight-streaming MFMA kernel is in gemm_mfma.hip.
#include <cstdint>

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

// Up to 16 rows: one wave per column of y.  A lane takes four consecutive k of its column's
// weight row per round (the wave 256) and multiplies them with the same k of every row of x
// (a few KB, cache hits); the rows' sums are then added across the wave in a fixed order.
// K % 4 == 0, ldx % 4 == 0.
__device__ __forceinline__ float4 load4(const float* p) { return *(const float4*)p; }
__device__ __forceinline__ float4 load4(const bf16* p) {
  const uint2 v = *(const uint2*)p;
  return make_float4(__uint_as_float(v.x << 16), __uint_as_float(v.x & 0xffff0000u), __uint_as_float(v.y << 16),
                     __uint_as_float(v.y & 0xffff0000u));
}

template <typename WT>
__global__ __launch_bounds__(256) void k_gemm_skinny(const float* __restrict__ x, int ldx, const WT* __restrict__ w,
                                                     float* __restrict__ y, int ldy, int rows, int n, int K) {
  const int lane = threadIdx.x & 63, c = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (c >= n) return;
  float acc[16];
#pragma unroll
  for (int r = 0; r < 16; ++r) acc[r] = 0.f;
  const WT* wr = w + (size_t)c * K;
  for (int k = lane * 4; k < K; k += 256) {
    const float4 a = load4(wr + k);
#pragma unroll
    for (int r = 0; r < 16; ++r)
      if (r < rows) {
        const float4 b = *(const float4*)(x + (size_t)r * ldx + k);
        acc[r] += a.x * b.x + a.y * b.y + a.z * b.z + a.w * b.w;
      }
  }
#pragma unroll
  for (int r = 0; r < 16; ++r)
    if (r < rows) {
      const float t = wave_sum(acc[r]);
      if (lane == 0) y[(size_t)r * ldy + c] = t;
    }
}

void launch_gemm_simple(const float* x, int ldx, const void* w, int dtype, float* y, int ldy,
                        int rows, int n, int K, hipStream_t s) {
  const bool aligned = ((uintptr_t)x & 15) == 0 && ((uintptr_t)w & 15) == 0;
  if (rows <= 16 && K % 4 == 0 && ldx % 4 == 0 && aligned) {
    dim3 gs((n + 3) / 4), bs(256);
    if (dtype == DT_BF16)
      hipLaunchKernelGGL(k_gemm_skinny<bf16>, gs, bs, 0, s, x, ldx, (const bf16*)w, y, ldy, rows, n, K);
    else
      hipLaunchKernelGGL(k_gemm_skinny<float>, gs, bs, 0, s, x, ldx, (const float*)w, y, ldy, rows, n, K);
    return;
  }
  dim3 g((n + 63) / 64, (rows + 63) / 64), b(256);
  if (dtype == DT_BF16)
    hipLaunchKernelGGL(k_gemm_simple<bf16>, g, b, 0, s, x, ldx, (const bf16*)w, y, ldy, rows, n, K);
  else
    hipLaunchKernelGGL(k_gemm_simple<float>, g, b, 0, s, x, ldx, (const float*)w, y, ldy, rows, n, K);
}

}  // namespace firp
