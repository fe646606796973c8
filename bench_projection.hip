// Standalone timing of the weight-streaming projection kernel (no Python, no PyTorch): for
// each [n, K] shape it cycles through a pool of weight matrices larger than every cache, so
// that each launch streams its weights from HBM, and prints the average launch time and the
// weight bytes per second.  `--copy` instead runs a plain device-to-device copy kernel of a
// known size: the reference that scales the FETCH_SIZE / WRITE_SIZE counters of a
// `rocprofv3 --pmc` run of this program.
//
//   bench_projection [rows] [n K [S nw]]      e.g.  bench_projection 67   |   bench_projection 67 5120 13824
//   bench_projection --copy
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "kernels.h"

using namespace firp;

#define CK(x)                                                                   \
  do {                                                                          \
    hipError_t e_ = (x);                                                        \
    if (e_ != hipSuccess) {                                                     \
      printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__);     \
      exit(1);                                                                  \
    }                                                                           \
  } while (0)

__global__ void k_plain_copy(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) dst[i] = src[i];
}

__global__ void k_fill_bf16(unsigned short* p, size_t n, unsigned seed) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) {
    unsigned h = (unsigned)(i * 2654435761u) ^ seed;
    h ^= h >> 15; h *= 2246822519u; h ^= h >> 13;
    // small values around +-0.02 with a varied mantissa
    p[i] = (unsigned short)(0x3c00u | (h & 0x80ffu));
  }
}

int main(int argc, char** argv) {
  hipEvent_t e0, e1;
  CK(hipEventCreate(&e0));
  CK(hipEventCreate(&e1));
  if (argc > 1 && !strcmp(argv[1], "--copy")) {
    const size_t bytes = (size_t)1 << 30;
    uint4 *src, *dst;
    CK(hipMalloc(&src, bytes));
    CK(hipMalloc(&dst, bytes));
    CK(hipMemset(src, 1, bytes));
    for (int i = 0; i < 4; ++i) hipLaunchKernelGGL(k_plain_copy, dim3(4096), dim3(256), 0, 0, src, dst, bytes / 16);
    CK(hipDeviceSynchronize());
    printf("plain copy kernel: 4 launches, each reads %zu bytes and writes %zu bytes\n", bytes, bytes);
    return 0;
  }
  int rows = argc > 1 ? atoi(argv[1]) : 67;
  struct Shape { int n, K; };
  // the LLaMA-2-13B projections: q|k|v, o, gate|up, down, lm-head
  std::vector<Shape> shapes = {{15360, 5120}, {5120, 5120}, {27648, 5120}, {5120, 13824}, {32000, 5120}};
  if (argc > 3) shapes = {{atoi(argv[2]), atoi(argv[3])}};
  int force_s = argc > 4 ? atoi(argv[4]) : 0, force_nw = argc > 5 ? atoi(argv[5]) : 0;
  for (auto sh : shapes) {
    size_t wbytes = (size_t)sh.n * sh.K * 2;
    int cnt = (int)std::max<size_t>(2, (size_t)3.0e9 / wbytes);
    unsigned short* pool;
    CK(hipMalloc(&pool, wbytes * cnt));
    hipLaunchKernelGGL(k_fill_bf16, dim3(8192), dim3(256), 0, 0, pool, wbytes * cnt / 2, 17u);
    // the kernel streams the fragment-major copies
    const size_t pbytes = gemm_packed_bytes(sh.n, sh.K);
    char* packed;
    CK(hipMalloc(&packed, pbytes * cnt));
    for (int i = 0; i < cnt; ++i)
      launch_pack_weights(wseg1(pool + (size_t)i * (wbytes / 2), sh.n), sh.n, sh.K, packed + (size_t)i * pbytes, 0);
    CK(hipDeviceSynchronize());
    CK(hipFree(pool));
    int rp = (rows + 15) / 16 * 16;
    unsigned short *xh, *xl;
    CK(hipMalloc(&xh, (size_t)rp * sh.K * 2));
    CK(hipMalloc(&xl, (size_t)rp * sh.K * 2));
    hipLaunchKernelGGL(k_fill_bf16, dim3(512), dim3(256), 0, 0, xh, (size_t)rp * sh.K, 3u);
    hipLaunchKernelGGL(k_fill_bf16, dim3(512), dim3(256), 0, 0, xl, (size_t)rp * sh.K, 5u);
    GemmPlan plan = force_nw ? gemm_mfma_plan_ex(rows, sh.n, sh.K, force_s, force_nw) : gemm_mfma_plan(rows, sh.n, sh.K, force_s);
    float* part;
    CK(hipMalloc(&part, (size_t)plan.S * rp * sh.n * 4));
    Act a{};
    a.hi = (bf16*)xh;
    a.lo = (bf16*)xl;
    a.ld = sh.K;
    auto run = [&](int i) {
      launch_gemm_mfma(a, packed + (size_t)(i % cnt) * pbytes, part, sh.n, (size_t)rp * sh.n, rows, sh.n, sh.K, plan, 0);
    };
    for (int i = 0; i < cnt; ++i) run(i);
    CK(hipDeviceSynchronize());
    int iters = cnt * 3;
    CK(hipEventRecord(e0));
    for (int i = 0; i < iters; ++i) run(i);
    CK(hipEventRecord(e1));
    CK(hipEventSynchronize(e1));
    float ms;
    CK(hipEventElapsedTime(&ms, e0, e1));
    double us = ms * 1e3 / iters;
    printf("rows %3d n %6d K %6d  splits %2d waves/wg %d grid %3d : %7.1f us/launch  %6.0f GB/s of weights  (%.1f MB/launch)\n",
           rows, sh.n, sh.K, plan.S, plan.nw, plan.grid, us, wbytes / us / 1e3, wbytes / 1e6);
    fflush(stdout);
    CK(hipFree(packed));
    CK(hipFree(xh));
    CK(hipFree(xl));
    CK(hipFree(part));
  }
  return 0;
}
