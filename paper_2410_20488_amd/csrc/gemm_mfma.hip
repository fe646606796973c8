// Weight-streaming skinny projection for bf16 weights on gfx950.
//
//   out[s][r][c] = sum_{k in split s} X[r][k] * W[c][k],   r < rows <= 128,  c < n
//
// The step is bound by streaming W from HBM once, so the kernel is built around that stream:
//  * every wave owns 16*MT rows of W and reads them straight from global memory into the
//    A-operand layout of v_mfma_f32_16x16x32_bf16 (lane = (row % 16, k-block of 8)): four lanes
//    cover 64 contiguous bytes of a row and two loads cover a 128-byte line; loads for the
//    stage after next are in flight while the current one is multiplied;
//  * the activations are the small operand: a stage's [16*NT rows][64 k] tile of both planes
//    (hi and lo bf16, see Act) is staged once per workgroup through LDS (double-buffered, row
//    pitch 144 B so that 128-bit reads of 8 consecutive rows hit distinct banks) and shared by
//    the four waves;
//  * fp32 accumulation in the MFMA accumulators; rows of X beyond `rows` and rows of W beyond
//    `n` are read from clamped addresses and never stored;
//  * K is cut into S contiguous splits so that (n / rows-per-workgroup) * S workgroups fill
//    the 256 CUs; each split leaves its own partial sum, added up by the consumer kernel
//    (deterministic, no atomics).
#include <algorithm>

#include "kernels.h"

namespace firp {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));

namespace {
constexpr int KC = 64;       // k elements per stage
constexpr int PITCH = 144;   // bytes per LDS row: 128 data + 16 pad

__device__ __forceinline__ bf16x8_t as_bf16x8(u32x4_t v) { return __builtin_bit_cast(bf16x8_t, v); }
}  // namespace

template <int NT, int MT, bool KTAIL>
__global__ __launch_bounds__(256, 2) void k_gemm_mfma(const bf16* __restrict__ xhi, const bf16* __restrict__ xlo,
                                                      int ldx, int rows, const bf16* __restrict__ w, int n, int K,
                                                      float* __restrict__ out, int ld_out, size_t part_stride,
                                                      int S, int k_per) {
  constexpr int XROWS = NT * 16;
  constexpr int PLANE = XROWS * PITCH;
  __shared__ __attribute__((aligned(16))) unsigned char lds[2][2 * PLANE];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int split = blockIdx.x % S, tile = blockIdx.x / S;
  const int n0 = tile * (64 * MT) + wave * (16 * MT);
  const int k_begin = split * k_per;
  const int k_end = min(K, k_begin + k_per);
  const int nstages = (k_end - k_begin + KC - 1) / KC;
  const int r16 = lane & 15, kb = lane >> 4;

  // W: lane (r16, kb) reads 16 B at byte j*64 + kb*16 of each 128-byte stage of its row
  const char* wp[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    int row = min(n0 + mt * 16 + r16, n - 1);
    wp[mt] = (const char*)w + ((size_t)row * K + k_begin) * 2 + kb * 16;
  }
  // X: thread -> (plane, row within a 16-row tile, 16-byte chunk of the 128-byte stage row)
  const int xplane = tid >> 7, xrow = (tid & 127) >> 3, xchunk = tid & 7;
  const char* xp[NT];
#pragma unroll
  for (int i = 0; i < NT; ++i) {
    int row = min(i * 16 + xrow, rows - 1);
    xp[i] = (const char*)(xplane ? xlo : xhi) + ((size_t)row * ldx + k_begin) * 2 + xchunk * 16;
  }
  const int xlds = xplane * PLANE + xrow * PITCH + xchunk * 16;
  const int blds = r16 * PITCH + kb * 16;

  auto load_w = [&](u32x4_t (&a)[MT][2], int stage) {
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        if constexpr (KTAIL) {
          bool ok = k_begin + stage * KC + j * 32 + kb * 8 < k_end;
          a[mt][j] = ok ? *(const u32x4_t*)(wp[mt] + (size_t)stage * (KC * 2) + j * 64) : u32x4_t{0, 0, 0, 0};
        } else {
          a[mt][j] = *(const u32x4_t*)(wp[mt] + (size_t)stage * (KC * 2) + j * 64);
        }
      }
  };
  auto load_x = [&](u32x4_t (&x)[NT], int stage) {
#pragma unroll
    for (int i = 0; i < NT; ++i) {
      if constexpr (KTAIL) {
        bool ok = k_begin + stage * KC + xchunk * 8 < k_end;
        x[i] = ok ? *(const u32x4_t*)(xp[i] + (size_t)stage * (KC * 2)) : u32x4_t{0, 0, 0, 0};
      } else {
        x[i] = *(const u32x4_t*)(xp[i] + (size_t)stage * (KC * 2));
      }
    }
  };

  f32x4_t acc[MT][NT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) acc[mt][nt] = f32x4_t{0.f, 0.f, 0.f, 0.f};

  u32x4_t a0[MT][2], a1[MT][2], a2[MT][2], xr[NT];
  if (nstages > 0) {
    load_w(a0, 0);
    load_x(xr, 0);
  }
  if (nstages > 1) load_w(a1, 1);

  for (int st = 0; st < nstages; ++st) {
    unsigned char* buf = lds[st & 1];
#pragma unroll
    for (int i = 0; i < NT; ++i) *(u32x4_t*)(buf + xlds + i * 16 * PITCH) = xr[i];
    if (st + 1 < nstages) load_x(xr, st + 1);
    if (st + 2 < nstages) load_w(a2, st + 2);
    __syncthreads();
#pragma unroll
    for (int j = 0; j < 2; ++j) {
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        const unsigned char* bp = buf + blds + nt * 16 * PITCH + j * 64;
        bf16x8_t bh = as_bf16x8(*(const u32x4_t*)bp);
        bf16x8_t bl = as_bf16x8(*(const u32x4_t*)(bp + PLANE));
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
          acc[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(a0[mt][j]), bh, acc[mt][nt], 0, 0, 0);
          acc[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(a0[mt][j]), bl, acc[mt][nt], 0, 0, 0);
        }
      }
    }
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        a0[mt][j] = a1[mt][j];
        a1[mt][j] = a2[mt][j];
      }
  }

  // accumulator layout: lane holds C[w-row 4*(lane/16) + i][x-row lane%16], i = 0..3
  float* o = out + (size_t)split * part_stride;
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    int c = n0 + mt * 16 + 4 * kb;
    if (c >= n) continue;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      int r = nt * 16 + r16;
      if (r < rows) *(f32x4_t*)(o + (size_t)r * ld_out + c) = acc[mt][nt];
    }
  }
}

bool gemm_mfma_supported(int rows, int n, int K) {
  return rows >= 1 && n >= 4 && n % 4 == 0 && K >= 8 && K % 8 == 0;
}

GemmPlan gemm_mfma_plan(int rows, int n, int K, int force_split) {
  GemmPlan p{};
  int nt = (std::min(rows, 128) + 15) / 16;
  const int nts[] = {1, 2, 3, 4, 5, 6, 8};
  for (int c : nts)
    if (c >= nt) {
      nt = c;
      break;
    }
  p.nt = nt;
  int tiles = (n + 127) / 128;
  int stages = (K + KC - 1) / KC;
  int S = force_split;
  if (S <= 0) {
    // enough workgroups for two per CU, never more splits than 8 nor fewer than 4 stages each
    S = std::max(1, std::min({8, 512 / tiles, stages / 4}));
  }
  S = std::max(1, std::min(S, stages));
  int per = (stages + S - 1) / S;
  S = (stages + per - 1) / per;  // no empty split
  p.S = force_split > 0 ? force_split : S;
  p.k_per = per * KC;
  p.grid = tiles * p.S;
  return p;
}

template <int NT>
static void launch_nt(const bf16* xhi, const bf16* xlo, int ldx, int rows, const bf16* w, int n, int K, float* out,
                      int ld, size_t part_stride, const GemmPlan& p, hipStream_t s) {
  bool tail = (K % KC) != 0;
  dim3 g(p.grid), b(256);
  if (tail)
    hipLaunchKernelGGL((k_gemm_mfma<NT, 2, true>), g, b, 0, s, xhi, xlo, ldx, rows, w, n, K, out, ld, part_stride, p.S, p.k_per);
  else
    hipLaunchKernelGGL((k_gemm_mfma<NT, 2, false>), g, b, 0, s, xhi, xlo, ldx, rows, w, n, K, out, ld, part_stride, p.S, p.k_per);
}

void launch_gemm_mfma(const Act& x, const bf16* w, float* out, int ld, size_t part_stride, int rows, int n,
                      int K, const GemmPlan& plan, hipStream_t s) {
  // more than 128 rows: row blocks of 128 (W is streamed once per block)
  for (int r0 = 0; r0 < rows; r0 += 128) {
    int rb = std::min(128, rows - r0);
    GemmPlan p = plan;
    p.nt = gemm_mfma_plan(rb, n, K, plan.S).nt;
    const bf16* xhi = x.hi + (size_t)r0 * x.ld;
    const bf16* xlo = x.lo + (size_t)r0 * x.ld;
    float* o = out + (size_t)r0 * ld;
    switch (p.nt) {
      case 1: launch_nt<1>(xhi, xlo, x.ld, rb, w, n, K, o, ld, part_stride, p, s); break;
      case 2: launch_nt<2>(xhi, xlo, x.ld, rb, w, n, K, o, ld, part_stride, p, s); break;
      case 3: launch_nt<3>(xhi, xlo, x.ld, rb, w, n, K, o, ld, part_stride, p, s); break;
      case 4: launch_nt<4>(xhi, xlo, x.ld, rb, w, n, K, o, ld, part_stride, p, s); break;
      case 5: launch_nt<5>(xhi, xlo, x.ld, rb, w, n, K, o, ld, part_stride, p, s); break;
      case 6: launch_nt<6>(xhi, xlo, x.ld, rb, w, n, K, o, ld, part_stride, p, s); break;
      default: launch_nt<8>(xhi, xlo, x.ld, rb, w, n, K, o, ld, part_stride, p, s); break;
    }
  }
}

}  // namespace firp
