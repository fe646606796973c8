// Kernel template of the weight-streaming skinny projection for bf16 weights on gfx950.
//
//   out[s][r][c] = sum_{k in split s} X[r][k] * W[c][k],   r < rows <= 128,  c < n
//
// The step is bound by streaming W from HBM once, so the kernel is built around that stream:
//  * every wave owns 16*MT rows of W and reads them straight from global memory into the
//    A-operand layout of v_mfma_f32_16x16x32_bf16 (lane = (row % 16, k-block of 8)).  W is kept
//    in a fragment-major copy made once (see gemm_packed_bytes): a load instruction then covers
//    1 KiB of contiguous memory, eight whole cache lines, instead of 64-byte halves of sixteen
//    lines that a second instruction touches again while they are still on their way - the
//    vector cache tracks few outstanding lines per CU and stalls on exactly that pattern.
//    Loads for three stages ahead are in flight while the current one is multiplied;
//  * the activations are the small operand: a stage's [16*NT rows][64 k] tile of both planes
//    (hi and lo bf16, see Act) is staged once per workgroup through LDS (double-buffered,
//    128-byte rows with the 16-byte pieces XOR-swizzled by the row number) and shared by
//    the workgroup's waves;
//  * fp32 accumulation in the MFMA accumulators; rows of X beyond `rows` and rows of W beyond
//    `n` are read from clamped addresses and never stored;
//  * K is cut into S contiguous splits so that (n / rows-per-workgroup) * S workgroups fill
//    the 256 CUs; each split leaves its own partial sum, added up by the consumer kernel
//    (deterministic, no atomics).
#pragma once
#include <algorithm>

#include "kernels.h"

namespace firp {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));

namespace {
constexpr int KC = 64;       // k elements per stage
constexpr int PITCH = 128;   // bytes per LDS row of the X tile (64 columns); no padding, see below

__device__ __forceinline__ bf16x8_t as_bf16x8(u32x4_t v) { return __builtin_bit_cast(bf16x8_t, v); }
}  // namespace

template <int NT, int MT, bool KTAIL, int NW>
__global__ __launch_bounds__(64 * NW, 2) void k_gemm_mfma(const bf16* __restrict__ xhi, const bf16* __restrict__ xlo,
                                                      int ldx, int rows, const char* __restrict__ wpk, int n, int K,
                                                      float* __restrict__ out, int ld_out, size_t part_stride,
                                                      int S, int k_per, int tiles) {
  constexpr int XROWS = NT * 16;
  constexpr int PLANE = XROWS * PITCH;
  __shared__ __attribute__((aligned(16))) unsigned char lds[2][2 * PLANE];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int item = xcd_item(blockIdx.x, gridDim.x);
  if (item >= tiles * S) return;
  const int split = item / tiles, tile = item - split * tiles;
  const int n0 = tile * (NW * 16 * MT) + wave * (16 * MT);
  const int k_begin = split * k_per;
  const int k_end = min(K, k_begin + k_per);
  const int nstages = (k_end - k_begin + KC - 1) / KC;
  const int r16 = lane & 15, kb = lane >> 4;

  // W: fragment (16-row tile, 32-column step) = 1 KiB, lane's 16 B at byte 16 * lane
  const int kp32 = ((K + KC - 1) / KC) * 2;   // 32-column steps of a zero-padded row
  const int n16 = (n + 15) >> 4;
  const char* wp[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    const int t16 = min((n0 >> 4) + mt, n16 - 1);
    wp[mt] = wpk + ((size_t)t16 * kp32 + (k_begin >> 5)) * 1024 + lane * 16;
  }
  // X: the stage tile is 2 planes x XROWS rows x 8 chunks of 16 B; chunk id -> thread round-robin
  constexpr int XCHUNKS = 2 * XROWS * 8;
  constexpr int XP = (XCHUNKS + 64 * NW - 1) / (64 * NW);  // loads per thread per stage
  const char* xp[XP];
  int xlds[XP], xck[XP];
#pragma unroll
  for (int i = 0; i < XP; ++i) {
    int c = min(tid + i * 64 * NW, XCHUNKS - 1);   // the clamp makes surplus threads repeat a chunk
    int plane = c / (XROWS * 8), xrow = (c % (XROWS * 8)) >> 3;
    int row = min(xrow, rows - 1);
    xp[i] = (const char*)(plane ? xlo : xhi) + ((size_t)row * ldx + k_begin) * 2 + (c & 7) * 16;
    xlds[i] = plane * PLANE + xrow * PITCH + (((c & 7) ^ (xrow & 7)) * 16);
    xck[i] = c & 7;
  }
  // 16-byte piece p of row r sits at slot p ^ (r % 8) of the row: the fragment reads (16 rows x one
  // piece per k-block) and the staging writes (8 pieces of a row per 8 lanes) are both free of
  // bank conflicts, which padded rows are not (measured: 144-byte rows read at half the rate)
  const int blds = r16 * PITCH + ((kb ^ (r16 & 7)) * 16);

  // (the padding of the copy is zero, so the last stage of a ragged K needs no guard here)
  auto load_w = [&](u32x4_t (&a)[MT][2], int stage) {
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int j = 0; j < 2; ++j)
        a[mt][j] = __builtin_nontemporal_load((const u32x4_t*)(wp[mt] + (size_t)stage * 2048 + j * 1024));
  };
  auto load_x = [&](u32x4_t (&x)[XP], int stage) {
#pragma unroll
    for (int i = 0; i < XP; ++i) {
      if constexpr (KTAIL) {
        bool ok = k_begin + stage * KC + xck[i] * 8 < k_end;
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

  // Software pipeline.  Loads return in issue order, so waiting for the X tile of a stage also
  // waits for every W load issued before it; what stays in flight during that wait is what was
  // issued after it.  X therefore runs two stages ahead (two register sets) and W three (four
  // sets): while a wave waits for X(st) the W loads of stages st+2 and st+3 are still in
  // flight.  The body is unrolled four times so that the rotation costs no register moves, and
  // every load is unconditional (stages past the end are clamped to the last one and ignored)
  // so that the compiler's wait counters stay exact.
  constexpr int XAHEAD = 2;
  u32x4_t a0[MT][2], a1[MT][2], a2[MT][2], a3[MT][2], x0[XP], x1[XP];
  const int last = nstages - 1;
  if (nstages > 0) {
    load_x(x0, 0);
    load_w(a0, 0);
    load_x(x1, min(1, last));
    load_w(a1, min(1, last));
    load_w(a2, min(2, last));
  }

  auto stage = [&](u32x4_t (&cur)[MT][2], u32x4_t (&nxt3)[MT][2], u32x4_t (&xc)[XP], int st) {
    unsigned char* buf = lds[st & 1];
#pragma unroll
    for (int i = 0; i < XP; ++i) *(u32x4_t*)(buf + xlds[i]) = xc[i];
    load_x(xc, min(st + XAHEAD, last));
    __syncthreads();
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      if (j == 1) {
        // The W loads go out in the middle of the stage's products, not in front of the barrier:
        // the vector cache's queue is full most of the time, an issuing wave waits for room in
        // it, and here that wait overlaps with the other waves' products instead of holding up
        // the whole workgroup at the barrier (measured at 67 rows: 3-8 % per 13B projection).
        __builtin_amdgcn_sched_barrier(0);
        load_w(nxt3, min(st + 3, last));
        __builtin_amdgcn_sched_barrier(0);
      }
      bf16x8_t bh[NT], bl[NT];
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        const unsigned char* bp = buf + (blds ^ (j * 64)) + nt * 16 * PITCH;
        bh[nt] = as_bf16x8(*(const u32x4_t*)bp);
        bl[nt] = as_bf16x8(*(const u32x4_t*)(bp + PLANE));
      }
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
          acc[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(cur[mt][j]), bh[nt], acc[mt][nt], 0, 0, 0);
          acc[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(cur[mt][j]), bl[nt], acc[mt][nt], 0, 0, 0);
        }
      }
    }
  };

  int st = 0;
  for (; st + 4 <= nstages; st += 4) {
    stage(a0, a3, x0, st);
    stage(a1, a0, x1, st + 1);
    stage(a2, a1, x0, st + 2);
    stage(a3, a2, x1, st + 3);
  }
  if (st < nstages) stage(a0, a3, x0, st);
  if (st + 1 < nstages) stage(a1, a0, x1, st + 1);
  if (st + 2 < nstages) stage(a2, a1, x0, st + 2);

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


// One translation unit per workgroup size instantiates this for every activation tile count.
template <int NW>
void launch_gemm_mfma_nw(const bf16* xhi, const bf16* xlo, int ldx, int rows, const char* w, int n, int K, float* out,
                         int ld, size_t part_stride, const GemmPlan& p, hipStream_t s);

#define FIRP_GEMM_INSTANTIATE(NW)                                                                                     \
  template <int NT>                                                                                                   \
  static void launch_nt_(const bf16* xhi, const bf16* xlo, int ldx, int rows, const char* w, int n, int K, float* out,\
                         int ld, size_t part_stride, const GemmPlan& p, hipStream_t s) {                              \
    dim3 g((p.grid + 7) & ~7), b(64 * NW);                                                                            \
    if (K % KC)                                                                                                       \
      hipLaunchKernelGGL((k_gemm_mfma<NT, 2, true, NW>), g, b, 0, s, xhi, xlo, ldx, rows, w, n, K, out, ld,           \
                         part_stride, p.S, p.k_per, p.grid / p.S);                                                    \
    else                                                                                                              \
      hipLaunchKernelGGL((k_gemm_mfma<NT, 2, false, NW>), g, b, 0, s, xhi, xlo, ldx, rows, w, n, K, out, ld,          \
                         part_stride, p.S, p.k_per, p.grid / p.S);                                                    \
  }                                                                                                                   \
  template <>                                                                                                         \
  void launch_gemm_mfma_nw<NW>(const bf16* xhi, const bf16* xlo, int ldx, int rows, const char* w, int n, int K,      \
                               float* out, int ld, size_t part_stride, const GemmPlan& p, hipStream_t s) {            \
    switch (p.nt) {                                                                                                   \
      case 1: launch_nt_<1>(xhi, xlo, ldx, rows, w, n, K, out, ld, part_stride, p, s); break;                         \
      case 2: launch_nt_<2>(xhi, xlo, ldx, rows, w, n, K, out, ld, part_stride, p, s); break;                         \
      case 3: launch_nt_<3>(xhi, xlo, ldx, rows, w, n, K, out, ld, part_stride, p, s); break;                         \
      case 4: launch_nt_<4>(xhi, xlo, ldx, rows, w, n, K, out, ld, part_stride, p, s); break;                         \
      case 5: launch_nt_<5>(xhi, xlo, ldx, rows, w, n, K, out, ld, part_stride, p, s); break;                         \
      case 6: launch_nt_<6>(xhi, xlo, ldx, rows, w, n, K, out, ld, part_stride, p, s); break;                         \
      default: launch_nt_<8>(xhi, xlo, ldx, rows, w, n, K, out, ld, part_stride, p, s); break;                        \
    }                                                                                                                 \
  }

}  // namespace firp
