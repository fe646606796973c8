// The projection for 129..256 activation rows in one pass over W.
//
//   out[s][r][c] = sum_{k in split s} X[r][k] * W[c][k],   r < rows <= 256,  c < n,  K % 64 == 0
//
// Same operands and the same result layout as the weight-streaming kernel (gemm_mfma_kernel.h):
// W in the fragment-major copy, X as hi/lo bf16 planes, split-K partial sums.  With this many
// rows the step is no longer bound by the HBM stream of W alone: per byte of W a workgroup also
// pulls the X tile through the CU's vector cache (which keeps only about 80 lines in flight,
// whether they come from HBM or from L2) and reads the activation fragments from LDS (which
// delivers 128-bit reads at full rate only from a conflict-free layout).  Both grow with rows / (rows of W per
// workgroup), and the LDS reads also with 1 / (rows of W per wave).  So:
//  * a workgroup of 8 waves owns 256 rows of W and up to 256 rows of X: the largest tile whose
//    accumulators (a quarter of a MiB) fit the register file with two waves per SIMD;
//  * the waves form a 4 x 2 grid: wave (wg, xg) multiplies 64 rows of W by half of the X rows, so
//    an activation fragment read from LDS feeds four MFMAs per plane instead of two;
//    (MW = 3 instead of 4 tiles of W per wave makes the workgroup's tile 192 rows of W: for
//    matrices whose 256-row tiles would leave a third of the CUs without work)
//  * W goes through LDS too (each fragment is used by two waves): a thread stages two 16-byte
//    pieces per 32-column half-stage in registers, three half-stages ahead; in LDS a fragment
//    keeps its 1 KiB lane order, so the reads are linear;
//  * X goes from global memory straight into LDS (global_load_lds, no staging registers: there
//    are none left), one 64-column stage ahead.  One instruction moves 8 rows x 128 B, whole
//    cache lines, into 1 KiB of LDS in lane order; the lane that lands at piece s of row r
//    fetches piece s ^ (r % 8) of that row, which keeps the 128-bit fragment reads of 8
//    consecutive rows on distinct banks without padding;
//  * LDS: two X stages (2 x 64 KiB at 256 rows) and two W half-stages (2 x 16 KiB) - all of it.
//    One barrier per half-stage.
#include <algorithm>
#include <type_traits>

#include "kernels.h"

namespace firp {

namespace {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));

__device__ __forceinline__ bf16x8_t as_bf16x8(u32x4_t v) { return __builtin_bit_cast(bf16x8_t, v); }

// One wave-wide direct load: lane L's 16 bytes at base + off[L] land at LDS byte lds + 16 L.
// Written as inline assembly on purpose: the compiler would make every later LDS access wait for
// a direct load it knows of (it cannot tell the LDS buffers apart), which would drain the weight
// loads in flight with it.  The waits for these loads are therefore explicit (wait_vmcnt).
__device__ __forceinline__ void load_to_lds_16(const void* base, unsigned off, unsigned lds) {
  // (one wait state between the scalar write of M0 and the instruction that reads it: the hazard
  // the compiler pads for in its own code and cannot see inside an asm statement)
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" : : "v"(off), "s"(base), "s"(lds) : "memory");
}

// Workgroup barrier after this wave's LDS writes have completed.  (Not __syncthreads(): no fence
// is needed beyond LDS, and the clobber keeps the compiler from moving memory accesses across.)
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" : : : "memory"); }

__device__ __forceinline__ unsigned lds_address(const void* p) {
  return (unsigned)(size_t)(const __attribute__((address_space(3))) unsigned char*)p;
}

// Wait until at most N vector-memory loads of this wave are outstanding.  Inline assembly with a
// memory clobber so that the compiler keeps the loads written before it before it: the count is
// only right for the program order as written.
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  asm volatile("s_waitcnt vmcnt(%0)" : : "n"(N) : "memory");
}

}  // namespace

// XT: 16-row activation tiles per wave (even); the workgroup takes 32 * XT rows of X.
// MW: 16-row tiles of W per wave (3 or 4); the workgroup takes 64 * MW rows of W.
template <int XT, int MW>
__global__ __launch_bounds__(512, 2) void k_gemm_tall(const bf16* __restrict__ xhi, const bf16* __restrict__ xlo, int ldx,
                                                      int rows, const char* __restrict__ wpk, int n, int K,
                                                      float* __restrict__ out, int ld_out, size_t part_stride, int S,
                                                      int k_per, int tiles) {
  constexpr int XR = 32 * XT;
  constexpr int XPLANE = XR * 128;   // one plane of a 64-column stage
  static_assert(XT % 2 == 0, "rows of the tile in units of 64");
  __shared__ __attribute__((aligned(1024))) unsigned char xb0[2 * XPLANE];
  __shared__ __attribute__((aligned(1024))) unsigned char xb1[2 * XPLANE];
  __shared__ __attribute__((aligned(1024))) unsigned char wb[2][16 * 1024];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);
  const int wg = wave & 3, xg = wave >> 2;
  const int item = xcd_item(blockIdx.x, gridDim.x);
  if (item >= tiles * S) return;
  const int split = item / tiles, tile = item - split * tiles;
  const int k_begin = split * k_per;
  const int k_end = min(K, k_begin + k_per);
  const int nstages = (k_end - k_begin) / 64;
  const int nh = 2 * nstages;   // 32-column half-stages
  const int r16 = lane & 15, kb = lane >> 4;

  // W: the tile's 4 MW fragments of a half-stage; this thread stages fragments wave and wave + 8
  // (with 12 fragments the waves 4..7 repeat fragment 11: every wave issues the same two loads,
  // and the repeated LDS writes store the same bytes).  Wave-uniform bases, one per-lane offset.
  constexpr int NF = 4 * MW;
  const int kp32 = (K / 64) * 2;
  const int n16 = (n + 15) >> 4;
  const char* wsrc[2];
  int wdst[2];
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int f = min(wave_u + 8 * i, NF - 1);
    const int t16 = min(tile * NF + f, n16 - 1);
    wsrc[i] = wpk + ((size_t)t16 * kp32 + (k_begin >> 5)) * 1024;
    wdst[i] = f * 1024 + lane * 16;
  }
  const unsigned woff = lane * 16;
  // X: a stage is 2 planes x XR/8 blocks of 8 rows x 128 B.  This wave moves blocks
  // wave + 8 j (j < XT/2) of both planes; its lane L fetches, for the row 8 (wave + 8 j) + L/8,
  // the piece (L % 8) ^ (L / 8): the same byte offset in both planes.
  const char* xbase[2] = {(const char*)xhi + (size_t)k_begin * 2, (const char*)xlo + (size_t)k_begin * 2};
  unsigned xoff[XT / 2];
#pragma unroll
  for (int j = 0; j < XT / 2; ++j) {
    const int row = min((tid >> 3) + 64 * j, rows - 1);
    xoff[j] = (unsigned)row * (unsigned)ldx * 2u + (unsigned)(((lane & 7) ^ (lane >> 3)) * 16);
  }

  auto load_w = [&](u32x4_t (&a)[2], int hs) {
#pragma unroll
    for (int i = 0; i < 2; ++i) a[i] = __builtin_nontemporal_load((const u32x4_t*)(wsrc[i] + (size_t)hs * 1024 + woff));
  };
  auto dma_x = [&](unsigned char* xbuf, int st) {
    const unsigned l0 = lds_address(xbuf) + wave_u * 1024;
#pragma unroll
    for (int i = 0; i < XT; ++i)
      load_to_lds_16(xbase[i & 1] + (size_t)st * 128, xoff[i >> 1], l0 + (i & 1) * XPLANE + (i >> 1) * 8192);
  };

  f32x4_t acc[MW][XT];
#pragma unroll
  for (int mt = 0; mt < MW; ++mt)
#pragma unroll
    for (int xt = 0; xt < XT; ++xt) acc[mt][xt] = f32x4_t{0.f, 0.f, 0.f, 0.f};

  // Every load is unconditional (half-stages past the end repeat the last one and are ignored) so
  // that the wait counters stay exact; W runs three half-stages ahead in four register sets, the
  // body is unrolled four times so that the rotation costs no moves.  The X stage st + 1 is
  // requested at the start of the second half of stage st (every wave has passed the barrier of
  // the first half by then, so nobody reads that buffer any more), before that half's W loads,
  // and must have landed before the barrier of the first half of stage st + 1.  Loads complete in
  // order and exactly two pairs of W loads are issued after it by then: "at most 4 outstanding"
  // means the X stage is in LDS.  The prologue issues its loads in the matching order.
  u32x4_t w0[2], w1[2], w2[2], w3[2];
  const int last = nstages - 1, lasth = nh - 1;
  if (nh > 0) {
    load_w(w0, 0);
    load_w(w1, min(1, lasth));
    dma_x(xb0, 0);
    load_w(w2, min(2, lasth));
  }
  const int arow = (wg * MW) * 1024 + lane * 16;
  // fragment reads: row 16 t + r16 is block 2 t + r16 / 8, line r16 % 8; piece (4 P + kb) ^ (r16 % 8)
  const int brow = xg * XT * 2048 + (r16 >> 3) * 1024 + (r16 & 7) * 128;
  const int bcol[2] = {((kb) ^ (r16 & 7)) * 16, ((4 + kb) ^ (r16 & 7)) * 16};

  auto half = [&](auto parity, unsigned char* xcur, unsigned char* xnext, u32x4_t (&cur)[2], u32x4_t (&nxt)[2], int hs,
                  bool live) {
    constexpr int P = decltype(parity)::value;
    unsigned char* wbuf = wb[P];
#pragma unroll
    for (int i = 0; i < 2; ++i) *(u32x4_t*)(wbuf + wdst[i]) = cur[i];
    if constexpr (P == 1) dma_x(xnext, min((hs >> 1) + 1, last));
    load_w(nxt, min(hs + 3, lasth));
    if constexpr (P == 0) wait_vmcnt<4>();
    lds_barrier();
    if (!live) return;   // a half-stage past the end: its loads, waits and barrier only (see below)
    bf16x8_t a[MW];
#pragma unroll
    for (int mt = 0; mt < MW; ++mt) a[mt] = as_bf16x8(*(const u32x4_t*)(wbuf + arow + mt * 1024));
#pragma unroll
    for (int xt = 0; xt < XT; ++xt) {
      const unsigned char* bp = xcur + brow + bcol[P] + xt * 2048;
      const bf16x8_t bh = as_bf16x8(*(const u32x4_t*)bp);
      const bf16x8_t bl = as_bf16x8(*(const u32x4_t*)(bp + XPLANE));
#pragma unroll
      for (int mt = 0; mt < MW; ++mt)
        acc[mt][xt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[mt], bh, acc[mt][xt], 0, 0, 0);
#pragma unroll
      for (int mt = 0; mt < MW; ++mt)
        acc[mt][xt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[mt], bl, acc[mt][xt], 0, 0, 0);
    }
  };

  std::integral_constant<int, 0> even;
  std::integral_constant<int, 1> odd;
  // The explicit waits count loads in program order, so every half-stage must issue exactly the
  // loads written here.  There is therefore no peeled tail (in one, the compiler drops the W loads
  // whose registers nobody reads any more, and "at most 4 outstanding" then no longer covers the
  // last X loads - seen as rare wrong values in the last rows of a tile): an odd stage count runs
  // one more stage of loads, waits and barriers without the multiplications.
  for (int hs = 0; hs < nh; hs += 4) {
    const bool live = hs + 2 < nh;   // nh is even
    half(even, xb0, xb1, w0, w3, hs, true);
    half(odd, xb0, xb1, w1, w0, hs + 1, true);
    half(even, xb1, xb0, w2, w1, hs + 2, live);
    half(odd, xb1, xb0, w3, w2, hs + 3, live);
  }
  wait_vmcnt<0>();   // nothing of this workgroup may still be on its way into LDS when it ends

  // accumulator layout: lane holds C[w-row 4*(lane/16) + i][x-row lane%16], i = 0..3
  float* o = out + (size_t)split * part_stride;
#pragma unroll
  for (int mt = 0; mt < MW; ++mt) {
    const int c = (tile * NF + wg * MW + mt) * 16 + 4 * kb;
    if (c >= n) continue;
#pragma unroll
    for (int xt = 0; xt < XT; ++xt) {
      const int r = (xg * XT + xt) * 16 + r16;
      if (r < rows) *(f32x4_t*)(o + (size_t)r * ld_out + c) = acc[mt][xt];
    }
  }
}

namespace {

template <int XT, int MW>
void launch_xt(const bf16* xhi, const bf16* xlo, int ldx, int rows, const char* w, int n, int K, float* out, int ld,
               size_t part_stride, const GemmPlan& p, hipStream_t s) {
  dim3 g((p.grid + 7) & ~7), b(512);
  hipLaunchKernelGGL((k_gemm_tall<XT, MW>), g, b, 0, s, xhi, xlo, ldx, rows, w, n, K, out, ld, part_stride, p.S, p.k_per,
                     p.grid / p.S);
}

}  // namespace

// 129 <= rows <= 256, K % 64 == 0; plan.nw is 8 or 6 (a workgroup owns 256 or 192 rows of W),
// plan.grid = tiles x S
void launch_gemm_tall(const bf16* xhi, const bf16* xlo, int ldx, int rows, const void* w_packed, int n, int K,
                      float* out, int ld, size_t part_stride, const GemmPlan& plan, hipStream_t s) {
  const char* w = (const char*)w_packed;
  if (plan.nw == 6) {
    if (rows <= 192) launch_xt<6, 3>(xhi, xlo, ldx, rows, w, n, K, out, ld, part_stride, plan, s);
    else launch_xt<8, 3>(xhi, xlo, ldx, rows, w, n, K, out, ld, part_stride, plan, s);
  } else {
    if (rows <= 192) launch_xt<6, 4>(xhi, xlo, ldx, rows, w, n, K, out, ld, part_stride, plan, s);
    else launch_xt<8, 4>(xhi, xlo, ldx, rows, w, n, K, out, ld, part_stride, plan, s);
  }
}

}  // namespace firp
