// Planning and dispatch of the weight-streaming projection (kernel in gemm_mfma_kernel.h).
#include "gemm_mfma_kernel.h"

namespace firp {

// the kernel for 129..256 rows (gemm_tall.hip); takes K % 64 == 0 only
void launch_gemm_tall(const bf16* xhi, const bf16* xlo, int ldx, int rows, const void* w_packed, int n, int K,
                      float* out, int ld, size_t part_stride, const GemmPlan& plan, hipStream_t s);
static bool tall_shape(int rows, int K) { return rows > 128 && K % 64 == 0; }

bool gemm_mfma_supported(int rows, int n, int K) {
  return rows >= 1 && n >= 4 && n % 4 == 0 && K >= 8 && K % 8 == 0;
}

// activation tiles of one pass of the streaming kernel: up to 8 (128 rows)
static int pick_nt(int rows) {
  int nt = (std::min(rows, 128) + 15) / 16;
  const int nts[] = {1, 2, 3, 4, 5, 6, 8};
  for (int c : nts)
    if (c >= nt) return c;
  return 8;
}


GemmPlan gemm_mfma_plan_ex(int rows, int n, int K, int S, int nw) {
  GemmPlan p{};
  p.nt = pick_nt(rows);
  p.nw = nw;
  int tiles = (n + nw * 32 - 1) / (nw * 32);
  int stages = (K + KC - 1) / KC;
  int s_eff = std::max(1, std::min(S, stages));
  int per = (stages + s_eff - 1) / s_eff;
  p.S = S;  // splits past the end of K find no stage and leave zeros
  p.k_per = per * KC;
  p.grid = tiles * p.S;
  p.row_block = (tall_shape(rows, K) && (nw == 8 || nw == 6)) ? 256 : 128;
  return p;
}

// A CU moves data at a capped rate however many workgroups it holds (its vector cache keeps only
// so many lines in flight), so a launch is as fast as its busiest CU: the plan puts at most one
// workgroup on each of the 256 CUs and picks waves per workgroup (nw: 32 rows of W each) and
// split factor S by a model of that CU's time, in units of one 4 KiB stage of one wave's W:
//   stages per workgroup x (nw + 0.6 x activation tiles)   W from HBM, the X tile (4 KiB per 16 rows
//                                                          and stage) from L2 at 0.6 of that cost
//   + rows x nw / 32                                       the partial sums it writes
//   + 6 per stage short of 8                               a pipeline that never fills
//   + S x rows x n / 2^18                                  the consumer kernel reading the partial sums
// The constants come from launch times measured over (S, nw) at the LLaMA-2 7B and 13B shapes
// (e.g. 5120 x 5120 at 67 rows: 8 x 5 waves; 4096 x 11008: 16 x 8).  Few waves with many
// activation tiles are excluded: two waves cannot keep a CU's memory pipeline busy.
static double plan_cost(int rows, int n, int K, int S, int nw, int nt) {
  const int stages = (K + KC - 1) / KC;
  const int per = (stages + S - 1) / S;
  const int r = std::min(rows, 256);
  return per * (nw + 0.6 * nt) + r * nw / 32.0 + 6.0 * std::max(0, 8 - per)
         + (double)S * r * n / 262144.0;   // and the consumer reads every partial sum back (spread over 256 CUs)
}

GemmPlan gemm_mfma_plan(int rows, int n, int K, int force_split) {
  const int stages = (K + KC - 1) / KC;
  const int n_cu = 256;
  const bool tall = tall_shape(rows, K);   // the 8-wave kernel for 129..256 rows per pass
  const int nt = tall ? (std::min(rows, 256) + 15) / 16 : pick_nt(rows);
  const int nw_hi = 8, nw_lo = tall ? 6 : std::min(4, std::max(2, nt));
  int best_nw = nw_hi, best_S = std::max(1, force_split);
  double best = -1.0;
  for (int nw = nw_hi; nw >= nw_lo; --nw) {
    if (tall && nw == 7) continue;   // that kernel's workgroups own 256 or 192 rows of W
    int tiles = (n + nw * 32 - 1) / (nw * 32);
    int s_lo = force_split > 0 ? force_split : 1, s_hi = force_split > 0 ? force_split : 16;
    for (int S = s_lo; S <= s_hi; ++S) {
      if (force_split <= 0 && S > 1 && stages / S < 4) break;
      int grid = tiles * S;
      if (grid > n_cu && !(nw == nw_hi && S == s_lo)) continue;   // (the fallback: several rounds)
      double cost = (double)((grid + n_cu - 1) / n_cu) * plan_cost(rows, n, K, S, nw, nt);
      if (best < 0.0 || cost < best - 1e-9) {
        best = cost;
        best_nw = nw;
        best_S = S;
      }
    }
  }
  return gemm_mfma_plan_ex(rows, n, K, best_S, best_nw);
}

size_t gemm_packed_bytes(int n, int K) {
  return (size_t)((n + 15) / 16) * (size_t)(((K + KC - 1) / KC) * 2) * 1024;
}

// One thread per 16-byte piece of the fragment-major copy.
__global__ void k_pack_weights(WSeg src, int n, int K, int kp32, size_t pieces, uint4* __restrict__ dst) {
  size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= pieces) return;
  const int lane = (int)(idx & 63);
  const size_t frag = idx >> 6;
  const int t16 = (int)(frag / kp32), ks = (int)(frag % kp32);
  const int row = t16 * 16 + (lane & 15), k = ks * 32 + (lane >> 4) * 8;
  union {
    uint4 v;
    unsigned short e[8];
  } u;
  u.v = make_uint4(0, 0, 0, 0);
  if (row < n && k < K) {
    const bf16* r = row < src.n0 ? src.w0 + (size_t)row * K
                    : row < src.n0 + src.n1 ? src.w1 + (size_t)(row - src.n0) * K
                                            : src.w2 + (size_t)(row - src.n0 - src.n1) * K;
    if (k + 8 <= K && (K & 7) == 0) {
      u.v = *(const uint4*)(r + k);
    } else {
      for (int i = 0; i < 8 && k + i < K; ++i) u.e[i] = r[k + i].v;
    }
  }
  dst[idx] = u.v;
}

void launch_pack_weights(const WSeg& src, int n, int K, void* dst, hipStream_t s) {
  const int kp32 = ((K + KC - 1) / KC) * 2;
  const size_t pieces = gemm_packed_bytes(n, K) / 16;
  const unsigned blocks = (unsigned)((pieces + 255) / 256);
  hipLaunchKernelGGL(k_pack_weights, dim3(blocks), dim3(256), 0, s, src, n, K, kp32, pieces, (uint4*)dst);
}

void launch_gemm_mfma(const Act& x, const void* w_packed, float* out, int ld, size_t part_stride, int rows, int n,
                      int K, const GemmPlan& plan, hipStream_t s) {
  // more rows than one pass takes: row blocks (W is streamed once per block)
  const int block = plan.row_block;
  for (int r0 = 0; r0 < rows; r0 += block) {
    int rb = std::min(block, rows - r0);
    GemmPlan p = plan;
    p.nt = pick_nt(rb);
    const bf16* xhi = x.hi + (size_t)r0 * x.ld;
    const bf16* xlo = x.lo + (size_t)r0 * x.ld;
    float* o = out + (size_t)r0 * ld;
    const char* w = (const char*)w_packed;
    if (rb > 128) {
      launch_gemm_tall(xhi, xlo, x.ld, rb, w, n, K, o, ld, part_stride, p, s);
      continue;
    }
    switch (p.nw) {
      case 2: launch_gemm_mfma_nw<2>(xhi, xlo, x.ld, rb, w, n, K, o, ld, part_stride, p, s); break;
      case 3: launch_gemm_mfma_nw<3>(xhi, xlo, x.ld, rb, w, n, K, o, ld, part_stride, p, s); break;
      case 4: launch_gemm_mfma_nw<4>(xhi, xlo, x.ld, rb, w, n, K, o, ld, part_stride, p, s); break;
      case 5: launch_gemm_mfma_nw<5>(xhi, xlo, x.ld, rb, w, n, K, o, ld, part_stride, p, s); break;
      case 6: launch_gemm_mfma_nw<6>(xhi, xlo, x.ld, rb, w, n, K, o, ld, part_stride, p, s); break;
      case 7: launch_gemm_mfma_nw<7>(xhi, xlo, x.ld, rb, w, n, K, o, ld, part_stride, p, s); break;
      default: launch_gemm_mfma_nw<8>(xhi, xlo, x.ld, rb, w, n, K, o, ld, part_stride, p, s); break;
    }
  }
}

}  // namespace firp
