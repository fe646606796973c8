// Shared device/host helpers of the FIRP step library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace firp {

// ---- element types -----------------------------------------------------------------------
struct bf16 {
  unsigned short v;
};

__device__ __forceinline__ float to_f32(float x) { return x; }
__device__ __forceinline__ float to_f32(bf16 x) { return __uint_as_float(((unsigned)x.v) << 16); }

// round-to-nearest-even fp32 -> bf16 with the hardware conversion (v_cvt_pk_bf16_f32)
typedef __bf16 bf16x2_hw __attribute__((ext_vector_type(2)));
typedef float f32x2_hw __attribute__((ext_vector_type(2)));
__device__ __forceinline__ bf16 f32_to_bf16(float f) {
  bf16 r;
  r.v = __builtin_bit_cast(unsigned short, (__bf16)f);
  return r;
}
// two values -> one 32-bit word, `a` in the low half
__device__ __forceinline__ unsigned pack2_bf16(float a, float b) {
  f32x2_hw v = {a, b};
  return __builtin_bit_cast(unsigned, __builtin_convertvector(v, bf16x2_hw));
}
// hi/lo planes of two values: hi = rne(v), lo = rne(v - hi)
__device__ __forceinline__ void split2_bf16(float a, float b, unsigned& hi, unsigned& lo) {
  hi = pack2_bf16(a, b);
  lo = pack2_bf16(a - __uint_as_float(hi << 16), b - __uint_as_float(hi & 0xffff0000u));
}

template <typename T>
__device__ __forceinline__ void store_elt(T* p, float v);
template <>
__device__ __forceinline__ void store_elt<float>(float* p, float v) { *p = v; }
template <>
__device__ __forceinline__ void store_elt<bf16>(bf16* p, float v) { *p = f32_to_bf16(v); }

// ---- activations handed to a projection -----------------------------------------------------
// fp32 models keep activations in fp32.  bf16 models hand the MFMA kernel two bf16 planes,
// hi = rne(v) and lo = rne(v - hi): together they carry ~16 mantissa bits, so rounding the
// activations costs no accuracy while both MFMA operands stay bf16.
struct Act {
  float* f32;  // [rows][ld] or nullptr
  bf16* hi;    // [rows][ld] or nullptr
  bf16* lo;
  int ld;
};

template <bool SPLIT>
__device__ __forceinline__ void act_store(const Act& a, size_t idx, float v) {
  if constexpr (SPLIT) {
    bf16 h = f32_to_bf16(v);
    a.hi[idx] = h;
    a.lo[idx] = f32_to_bf16(v - to_f32(h));
  } else {
    a.f32[idx] = v;
  }
}

// four consecutive activations (idx % 4 == 0): one 8-byte store per plane
template <bool SPLIT>
__device__ __forceinline__ void act_store4(const Act& a, size_t idx, float v0, float v1, float v2, float v3) {
  if constexpr (SPLIT) {
    uint2 ph, pl;
    split2_bf16(v0, v1, ph.x, pl.x);
    split2_bf16(v2, v3, ph.y, pl.y);
    *(uint2*)(a.hi + idx) = ph;
    *(uint2*)(a.lo + idx) = pl;
  } else {
    *(float4*)(a.f32 + idx) = make_float4(v0, v1, v2, v3);
  }
}

// ---- workgroup -> work item of a projection launch -------------------------------------------
// Work item of a workgroup.  The hardware deals workgroups to the 8 XCDs (each with its own L2)
// round-robin by id, and all workgroups of one split read the same columns of X: the items are
// therefore numbered split by split and XCD x takes the contiguous items [x, x + 1) * grid / 8, so
// that a split's slice of X is fetched into one or two L2s instead of all eight.  The launch is
// padded to a multiple of 8 workgroups; the surplus ones (item >= tiles * S) leave at once.
__device__ __forceinline__ int xcd_item(int block, int launched) { return (block & 7) * (launched >> 3) + (block >> 3); }

// ---- split-K partial sums ------------------------------------------------------------------
// A projection leaves S partial products [S][rows][n] (fp32); its consumer adds them up.
struct Partial {
  const float* p;
  int S;
  size_t stride;  // elements between consecutive splits
  int ld;         // n
};

__device__ __forceinline__ float partial_sum(const Partial& q, size_t idx) {
  float v = q.p[idx];
  for (int s = 1; s < q.S; ++s) v += q.p[idx + (size_t)s * q.stride];
  return v;
}

// ---- row scale of an RMSNorm, applied after the projection --------------------------------
// The norm kernel hands the projection x * gain and leaves the sum of squares of every row in P
// pieces; the projection is linear, so the consumer of its output multiplies by
// 1 / sqrt(mean(x^2) + eps) instead.  This lets the norm run on several workgroups per row
// without a second pass.  ss == nullptr: no scale.
struct RowScale {
  const float* ss;   // [rows][FIRP_NORM_PIECES]
  int pieces;
  float inv_d, eps;
};
#define FIRP_NORM_PIECES 8
__device__ __forceinline__ float row_scale(const RowScale& rs, int r) {
  if (!rs.ss) return 1.0f;
  float t = 0.f;
  for (int p = 0; p < rs.pieces; ++p) t += rs.ss[(size_t)r * FIRP_NORM_PIECES + p];
  return 1.0f / sqrtf(t * rs.inv_d + rs.eps);
}

// ---- per-row tables of one step (device) ---------------------------------------------------
// Rows of a step: the tree nodes of every sequence first (sequence-major), then the pseudo rows.
// `local` is the row's index inside its own sequence (node id, or N + pseudo index): its K/V
// live at cache slot p0[seq] + local and bit `local` of another row's mask says "visible".
#define FIRP_MASK_WORDS 4
struct RowTab {
  const int* seq;
  const int* local;
  const int* pos_off;                // position id = p0[seq] + pos_off
  const unsigned long long* mask;    // [rows][FIRP_MASK_WORDS]
};

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

// block-wide sum for blockDim.x == 256 (4 waves)
__device__ __forceinline__ float block_sum_256(float v, float* smem4) {
  v = wave_sum(v);
  int w = threadIdx.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) smem4[w] = v;
  __syncthreads();
  return smem4[0] + smem4[1] + smem4[2] + smem4[3];
}

// block-wide sum for any blockDim.x that is a multiple of 64 (up to 16 waves)
__device__ __forceinline__ float block_sum(float v, float* smem16) {
  v = wave_sum(v);
  int w = threadIdx.x >> 6, nw = blockDim.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) smem16[w] = v;
  __syncthreads();
  float t = 0.f;
  for (int i = 0; i < nw; ++i) t += smem16[i];
  return t;
}

}  // namespace firp
