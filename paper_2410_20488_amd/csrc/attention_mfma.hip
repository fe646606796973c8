// Tree-masked flash-decode attention for a bf16 KV cache on gfx950 (MFMA 16x16x32 bf16).
//
// Grid = (splits over cache length, kv heads, sequences).  A workgroup owns one contiguous
// chunk of keys of one kv head.  Its work items are "pairs" (16-row tile of the sequence's
// step rows, q head of the kv group); every wave takes up to two pairs at a time and sweeps
// the chunk in blocks of 32 keys, reading K and V^T straight from the cache into MFMA operand
// layout (the waves of a workgroup read the same lines, so HBM sees them once):
//   S^T = K . Q^T   A = K block (lane = key, 8 dims), B = Q (lane = row, 8 dims), hi and lo
//                   planes of Q accumulated into the same tile.  The key <-> MFMA-row map is
//                   chosen so that a lane ends up with 8 consecutive keys of its row, which is
//                   exactly the B layout the next product needs - no shuffle in between;
//   online softmax  fp32, max over the lane's 8 scores and 2 cross-lane steps, mask applied
//                   only in blocks that reach past the committed cache: key p0 + c is visible
//                   to a row iff bit c of the row's mask is set;
//   O^T += V^T . P  A = V^T block (lane = dim, 8 keys, contiguous because V is stored
//                   transposed), B = P as hi and lo bf16 planes.
// Each (row, q head, split) leaves (max, sum, unnormalised output); k_attn_combine merges the
// splits and writes the activation planes for the output projection.
#include <algorithm>

#include "kernels.h"

namespace firp {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));

namespace {
__device__ __forceinline__ bf16x8_t as_bf16x8(u32x4_t v) { return __builtin_bit_cast(bf16x8_t, v); }
__device__ __forceinline__ unsigned pack_bf16(float a, float b) {
  return (unsigned)f32_to_bf16(a).v | ((unsigned)f32_to_bf16(b).v << 16);
}
constexpr int PAIRS = 2;
}  // namespace

// Where the rows of one sequence live in the step's global row order: local id -> row.
struct SeqRows {
  int n_real_per_seq;    // N
  int n_pseudo_per_seq;  // P (0 in the layers below the FIRP layer)
  int real_total;        // B * N
};
__device__ __forceinline__ int global_row(const SeqRows& sr, int b, int local) {
  return local < sr.n_real_per_seq ? b * sr.n_real_per_seq + local
                                   : sr.real_total + b * sr.n_pseudo_per_seq + (local - sr.n_real_per_seq);
}

template <int DH>
__global__ __launch_bounds__(256, 1) void k_attention_mfma(const bf16* __restrict__ qhi, const bf16* __restrict__ qlo,
                                                          int ldq, int n_q_heads, SeqRows sr, int n_local,
                                                          const unsigned long long* __restrict__ row_mask,
                                                          const int* __restrict__ p0v, KvView kv, int chunk,
                                                          float* __restrict__ part_o, float* __restrict__ part_ml,
                                                          int splits) {
  constexpr int DS = DH / 32;  // k-steps of the score product
  constexpr int DT = DH / 16;  // 16-dim tiles of the output
  const int split = blockIdx.x, hk = blockIdx.y, b = blockIdx.z;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, n_waves = blockDim.x >> 6;
  const int r16 = lane & 15, kb = lane >> 4;
  const int G = n_q_heads / kv.n_kv_heads;
  const int n_tiles = (n_local + 15) >> 4;
  const int n_pairs = n_tiles * G;
  const int p0 = p0v[b];
  const int n_keys = p0 + n_local;
  const int key_begin = split * chunk;
  const int key_end = min(n_keys, key_begin + chunk);
  const bf16* Kb = (const bf16*)kv.k + (size_t)b * kv.seq_stride + (size_t)hk * kv.slots * DH;
  const bf16* Vt = (const bf16*)kv.v + (size_t)b * kv.seq_stride + (size_t)hk * DH * kv.slots;
  const float sc = 1.4426950408889634f / sqrtf((float)DH);  // log2(e) / sqrt(dh)
  const float NEG = -__builtin_inff();

  for (int pp = wave * PAIRS; pp < n_pairs; pp += n_waves * PAIRS) {
    // ---- this wave's pairs: Q fragments, masks, running state
    u32x4_t q[PAIRS][DS][2];
    unsigned long long mk[PAIRS][FIRP_MASK_WORDS];
    int row_of[PAIRS], head_of[PAIRS];
    bool live[PAIRS];
#pragma unroll
    for (int p = 0; p < PAIRS; ++p) {
      int pi = min(pp + p, n_pairs - 1);
      live[p] = pp + p < n_pairs;
      int tile = pi / G, g = pi % G;
      int local = min(tile * 16 + r16, n_local - 1);
      int row = global_row(sr, b, local);
      row_of[p] = (tile * 16 + r16 < n_local) ? row : -1;
      head_of[p] = hk * G + g;
      const size_t qoff = (size_t)row * ldq + (size_t)head_of[p] * DH + kb * 8;
#pragma unroll
      for (int ds = 0; ds < DS; ++ds) {
        q[p][ds][0] = *(const u32x4_t*)(qhi + qoff + ds * 32);
        q[p][ds][1] = *(const u32x4_t*)(qlo + qoff + ds * 32);
      }
#pragma unroll
      for (int wd = 0; wd < FIRP_MASK_WORDS; ++wd) mk[p][wd] = row_mask[(size_t)row * FIRP_MASK_WORDS + wd];
    }
    f32x4_t o[PAIRS][DT];
    float m_run[PAIRS], l_run[PAIRS];
#pragma unroll
    for (int p = 0; p < PAIRS; ++p) {
      m_run[p] = NEG;
      l_run[p] = 0.f;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) o[p][dt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    }

    // ---- sweep the chunk, 32 keys per block
    auto load_kv = [&](u32x4_t (&kf)[2][DS], u32x4_t (&vf)[DT], int k0) {
      // K rows of the two 16-key tiles: MFMA row m <-> key 8*(m/4) + (m%4) (+4 for the second)
      const int key_a = k0 + 8 * (r16 >> 2) + (r16 & 3);
#pragma unroll
      for (int t2 = 0; t2 < 2; ++t2) {
        const bf16* kr = Kb + (size_t)min(key_a + 4 * t2, kv.slots - 1) * DH + kb * 8;
#pragma unroll
        for (int ds = 0; ds < DS; ++ds) kf[t2][ds] = *(const u32x4_t*)(kr + ds * 32);
      }
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) vf[dt] = *(const u32x4_t*)(Vt + (size_t)(dt * 16 + r16) * kv.slots + k0 + 8 * kb);
    };
    auto block = [&](u32x4_t (&kf)[2][DS], u32x4_t (&vf)[DT], int k0) {
      const bool need_mask = k0 + 32 > p0;
#pragma unroll
      for (int p = 0; p < PAIRS; ++p) {
        if (!live[p]) continue;
        f32x4_t s[2];
#pragma unroll
        for (int t2 = 0; t2 < 2; ++t2) {
          s[t2] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int ds = 0; ds < DS; ++ds) {
            s[t2] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(kf[t2][ds]), as_bf16x8(q[p][ds][0]), s[t2], 0, 0, 0);
            s[t2] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(kf[t2][ds]), as_bf16x8(q[p][ds][1]), s[t2], 0, 0, 0);
          }
        }
        // lane holds scores of row r16 at keys k0 + 8*kb + 4*t2 + i
        float e[8];
#pragma unroll
        for (int t2 = 0; t2 < 2; ++t2)
#pragma unroll
          for (int i = 0; i < 4; ++i) e[t2 * 4 + i] = s[t2][i] * sc;
        if (need_mask) {
#pragma unroll
          for (int j = 0; j < 8; ++j) {
            int key = k0 + 8 * kb + j;
            int c = key - p0;
            int wd = c >> 6;
            unsigned long long word = wd == 0 ? mk[p][0] : wd == 1 ? mk[p][1] : wd == 2 ? mk[p][2] : mk[p][3];
            bool vis = key < p0 || (c < n_local && ((word >> (c & 63)) & 1ull));
            e[j] = vis ? e[j] : NEG;
          }
        }
        float mx = e[0];
#pragma unroll
        for (int j = 1; j < 8; ++j) mx = fmaxf(mx, e[j]);
        mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        float m_new = fmaxf(m_run[p], mx);
        float m_use = (m_new == NEG) ? 0.f : m_new;
        float alpha = exp2f(m_run[p] - m_use);
        m_run[p] = m_new;
        float psum = 0.f;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          e[j] = exp2f(e[j] - m_use);
          psum += e[j];
        }
        l_run[p] = l_run[p] * alpha + psum;
        // probabilities as two bf16 planes (hi + lo), like every other MFMA activation operand
        float eh[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) eh[j] = to_f32(f32_to_bf16(e[j]));
        u32x4_t pf, pl;
        pf.x = pack_bf16(eh[0], eh[1]);
        pf.y = pack_bf16(eh[2], eh[3]);
        pf.z = pack_bf16(eh[4], eh[5]);
        pf.w = pack_bf16(eh[6], eh[7]);
        pl.x = pack_bf16(e[0] - eh[0], e[1] - eh[1]);
        pl.y = pack_bf16(e[2] - eh[2], e[3] - eh[3]);
        pl.z = pack_bf16(e[4] - eh[4], e[5] - eh[5]);
        pl.w = pack_bf16(e[6] - eh[6], e[7] - eh[7]);
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
          o[p][dt] *= alpha;
          o[p][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(vf[dt]), as_bf16x8(pf), o[p][dt], 0, 0, 0);
          o[p][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(vf[dt]), as_bf16x8(pl), o[p][dt], 0, 0, 0);
        }
      }
    };
    // two register sets: the loads of block i+1 are in flight while block i is multiplied
    u32x4_t kfa[2][DS], vfa[DT], kfb[2][DS], vfb[DT];
    const int k_last = max(key_begin, ((key_end - 1) >> 5) << 5);   // start of the last block
    if (key_begin < key_end) load_kv(kfa, vfa, key_begin);
    int k0 = key_begin;
    for (; k0 + 32 < key_end; k0 += 64) {
      load_kv(kfb, vfb, k0 + 32);
      block(kfa, vfa, k0);
      load_kv(kfa, vfa, min(k0 + 64, k_last));
      block(kfb, vfb, k0 + 32);
    }
    if (k0 < key_end) block(kfa, vfa, k0);

    // ---- leave this split's partial result: lane holds O[row r16][dim dt*16 + 4*kb + i]
#pragma unroll
    for (int p = 0; p < PAIRS; ++p) {
      if (!live[p] || row_of[p] < 0) continue;
      float l = l_run[p];
      l += __shfl_xor(l, 16, 64);
      l += __shfl_xor(l, 32, 64);
      size_t base = ((size_t)row_of[p] * n_q_heads + head_of[p]) * splits + split;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) *(f32x4_t*)(part_o + base * DH + dt * 16 + 4 * kb) = o[p][dt];
      if (kb == 0) {
        part_ml[base * 2 + 0] = m_run[p];
        part_ml[base * 2 + 1] = l;
      }
    }
  }
}

// Merge the splits of one (row, q head): O = sum_s 2^(m_s - M) o_s / sum_s 2^(m_s - M) l_s.
// blockDim = (dh/4, heads per block); blockIdx = (row, head group).
template <bool SPLIT>
__global__ void k_attn_combine(const float* __restrict__ part_o, const float* __restrict__ part_ml, int splits,
                               int n_q_heads, int dh, Act out) {
  int r = blockIdx.x, h = blockIdx.y * blockDim.y + threadIdx.y;
  if (h >= n_q_heads) return;
  size_t base = ((size_t)r * n_q_heads + h) * splits;
  float M = -__builtin_inff();
  for (int s = 0; s < splits; ++s) M = fmaxf(M, part_ml[(base + s) * 2]);
  float L = 0.f;
  for (int s = 0; s < splits; ++s) L += exp2f(part_ml[(base + s) * 2] - M) * part_ml[(base + s) * 2 + 1];
  float inv = 1.0f / L;
  int d = threadIdx.x * 4;
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int s = 0; s < splits; ++s) {
    float w = exp2f(part_ml[(base + s) * 2] - M);
    if (w == 0.f) continue;  // an empty split may hold stale values
    float4 v = *(const float4*)(part_o + (base + s) * dh + d);
    acc.x += w * v.x;
    acc.y += w * v.y;
    acc.z += w * v.z;
    acc.w += w * v.w;
  }
  act_store4<SPLIT>(out, (size_t)r * out.ld + (size_t)h * dh + d, acc.x * inv, acc.y * inv, acc.z * inv, acc.w * inv);
}

bool attention_mfma_supported(int head_dim, int dtype) {
  return dtype == DT_BF16 && (head_dim == 32 || head_dim == 64 || head_dim == 128);
}

size_t attention_mfma_scratch_floats(int rows, int n_q_heads, int head_dim) {
  return (size_t)rows * n_q_heads * FIRP_ATTN_MAX_SPLITS * (head_dim + 2);
}

void launch_attention_mfma(const Act& q, int rows, int n_q_heads, int B, int n_real_per_seq, int n_pseudo_per_seq,
                           const RowTab& rt, const int* p0, int max_ctx_now, const KvView& kv, float* scratch,
                           const Act& out, hipStream_t s) {
  const int n_local = n_real_per_seq + n_pseudo_per_seq;
  const int dh = kv.head_dim;
  SeqRows sr{n_real_per_seq, n_pseudo_per_seq, B * n_real_per_seq};
  // chunks of whole 32-key blocks; about one workgroup per CU
  int n_keys = max_ctx_now + n_local;
  int blocks = (n_keys + 31) / 32;
  int want = std::max(1, 256 / std::max(1, kv.n_kv_heads * B));
  int splits = std::max(1, std::min({want, blocks, FIRP_ATTN_MAX_SPLITS}));
  int chunk = ((blocks + splits - 1) / splits) * 32;
  splits = (n_keys + chunk - 1) / chunk;
  const int G = n_q_heads / kv.n_kv_heads;
  int n_pairs = ((n_local + 15) / 16) * G;
  int n_waves = std::max(1, std::min(4, (n_pairs + PAIRS - 1) / PAIRS));
  float* part_o = scratch;
  float* part_ml = scratch + (size_t)rows * n_q_heads * FIRP_ATTN_MAX_SPLITS * dh;
  dim3 g(splits, kv.n_kv_heads, B), blk(64 * n_waves);
  if (dh == 128)
    hipLaunchKernelGGL(k_attention_mfma<128>, g, blk, 0, s, q.hi, q.lo, q.ld, n_q_heads, sr, n_local, rt.mask, p0, kv, chunk, part_o, part_ml, splits);
  else if (dh == 64)
    hipLaunchKernelGGL(k_attention_mfma<64>, g, blk, 0, s, q.hi, q.lo, q.ld, n_q_heads, sr, n_local, rt.mask, p0, kv, chunk, part_o, part_ml, splits);
  else
    hipLaunchKernelGGL(k_attention_mfma<32>, g, blk, 0, s, q.hi, q.lo, q.ld, n_q_heads, sr, n_local, rt.mask, p0, kv, chunk, part_o, part_ml, splits);
  int hpb = std::max(1, 256 / (dh / 4));
  dim3 gc(rows, (n_q_heads + hpb - 1) / hpb), bc(dh / 4, hpb);
  hipLaunchKernelGGL(k_attn_combine<true>, gc, bc, 0, s, part_o, part_ml, splits, n_q_heads, dh, out);
}

}  // namespace firp
