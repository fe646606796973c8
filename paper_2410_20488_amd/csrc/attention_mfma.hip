// Tree-masked flash-decode attention for a bf16 KV cache on gfx950 (MFMA 16x16x32 bf16).
//
// Grid = (splits over cache length, kv heads, sequences); 8 waves per workgroup, two per SIMD:
// one wave issues an MFMA at most every 16 cycles and its softmax arithmetic sits between the
// two products, so a second wave per SIMD is what fills the matrix pipe.  A workgroup owns one
// contiguous chunk of keys of one kv head and sweeps it in blocks of 32 keys.  Its work items
// are "pairs" (16-row tile of the sequence's step rows, q head of the kv group), dealt out one
// per wave first, up to two per wave.  Every block of K and V^T is fetched once per workgroup:
// each wave loads an eighth of the block's MFMA operand fragments (global -> registers, three
// blocks ahead), drops them into one of two LDS buffers in the lane order the MFMA wants, and
// after a barrier every wave reads all fragments back with conflict-free 16-byte LDS reads.
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
#include <type_traits>

#include "kernels.h"

namespace firp {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));

namespace {
__device__ __forceinline__ bf16x8_t as_bf16x8(u32x4_t v) { return __builtin_bit_cast(bf16x8_t, v); }
constexpr int PAIRS = 2;
constexpr int NWAVES = 8;
}  // namespace

// Where the rows of one sequence live in the step's global row order: local id -> row.  The
// tree nodes of all sequences come first (sequence-major); the pseudo rows follow step by step:
// pseudo row i of anchor a of sequence b has local id N + i*A + a and sits behind the pseudo rows
// of all earlier steps of all sequences, so that the rows alive at a layer are a prefix.
struct SeqRows {
  int n_real_per_seq;     // N
  int n_anchor_per_seq;   // A
  int real_total;         // B * N
  int anchor_total;       // B * A
};
__device__ __forceinline__ int global_row(const SeqRows& sr, int b, int local) {
  if (local < sr.n_real_per_seq) return b * sr.n_real_per_seq + local;
  const int q = local - sr.n_real_per_seq, i = q / sr.n_anchor_per_seq, a = q - i * sr.n_anchor_per_seq;
  return sr.real_total + i * sr.anchor_total + b * sr.n_anchor_per_seq + a;
}

// ------------------------------------------------------------------------------------------
// Producer of the attention operands for one layer: sums the split-K partials of the q|k|v
// projection, applies the row scale of the norm before it and the rotary embedding (half-split
// pairs (j, j + dh/2), cos/sin from the step's table), and writes
//   Q   as MFMA B-operand fragments: for (sequence, 16-row tile, q head) 2*dh/32 blocks of 1 KiB,
//       block 2*ds + plane holding at byte 16 * (16 * kb + r16) the 8 dims 32 ds + 8 kb ... of row
//       16 tile + r16 (plane 0 = hi, 1 = lo), so that the attention kernel loads a fragment with
//       one fully coalesced instruction;
//   K   into the cache row of slot p0 + local (16-byte stores);
//   V^T through an LDS transpose, so that a store instruction writes runs of 16 consecutive
//       slots of a dim instead of one element of 64 different dims.
// blockIdx = (sequence * tiles + tile, group of 128/dh heads); 2*dh threads per head: thread
// (r16, c), c fastest, owns dims [4c, 4c+4) and their rotation partners [4c + dh/2, ...), so a
// wave reads whole rows of the partial sums in 16-byte pieces.
// SMAX: upper bound of the split factor of the instance (its loads are all in flight at once).
template <int DH, int SMAX>
__global__ __launch_bounds__(256) void k_rope_kv_tiles(Partial qkv, RowScale rs, int n_q_heads, SeqRows sr,
                                                       int n_local, int n_tiles, int seq0,
                                                       const int* __restrict__ p0v, const float2* __restrict__ tab,
                                                       bf16* __restrict__ q_frag, KvView kv) {
  constexpr int TPH = 2 * DH, HPB = 256 / TPH, HALF = DH / 2, DS = DH / 32, CPR = DH / 8;  // chunks per row
  __shared__ unsigned short vt_lds[HPB][16][DH + 8];
  const int tile = blockIdx.x % n_tiles, b = blockIdx.x / n_tiles;
  const int hsel = threadIdx.x / TPH, t = threadIdx.x % TPH;
  const int Hkv = kv.n_kv_heads, heads = n_q_heads + 2 * Hkv;
  const int h = blockIdx.y * HPB + hsel;
  const int c = t % CPR, r16 = t / CPR;
  const int local = tile * 16 + r16;
  const bool valid = local < n_local && h < heads;
  const int bs = seq0 + b;   // sequence whose cache this launch works on (b counts inside the launch)
  const int p0 = p0v[bs];
  if (valid) {
    const int row = global_row(sr, b, local);
    const size_t col = (size_t)row * qkv.ld + (size_t)h * DH + 4 * c;
    // all splits' loads in flight at once (split-K never exceeds 16)
    float4 va[SMAX], vb[SMAX];
#pragma unroll
    for (int u = 0; u < SMAX; ++u)
      if (u < qkv.S) {
        const float* pp = qkv.p + (size_t)u * qkv.stride + col;
        va[u] = *(const float4*)pp;
        vb[u] = *(const float4*)(pp + HALF);
      }
    float x1[4] = {0.f, 0.f, 0.f, 0.f}, x2[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int u = 0; u < SMAX; ++u)
      if (u < qkv.S) {
        x1[0] += va[u].x; x1[1] += va[u].y; x1[2] += va[u].z; x1[3] += va[u].w;
        x2[0] += vb[u].x; x2[1] += vb[u].y; x2[2] += vb[u].z; x2[3] += vb[u].w;
      }
    const float scale = row_scale(rs, row);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      x1[i] *= scale;
      x2[i] *= scale;
    }
    if (h < n_q_heads + Hkv) {
      const float4* cs = (const float4*)(tab + (size_t)row * HALF + 4 * c);
      const float4 w01 = cs[0], w23 = cs[1];   // (cos, sin) of dims 4c .. 4c+3
      const float co[4] = {w01.x, w01.z, w23.x, w23.z}, si[4] = {w01.y, w01.w, w23.y, w23.w};
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float y1 = x1[i] * co[i] - x2[i] * si[i], y2 = x2[i] * co[i] + x1[i] * si[i];
        x1[i] = y1;
        x2[i] = y2;
      }
    }
    if (h < n_q_heads) {
      bf16* fb = q_frag + ((size_t)(b * n_tiles + tile) * n_q_heads + h) * (size_t)(DS * 2 * 512);
#pragma unroll
      for (int half = 0; half < 2; ++half) {
        const float* x = half ? x2 : x1;
        const int c8 = (c >> 1) + half * (DH / 16);   // chunk of 8 dims: k-step c8/4, k-block c8%4
        uint2 hi, lo;
        split2_bf16(x[0], x[1], hi.x, lo.x);
        split2_bf16(x[2], x[3], hi.y, lo.y);
        bf16* dst = fb + (size_t)((c8 >> 2) * 2) * 512 + ((c8 & 3) * 16 + r16) * 8 + (c & 1) * 4;
        *(uint2*)dst = hi;
        *(uint2*)(dst + 512) = lo;
      }
    } else if (h < n_q_heads + Hkv) {
      const int hk = h - n_q_heads;
      bf16* krow = (bf16*)kv.k + (size_t)bs * kv.seq_stride + ((size_t)hk * kv.slots + (size_t)(p0 + local)) * DH;
      *(uint2*)(krow + 4 * c) = make_uint2(pack2_bf16(x1[0], x1[1]), pack2_bf16(x1[2], x1[3]));
      *(uint2*)(krow + 4 * c + HALF) = make_uint2(pack2_bf16(x2[0], x2[1]), pack2_bf16(x2[2], x2[3]));
    } else {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        vt_lds[hsel][r16][4 * c + i] = f32_to_bf16(x1[i]).v;
        vt_lds[hsel][r16][4 * c + HALF + i] = f32_to_bf16(x2[i]).v;
      }
    }
  }
  __syncthreads();
  if (h >= n_q_heads + Hkv && h < heads) {
    const int hv = h - n_q_heads - Hkv;
    // slots p0 + 16 tile + rr of every dim: pairs of rows that start at an even slot go out as one
    // 4-byte store (item j of a dim covers rows 2j - off and 2j - off + 1, off = parity of the
    // tile's first slot)
    const int sb = p0 + tile * 16, off = sb & 1;
    unsigned short* vt = (unsigned short*)kv.v + (size_t)bs * kv.seq_stride + (size_t)hv * DH * kv.slots + sb;
    for (int idx = t; idx < DH * 9; idx += TPH) {
      const int dim = idx / 9, j = idx - dim * 9;
      const int r0 = 2 * j - off, r1 = r0 + 1;
      const bool ok0 = r0 >= 0 && r0 < 16 && tile * 16 + r0 < n_local;
      const bool ok1 = r1 < 16 && tile * 16 + r1 < n_local;
      unsigned short* dst = vt + (size_t)dim * kv.slots;
      if (ok0 && ok1)
        *(unsigned*)(dst + r0) = (unsigned)vt_lds[hsel][r0][dim] | ((unsigned)vt_lds[hsel][r1][dim] << 16);
      else if (ok0)
        dst[r0] = vt_lds[hsel][r0][dim];
      else if (ok1)
        dst[r1] = vt_lds[hsel][r1][dim];
    }
  }
}

size_t attention_q_frag_elems(int rows, int max_batch, int n_q_heads, int head_dim) {
  return (size_t)(rows + 16 * max_batch) * n_q_heads * head_dim * 2;
}

void launch_rope_kv_tiles(const Partial& qkv, const RowScale& rs, int n_q_heads, int B, int n_real_per_seq,
                          int n_pseudo_per_seq, int n_anchor_per_seq, int seq0, const int* p0, const float2* tab,
                          bf16* q_frag, const KvView& kv, hipStream_t s) {
  const int n_local = n_real_per_seq + n_pseudo_per_seq, n_tiles = (n_local + 15) / 16;
  SeqRows sr{n_real_per_seq, std::max(1, n_anchor_per_seq), B * n_real_per_seq, B * n_anchor_per_seq};
  const int dh = kv.head_dim, heads = n_q_heads + 2 * kv.n_kv_heads, hpb = 128 / dh;
  dim3 g(B * n_tiles, (heads + hpb - 1) / hpb), blk(256);
  auto go = [&](auto kern) { hipLaunchKernelGGL(kern, g, blk, 0, s, qkv, rs, n_q_heads, sr, n_local, n_tiles, seq0, p0, tab, q_frag, kv); };
  const int sm = qkv.S <= 4 ? 4 : qkv.S <= 8 ? 8 : 16;
  if (dh == 128) {
    if (sm == 4) go(k_rope_kv_tiles<128, 4>); else if (sm == 8) go(k_rope_kv_tiles<128, 8>); else go(k_rope_kv_tiles<128, 16>);
  } else if (dh == 64) {
    if (sm == 4) go(k_rope_kv_tiles<64, 4>); else if (sm == 8) go(k_rope_kv_tiles<64, 8>); else go(k_rope_kv_tiles<64, 16>);
  } else {
    if (sm == 4) go(k_rope_kv_tiles<32, 4>); else if (sm == 8) go(k_rope_kv_tiles<32, 8>); else go(k_rope_kv_tiles<32, 16>);
  }
}

template <int DH>
__global__ __launch_bounds__(64 * NWAVES, 1) void k_attention_mfma(const bf16* __restrict__ q_frag,
                                                          int n_q_heads, SeqRows sr, int n_local,
                                                          const unsigned long long* __restrict__ row_mask,
                                                          const int* __restrict__ p0v, int seq0, KvView kv,
                                                          float* __restrict__ part_o, float* __restrict__ part_ml,
                                                          int splits) {
  constexpr int DS = DH / 32;       // k-steps of the score product
  constexpr int DT = DH / 16;       // 16-dim tiles of the output
  constexpr int NF = 2 * DS + DT;   // operand fragments (64 lanes x 16 B) of one 32-key block
  constexpr int FPW = (NF + NWAVES - 1) / NWAVES;   // fragments each wave fetches
  static_assert(NF % NWAVES == 0 || NF < NWAVES, "fragments must divide over the waves");
  const int split = blockIdx.x, hk = blockIdx.y, b = blockIdx.z;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r16 = lane & 15, kb = lane >> 4;
  const int G = n_q_heads / kv.n_kv_heads;
  const int n_tiles = (n_local + 15) >> 4;
  const int n_pairs = n_tiles * G;
  const int bs = seq0 + b;   // sequence whose cache this launch reads (b counts inside the launch)
  const int p0 = p0v[bs];
  const int n_keys = p0 + n_local;
  // The sequence's keys in `splits` chunks of whole 32-key blocks.  The chunk length follows
  // from the committed length on the device, so that no launch argument changes from step to
  // step (a captured launch can be replayed as the context grows).
  const int chunk = ((((n_keys + 31) >> 5) + splits - 1) / splits) << 5;
  const int key_begin = split * chunk;
  if (key_begin >= n_keys) {
    // a split past the end of a short context: leave the neutral element (weight 0) for the merge
    for (int idx = threadIdx.x; idx < n_local * G; idx += blockDim.x) {
      const int local = idx / G, head = hk * G + idx % G;
      const size_t base = ((size_t)global_row(sr, b, local) * n_q_heads + head) * splits + split;
      part_ml[base * 2 + 0] = -__builtin_inff();
      part_ml[base * 2 + 1] = 0.f;
    }
    return;
  }
  // last block the launch geometry allows (key_begin < n_keys <= slots, both multiples of 32 apart)
  const int hard_last = (min(key_begin + chunk, kv.slots) - key_begin - 32) >> 5;
  const int key_end = min(n_keys, key_begin + chunk);
  const int nb = key_end > key_begin ? (key_end - key_begin + 31) >> 5 : 0;   // blocks of this chunk
  const int last = nb - 1;
  const bf16* Kb = (const bf16*)kv.k + (size_t)(seq0 + b) * kv.seq_stride + (size_t)hk * kv.slots * DH;
  const bf16* Vt = (const bf16*)kv.v + (size_t)(seq0 + b) * kv.seq_stride + (size_t)hk * DH * kv.slots;
  const float sc = 1.4426950408889634f / sqrtf((float)DH);  // log2(e) / sqrt(dh)
  const float NEG = -__builtin_inff();

  __shared__ u32x4_t kv_lds[2][NF][64];
  // every row's mask words (two zero words behind them) sit in its wave's corner of LDS, where
  // the blocks that reach past the committed cache pick the word they need by index
  __shared__ unsigned long long mk_lds[NWAVES * PAIRS * 16][FIRP_MASK_WORDS + 2];

  // This wave fetches fragments f = NWAVES*j + wave (with fewer fragments than waves, several
  // waves fetch and store the same one).  Fragments [0, 2*DS) are K: (16-key tile t2,
  // k-step ds), MFMA row m <-> key 8*(m/4) + (m%4) + 4*t2; the rest are V^T: 16-dim tile dt.
  // A fragment's address is linear in the block's first key.
  const char* fbase[FPW];
  int fstep[FPW];   // bytes per key
#pragma unroll
  for (int j = 0; j < FPW; ++j) {
    const int f = (NWAVES * j + wave) % NF;
    if (f < 2 * DS) {
      const int t2 = f / DS, ds = f % DS;
      fbase[j] = (const char*)(Kb + (size_t)(8 * (r16 >> 2) + (r16 & 3) + 4 * t2) * DH + kb * 8 + ds * 32);
      fstep[j] = DH * 2;
    } else {
      const int dt = f - 2 * DS;
      fbase[j] = (const char*)(Vt + (size_t)(dt * 16 + r16) * kv.slots + 8 * kb);
      fstep[j] = 2;
    }
  }
  // every load is unconditional (blocks past the end repeat the last one and are never used) so
  // that the compiler's wait counters stay exact
  auto fetch = [&](u32x4_t (&g)[FPW], int blk, int bound) {
    const size_t key = (size_t)(key_begin + 32 * min(blk, bound));
#pragma unroll
    for (int j = 0; j < FPW; ++j) g[j] = *(const u32x4_t*)(fbase[j] + key * fstep[j]);
  };
  auto stash = [&](const u32x4_t (&g)[FPW], int buf) {
#pragma unroll
    for (int j = 0; j < FPW; ++j) kv_lds[buf][(NWAVES * j + wave) % NF][lane] = g[j];
  };

  // a sweep covers up to NWAVES * PAIRS pairs: pair `first + wave + NWAVES*p` is this wave's p-th
  const int n_sweeps = (n_pairs + NWAVES * PAIRS - 1) / (NWAVES * PAIRS);
  for (int sweep = 0; sweep < n_sweeps; ++sweep) {
    const int first = sweep * NWAVES * PAIRS;
    int n_live = 0;
#pragma unroll
    for (int p = 0; p < PAIRS; ++p) n_live += first + wave + NWAVES * p < n_pairs;
    // ---- this wave's pairs: Q fragments, masks, running state.  Q and the masks are cache
    // hits and are asked for first (loads return in order); the first three K/V blocks follow.
    u32x4_t q[PAIRS][DS][2];
    unsigned long long mw[PAIRS][FIRP_MASK_WORDS];
    int row_of[PAIRS], head_of[PAIRS];
#pragma unroll
    for (int p = 0; p < PAIRS; ++p) {
      int pi = min(first + wave + NWAVES * p, n_pairs - 1);
      int tile = pi / G, g = pi % G;
      int local = min(tile * 16 + r16, n_local - 1);
      int row = global_row(sr, b, local);
      row_of[p] = (tile * 16 + r16 < n_local) ? row : -1;
      head_of[p] = hk * G + g;
      if (p < n_live) {
        const bf16* fb = q_frag + ((size_t)(b * n_tiles + tile) * n_q_heads + head_of[p]) * (size_t)(DS * 2 * 512) + lane * 8;
#pragma unroll
        for (int ds = 0; ds < DS; ++ds) {
          q[p][ds][0] = *(const u32x4_t*)(fb + (ds * 2) * 512);
          q[p][ds][1] = *(const u32x4_t*)(fb + (ds * 2 + 1) * 512);
        }
      } else {
#pragma unroll
        for (int ds = 0; ds < DS; ++ds) q[p][ds][0] = q[p][ds][1] = u32x4_t{0, 0, 0, 0};
      }
#pragma unroll
      for (int wd = 0; wd < FIRP_MASK_WORDS; ++wd) mw[p][wd] = row_mask[(size_t)row * FIRP_MASK_WORDS + wd];
    }
    u32x4_t g0[FPW], g1[FPW], g2[FPW];
    fetch(g0, 0, hard_last);
    fetch(g1, 1, hard_last);
    fetch(g2, 2, hard_last);
    if (kb == 0) {
#pragma unroll
      for (int p = 0; p < PAIRS; ++p) {
        unsigned long long* mrow = mk_lds[(wave * PAIRS + p) * 16 + r16];
#pragma unroll
        for (int wd = 0; wd < FIRP_MASK_WORDS; ++wd) mrow[wd] = mw[p][wd];
        mrow[FIRP_MASK_WORDS] = 0ull;
        mrow[FIRP_MASK_WORDS + 1] = 0ull;
      }
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

    // One block of 32 keys against NP pairs, in three phases so that the pairs' independent
    // MFMA chains and softmax arithmetic interleave: scores, softmax, output.
    auto block = [&](auto np_tag, int buf, int k0) {
      constexpr int NP = decltype(np_tag)::value;
      f32x4_t s[NP][2];
#pragma unroll
      for (int p = 0; p < NP; ++p)
#pragma unroll
        for (int t2 = 0; t2 < 2; ++t2) s[p][t2] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ds = 0; ds < DS; ++ds)
#pragma unroll
        for (int t2 = 0; t2 < 2; ++t2) {
          const bf16x8_t kf = as_bf16x8(kv_lds[buf][t2 * DS + ds][lane]);
#pragma unroll
          for (int p = 0; p < NP; ++p) {
            s[p][t2] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf, as_bf16x8(q[p][ds][0]), s[p][t2], 0, 0, 0);
            s[p][t2] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf, as_bf16x8(q[p][ds][1]), s[p][t2], 0, 0, 0);
          }
        }
      // lane holds the raw scores of row r16 at keys k0 + 8*kb + j, j = 4*t2 + i
      float e[NP][8];
#pragma unroll
      for (int p = 0; p < NP; ++p)
#pragma unroll
        for (int t2 = 0; t2 < 2; ++t2)
#pragma unroll
          for (int i = 0; i < 4; ++i) e[p][t2 * 4 + i] = s[p][t2][i];
      if (k0 + 32 > p0) {
        // bit j of `vis`: key k0 + 8*kb + j is visible to this lane's row
        const int c0 = k0 + 8 * kb - p0;  // step-local index of the lane's first key
#pragma unroll
        for (int p = 0; p < NP; ++p) {
          const unsigned long long* mrow = mk_lds[(wave * PAIRS + p) * 16 + r16];
          unsigned vis;
          if (c0 <= -8) {
            vis = 0xffu;
          } else if (c0 < 0) {
            vis = (unsigned)(mrow[0] << (-c0)) | ((1u << (-c0)) - 1u);
          } else {
            const int wd = min(c0 >> 6, FIRP_MASK_WORDS), sh = c0 & 63;
            vis = (unsigned)(mrow[wd] >> sh);
            if (sh > 56) vis |= (unsigned)(mrow[wd + 1] << (64 - sh));
          }
#pragma unroll
          for (int j = 0; j < 8; ++j) e[p][j] = ((vis >> j) & 1u) ? e[p][j] : NEG;
        }
      }
      float mx[NP];
#pragma unroll
      for (int p = 0; p < NP; ++p)
        mx[p] = fmaxf(fmaxf(fmaxf(e[p][0], e[p][1]), fmaxf(e[p][2], e[p][3])),
                      fmaxf(fmaxf(e[p][4], e[p][5]), fmaxf(e[p][6], e[p][7])));
#pragma unroll
      for (int p = 0; p < NP; ++p) mx[p] = fmaxf(mx[p], __shfl_xor(mx[p], 16, 64));
#pragma unroll
      for (int p = 0; p < NP; ++p) mx[p] = fmaxf(mx[p], __shfl_xor(mx[p], 32, 64)) * sc;
      // The reference point m_run of the exponentials only has to stay within 2^8 of the true
      // running maximum (any reference gives the same quotient in the end), so the rescale of
      // the accumulators is taken only when some row of a tile moved further than that.
      bool moved = false;   // stays false for a row with nothing visible yet
#pragma unroll
      for (int p = 0; p < NP; ++p) moved |= mx[p] > m_run[p] + 8.0f;
      if (__builtin_amdgcn_ballot_w64(moved) != 0ull) {
#pragma unroll
        for (int p = 0; p < NP; ++p) {
          const float m_new = fmaxf(m_run[p], mx[p]);
          const float alpha = (m_new == NEG) ? 1.0f : __builtin_amdgcn_exp2f(m_run[p] - m_new);
          m_run[p] = m_new;
          l_run[p] *= alpha;
#pragma unroll
          for (int dt = 0; dt < DT; ++dt) o[p][dt] *= alpha;
        }
      }
      // probabilities as two bf16 planes (hi + lo), like every other MFMA activation operand
      u32x4_t pf[NP], pw[NP];
#pragma unroll
      for (int p = 0; p < NP; ++p) {
        const float nm = (m_run[p] == NEG) ? 0.f : -m_run[p];
        float psum = 0.f;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          e[p][j] = __builtin_amdgcn_exp2f(__builtin_fmaf(e[p][j], sc, nm));
          psum += e[p][j];
        }
        l_run[p] += psum;
        unsigned h[4], l[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) split2_bf16(e[p][2 * j], e[p][2 * j + 1], h[j], l[j]);
        pf[p] = u32x4_t{h[0], h[1], h[2], h[3]};
        pw[p] = u32x4_t{l[0], l[1], l[2], l[3]};
      }
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) {
        const bf16x8_t vf = as_bf16x8(kv_lds[buf][2 * DS + dt][lane]);
#pragma unroll
        for (int p = 0; p < NP; ++p) {
          o[p][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, as_bf16x8(pf[p]), o[p][dt], 0, 0, 0);
          o[p][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, as_bf16x8(pw[p]), o[p][dt], 0, 0, 0);
        }
      }
    };
    // ---- sweep the chunk.  Step i: barrier (block i is in LDS buffer i&1 and nobody still
    // reads the other buffer), multiply block i, then move block i+1 from its register set to
    // the other buffer and send that set for block i+4.
    auto step = [&](u32x4_t (&gnext)[FPW], int i) {
      __syncthreads();
      const int k0 = key_begin + 32 * i;
      if (n_live == PAIRS)
        block(std::integral_constant<int, PAIRS>{}, i & 1, k0);
      else if (n_live == 1)
        block(std::integral_constant<int, 1>{}, i & 1, k0);
      stash(gnext, (i + 1) & 1);
      fetch(gnext, i + 4, last);
    };
    if (nb > 0) {
      stash(g0, 0);
      fetch(g0, 3, last);
      int i = 0;
      for (; i + 3 <= nb; i += 3) {
        step(g1, i);
        step(g2, i + 1);
        step(g0, i + 2);
      }
      if (i < nb) step(g1, i);
      if (i + 1 < nb) step(g2, i + 1);
    }
    __syncthreads();   // the next sweep overwrites both buffers

    // ---- leave this split's partial result: lane holds O[row r16][dim dt*16 + 4*kb + i]
#pragma unroll
    for (int p = 0; p < PAIRS; ++p) {
      if (p >= n_live || row_of[p] < 0) continue;
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
  // all loads of a thread are issued before any is used (splits <= FIRP_ATTN_MAX_SPLITS = 16)
  const int d = threadIdx.x * 4;
  float2 ml[16];
  float4 v[16];
#pragma unroll
  for (int s = 0; s < 16; ++s)
    if (s < splits) {
      ml[s] = *(const float2*)(part_ml + (base + s) * 2);
      v[s] = *(const float4*)(part_o + (base + s) * dh + d);
    }
  float M = -__builtin_inff();
#pragma unroll
  for (int s = 0; s < 16; ++s)
    if (s < splits) M = fmaxf(M, ml[s].x);
  float L = 0.f;
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
  for (int s = 0; s < 16; ++s)
    if (s < splits) {
      const float w = exp2f(ml[s].x - M);
      L += w * ml[s].y;
      if (w != 0.f) {  // an empty split may hold stale values
        acc.x += w * v[s].x;
        acc.y += w * v[s].y;
        acc.z += w * v[s].z;
        acc.w += w * v[s].w;
      }
    }
  const float inv = 1.0f / L;
  act_store4<SPLIT>(out, (size_t)r * out.ld + (size_t)h * dh + d, acc.x * inv, acc.y * inv, acc.z * inv, acc.w * inv);
}

bool attention_mfma_supported(int head_dim, int dtype) {
  return dtype == DT_BF16 && (head_dim == 32 || head_dim == 64 || head_dim == 128);
}

size_t attention_mfma_scratch_floats(int rows, int n_q_heads, int head_dim) {
  return (size_t)rows * n_q_heads * FIRP_ATTN_MAX_SPLITS * (head_dim + 2);
}

void launch_attention_mfma(const bf16* q_frag, int rows, int n_q_heads, int B, int n_real_per_seq, int n_pseudo_per_seq,
                           int n_anchor_per_seq, int seq0, const RowTab& rt, const int* p0, int max_ctx_now, const KvView& kv, float* scratch,
                           const Act& out, hipStream_t s) {
  const int n_local = n_real_per_seq + n_pseudo_per_seq;
  const int dh = kv.head_dim;
  SeqRows sr{n_real_per_seq, std::max(1, n_anchor_per_seq), B * n_real_per_seq, B * n_anchor_per_seq};
  // about one workgroup per CU; the count of splits depends on the context length only while the
  // context is shorter than that many 32-key blocks
  int n_keys = max_ctx_now + n_local;
  int blocks = (n_keys + 31) / 32;
  int want = std::max(1, 256 / std::max(1, kv.n_kv_heads * B));
  int splits = std::max(1, std::min({want, blocks, FIRP_ATTN_MAX_SPLITS}));
  float* part_o = scratch;
  float* part_ml = scratch + (size_t)rows * n_q_heads * FIRP_ATTN_MAX_SPLITS * dh;
  dim3 g(splits, kv.n_kv_heads, B), blk(64 * NWAVES);
  if (dh == 128)
    hipLaunchKernelGGL(k_attention_mfma<128>, g, blk, 0, s, q_frag, n_q_heads, sr, n_local, rt.mask, p0, seq0, kv, part_o, part_ml, splits);
  else if (dh == 64)
    hipLaunchKernelGGL(k_attention_mfma<64>, g, blk, 0, s, q_frag, n_q_heads, sr, n_local, rt.mask, p0, seq0, kv, part_o, part_ml, splits);
  else
    hipLaunchKernelGGL(k_attention_mfma<32>, g, blk, 0, s, q_frag, n_q_heads, sr, n_local, rt.mask, p0, seq0, kv, part_o, part_ml, splits);
  int hpb = std::max(1, 256 / (dh / 4));
  dim3 gc(rows, (n_q_heads + hpb - 1) / hpb), bc(dh / 4, hpb);
  hipLaunchKernelGGL(k_attn_combine<true>, gc, bc, 0, s, part_o, part_ml, splits, n_q_heads, dh, out);
}

}  // namespace firp
