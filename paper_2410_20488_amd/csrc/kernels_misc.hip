// Everything of the step that is not a projection or attention: candidate fill, embedding
// gather, fused residual-add + RMSNorm, rotary + KV append, SwiGLU, the FIRP map's gather /
// scatter, argmax / top-b over the logits, greedy verification, KV compaction.
#include <algorithm>

#include "kernels.h"

namespace firp {

// ------------------------------------------------------------------------------------------
// Candidate fill (Inference stage: the tree verified now was drafted by the previous step).
// Node v at depth j carries drafts[j-1][rank[v]]; without valid drafts every candidate is -1,
// which no greedy token equals, so the step accepts nothing beyond the root.
__global__ void k_fill_tokens(SeqState st, TreeTab tt, const int* injected) {
  int b = blockIdx.x;
  for (int v = threadIdx.x; v < tt.n_nodes; v += blockDim.x) {
    int t;
    if (v == 0) {
      t = st.root_tok[b];
    } else if (injected) {
      t = injected[b * tt.n_nodes + v];
    } else {
      int lvl = tt.level[v];
      t = (st.drafts_valid[b] && lvl <= st.k) ? st.drafts[(b * st.k + lvl - 1) * st.b_max + tt.rank[v]] : -1;
    }
    st.tok[b * tt.n_nodes + v] = t;
  }
}

void launch_fill_tokens(const SeqState& st, const TreeTab& tt, int B, const int* injected,
                        hipStream_t s) {
  hipLaunchKernelGGL(k_fill_tokens, dim3(B), dim3(64), 0, s, st, tt, injected);
}

// ------------------------------------------------------------------------------------------
template <typename WT>
__global__ void k_embed(const WT* __restrict__ E, const int* __restrict__ tok, int d, int vocab, float* x) {
  int r = blockIdx.x;
  int t = tok[r];
  if (t < 0 || t >= vocab) t = 0;  // "no candidate" (-1), or an id derived from non-finite logits
  const WT* e = E + (size_t)t * d;
  for (int i = threadIdx.x; i < d; i += blockDim.x) x[(size_t)r * d + i] = to_f32(e[i]);
}

void launch_embed(const void* embed, int dtype, const int* tok, int rows, int d, int vocab, float* x,
                  hipStream_t s) {
  if (dtype == DT_BF16)
    hipLaunchKernelGGL(k_embed<bf16>, dim3(rows), dim3(256), 0, s, (const bf16*)embed, tok, d, vocab, x);
  else
    hipLaunchKernelGGL(k_embed<float>, dim3(rows), dim3(256), 0, s, (const float*)embed, tok, d, vocab, x);
}

// ------------------------------------------------------------------------------------------
// Residual update + RMSNorm: x[r] += sum_s part[s][r]; act[r] = x[r] * g, and the sum of squares
// of the row in pieces (the 1/rms factor is applied by whoever consumes the projection of act,
// see RowScale).  blockIdx = (row, piece): a piece is 1024 columns, one float4 per thread, all
// loads of a thread independent 128-bit loads.
template <typename GT, bool SPLIT, bool NORM, int SMAX>
__global__ __launch_bounds__(256) void k_add_rmsnorm(float* x, Partial part, int d, const GT* __restrict__ gain,
                                                     Act out, float* __restrict__ ss_out) {
  __shared__ float red[4];
  const int r = blockIdx.x, piece = blockIdx.y;
  const int i = piece * 256 + threadIdx.x;   // float4 index in the row
  float ss = 0.f;
  if (i < (d >> 2)) {
    float4* xr = (float4*)(x + (size_t)r * d);
    float4 a = xr[i];
    if (part.p) {
      const float* pp = part.p + (size_t)r * part.ld + (size_t)i * 4;
      float4 q[SMAX];
#pragma unroll
      for (int sp = 0; sp < SMAX; ++sp)
        if (sp < part.S) q[sp] = *(const float4*)(pp + (size_t)sp * part.stride);
#pragma unroll
      for (int sp = 0; sp < SMAX; ++sp)
        if (sp < part.S) {
          a.x += q[sp].x;
          a.y += q[sp].y;
          a.z += q[sp].z;
          a.w += q[sp].w;
        }
      xr[i] = a;
    }
    if constexpr (NORM) {
      ss = a.x * a.x + a.y * a.y + a.z * a.z + a.w * a.w;
      act_store4<SPLIT>(out, (size_t)r * out.ld + (size_t)i * 4, a.x * to_f32(gain[i * 4 + 0]),
                        a.y * to_f32(gain[i * 4 + 1]), a.z * to_f32(gain[i * 4 + 2]), a.w * to_f32(gain[i * 4 + 3]));
    }
  }
  if constexpr (NORM) {
    ss = block_sum_256(ss, red);
    if (threadIdx.x == 0) ss_out[(size_t)r * FIRP_NORM_PIECES + piece] = ss;
  }
}

int norm_pieces(int d) { return (d / 4 + 255) / 256; }

void launch_add_rmsnorm(float* x, const Partial& part, int rows, int d, const void* gain, int dtype, const Act& out,
                        bool split, float* ss_out, hipStream_t s) {
  dim3 g(rows, norm_pieces(d)), b(256);
  const int S = part.p ? part.S : 0;
  if (dtype == DT_BF16 && split) {
    if (S <= 4)
      hipLaunchKernelGGL((k_add_rmsnorm<bf16, true, true, 4>), g, b, 0, s, x, part, d, (const bf16*)gain, out, ss_out);
    else if (S <= 8)
      hipLaunchKernelGGL((k_add_rmsnorm<bf16, true, true, 8>), g, b, 0, s, x, part, d, (const bf16*)gain, out, ss_out);
    else
      hipLaunchKernelGGL((k_add_rmsnorm<bf16, true, true, 16>), g, b, 0, s, x, part, d, (const bf16*)gain, out, ss_out);
  } else if (dtype == DT_BF16) {
    hipLaunchKernelGGL((k_add_rmsnorm<bf16, false, true, 16>), g, b, 0, s, x, part, d, (const bf16*)gain, out, ss_out);
  } else {
    hipLaunchKernelGGL((k_add_rmsnorm<float, false, true, 16>), g, b, 0, s, x, part, d, (const float*)gain, out, ss_out);
  }
}

void launch_add_partial(float* x, const Partial& part, int rows, int d, hipStream_t s) {
  Act none{};
  hipLaunchKernelGGL((k_add_rmsnorm<float, false, false, 16>), dim3(rows, norm_pieces(d)), dim3(256), 0, s, x, part, d,
                     (const float*)nullptr, none, (float*)nullptr);
}

// ------------------------------------------------------------------------------------------
// Rotary embedding (half-split pairs (j, j+dh/2), angle pos * base^(-2j/dh)) on q and k at the
// row's position id p0 + pos_off (tree nodes keep their original positions; siblings share
// one), then K and V^T go to cache slot p0 + local.  cos/sin come from a per-step table whose
// angles are formed in fp64: at positions in the thousands an fp32 product would already be
// off by 1e-4 rad.
__global__ void k_rope_table(RowTab rt, const int* __restrict__ p0, int half, float rope_base, float2* tab) {
  int r = blockIdx.x, j = threadIdx.x;
  if (j >= half) return;
  double inv_freq = exp2(-(double)j / (double)half * log2((double)rope_base));
  double ang = (double)(p0[rt.seq[r]] + rt.pos_off[r]) * inv_freq;
  double sd, cd;
  sincos(ang, &sd, &cd);
  tab[(size_t)r * half + j] = make_float2((float)cd, (float)sd);
}

void launch_rope_table(const RowTab& rt, const int* p0, int rows, int head_dim, float rope_base, float2* tab,
                       hipStream_t s) {
  hipLaunchKernelGGL(k_rope_table, dim3(rows), dim3(head_dim / 2), 0, s, rt, p0, head_dim / 2, rope_base, tab);
}

// blockDim = (dh/2, heads per block); blockIdx = (row, head group)
template <typename KT, bool SPLIT>
__global__ void k_rope_kv(Partial qkv, RowScale rs, int n_q_heads, RowTab rt, const int* __restrict__ p0,
                          const float2* __restrict__ tab, Act q_out, KvView kv) {
  int r = blockIdx.x, h = blockIdx.y * blockDim.y + threadIdx.y, j = threadIdx.x;
  int dh = kv.head_dim, half = dh >> 1, Hkv = kv.n_kv_heads;
  if (h >= n_q_heads + 2 * Hkv) return;
  int b = rt.seq[r];
  size_t row_off = (size_t)r * qkv.ld;
  const float scale = row_scale(rs, r);
  float x1 = partial_sum(qkv, row_off + (size_t)h * dh + j) * scale;
  float x2 = partial_sum(qkv, row_off + (size_t)h * dh + j + half) * scale;
  if (h < n_q_heads + Hkv) {
    float2 cs = tab[(size_t)r * half + j];
    float y1 = x1 * cs.x - x2 * cs.y, y2 = x2 * cs.x + x1 * cs.y;
    if (h < n_q_heads) {
      act_store<SPLIT>(q_out, (size_t)r * q_out.ld + (size_t)h * dh + j, y1);
      act_store<SPLIT>(q_out, (size_t)r * q_out.ld + (size_t)h * dh + j + half, y2);
    } else {
      int hk = h - n_q_heads;
      size_t slot = (size_t)(p0[b] + rt.local[r]);
      KT* krow = (KT*)kv.k + (size_t)b * kv.seq_stride + ((size_t)hk * kv.slots + slot) * dh;
      store_elt<KT>(krow + j, y1);
      store_elt<KT>(krow + j + half, y2);
    }
  } else {
    int hv = h - n_q_heads - Hkv;
    size_t slot = (size_t)(p0[b] + rt.local[r]);
    KT* vt = (KT*)kv.v + (size_t)b * kv.seq_stride + (size_t)hv * dh * kv.slots + slot;
    store_elt<KT>(vt + (size_t)j * kv.slots, x1);
    store_elt<KT>(vt + (size_t)(j + half) * kv.slots, x2);
  }
}

void launch_rope_kv(const Partial& qkv, const RowScale& rs, int rows, int n_q_heads, const RowTab& rt, const int* p0,
                    const float2* tab, const Act& q_out, bool split, const KvView& kv, int dtype,
                    hipStream_t s) {
  int half = kv.head_dim / 2;
  int hpb = std::max(1, 256 / half);
  int heads = n_q_heads + 2 * kv.n_kv_heads;
  dim3 g(rows, (heads + hpb - 1) / hpb), b(half, hpb);
  if (dtype == DT_BF16) {
    if (split)
      hipLaunchKernelGGL((k_rope_kv<bf16, true>), g, b, 0, s, qkv, rs, n_q_heads, rt, p0, tab, q_out, kv);
    else
      hipLaunchKernelGGL((k_rope_kv<bf16, false>), g, b, 0, s, qkv, rs, n_q_heads, rt, p0, tab, q_out, kv);
  } else {
    hipLaunchKernelGGL((k_rope_kv<float, false>), g, b, 0, s, qkv, rs, n_q_heads, rt, p0, tab, q_out, kv);
  }
}

// ------------------------------------------------------------------------------------------
// SwiGLU: act = silu(gate) * up, gate = columns [0,F), up = columns [F,2F) of the partials.
// Four columns per thread (F % 4 == 0).
template <bool SPLIT>
__global__ void k_swiglu(Partial gu, RowScale rs, int F, Act out) {
  int r = blockIdx.y;
  int j = (blockIdx.x * blockDim.x + threadIdx.x) * 4;
  if (j >= F) return;
  const float* pg = gu.p + (size_t)r * gu.ld + j;
  float4 g = make_float4(0.f, 0.f, 0.f, 0.f), u = g;
  // four splits' loads in flight at a time
  for (int sp0 = 0; sp0 < gu.S; sp0 += 4) {
    float4 a[4], b[4];
#pragma unroll
    for (int e = 0; e < 4; ++e)
      if (sp0 + e < gu.S) {
        a[e] = *(const float4*)(pg + (size_t)(sp0 + e) * gu.stride);
        b[e] = *(const float4*)(pg + F + (size_t)(sp0 + e) * gu.stride);
      }
#pragma unroll
    for (int e = 0; e < 4; ++e)
      if (sp0 + e < gu.S) {
        g.x += a[e].x; g.y += a[e].y; g.z += a[e].z; g.w += a[e].w;
        u.x += b[e].x; u.y += b[e].y; u.z += b[e].z; u.w += b[e].w;
      }
  }
  const float scale = row_scale(rs, r);
  g.x *= scale; g.y *= scale; g.z *= scale; g.w *= scale;
  u.x *= scale; u.y *= scale; u.z *= scale; u.w *= scale;
  act_store4<SPLIT>(out, (size_t)r * out.ld + j, g.x / (1.0f + expf(-g.x)) * u.x, g.y / (1.0f + expf(-g.y)) * u.y,
                    g.z / (1.0f + expf(-g.z)) * u.z, g.w / (1.0f + expf(-g.w)) * u.w);
}

void launch_swiglu(const Partial& gate_up, const RowScale& rs, int rows, int d_ffn, const Act& out, bool split,
                   hipStream_t s) {
  dim3 g((d_ffn / 4 + 255) / 256, rows), b(256);
  if (split)
    hipLaunchKernelGGL(k_swiglu<true>, g, b, 0, s, gate_up, rs, d_ffn, out);
  else
    hipLaunchKernelGGL(k_swiglu<false>, g, b, 0, s, gate_up, rs, d_ffn, out);
}

// ------------------------------------------------------------------------------------------
// FIRP map, Eq. 3: pseudo hidden state i of anchor a is W_i x_a + b_i on the raw residual
// stream.  gather: rows of x -> projection input; scatter: projection output (+bias) -> x.
template <bool SPLIT>
__global__ void k_gather_rows(const float* __restrict__ x, const int* __restrict__ src, int d, Act out) {
  int g = blockIdx.x;
  const float* xr = x + (size_t)src[g] * d;
  for (int i = threadIdx.x; i < d; i += blockDim.x) act_store<SPLIT>(out, (size_t)g * out.ld + i, xr[i]);
}

void launch_gather_rows(const float* x, const int* src_rows, int rows, int d, const Act& out,
                        bool split, hipStream_t s) {
  if (split)
    hipLaunchKernelGGL(k_gather_rows<true>, dim3(rows), dim3(256), 0, s, x, src_rows, d, out);
  else
    hipLaunchKernelGGL(k_gather_rows<false>, dim3(rows), dim3(256), 0, s, x, src_rows, d, out);
}

// y holds the k maps' outputs side by side (map i in columns [i*d, (i+1)*d)), or one map's output
// (k_in_y == 1, map index i0).  blockIdx = (anchor row, map, column chunk).
template <typename BT>
__global__ void k_scatter_pseudo(Partial y, int d, int k, int i0, int k_in_y, PseudoBias bias, float* x,
                                 int first_pseudo_row) {
  // map i0 + blockIdx.y; its rows start at first_pseudo_row + blockIdx.y * (anchor rows)
  const int g = blockIdx.x, i = i0 + blockIdx.y;
  float* xr = x + (size_t)(first_pseudo_row + (int)blockIdx.y * (int)gridDim.x + g) * d;
  const BT* bi = (const BT*)bias.b[i];
  const int c = blockIdx.z * blockDim.x + threadIdx.x;
  if (c >= d) return;
  float v = partial_sum(y, (size_t)g * y.ld + (size_t)blockIdx.y * d + c);
  if (bi) v += to_f32(bi[c]);
  xr[c] = v;
}

void launch_scatter_pseudo(const Partial& y, int n_anchor_rows, int d, int k, int i0, int k_in_y,
                           const PseudoBias& bias, int dtype, float* x, int first_pseudo_row, hipStream_t s) {
  dim3 g(n_anchor_rows, k_in_y, (d + 255) / 256);
  if (dtype == DT_BF16)
    hipLaunchKernelGGL(k_scatter_pseudo<bf16>, g, dim3(256), 0, s, y, d, k, i0, k_in_y, bias, x, first_pseudo_row);
  else
    hipLaunchKernelGGL(k_scatter_pseudo<float>, g, dim3(256), 0, s, y, d, k, i0, k_in_y, bias, x, first_pseudo_row);
}

// ------------------------------------------------------------------------------------------
// Greedy token of real rows, top-b of pseudo rows.  Order: larger logit first, ties to the
// lower token id.
struct Best {
  float v;
  int id;
};
__device__ __forceinline__ bool better(float v, int id, const Best& o) {
  return v > o.v || (v == o.v && id < o.id);
}

// Two levels.  k_argmax_part: blockIdx = (row, vocabulary segment); one pass over the segment,
// every thread keeps the best BM entries of its strided share in registers (sorted insertion),
// then `want` rounds of a block-wide arg-best over the threads' current heads leave the
// segment's best entries, in order, in cand[row][segment][BM].  k_argmax_merge: one block per
// row picks the row's top entries out of the segments' candidates the same way.
#define FIRP_ARGMAX_SEGS 8
template <int BM>
__global__ __launch_bounds__(256) void k_argmax_part(Partial lg, RowScale rs, float* logits_out, int real_rows,
                                                     int vocab, int b_max, Best* __restrict__ cand) {
  __shared__ float sv[256];
  __shared__ int si[256];
  const int r = blockIdx.x, seg = blockIdx.y, tid = threadIdx.x;
  const size_t off = (size_t)r * lg.ld;
  const bool copy = logits_out && (lg.S > 1 || logits_out != lg.p || rs.ss);
  const int want = (r < real_rows) ? 1 : b_max;
  const float scale = row_scale(rs, r);
  const int seg_len = ((vocab + FIRP_ARGMAX_SEGS - 1) / FIRP_ARGMAX_SEGS + 3) & ~3;
  const int t0 = seg * seg_len, t1 = min(vocab, t0 + seg_len);
  Best mine[BM];
#pragma unroll
  for (int e = 0; e < BM; ++e) mine[e] = Best{-__builtin_inff(), 0x7fffffff};
  for (int t = t0 + tid; t < t1; t += 256) {
    float v = partial_sum(lg, off + t) * scale;
    if (copy) logits_out[(size_t)r * vocab + t] = v;
    if (better(v, t, mine[BM - 1])) {
      mine[BM - 1] = Best{v, t};
#pragma unroll
      for (int e = BM - 1; e > 0; --e)
        if (better(mine[e].v, mine[e].id, mine[e - 1])) {
          Best tmp = mine[e - 1];
          mine[e - 1] = mine[e];
          mine[e] = tmp;
        }
    }
  }
  Best* out = cand + ((size_t)r * FIRP_ARGMAX_SEGS + seg) * BM;
  for (int p = 0; p < want; ++p) {
    sv[tid] = mine[0].v;
    si[tid] = mine[0].id;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
      if (tid < w) {
        Best o{sv[tid + w], si[tid + w]};
        Best m{sv[tid], si[tid]};
        if (better(o.v, o.id, m)) {
          sv[tid] = o.v;
          si[tid] = o.id;
        }
      }
      __syncthreads();
    }
    const Best win{sv[0], si[0]};
    __syncthreads();
    if (mine[0].id == win.id && win.id != 0x7fffffff) {  // the owner pops its head
#pragma unroll
      for (int e = 0; e + 1 < BM; ++e) mine[e] = mine[e + 1];
      mine[BM - 1] = Best{-__builtin_inff(), 0x7fffffff};
    }
    if (tid == 0) out[p] = win;
  }
}

template <int BM>
__global__ __launch_bounds__(64) void k_argmax_merge(const Best* __restrict__ cand, int real_rows, int vocab,
                                                     int b_max, int* amax, int* top) {
  const int r = blockIdx.x, lane = threadIdx.x;
  const int want = (r < real_rows) ? 1 : b_max;
  // lane = (segment, slot) for up to 8 segments x 8 slots; with BM = 16 a lane holds two slots
  constexpr int PER = (FIRP_ARGMAX_SEGS * BM + 63) / 64;
  Best mine[PER];
#pragma unroll
  for (int e = 0; e < PER; ++e) {
    const int idx = lane * PER + e;           // consecutive slots of one segment are in order
    const int slot = idx % BM;
    mine[e] = (idx < FIRP_ARGMAX_SEGS * BM && slot < want) ? cand[(size_t)r * FIRP_ARGMAX_SEGS * BM + idx]
                                                           : Best{-__builtin_inff(), 0x7fffffff};
  }
  for (int p = 0; p < want; ++p) {
    Best m = mine[0];
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
      Best other{__shfl_xor(m.v, o, 64), __shfl_xor(m.id, o, 64)};
      if (better(other.v, other.id, m)) m = other;
    }
    int win = m.id;
    if (mine[0].id == win && win != 0x7fffffff) {
#pragma unroll
      for (int e = 0; e + 1 < PER; ++e) mine[e] = mine[e + 1];
      mine[PER - 1] = Best{-__builtin_inff(), 0x7fffffff};
    }
    if (win >= vocab) win = 0;  // only when every remaining logit is NaN
    if (lane == 0) {
      if (r < real_rows)
        amax[r] = win;
      else
        top[(size_t)(r - real_rows) * b_max + p] = win;
    }
  }
}

size_t argmax_scratch_bytes(int rows, int b_max) {
  return (size_t)rows * FIRP_ARGMAX_SEGS * (b_max <= 8 ? 8 : 16) * sizeof(Best);
}

void launch_argmax_topb(const Partial& logits, const RowScale& rs, float* logits_out, int real_rows, int rows,
                        int vocab, int b_max, int* amax, int* top, void* scratch, hipStream_t s) {
  Best* cand = (Best*)scratch;
  dim3 g(rows, FIRP_ARGMAX_SEGS);
  if (b_max <= 8) {
    hipLaunchKernelGGL(k_argmax_part<8>, g, dim3(256), 0, s, logits, rs, logits_out, real_rows, vocab, b_max, cand);
    hipLaunchKernelGGL(k_argmax_merge<8>, dim3(rows), dim3(64), 0, s, cand, real_rows, vocab, b_max, amax, top);
  } else {
    hipLaunchKernelGGL(k_argmax_part<16>, g, dim3(256), 0, s, logits, rs, logits_out, real_rows, vocab, b_max, cand);
    hipLaunchKernelGGL(k_argmax_merge<16>, dim3(rows), dim3(64), 0, s, cand, real_rows, vocab, b_max, amax, top);
  }
}

// ------------------------------------------------------------------------------------------
// Training stage, Eq. 4: kl[q] = KL(softmax(logits[n + q]), softmax(logits[q + step])) for
// q < n - step, with KL(A, B) = sum_t A_t (log A_t - log B_t).  One block per q; three passes
// over the two rows (maxima, normalisers, the sum).
__global__ __launch_bounds__(256) void k_kl_rows(const float* __restrict__ logits, int vocab, int n, int step,
                                                 float* __restrict__ kl) {
  __shared__ float red[4];
  const int q = blockIdx.x;
  const float* a = logits + (size_t)(n + q) * vocab;
  const float* b = logits + (size_t)(q + step) * vocab;
  float ma = -__builtin_inff(), mb = -__builtin_inff();
  for (int t = threadIdx.x; t < vocab; t += 256) {
    ma = fmaxf(ma, a[t]);
    mb = fmaxf(mb, b[t]);
  }
  ma = wave_max(ma);
  mb = wave_max(mb);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ma;
  __syncthreads();
  ma = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = mb;
  __syncthreads();
  mb = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
  float sa = 0.f, sb = 0.f;
  for (int t = threadIdx.x; t < vocab; t += 256) {
    sa += expf(a[t] - ma);
    sb += expf(b[t] - mb);
  }
  sa = block_sum_256(sa, red);
  sb = block_sum_256(sb, red);
  const float la = ma + logf(sa), lb = mb + logf(sb);   // log normalisers
  float acc = 0.f;
  for (int t = threadIdx.x; t < vocab; t += 256) {
    const float lpa = a[t] - la;
    acc += expf(lpa) * (lpa - (b[t] - lb));
  }
  acc = block_sum_256(acc, red);
  if (threadIdx.x == 0) kl[q] = acc;
}

void launch_kl_rows(const float* logits, int vocab, int n, int step, float* kl, hipStream_t s) {
  hipLaunchKernelGGL(k_kl_rows, dim3(n - step), dim3(256), 0, s, logits, vocab, n, step, kl);
}

// ------------------------------------------------------------------------------------------
// Greedy verification (Inference stage): from the root, emit the greedy token of the current
// node and move to the child that carries it (lowest node id if several do); stop when none
// does.  Then read the next drafts off the pseudo rows of the node that ends the path.
__global__ void k_verify_select(SeqState st, TreeTab tt) {
  int b = blockIdx.x;
  int N = tt.n_nodes;
  int* res = st.result + b * FIRP_RESULT_STRIDE;
  __shared__ int s_cur;
  if (threadIdx.x == 0) {
    const int* tok = st.tok + b * N;
    const int* amax = st.amax + b * N;
    int cur = 0, n = 0;
    int* out_tok = res + 3;
    int* out_path = res + 3 + (st.k_cap + 1);
    while (true) {
      int t = amax[cur];
      out_tok[n] = t;
      out_path[n] = cur;
      ++n;
      int nxt = -1;
      for (int e = tt.child_start[cur]; e < tt.child_start[cur + 1]; ++e) {
        int c = tt.child_list[e];
        if (tok[c] == t) {
          nxt = c;
          break;
        }
      }
      if (nxt < 0 || n > st.k_cap) break;  // n <= k_cap + 1 by the depth check on the host
      cur = nxt;
    }
    int pb = tt.pseudo_base[cur];
    res[0] = n;
    res[1] = (pb >= 0 && st.k > 0) ? 1 : 0;
    res[2] = st.p0[b];  // cache length before this step's commit
    st.p0[b] += n;
    st.root_tok[b] = out_tok[n - 1];
    st.drafts_valid[b] = res[1];
    s_cur = cur;
  }
  __syncthreads();
  int pb = tt.pseudo_base[s_cur];
  if (pb >= 0 && st.k > 0) {
    // pseudo rows are ordered step by step: step i of anchor a of sequence b is pseudo row
    // i * (B * A) + b * A + a
    const int B = gridDim.x, A = tt.n_anchor, a = pb - N;
    for (int e = threadIdx.x; e < st.k * st.b_max; e += blockDim.x) {
      const int i = e / st.b_max, j = e - i * st.b_max;
      st.drafts[(size_t)b * st.k * st.b_max + e] = st.top[((size_t)i * B * A + (size_t)b * A + a) * st.b_max + j];
    }
  }
}

void launch_verify_select(const SeqState& st, const TreeTab& tt, int B, hipStream_t s) {
  hipLaunchKernelGGL(k_verify_select, dim3(B), dim3(64), 0, s, st, tt);
}

// ------------------------------------------------------------------------------------------
// Commit: the accepted path's nodes sit at slots p0 + path[j]; move them to p0 + j.  Nodes are
// in topological order so path[j] >= j: every destination lies at or before its source.  All
// sources are read before any destination is written.
template <typename KT>
__global__ __launch_bounds__(256) void k_kv_compact(KvView kv0, size_t layer_stride, SeqState st) {
  int layer = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  const int* res = st.result + b * FIRP_RESULT_STRIDE;
  int n = res[0], p0 = res[2];
  const int* path = res + 3 + (st.k_cap + 1);
  bool moved = false;
  for (int j = 1; j < n; ++j) moved |= (path[j] != j);
  if (!moved) return;
  int dh = kv0.head_dim, e = threadIdx.x;
  KT* K = (KT*)kv0.k + (size_t)b * kv0.seq_stride + (size_t)layer * layer_stride + (size_t)h * kv0.slots * dh;
  KT* Vt = (KT*)kv0.v + (size_t)b * kv0.seq_stride + (size_t)layer * layer_stride + (size_t)h * dh * kv0.slots;
  KT kk[FIRP_MAX_COMMIT], vv[FIRP_MAX_COMMIT];
  if (e < dh) {
#pragma unroll
    for (int j = 1; j < FIRP_MAX_COMMIT; ++j)
      if (j < n) {
        kk[j] = K[(size_t)(p0 + path[j]) * dh + e];
        vv[j] = Vt[(size_t)e * kv0.slots + p0 + path[j]];
      }
  }
  __syncthreads();
  if (e < dh) {
#pragma unroll
    for (int j = 1; j < FIRP_MAX_COMMIT; ++j)
      if (j < n) {
        K[(size_t)(p0 + j) * dh + e] = kk[j];
        Vt[(size_t)e * kv0.slots + p0 + j] = vv[j];
      }
  }
}

void launch_kv_compact(const KvView& kv0, size_t layer_stride, int n_layers, int B, const SeqState& st,
                       int dtype, hipStream_t s) {
  dim3 g(n_layers, kv0.n_kv_heads, B), blk(256);
  if (dtype == DT_BF16)
    hipLaunchKernelGGL(k_kv_compact<bf16>, g, blk, 0, s, kv0, layer_stride, st);
  else
    hipLaunchKernelGGL(k_kv_compact<float>, g, blk, 0, s, kv0, layer_stride, st);
}

// ------------------------------------------------------------------------------------------
__global__ void k_advance_by(int* p0, int seq, int n) { p0[seq] += n; }
void launch_advance_by(int* p0, int seq, int n, hipStream_t s) {
  hipLaunchKernelGGL(k_advance_by, dim3(1), dim3(1), 0, s, p0, seq, n);
}

__global__ void k_set_root(SeqState st, int seq, int token, int p0) {
  st.root_tok[seq] = token;
  st.drafts_valid[seq] = 0;
  st.p0[seq] = p0;
}
void launch_set_root(const SeqState& st, int seq, int token, int p0, hipStream_t s) {
  hipLaunchKernelGGL(k_set_root, dim3(1), dim3(1), 0, s, st, seq, token, p0);
}

// ------------------------------------------------------------------------------------------
// helpers of the standalone projection entry
__global__ void k_split_act(const float* __restrict__ x, int ld, Act out) {
  int r = blockIdx.x;
  for (int i = threadIdx.x; i < ld; i += blockDim.x) act_store<true>(out, (size_t)r * out.ld + i, x[(size_t)r * ld + i]);
}
void launch_split_act(const float* x, int rows, int ld, const Act& out, hipStream_t s) {
  hipLaunchKernelGGL(k_split_act, dim3(rows), dim3(256), 0, s, x, ld, out);
}

__global__ void k_reduce_partials(Partial p, float* y) {
  int r = blockIdx.y;
  int c = blockIdx.x * blockDim.x + threadIdx.x;
  if (c < p.ld) y[(size_t)r * p.ld + c] = partial_sum(p, (size_t)r * p.ld + c);
}
void launch_reduce_partials(const Partial& p, float* y, int rows, hipStream_t s) {
  hipLaunchKernelGGL(k_reduce_partials, dim3((p.ld + 255) / 256, rows), dim3(256), 0, s, p, y);
}

// ------------------------------------------------------------------------------------------
// A plain streaming read (the measured ceiling the step's bandwidth is compared with): nothing
// but loads.  They carry the non-temporal hint like the projection's weight loads (measured: 6.9 TB/s
// against 6.1 TB/s without it).
__device__ __forceinline__ uint4 nt_load16(const uint4* p) {
  typedef unsigned int u4 __attribute__((ext_vector_type(4)));
  const u4 r = __builtin_nontemporal_load((const u4*)p);
  return make_uint4(r.x, r.y, r.z, r.w);
}
// Every wave walks two private contiguous runs, 1 KiB per instruction and 4 KiB ahead in each (the
// projection's shape of traffic); what the runs leave over is read with a grid-wide stride.
__global__ __launch_bounds__(512) void k_stream_read(const uint4* __restrict__ src, size_t n16, unsigned* __restrict__ sink) {
  constexpr int STREAMS = 2, DEPTH = 4;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, wpb = blockDim.x >> 6;
  const size_t nstreams = (size_t)gridDim.x * wpb * STREAMS;
  const size_t per = n16 / nstreams / (64 * DEPTH) * (64 * DEPTH);   // 16-byte items of one run
  const size_t s0 = ((size_t)blockIdx.x * wpb + wave) * STREAMS;
  uint4 acc = make_uint4(0, 0, 0, 0);
  for (size_t off = 0; off < per; off += 64 * DEPTH) {
    uint4 v[STREAMS][DEPTH];
#pragma unroll
    for (int st = 0; st < STREAMS; ++st)
#pragma unroll
      for (int j = 0; j < DEPTH; ++j) v[st][j] = nt_load16(src + (s0 + st) * per + off + j * 64 + lane);
#pragma unroll
    for (int st = 0; st < STREAMS; ++st)
#pragma unroll
      for (int j = 0; j < DEPTH; ++j) {
        acc.x ^= v[st][j].x;
        acc.y ^= v[st][j].y;
        acc.z ^= v[st][j].z;
        acc.w ^= v[st][j].w;
      }
  }
  for (size_t i = nstreams * per + (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16;
       i += (size_t)gridDim.x * blockDim.x) {
    uint4 v = nt_load16(src + i);
    acc.x ^= v.x;
    acc.y ^= v.y;
    acc.z ^= v.z;
    acc.w ^= v.w;
  }
  if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x9e3779b9u) sink[0] = acc.x;   // keeps the loads alive; practically never taken
}

void launch_stream_read(const void* src, size_t bytes, unsigned* sink, hipStream_t s) {
  hipLaunchKernelGGL(k_stream_read, dim3(512), dim3(512), 0, s, (const uint4*)src, bytes / 16, sink);
}

}  // namespace firp
