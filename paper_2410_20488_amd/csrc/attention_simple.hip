// Plain tree-masked attention: one workgroup per (row, q-head) walks the row's visible keys.
// Visible = every committed cache slot [0, p0) plus the step slots p0 + c whose bit c is set
// in the row's mask (Tree attention: a node sees its ancestors and itself; a pseudo row also
// sees the earlier pseudo rows of its anchor).  fp32 softmax with max subtraction.
#include "kernels.h"

namespace firp {

template <bool SPLIT>
__device__ __forceinline__ float act_load(const Act& a, size_t idx) {
  if constexpr (SPLIT)
    return to_f32(a.hi[idx]) + to_f32(a.lo[idx]);
  else
    return a.f32[idx];
}

template <typename KT, bool SPLIT>
__global__ __launch_bounds__(256) void k_attention_simple(Act q, int n_q_heads, RowTab rt,
                                                          const int* __restrict__ p0, KvView kv, Act out,
                                                          int n_local) {
  extern __shared__ float smem[];
  __shared__ float red[4];
  int r = blockIdx.x, h = blockIdx.y, tid = threadIdx.x;
  int dh = kv.head_dim;
  float* qs = smem;            // [dh]
  float* sc = smem + dh;       // [keys]
  int b = rt.seq[r];
  int ctx = p0[b];
  int hk = h / (n_q_heads / kv.n_kv_heads);
  const KT* K = (const KT*)kv.k + (size_t)b * kv.seq_stride + (size_t)hk * kv.slots * dh;
  const KT* Vt = (const KT*)kv.v + (size_t)b * kv.seq_stride + (size_t)hk * dh * kv.slots;
  const unsigned long long* mask = rt.mask + (size_t)r * FIRP_MASK_WORDS;
  for (int i = tid; i < dh; i += 256) qs[i] = act_load<SPLIT>(q, (size_t)r * q.ld + (size_t)h * dh + i);
  __syncthreads();
  int nkeys = ctx + n_local;
  float scale = 1.0f / sqrtf((float)dh);
  float mx = -__builtin_inff();
  for (int j = tid; j < nkeys; j += 256) {
    bool vis = j < ctx || ((mask[(j - ctx) >> 6] >> ((j - ctx) & 63)) & 1ull);
    float s = -__builtin_inff();
    if (vis) {
      const KT* kr = K + (size_t)j * dh;
      float a = 0.f;
      for (int i = 0; i < dh; ++i) a += qs[i] * to_f32(kr[i]);
      s = a * scale;
    }
    sc[j] = s;
    mx = fmaxf(mx, s);
  }
  mx = wave_max(mx);
  __syncthreads();
  if ((tid & 63) == 0) red[tid >> 6] = mx;
  __syncthreads();
  mx = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
  float sum = 0.f;
  for (int j = tid; j < nkeys; j += 256) {
    float e = (sc[j] == -__builtin_inff()) ? 0.f : expf(sc[j] - mx);
    sc[j] = e;
    sum += e;
  }
  sum = block_sum_256(sum, red);
  float inv = 1.0f / sum;
  for (int d = tid; d < dh; d += 256) {
    const KT* vr = Vt + (size_t)d * kv.slots;
    float o = 0.f;
    for (int j = 0; j < nkeys; ++j) o += sc[j] * to_f32(vr[j]);
    act_store<SPLIT>(out, (size_t)r * out.ld + (size_t)h * dh + d, o * inv);
  }
}

void launch_attention_simple(const Act& q, bool split, int rows, int n_q_heads, const RowTab& rt,
                             const int* p0, const KvView& kv, int dtype, const Act& out,
                             int n_local, int max_keys, hipStream_t s) {
  dim3 g(rows, n_q_heads), b(256);
  size_t sm = (size_t)(kv.head_dim + max_keys) * sizeof(float);
  if (dtype == DT_BF16) {
    if (split)
      hipLaunchKernelGGL((k_attention_simple<bf16, true>), g, b, sm, s, q, n_q_heads, rt, p0, kv, out, n_local);
    else
      hipLaunchKernelGGL((k_attention_simple<bf16, false>), g, b, sm, s, q, n_q_heads, rt, p0, kv, out, n_local);
  } else {
    hipLaunchKernelGGL((k_attention_simple<float, false>), g, b, sm, s, q, n_q_heads, rt, p0, kv, out, n_local);
  }
}

}  // namespace firp
