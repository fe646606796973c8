// Launchers of the step's kernels.  Everything is enqueued on the given stream; nothing here
// synchronises or allocates.
#pragma once
#include "common.h"

namespace firp {

enum { DT_F32 = 0, DT_BF16 = 1 };

// KV cache of one layer.  K: [B][Hkv][slots][dh]; V is stored transposed, [B][Hkv][dh][slots],
// so that the P.V contraction reads keys contiguously.  seq_stride = elements between sequences.
struct KvView {
  void* k;
  void* v;
  size_t seq_stride;
  int slots;  // per (sequence, head): max_ctx + step rows, multiple of 64
  int n_kv_heads, head_dim;
};

// Node tables of the tree (device), shared by all sequences of a step.
struct TreeTab {
  const int* parent;
  const int* level;       // depth of node v (root 0)
  const int* rank;
  const int* child_start; // CSR over children, [N+1]
  const int* child_list;  // [N-1]
  const int* pseudo_base; // local row of the first pseudo row (step 1) of node v, or -1; the
                          // row of step i is n_anchor further per step
  int n_nodes;
  int n_pseudo;           // pseudo rows per sequence (k * n_anchor)
  int n_anchor;           // anchors per sequence
};

// Per-sequence decoding state (device).
struct SeqState {
  int* p0;           // [B] committed cache length
  int* root_tok;     // [B] last emitted token = next root
  int* drafts;       // [B][k][b_max]
  int* drafts_valid; // [B]
  int* tok;          // [B][N] token of every node of the running step
  int* amax;         // [B*N] greedy token per real row
  int* top;          // [B*P][b_max] top-b ids per pseudo row
  int* result;       // [B][RESULT_STRIDE]: n_emitted, drafts_valid, p0 before, tokens[k_cap+1], path[k_cap+1]
  int k, b_max, k_cap;
};
#define FIRP_RESULT_STRIDE 40
#define FIRP_MAX_COMMIT 9   // deepest tree level + 1

void launch_fill_tokens(const SeqState& st, const TreeTab& tt, int B, const int* injected,
                        hipStream_t s);
void launch_embed(const void* embed, int dtype, const int* tok, int rows, int d, int vocab, float* x,
                  hipStream_t s);
// x[r] += sum of partials (if part.p), then act = x[r] * gain and ss_out[r][piece] = the row's
// sums of squares (see RowScale: the 1/rms factor is applied after the projection).
int norm_pieces(int d);
void launch_add_rmsnorm(float* x, const Partial& part, int rows, int d, const void* gain, int dtype, const Act& out,
                        bool split, float* ss_out, hipStream_t s);
// Only the residual update, no norm output (used before the projection at the FIRP layer).
void launch_add_partial(float* x, const Partial& part, int rows, int d, hipStream_t s);
// qkv partials -> rotary q (activation planes, [rows][Hq*dh]) and K / V^T into the cache.
void launch_rope_table(const RowTab& rt, const int* p0, int rows, int head_dim, float rope_base,
                       float2* tab, hipStream_t s);   // cos/sin of every row's position, once per step
void launch_rope_kv(const Partial& qkv, const RowScale& rs, int rows, int n_q_heads, const RowTab& rt, const int* p0,
                    const float2* tab, const Act& q_out, bool split, const KvView& kv, int dtype,
                    hipStream_t s);
void launch_swiglu(const Partial& gate_up, const RowScale& rs, int rows, int d_ffn, const Act& out, bool split,
                   hipStream_t s);
// FIRP map (Eq. 3): gather anchor rows of the residual stream as projection input ...
void launch_gather_rows(const float* x, const int* src_rows, int rows, int d, const Act& out,
                        bool split, hipStream_t s);
// ... and scatter the maps' outputs (+ bias) to the pseudo rows: y holds `k_in_y` maps side by
// side starting with map i0; anchor row g of the j-th of them goes to row first_pseudo_row +
// j * n_anchor_rows + g (pseudo rows are ordered step by step).
struct PseudoBias {
  const void* b[8];  // per map, nullptr = none
};
void launch_scatter_pseudo(const Partial& y, int n_anchor_rows, int d, int k, int i0, int k_in_y,
                           const PseudoBias& bias, int dtype, float* x, int first_pseudo_row, hipStream_t s);
// greedy token of every real row and top-b of every pseudo row; also leaves summed logits.
// (two launches: per vocabulary segment, then a merge; `scratch` >= argmax_scratch_bytes)
size_t argmax_scratch_bytes(int rows, int b_max);
void launch_argmax_topb(const Partial& logits, const RowScale& rs, float* logits_out, int real_rows, int rows,
                        int vocab, int b_max, int* amax, int* top, void* scratch, hipStream_t s);
// Training stage, Eq. 4: kl[q] = KL(softmax(logits[n+q]) , softmax(logits[q+step])), q < n - step
void launch_kl_rows(const float* logits, int vocab, int n, int step, float* kl, hipStream_t s);
void launch_verify_select(const SeqState& st, const TreeTab& tt, int B, hipStream_t s);
// move the accepted path's K/V to the front of the step's slots; advances nothing.
void launch_kv_compact(const KvView& kv_layer0, size_t layer_stride, int n_layers, int B,
                       const SeqState& st, int dtype, hipStream_t s);
void launch_advance_by(int* p0, int seq, int n, hipStream_t s);           // prefill chunk
void launch_set_root(const SeqState& st, int seq, int token, int p0, hipStream_t s);

// plain attention: every (row, head) walks its visible keys
void launch_attention_simple(const Act& q, bool split, int rows, int n_q_heads, const RowTab& rt,
                             const int* p0, const KvView& kv, int dtype, const Act& out,
                             int n_local, int max_keys, hipStream_t s);

// MFMA flash-decode attention over a bf16 cache; see attention_mfma.hip.  `scratch` holds the
// per-split partial results (attention_mfma_scratch_floats floats).
#define FIRP_ATTN_MAX_SPLITS 16
bool attention_mfma_supported(int head_dim, int dtype);
size_t attention_mfma_scratch_floats(int rows, int n_q_heads, int head_dim);
void launch_attention_mfma(const bf16* q_frag, int rows, int n_q_heads, int B, int n_real_per_seq,
                           int n_pseudo_per_seq, int n_anchor_per_seq, int seq0, const RowTab& rt, const int* p0, int max_ctx_now,
                           const KvView& kv, float* scratch, const Act& out, hipStream_t s);
// (seq0: first sequence of the launch; a prefill chunk runs one sequence as a batch of one.)
// Its operand producer (replaces launch_rope_kv on this path): q as MFMA fragments in q_frag
// (attention_q_frag_elems bf16 elements), K and V^T into the cache.
size_t attention_q_frag_elems(int rows, int max_batch, int n_q_heads, int head_dim);
void launch_rope_kv_tiles(const Partial& qkv, const RowScale& rs, int n_q_heads, int B, int n_real_per_seq,
                          int n_pseudo_per_seq, int n_anchor_per_seq, int seq0, const int* p0, const float2* tab, bf16* q_frag, const KvView& kv,
                          hipStream_t s);

// plain tiled projection: y[S=1][rows][n] = x_f32[rows][K] . W[n][K]^T
void launch_gemm_simple(const float* x, int ldx, const void* w, int dtype, float* y, int ldy,
                        int rows, int n, int K, hipStream_t s);

// MFMA weight-streaming projection for bf16 weights; see gemm_mfma.hip
struct GemmPlan {
  int S;        // split-K factor
  int k_per;    // K elements per split (multiple of 64)
  int nt;       // 16-row activation tiles of one pass of the streaming kernel (up to 8)
  int nw;       // waves per workgroup (each owns 32 rows of W): 2..8
  int grid;
  int row_block;  // activation rows one launch takes: 128, or 256 (the kernel for 129..256 rows)
};
GemmPlan gemm_mfma_plan_ex(int rows, int n, int K, int S, int nw);
bool gemm_mfma_supported(int rows, int n, int K);
GemmPlan gemm_mfma_plan(int rows, int n, int K, int force_split);  // force_split 0 = choose
// Up to three row-major [n_i][K] matrices stacked along n (rows [0,n0) from w0, the next n1 from
// w1, the rest from w2).  A single matrix has n0 >= n.
struct WSeg {
  const bf16 *w0, *w1, *w2;
  int n0, n1;
};
inline WSeg wseg1(const void* w, int n) { return WSeg{(const bf16*)w, nullptr, nullptr, n, 0}; }
// The kernel streams W from a fragment-major copy: the [n][K] matrix, zero-padded to multiples
// of 16 rows and 64 columns, cut into 16-row x 32-column fragments; fragment (t, s) is the
// 1 KiB block number t * (Kpad / 32) + s and holds, at byte 16 * lane, the 8 elements
// W[16 t + lane % 16][32 s + 8 (lane / 16) ...]: exactly the A operand of one
// v_mfma_f32_16x16x32_bf16, so that a wave's load instruction covers eight whole cache lines.
size_t gemm_packed_bytes(int n, int K);
void launch_pack_weights(const WSeg& src, int n, int K, void* dst, hipStream_t s);
// partials[s][r][c] at out + s*part_stride + r*ld + c for c < n
void launch_gemm_mfma(const Act& x, const void* w_packed, float* out, int ld, size_t part_stride, int rows,
                      int n, int K, const GemmPlan& plan, hipStream_t s);
void launch_split_act(const float* x, int rows, int ld, const Act& out, hipStream_t s);
void launch_reduce_partials(const Partial& p, float* y, int rows, hipStream_t s);
void launch_stream_read(const void* src, size_t bytes, unsigned* sink, hipStream_t s);

}  // namespace firp
