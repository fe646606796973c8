// Step engine and C ABI: validates, parses the tree (host), sequences the kernels of
// firp_prefill / firp_step on the caller's stream, owns the carve-up of the workspace.
#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <string>
#include <vector>

#include "../../include/firp.h"
#include "kernels.h"

using namespace firp;

// Rows of the partial-sum buffer are padded by one 128-byte line: projection widths are
// multiples of 1024 floats, and rows a multiple of 4 KB apart would all fall on one memory channel.
#define FIRP_PART_PAD 32

namespace {

std::string g_init_error;

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

struct Carver {
  char* base;
  size_t off = 0;
  template <typename T>
  T* take(size_t count) {
    off = align_up(off, 256);
    T* p = base ? reinterpret_cast<T*>(base + off) : nullptr;
    off += count * sizeof(T);
    return p;
  }
};

struct HostTree {
  int B = 0, N = 0, P = 0, k = 0, n_anchor = 0, max_depth = 0;
  std::vector<int> parent, rank, depth;
  std::vector<uint8_t> anchor;
  bool same(int B_, int k_, const std::vector<int>& par, const std::vector<int>& rk,
            const std::vector<uint8_t>& an) const {
    return B == B_ && k == k_ && parent == par && rank == rk && anchor == an;
  }
};

// The per-row and per-node tables of one topology (device), one contiguous block per slot so
// that a new topology is uploaded with a single copy.  A few slots are kept: decoding alternates
// between the full tree and its root-only sub-tree (a path that ends at a non-anchor leaves no
// drafts), and neither switch may cost an upload.
#define FIRP_TOPO_SLOTS 4
struct TopoLayout {   // byte offsets inside a slot
  size_t seq, local, pos, mask, parent, level, rank, cstart, clist, pbase, psrc, bytes;
};
// What a captured step depends on besides the topology: when any of it differs, the step is
// captured again.
struct GraphKey {
  int B = 0, injected = 0, keep_logits = 0, gemm_kind = 0, attn_kind = 0;
  bool operator==(const GraphKey& o) const {
    return B == o.B && injected == o.injected && keep_logits == o.keep_logits && gemm_kind == o.gemm_kind &&
           attn_kind == o.attn_kind;
  }
};
struct TopoSlot {
  char* base = nullptr;
  HostTree key;
  bool valid = false;
  unsigned long long last_use = 0;
  // the decoding step on this topology as a captured graph: [0] with the library's own drafts,
  // [1] with injected candidates
  hipGraphExec_t exec[2] = {nullptr, nullptr};
  GraphKey gkey[2];
};

}  // namespace

struct firp_ctx {
  firp_model_desc d{};
  int k = 0, dtype = 0;
  std::vector<int> tl;  // prediction layer of every step (k entries, non-decreasing)
  bool split = false;   // activations as hi/lo bf16 planes (MFMA projection)
  int gemm_kind = 0;    // 0 plain, 1 MFMA
  int attn_kind = 0;    // 0 plain, 1 MFMA flash-decode (needs the bf16 planes of q)
  bool cache_clean = false;  // the KV cache holds only finite values (zero-filled once)
  bool keep_logits = false;  // option "keep_logits": the lm-head's consumer also writes all logits
  bool force_logits = false; // ... for the running call only (the training forward reads them)
  bool last_has_logits = false;
  float* attn_scratch = nullptr;
  void* argmax_scratch = nullptr;
  bf16* q_frag = nullptr;      // q of the running layer as MFMA fragments (MFMA attention)
  float* norm_ss = nullptr;    // [rows][FIRP_NORM_PIECES] sums of squares left by the last norm
  float2* rope_tab = nullptr;  // [rows][dh/2] (cos, sin) of the running step
  hipStream_t stream = nullptr;
  // weights
  const void* embed = nullptr;
  const void* norm_final = nullptr;
  const void* lm_head = nullptr;
  std::vector<const void*> wq, wk, wv, wo, wg, wu, wd, n1, n2, pw, pb;
  // fragment-major copies of the projection matrices (bf16 models; see gemm_packed_bytes):
  // q|k|v and gate|up stacked along n, made on the stream by the first prefill
  std::vector<void*> pk_qkv, pk_o, pk_gu, pk_d, pk_proj;
  void* pk_head = nullptr;
  bool pk_proj_stacked = false;
  bool packed = false;
  // geometry
  int Rmax = 0, Rpad = 0, slots = 0, qkv_ld = 0, esize = 0;
  size_t kv_layer_stride = 0, kv_seq_stride = 0;
  // device buffers
  float* x = nullptr;
  float* part = nullptr;
  size_t part_elems = 0;
  float* logits = nullptr;
  Act act_d{}, act_q{}, act_o{}, act_f{}, act_p{};
  void* kcache = nullptr;
  void* vcache = nullptr;
  int *rt_seq = nullptr, *rt_local = nullptr, *rt_pos = nullptr;
  unsigned long long* rt_mask = nullptr;
  int *tt_parent = nullptr, *tt_level = nullptr, *tt_rank = nullptr, *tt_cstart = nullptr,
      *tt_clist = nullptr, *tt_pbase = nullptr, *pseudo_src = nullptr, *injected = nullptr;
  SeqState st{};
  // host state
  int batch = 0;
  bool prefilled = false;
  std::vector<int> p0, drafts_valid;
  TopoLayout tl_off{};
  TopoSlot slot[FIRP_TOPO_SLOTS + 1];   // the last one: prefill chunks and the training forward (never cached)
  int cur_slot = -1;     // slot the table pointers above point into
  unsigned long long use_clock = 0;
  long topo_uploads = 0;  // topologies uploaded since firp_init (a cached one costs none)
  // option "graph": replay the step of a resident topology as a captured HIP graph: 0 never, 1
  // whenever possible, 2 (default) where it pays: measured on MI355X, a replay starts about 40 us
  // later than the first directly launched kernel, which a step of a few hundred kernels wins
  // back only while its kernels are short (0.19 against 0.24 ms per step at 4 layers of width 256,
  // equal at the 7B shape, 0.04 ms slower at 13B): steps that stream at most 8 GB of weights
  int graph_mode = 2;
  bool use_graph = true;
  bool graph_broken = false; // the stream cannot be captured (e.g. the default stream): launch directly
  long graph_launches = 0, graph_captures = 0;
  HostTree cur;          // topology of the current slot
  bool tables_valid = false;
  int last_rows = 0, last_N = 0, last_P = 0, last_steps = 0;  // last_steps: pseudo rows per anchor
  // optional timing of the projection launches (HIP events on the library's stream)
  bool time_gemm = false;
  std::vector<hipEvent_t> ev;
  size_t ev_used = 0;
  double gemm_ms = 0.0, gemm_bytes = 0.0;
  long gemm_launches = 0;
  hipEvent_t ev_empty[2] = {nullptr, nullptr};   // a bracket with nothing in it, once per timed step
  double empty_ms = 0.0;
  long empty_n = 0;
  int* h_result = nullptr;  // pinned when a device is present
  bool h_result_pinned = true;
  std::string err;

  firp_status fail(firp_status code, const char* fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    err = buf;
    return code;
  }
};

static_assert(FIRP_MAX_K <= 8, "PseudoBias holds 8 maps");

namespace {

bool desc_ok(const firp_model_desc* d, int k, std::string& why) {
  auto bad = [&](const char* m) {
    why = m;
    return false;
  };
  if (!d) return bad("desc is NULL");
  if (d->n_layers < 1 || d->d_model < 1 || d->n_q_heads < 1 || d->n_kv_heads < 1 || d->head_dim < 2 ||
      d->d_ffn < 1 || d->vocab < 2)
    return bad("non-positive model dimension");
  if (d->head_dim % 2 || d->head_dim > 256) return bad("head_dim must be even and <= 256");
  if (d->d_model % 4 || d->d_model > 8192 || d->d_ffn % 4) return bad("d_model must be a multiple of 4 and <= 8192, d_ffn a multiple of 4");
  if (d->n_q_heads % d->n_kv_heads) return bad("n_q_heads must be a multiple of n_kv_heads");
  if (d->dtype != FIRP_F32 && d->dtype != FIRP_BF16) return bad("unknown dtype");
  if (!(d->rms_eps > 0.f) || !(d->rope_base > 1.f)) return bad("rms_eps / rope_base out of range");
  if (d->max_ctx < 1 || d->max_batch < 1 || d->max_nodes < 1) return bad("non-positive capacity");
  if (d->max_rows < d->max_nodes || d->max_rows > FIRP_MAX_ROWS) return bad("max_rows must be in [max_nodes, 256]");
  if (d->b_max < 1 || d->b_max > FIRP_MAX_B || d->b_max > d->vocab) return bad("b_max out of range");
  if (k < 0 || k > FIRP_MAX_K) return bad("k out of range");
  return true;
}

// One carve-up serves firp_workspace_bytes (base == nullptr) and firp_init.
size_t carve(firp_ctx* c, char* base) {
  const firp_model_desc& d = c->d;
  Carver cv{base};
  int R = c->Rmax, Rp = c->Rpad;
  size_t es = c->esize;
  int qd = d.n_q_heads * d.head_dim;
  c->x = cv.take<float>((size_t)Rp * d.d_model);
  c->part = cv.take<float>(c->part_elems);
  c->logits = cv.take<float>((size_t)Rp * d.vocab);
  c->attn_scratch = cv.take<float>(attention_mfma_scratch_floats(Rp, d.n_q_heads, d.head_dim));
  c->rope_tab = cv.take<float2>((size_t)Rp * d.head_dim / 2);
  c->argmax_scratch = cv.take<char>(argmax_scratch_bytes(Rp, d.b_max));
  c->norm_ss = cv.take<float>((size_t)Rp * FIRP_NORM_PIECES);
  c->q_frag = cv.take<bf16>(attention_q_frag_elems(Rp, d.max_batch, d.n_q_heads, d.head_dim));
  auto act = [&](Act& a, int ld) {
    a.ld = ld;
    a.f32 = cv.take<float>((size_t)Rp * ld);
    a.hi = cv.take<bf16>((size_t)Rp * ld);
    a.lo = cv.take<bf16>((size_t)Rp * ld);
  };
  act(c->act_d, d.d_model);
  act(c->act_q, qd);
  act(c->act_o, qd);
  act(c->act_f, d.d_ffn);
  act(c->act_p, d.d_model);
  if (c->dtype == FIRP_BF16) {
    auto pk = [&](int n, int K) { return (void*)cv.take<char>(gemm_packed_bytes(n, K)); };
    c->pk_qkv.assign(d.n_layers, nullptr);
    c->pk_o.assign(d.n_layers, nullptr);
    c->pk_gu.assign(d.n_layers, nullptr);
    c->pk_d.assign(d.n_layers, nullptr);
    c->pk_proj.assign(c->k, nullptr);
    for (int i = 0; i < d.n_layers; ++i) {
      c->pk_qkv[i] = pk(c->qkv_ld, d.d_model);
      c->pk_o[i] = pk(d.d_model, qd);
      c->pk_gu[i] = pk(2 * d.d_ffn, d.d_model);
      c->pk_d[i] = pk(d.d_model, d.d_ffn);
    }
    // the k maps back to back: with d a multiple of 16 this is also the copy of the stacked
    // [k*d][d] matrix, so one launch can stream all of them
    for (int i = 0; i < c->k; ++i) c->pk_proj[i] = pk(d.d_model, d.d_model);
    c->pk_proj_stacked = d.d_model % 16 == 0 && (gemm_packed_bytes(d.d_model, d.d_model) % 256) == 0;
    c->pk_head = pk(d.vocab, d.d_model);
  }
  size_t kv_elems = (size_t)d.max_batch * c->kv_seq_stride;
  c->kcache = cv.take<char>(kv_elems * es);
  c->vcache = cv.take<char>(kv_elems * es);
  {
    // layout of one slot (R rows, N nodes)
    Carver lay{nullptr};
    auto off = [&](size_t bytes) {
      lay.off = align_up(lay.off, 256);
      size_t o = lay.off;
      lay.off += bytes;
      return o;
    };
    int N = d.max_rows;  // prefill chunks use the node tables' row arrays only
    TopoLayout& t = c->tl_off;
    t.seq = off((size_t)R * 4);
    t.local = off((size_t)R * 4);
    t.pos = off((size_t)R * 4);
    t.mask = off((size_t)R * FIRP_MASK_WORDS * 8);
    t.parent = off((size_t)N * 4);
    t.level = off((size_t)N * 4);
    t.rank = off((size_t)N * 4);
    t.cstart = off((size_t)(N + 1) * 4);
    t.clist = off((size_t)N * 4);
    t.pbase = off((size_t)N * 4);
    t.psrc = off((size_t)R * 4);
    t.bytes = align_up(lay.off, 256);
    for (auto& sl : c->slot) sl.base = cv.take<char>(t.bytes);
  }
  c->injected = cv.take<int>(R);
  int B = d.max_batch;
  c->st.p0 = cv.take<int>(B);
  c->st.root_tok = cv.take<int>(B);
  c->st.drafts = cv.take<int>((size_t)B * std::max(c->k, 1) * d.b_max);
  c->st.drafts_valid = cv.take<int>(B);
  c->st.tok = cv.take<int>(R);
  c->st.amax = cv.take<int>(R);
  c->st.top = cv.take<int>((size_t)R * d.b_max);
  c->st.result = cv.take<int>((size_t)B * FIRP_RESULT_STRIDE);
  c->st.k = c->k;
  c->st.b_max = d.b_max;
  c->st.k_cap = FIRP_MAX_K;
  return align_up(cv.off, 256);
}

void setup_geometry(firp_ctx* c, const firp_model_desc* d, int k) {
  c->d = *d;
  c->k = k;
  c->dtype = d->dtype;
  c->esize = d->dtype == FIRP_BF16 ? 2 : 4;
  c->Rmax = d->max_batch * d->max_rows;
  c->Rpad = (int)align_up(c->Rmax, 16);
  c->slots = (int)align_up((size_t)d->max_ctx + d->max_rows, 64);
  c->qkv_ld = (d->n_q_heads + 2 * d->n_kv_heads) * d->head_dim;
  c->kv_layer_stride = (size_t)d->n_kv_heads * c->slots * d->head_dim;
  c->kv_seq_stride = (size_t)d->n_layers * c->kv_layer_stride;
  // split-K partial sums: the widest projection output times the largest split factor used
  size_t widest = std::max<size_t>({(size_t)d->vocab, (size_t)2 * d->d_ffn, (size_t)c->qkv_ld, (size_t)d->d_model});
  c->part_elems = (size_t)c->Rpad * (widest + FIRP_PART_PAD) * 8;
}

#define HIPCHK(call)                                                                         \
  do {                                                                                       \
    hipError_t e_ = (call);                                                                  \
    if (e_ != hipSuccess) return c->fail(FIRP_EDEVICE, "%s failed: %s", #call, hipGetErrorString(e_)); \
  } while (0)

KvView kv_view(const firp_ctx* c, int layer) {
  KvView v;
  v.k = (char*)c->kcache + (size_t)layer * c->kv_layer_stride * c->esize;
  v.v = (char*)c->vcache + (size_t)layer * c->kv_layer_stride * c->esize;
  v.seq_stride = c->kv_seq_stride;
  v.slots = c->slots;
  v.n_kv_heads = c->d.n_kv_heads;
  v.head_dim = c->d.head_dim;
  return v;
}

RowTab row_tab(const firp_ctx* c) { return RowTab{c->rt_seq, c->rt_local, c->rt_pos, c->rt_mask}; }
TreeTab tree_tab(const firp_ctx* c, int N, int P) {
  return TreeTab{c->tt_parent, c->tt_level, c->tt_rank, c->tt_cstart, c->tt_clist, c->tt_pbase, N, P,
                 c->k > 0 ? P / c->k : 0};
}

void select_slot(firp_ctx* c, int i) {
  char* b = c->slot[i].base;
  const TopoLayout& t = c->tl_off;
  c->rt_seq = (int*)(b + t.seq);
  c->rt_local = (int*)(b + t.local);
  c->rt_pos = (int*)(b + t.pos);
  c->rt_mask = (unsigned long long*)(b + t.mask);
  c->tt_parent = (int*)(b + t.parent);
  c->tt_level = (int*)(b + t.level);
  c->tt_rank = (int*)(b + t.rank);
  c->tt_cstart = (int*)(b + t.cstart);
  c->tt_clist = (int*)(b + t.clist);
  c->tt_pbase = (int*)(b + t.pbase);
  c->pseudo_src = (int*)(b + t.psrc);
  c->cur_slot = i;
}

// y = act . W^T into the partial-sum buffer at column `col` of rows that are `ld` wide.
// `like`: an earlier projection into the same rows whose split factor must be matched.
Partial project(firp_ctx* c, const Act& in, const void* w, const void* w_packed, int rows, int n, int K, int ld,
                int col, const Partial* like) {
  Partial out;
  out.ld = ld + FIRP_PART_PAD;
  out.stride = (size_t)c->Rpad * out.ld;
  out.p = c->part;
  if (c->gemm_kind == 1 && w_packed && gemm_mfma_supported(rows, n, K)) {
    GemmPlan plan = gemm_mfma_plan(rows, n, K, like ? like->S : 0);
    if ((size_t)plan.S * out.stride > c->part_elems)  // never outgrow the partial-sum buffer
      plan = gemm_mfma_plan(rows, n, K, (int)std::max<size_t>(1, c->part_elems / out.stride));
    bool timed = c->time_gemm && c->ev_used + 2 <= c->ev.size();
    if (timed) (void)hipEventRecord(c->ev[c->ev_used++], c->stream);
    launch_gemm_mfma(in, w_packed, c->part + col, out.ld, out.stride, rows, n, K, plan, c->stream);
    if (timed) {
      (void)hipEventRecord(c->ev[c->ev_used++], c->stream);
      c->gemm_bytes += 2.0 * (double)n * (double)K;
      c->gemm_launches += (rows + plan.row_block - 1) / plan.row_block;
    }
    out.S = plan.S;
  } else {
    launch_gemm_simple(in.f32, in.ld, w, c->dtype, c->part + col, out.ld, rows, n, K, c->stream);
    out.S = 1;
  }
  return out;
}

// Up to three matrices sharing the input, written side by side (q|k|v, gate|up): one launch of
// the MFMA kernel, or one plain launch per matrix.
Partial project_stacked(firp_ctx* c, const Act& in, const void* w0, int n0, const void* w1, int n1,
                        const void* w2, int n2, const void* w_packed, int rows, int K) {
  int n = n0 + n1 + n2;
  if (c->gemm_kind == 1 && w_packed && gemm_mfma_supported(rows, n, K)) {
    Partial out;
    out.ld = n + FIRP_PART_PAD;
    out.stride = (size_t)c->Rpad * out.ld;
    out.p = c->part;
    GemmPlan plan = gemm_mfma_plan(rows, n, K, 0);
    if ((size_t)plan.S * out.stride > c->part_elems)
      plan = gemm_mfma_plan(rows, n, K, (int)std::max<size_t>(1, c->part_elems / out.stride));
    bool timed = c->time_gemm && c->ev_used + 2 <= c->ev.size();
    if (timed) (void)hipEventRecord(c->ev[c->ev_used++], c->stream);
    launch_gemm_mfma(in, w_packed, c->part, out.ld, out.stride, rows, n, K, plan, c->stream);
    if (timed) {
      (void)hipEventRecord(c->ev[c->ev_used++], c->stream);
      c->gemm_bytes += 2.0 * (double)n * (double)K;
      c->gemm_launches += (rows + plan.row_block - 1) / plan.row_block;
    }
    out.S = plan.S;
    return out;
  }
  Partial q = project(c, in, w0, nullptr, rows, n0, K, n, 0, nullptr);
  project(c, in, w1, nullptr, rows, n1, K, n, n0, &q);
  if (n2 > 0) project(c, in, w2, nullptr, rows, n2, K, n, n0 + n1, &q);
  return q;
}

// Every projection shape of the model is one the MFMA kernel takes.
bool mfma_shapes_ok(const firp_model_desc& d, int qkv_ld) {
  const int qd = d.n_q_heads * d.head_dim;
  return gemm_mfma_supported(1, qkv_ld, d.d_model) && gemm_mfma_supported(1, d.d_model, qd) &&
         gemm_mfma_supported(1, 2 * d.d_ffn, d.d_model) && gemm_mfma_supported(1, d.d_model, d.d_ffn) &&
         gemm_mfma_supported(1, d.vocab, d.d_model);
}

// bytes of weights one decoding step streams
double step_weight_bytes(const firp_ctx* c) {
  const firp_model_desc& d = c->d;
  const double qd = (double)d.n_q_heads * d.head_dim, kvd = (double)d.n_kv_heads * d.head_dim;
  const double layer = d.d_model * (2 * qd + 2 * kvd) + 3.0 * d.d_model * d.d_ffn;
  return c->esize * (d.n_layers * layer + (double)d.vocab * d.d_model + (double)c->k * d.d_model * d.d_model);
}

// Make the fragment-major copies of the projection matrices (once, on the library's stream).
void ensure_packed(firp_ctx* c) {
  if (c->packed || c->dtype != FIRP_BF16 || c->pk_qkv.empty()) return;
  const firp_model_desc& d = c->d;
  const int qd = d.n_q_heads * d.head_dim, kvd = d.n_kv_heads * d.head_dim;
  hipStream_t s = c->stream;
  for (int i = 0; i < d.n_layers; ++i) {
    launch_pack_weights(WSeg{(const bf16*)c->wq[i], (const bf16*)c->wk[i], (const bf16*)c->wv[i], qd, kvd},
                        c->qkv_ld, d.d_model, c->pk_qkv[i], s);
    launch_pack_weights(wseg1(c->wo[i], d.d_model), d.d_model, qd, c->pk_o[i], s);
    launch_pack_weights(WSeg{(const bf16*)c->wg[i], (const bf16*)c->wu[i], nullptr, d.d_ffn, d.d_ffn},
                        2 * d.d_ffn, d.d_model, c->pk_gu[i], s);
    launch_pack_weights(wseg1(c->wd[i], d.d_model), d.d_model, d.d_ffn, c->pk_d[i], s);
  }
  for (int i = 0; i < c->k; ++i) launch_pack_weights(wseg1(c->pw[i], d.d_model), d.d_model, d.d_model, c->pk_proj[i], s);
  launch_pack_weights(wseg1(c->lm_head, d.vocab), d.vocab, d.d_model, c->pk_head, s);
  c->packed = true;
}

// The decoder over B sequences of N real rows each; with n_anchor > 0 the pseudo rows of step i
// (n_anchor per sequence) join at layer tl[i] (Eq. 3 on the residual stream entering it).  With
// `head`, ends with final norm, lm-head and argmax / top-b.
// Only the maps [map_lo, map_hi) take part (all k of them in a decoding step, one in the
// training forward); seq0 is the first sequence of the launch.
firp_status forward(firp_ctx* c, int B, int N, int n_anchor, bool head, int max_ctx_now, int seq0, int map_lo,
                    int map_hi) {
  if (c->gemm_kind == 1) ensure_packed(c);
  const firp_model_desc& d = c->d;
  hipStream_t s = c->stream;
  RowTab rt = row_tab(c);
  const bool sp = c->split;
  const int qd = d.n_q_heads * d.head_dim, kvd = d.n_kv_heads * d.head_dim;
  const int real_rows = B * N, n_anchor_rows = B * n_anchor;
  const int k_act = n_anchor > 0 ? map_hi - map_lo : 0;
  launch_embed(c->embed, c->dtype, c->st.tok, real_rows, d.d_model, d.vocab, c->x, s);
  launch_rope_table(rt, c->st.p0, real_rows + k_act * n_anchor_rows, d.head_dim, d.rope_base, c->rope_tab, s);
  Partial pending{};  // projection output not yet added to the residual stream
  // 1/rms of the latest norm, applied by the kernel that consumes the projection behind it
  const RowScale rs{c->norm_ss, norm_pieces(d.d_model), 1.0f / (float)d.d_model, d.rms_eps};
  int pending_rows = 0;
  int m = 0;  // steps whose pseudo rows are alive
  PseudoBias pbias{};
  for (int i = 0; i < c->k; ++i) pbias.b[i] = c->pb.empty() ? nullptr : c->pb[i];
  for (int layer = 0; layer <= d.n_layers; ++layer) {
    int m_new = m;
    while (m_new < k_act && c->tl[map_lo + m_new] == layer) ++m_new;
    if (m_new > m) {
      // FIRP map (Eq. 3) of steps [m, m_new) on the raw residual stream of the anchor rows
      if (pending.p) launch_add_partial(c->x, pending, pending_rows, d.d_model, s);
      pending = Partial{};
      launch_gather_rows(c->x, c->pseudo_src, n_anchor_rows, d.d_model, c->act_p, sp, s);
      const int nm = m_new - m;
      if (c->gemm_kind == 1 && c->packed && c->pk_proj_stacked && gemm_mfma_supported(n_anchor_rows, nm * d.d_model, d.d_model)) {
        // the maps share their input: one projection over the stacked copy, one scatter
        Partial y = project(c, c->act_p, nullptr, c->pk_proj[map_lo + m], n_anchor_rows, nm * d.d_model, d.d_model,
                            nm * d.d_model, 0, nullptr);
        launch_scatter_pseudo(y, n_anchor_rows, d.d_model, c->k, map_lo + m, nm, pbias, c->dtype, c->x,
                              real_rows + m * n_anchor_rows, s);
      } else {
        for (int j = m; j < m_new; ++j) {
          const int i = map_lo + j;
          Partial y = project(c, c->act_p, c->pw[i], c->packed ? c->pk_proj[i] : nullptr, n_anchor_rows, d.d_model,
                              d.d_model, d.d_model, 0, nullptr);
          launch_scatter_pseudo(y, n_anchor_rows, d.d_model, c->k, i, 1, pbias, c->dtype, c->x,
                                real_rows + j * n_anchor_rows, s);
        }
      }
      m = m_new;
    }
    const int rows = real_rows + m * n_anchor_rows;
    const int n_local = N + m * n_anchor;
    if (layer == d.n_layers) {
      if (!head) {
        if (pending.p) launch_add_partial(c->x, pending, pending_rows, d.d_model, s);
        break;
      }
      launch_add_rmsnorm(c->x, pending, rows, d.d_model, c->norm_final, c->dtype, c->act_d, sp, c->norm_ss, s);
      Partial lg = project(c, c->act_d, c->lm_head, c->packed ? c->pk_head : nullptr, rows, d.vocab, d.d_model,
                           d.vocab, 0, nullptr);
      // the logits themselves are written only on request (tests, the training forward): the step
      // needs the greedy token of every node and the top-b ids of every pseudo row, nothing else
      const bool want_logits = c->keep_logits || c->force_logits;
      launch_argmax_topb(lg, rs, want_logits ? c->logits : nullptr, real_rows, rows, d.vocab, d.b_max, c->st.amax,
                         c->st.top, c->argmax_scratch, s);
      c->last_has_logits = want_logits;
      break;
    }
    // the pending partials cover `pending_rows` rows; rows beyond (new pseudo rows) have none
    if (pending.p && pending_rows < rows) {
      launch_add_partial(c->x, pending, pending_rows, d.d_model, s);
      pending = Partial{};
    }
    launch_add_rmsnorm(c->x, pending, rows, d.d_model, c->n1[layer], c->dtype, c->act_d, sp, c->norm_ss, s);
    Partial q = project_stacked(c, c->act_d, c->wq[layer], qd, c->wk[layer], kvd, c->wv[layer], kvd,
                                c->packed ? c->pk_qkv[layer] : nullptr, rows, d.d_model);
    KvView kv = kv_view(c, layer);
    if (c->attn_kind == 1 && sp) {
      launch_rope_kv_tiles(q, rs, d.n_q_heads, B, N, n_local - N, n_anchor, seq0, c->st.p0, c->rope_tab, c->q_frag, kv,
                           s);
      launch_attention_mfma(c->q_frag, rows, d.n_q_heads, B, N, n_local - N, n_anchor, seq0, rt, c->st.p0, max_ctx_now,
                            kv, c->attn_scratch, c->act_o, s);
    } else {
      launch_rope_kv(q, rs, rows, d.n_q_heads, rt, c->st.p0, c->rope_tab, c->act_q, sp, kv, c->dtype, s);
      launch_attention_simple(c->act_q, sp, rows, d.n_q_heads, rt, c->st.p0, kv, c->dtype, c->act_o, n_local,
                              max_ctx_now + n_local, s);
    }
    Partial o = project(c, c->act_o, c->wo[layer], c->packed ? c->pk_o[layer] : nullptr, rows, d.d_model, qd,
                        d.d_model, 0, nullptr);
    launch_add_rmsnorm(c->x, o, rows, d.d_model, c->n2[layer], c->dtype, c->act_d, sp, c->norm_ss, s);
    Partial g = project_stacked(c, c->act_d, c->wg[layer], d.d_ffn, c->wu[layer], d.d_ffn, nullptr, 0,
                                c->packed ? c->pk_gu[layer] : nullptr, rows, d.d_model);
    launch_swiglu(g, rs, rows, d.d_ffn, c->act_f, sp, s);
    pending = project(c, c->act_f, c->wd[layer], c->packed ? c->pk_d[layer] : nullptr, rows, d.d_model, d.d_ffn,
                      d.d_model, 0, nullptr);
    pending_rows = rows;
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return c->fail(FIRP_EDEVICE, "kernel launch failed: %s", hipGetErrorString(e));
  return FIRP_OK;
}

// Host-side tree parser: depths, ancestor masks, child lists, pseudo-row table; uploads the
// per-row and per-node tables for `B` sequences sharing the topology.
firp_status upload_tree(firp_ctx* c, int B, const std::vector<int>& parent, const std::vector<int>& rank,
                        const std::vector<uint8_t>& anchor) {
  int N = (int)parent.size(), k = c->k;
  ++c->use_clock;
  // a topology seen before still has its tables on the device
  for (int i = 0; i < FIRP_TOPO_SLOTS; ++i) {
    TopoSlot& sl = c->slot[i];
    if (sl.valid && sl.key.same(B, k, parent, rank, anchor)) {
      sl.last_use = c->use_clock;
      if (c->cur_slot != i) select_slot(c, i);
      c->cur = sl.key;
      c->tables_valid = true;
      return FIRP_OK;
    }
  }
  int victim = 0;
  for (int i = 0; i < FIRP_TOPO_SLOTS; ++i) {
    if (!c->slot[i].valid) {
      victim = i;
      break;
    }
    if (c->slot[i].last_use < c->slot[victim].last_use) victim = i;
  }
  std::vector<int> depth(N, 0), pbase(N, -1), cstart(N + 1, 0), clist(std::max(N - 1, 1), 0);
  std::vector<std::vector<unsigned long long>> m(N, std::vector<unsigned long long>(FIRP_MASK_WORDS, 0));
  int n_anchor = 0;
  for (int v = 0; v < N; ++v) {
    if (v > 0) {
      depth[v] = depth[parent[v]] + 1;
      m[v] = m[parent[v]];
      cstart[parent[v] + 1]++;
    }
    m[v][v >> 6] |= 1ull << (v & 63);
    if (anchor[v] && k > 0) pbase[v] = N + n_anchor++;   // step 1; step i is n_anchor further per step
  }
  for (int v = 0; v < N; ++v) cstart[v + 1] += cstart[v];
  {
    std::vector<int> fill(cstart.begin(), cstart.end() - 1);
    for (int v = 1; v < N; ++v) clist[fill[parent[v]]++] = v;  // ascending node id per parent
  }
  const int P = k * n_anchor;
  // one host image of the slot, one copy
  const TopoLayout& t = c->tl_off;
  std::vector<char> img(t.bytes, 0);
  int* seq = (int*)(img.data() + t.seq);
  int* local = (int*)(img.data() + t.local);
  int* pos = (int*)(img.data() + t.pos);
  unsigned long long* mask = (unsigned long long*)(img.data() + t.mask);
  int* psrc = (int*)(img.data() + t.psrc);
  for (int b = 0; b < B; ++b) {
    for (int v = 0; v < N; ++v) {
      int r = b * N + v;
      seq[r] = b;
      local[r] = v;
      pos[r] = depth[v];
      std::copy(m[v].begin(), m[v].end(), mask + (size_t)r * FIRP_MASK_WORDS);
    }
    for (int v = 0; v < N; ++v) {
      if (pbase[v] < 0) continue;
      const int a_idx = pbase[v] - N;
      psrc[b * n_anchor + a_idx] = b * N + v;
      std::vector<unsigned long long> mm = m[v];
      for (int i = 0; i < k; ++i) {
        // local id N + i*A + a; global row behind the pseudo rows of all earlier steps
        int loc = N + i * n_anchor + a_idx;
        int r = B * N + i * (B * n_anchor) + b * n_anchor + a_idx;
        mm[loc >> 6] |= 1ull << (loc & 63);  // pseudo row i sees the earlier pseudo rows of its anchor
        seq[r] = b;
        local[r] = loc;
        pos[r] = depth[v] + i + 1;
        std::copy(mm.begin(), mm.end(), mask + (size_t)r * FIRP_MASK_WORDS);
      }
    }
  }
  std::copy(parent.begin(), parent.end(), (int*)(img.data() + t.parent));
  std::copy(depth.begin(), depth.end(), (int*)(img.data() + t.level));
  std::copy(rank.begin(), rank.end(), (int*)(img.data() + t.rank));
  std::copy(cstart.begin(), cstart.end(), (int*)(img.data() + t.cstart));
  std::copy(clist.begin(), clist.end(), (int*)(img.data() + t.clist));
  std::copy(pbase.begin(), pbase.end(), (int*)(img.data() + t.pbase));
  hipStream_t s = c->stream;
  TopoSlot& sl = c->slot[victim];
  sl.valid = false;
  for (auto& ex : sl.exec)
    if (ex) {
      (void)hipGraphExecDestroy(ex);
      ex = nullptr;
    }
  HIPCHK(hipStreamSynchronize(s));  // an earlier step may still read the slot that is overwritten
  HIPCHK(hipMemcpy(sl.base, img.data(), t.bytes, hipMemcpyHostToDevice));
  ++c->topo_uploads;
  sl.key.B = B;
  sl.key.N = N;
  sl.key.P = P;
  sl.key.k = k;
  sl.key.n_anchor = n_anchor;
  sl.key.parent = parent;
  sl.key.rank = rank;
  sl.key.anchor = anchor;
  sl.key.depth = depth;
  sl.key.max_depth = *std::max_element(depth.begin(), depth.end());
  sl.valid = true;
  sl.last_use = c->use_clock;
  select_slot(c, victim);
  c->cur = sl.key;
  c->tables_valid = true;
  return FIRP_OK;
}

// masked keys are multiplied by a zero probability: the cache must never hold NaN or Inf
firp_status ensure_cache_clean(firp_ctx* c) {
  if (c->cache_clean) return FIRP_OK;
  size_t bytes = (size_t)c->d.max_batch * c->kv_seq_stride * c->esize;
  HIPCHK(hipMemsetAsync(c->kcache, 0, bytes, c->stream));
  HIPCHK(hipMemsetAsync(c->vcache, 0, bytes, c->stream));
  c->cache_clean = true;
  return FIRP_OK;
}

firp_status check_tree(firp_ctx* c, const firp_tree* t, bool injected, std::vector<int>& parent,
                       std::vector<int>& rank, std::vector<uint8_t>& anchor, int& max_depth) {
  if (!t || !t->parent || (t->n_nodes > 1 && !t->rank)) return c->fail(FIRP_EINVAL, "tree or its arrays are NULL");
  int N = t->n_nodes;
  if (N < 1) return c->fail(FIRP_EINVAL, "tree has no root");
  if (N > c->d.max_nodes) return c->fail(FIRP_ECAPACITY, "tree has %d nodes, max_nodes is %d", N, c->d.max_nodes);
  if (t->parent[0] != -1) return c->fail(FIRP_EINVAL, "parent[0] must be -1");
  parent.assign(t->parent, t->parent + N);
  rank.assign(N, 0);
  anchor.assign(N, 1);
  std::vector<int> depth(N, 0);
  max_depth = 0;
  int n_anchor = 0;
  for (int v = 0; v < N; ++v) {
    if (v > 0) {
      if (parent[v] < 0 || parent[v] >= v) return c->fail(FIRP_EINVAL, "parent[%d] = %d is not an earlier node", v, parent[v]);
      rank[v] = t->rank[v];
      if (rank[v] < 0 || rank[v] >= c->d.b_max) return c->fail(FIRP_EINVAL, "rank[%d] = %d outside [0, b_max)", v, rank[v]);
      depth[v] = depth[parent[v]] + 1;
      max_depth = std::max(max_depth, depth[v]);
    }
    if (t->anchor) anchor[v] = t->anchor[v] ? 1 : 0;
    if (c->k == 0) anchor[v] = 0;
    n_anchor += anchor[v];
  }
  if (max_depth > FIRP_MAX_K) return c->fail(FIRP_EINVAL, "tree is %d levels deep, at most %d are supported", max_depth, FIRP_MAX_K);
  (void)injected;
  int T = N + c->k * n_anchor;
  if (T > c->d.max_rows) return c->fail(FIRP_ECAPACITY, "step needs %d rows (N + k*anchors), max_rows is %d", T, c->d.max_rows);
  return FIRP_OK;
}

firp_status run_step(firp_ctx* c, const firp_tree* tree, const int32_t* node_tokens, int32_t* accepted,
                     int32_t* n_accepted) {
  if (!c) return FIRP_EINVAL;
  if (!accepted || !n_accepted) return c->fail(FIRP_EINVAL, "output pointer is NULL");
  if (!c->prefilled) return c->fail(FIRP_ESTATE, "firp_step before firp_prefill");
  std::vector<int> parent, rank;
  std::vector<uint8_t> anchor;
  int max_depth = 0;
  firp_status st = check_tree(c, tree, node_tokens != nullptr, parent, rank, anchor, max_depth);
  if (st != FIRP_OK) return st;
  int B = c->batch;
  int N_in = (int)parent.size();
  bool any_valid = false;
  for (int b = 0; b < B; ++b) any_valid |= c->drafts_valid[b] != 0;
  if (!node_tokens && !any_valid && N_in > 1) {
    // no sequence has drafts: the step degenerates to the root-only sub-tree
    parent = {-1};
    rank = {0};
    anchor = {anchor[0]};
    max_depth = 0;
  }
  int N = (int)parent.size();
  int n_anchor = 0;
  for (auto a : anchor) n_anchor += a;
  int P = c->k * n_anchor, T = N + P;
  int ctx_max = 0;
  for (int b = 0; b < B; ++b) {
    if (c->p0[b] + max_depth + 1 > c->d.max_ctx)
      return c->fail(FIRP_ECAPACITY, "sequence %d: %d cached + %d new tokens exceed max_ctx %d", b, c->p0[b], max_depth + 1, c->d.max_ctx);
    ctx_max = std::max(ctx_max, c->p0[b]);
  }
  if (!(c->attn_kind == 1 && c->split) && (size_t)(c->d.head_dim + ctx_max + T) * sizeof(float) > 64 * 1024)
    return c->fail(FIRP_ECAPACITY, "context of %d tokens exceeds the plain attention kernel's limit", ctx_max);
  st = upload_tree(c, B, parent, rank, anchor);
  if (st != FIRP_OK) return st;
  hipStream_t s = c->stream;
  const int* inj = nullptr;
  if (node_tokens) {
    if (N != N_in) return c->fail(FIRP_EINVAL, "internal: injected tokens with a substituted tree");
    HIPCHK(hipMemcpyAsync(c->injected, node_tokens, (size_t)B * N * sizeof(int), hipMemcpyHostToDevice, s));
    inj = c->injected;
  }
  const bool empty_bracket = c->time_gemm && c->ev_empty[0];
  // the step's kernels, from candidate fill to the KV commit
  auto enqueue = [&]() -> firp_status {
    launch_fill_tokens(c->st, tree_tab(c, N, P), B, inj, s);
    if (empty_bracket) {
      (void)hipEventRecord(c->ev_empty[0], s);
      (void)hipEventRecord(c->ev_empty[1], s);
    }
    firp_status fs = forward(c, B, N, n_anchor, true, ctx_max, 0, 0, c->k);
    if (fs != FIRP_OK) return fs;
    launch_verify_select(c->st, tree_tab(c, N, P), B, s);
    launch_kv_compact(kv_view(c, 0), c->kv_layer_stride, c->d.n_layers, B, c->st, c->dtype, s);
    return FIRP_OK;
  };
  // Replayed as a captured graph when nothing the kernels are launched with can change between
  // steps: MFMA kernels (the attention launch takes its chunk length from the device), a
  // context long enough that the number of attention splits no longer depends on it, packed
  // weights in place, no event brackets.  Everything else the kernels read is device state.
  const int want_splits = std::min(FIRP_ATTN_MAX_SPLITS, std::max(1, 256 / std::max(1, c->d.n_kv_heads * B)));
  int ctx_min = ctx_max;
  for (int b = 0; b < B; ++b) ctx_min = std::min(ctx_min, c->p0[b]);
  const bool graphable = c->use_graph && !c->graph_broken && !c->time_gemm && c->attn_kind == 1 && c->split &&
                         c->gemm_kind == 1 && c->packed && c->cur_slot >= 0 && c->cur_slot < FIRP_TOPO_SLOTS &&
                         (ctx_min + N) / 32 >= want_splits;
  bool launched = false;
  if (graphable) {
    TopoSlot& sl = c->slot[c->cur_slot];
    GraphKey key;
    key.B = B;
    key.injected = inj ? 1 : 0;
    key.keep_logits = c->keep_logits ? 1 : 0;
    key.gemm_kind = c->gemm_kind;
    key.attn_kind = c->attn_kind;
    hipGraphExec_t& exec = sl.exec[key.injected];
    if (exec && !(sl.gkey[key.injected] == key)) {
      (void)hipGraphExecDestroy(exec);
      exec = nullptr;
    }
    if (!exec) {
      if (hipStreamBeginCapture(s, hipStreamCaptureModeThreadLocal) != hipSuccess) {
        (void)hipGetLastError();
        c->graph_broken = true;
      } else {
        firp_status fs = enqueue();
        hipGraph_t g = nullptr;
        hipError_t e = hipStreamEndCapture(s, &g);
        if (fs == FIRP_OK && e == hipSuccess && g && hipGraphInstantiate(&exec, g, nullptr, nullptr, 0) == hipSuccess) {
          sl.gkey[key.injected] = key;
          ++c->graph_captures;
        } else {
          (void)hipGetLastError();
          exec = nullptr;
          c->graph_broken = true;
        }
        if (g) (void)hipGraphDestroy(g);
        if (fs != FIRP_OK) return fs;
      }
    }
    if (exec) {
      HIPCHK(hipGraphLaunch(exec, s));
      c->last_has_logits = c->keep_logits;
      ++c->graph_launches;
      launched = true;
    }
  }
  if (!launched) {
    st = enqueue();
    if (st != FIRP_OK) return st;
  }
  HIPCHK(hipMemcpyAsync(c->h_result, c->st.result, (size_t)B * FIRP_RESULT_STRIDE * sizeof(int), hipMemcpyDeviceToHost, s));
  HIPCHK(hipStreamSynchronize(s));
  for (size_t i = 0; i + 1 < c->ev_used; i += 2) {
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, c->ev[i], c->ev[i + 1]) == hipSuccess) c->gemm_ms += ms;
  }
  c->ev_used = 0;
  if (empty_bracket) {
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, c->ev_empty[0], c->ev_empty[1]) == hipSuccess) {
      c->empty_ms += ms;
      c->empty_n += 1;
    }
  }
  for (int b = 0; b < B; ++b) {
    const int* r = c->h_result + b * FIRP_RESULT_STRIDE;
    n_accepted[b] = r[0];
    for (int j = 0; j < r[0]; ++j) accepted[b * (FIRP_MAX_K + 1) + j] = r[3 + j];
    c->drafts_valid[b] = r[1];
    c->p0[b] = r[2] + r[0];
  }
  c->last_rows = B * T;
  c->last_N = N;
  c->last_P = P;
  c->last_steps = c->k;
  return FIRP_OK;
}

}  // namespace

// ============================================================================ C ABI

extern "C" {

size_t firp_workspace_bytes(const firp_model_desc* desc, int32_t k) {
  std::string why;
  if (!desc_ok(desc, k, why)) return 0;
  firp_ctx tmp;
  setup_geometry(&tmp, desc, k);
  return carve(&tmp, nullptr);
}

firp_status firp_init(firp_ctx** out, const firp_model_desc* desc, const firp_weights* w,
                      const void* const* proj_w, const void* const* proj_b, int32_t layer_l, int32_t k,
                      void* workspace, size_t workspace_bytes, void* hip_stream) {
  int32_t layers[FIRP_MAX_K];
  for (int i = 0; i < FIRP_MAX_K; ++i) layers[i] = layer_l;
  if (desc && (layer_l < 0 || layer_l > desc->n_layers)) {
    if (out) *out = nullptr;
    g_init_error = "layer_l outside [0, n_layers]";
    return FIRP_EINVAL;
  }
  return firp_init_layers(out, desc, w, proj_w, proj_b, layers, k, workspace, workspace_bytes, hip_stream);
}

firp_status firp_init_layers(firp_ctx** out, const firp_model_desc* desc, const firp_weights* w,
                             const void* const* proj_w, const void* const* proj_b, const int32_t* layers,
                             int32_t k, void* workspace, size_t workspace_bytes, void* hip_stream) {
  auto bad = [&](firp_status code, const std::string& m) {
    g_init_error = m;
    return code;
  };
  if (!out) return bad(FIRP_EINVAL, "out is NULL");
  *out = nullptr;
  std::string why;
  if (!desc_ok(desc, k, why)) return bad(FIRP_EINVAL, why);
  if (k > 0 && !layers) return bad(FIRP_EINVAL, "layers is NULL with k > 0");
  for (int i = 0; i < k; ++i) {
    if (layers[i] < 0 || layers[i] > desc->n_layers) return bad(FIRP_EINVAL, "a prediction layer is outside [0, n_layers]");
    if (i > 0 && layers[i] < layers[i - 1]) return bad(FIRP_EINVAL, "prediction layers must not decrease");
  }
  if (!w || !w->embed || !w->wq || !w->wk || !w->wv || !w->wo || !w->w_gate || !w->w_up || !w->w_down ||
      !w->norm_attn || !w->norm_mlp || !w->norm_final || !w->lm_head)
    return bad(FIRP_EINVAL, "a weight pointer is NULL");
  for (int i = 0; i < desc->n_layers; ++i)
    if (!w->wq[i] || !w->wk[i] || !w->wv[i] || !w->wo[i] || !w->w_gate[i] || !w->w_up[i] || !w->w_down[i] ||
        !w->norm_attn[i] || !w->norm_mlp[i])
      return bad(FIRP_EINVAL, "a per-layer weight pointer is NULL");
  if (k > 0) {
    if (!proj_w) return bad(FIRP_EINVAL, "proj_w is NULL with k > 0");
    for (int i = 0; i < k; ++i)
      if (!proj_w[i] || (proj_b && !proj_b[i])) return bad(FIRP_EINVAL, "a projection pointer is NULL");
  }
  if (!workspace) return bad(FIRP_EINVAL, "workspace is NULL");
  if (((uintptr_t)workspace) & 255) return bad(FIRP_EINVAL, "workspace is not 256-byte aligned");
  firp_ctx* c = new firp_ctx;
  setup_geometry(c, desc, k);
  c->tl.assign(layers, layers + k);
  size_t need = carve(c, (char*)workspace);
  if (workspace_bytes < need) {
    delete c;
    return bad(FIRP_ECAPACITY, "workspace too small");
  }
  c->stream = (hipStream_t)hip_stream;
  c->embed = w->embed;
  c->norm_final = w->norm_final;
  c->lm_head = w->lm_head;
  int L = desc->n_layers;
  c->wq.assign(w->wq, w->wq + L);
  c->wk.assign(w->wk, w->wk + L);
  c->wv.assign(w->wv, w->wv + L);
  c->wo.assign(w->wo, w->wo + L);
  c->wg.assign(w->w_gate, w->w_gate + L);
  c->wu.assign(w->w_up, w->w_up + L);
  c->wd.assign(w->w_down, w->w_down + L);
  c->n1.assign(w->norm_attn, w->norm_attn + L);
  c->n2.assign(w->norm_mlp, w->norm_mlp + L);
  if (k > 0) {
    c->pw.assign(proj_w, proj_w + k);
    if (proj_b) c->pb.assign(proj_b, proj_b + k);
  }
  // bf16 models stream weights through MFMA (when every projection shape fits the kernel)
  c->gemm_kind = (desc->dtype == FIRP_BF16 && mfma_shapes_ok(*desc, c->qkv_ld)) ? 1 : 0;
  c->split = c->gemm_kind == 1;
  c->attn_kind = (c->split && attention_mfma_supported(desc->head_dim, desc->dtype)) ? 1 : 0;
  c->use_graph = step_weight_bytes(c) <= 8e9;
  c->p0.assign(desc->max_batch, 0);
  c->drafts_valid.assign(desc->max_batch, 0);
  size_t res_bytes = (size_t)desc->max_batch * FIRP_RESULT_STRIDE * sizeof(int);
  if (hipHostMalloc((void**)&c->h_result, res_bytes, hipHostMallocDefault) != hipSuccess) {
    // no usable device (host-only validation runs): an ordinary buffer keeps the context usable
    (void)hipGetLastError();
    c->h_result = (int*)calloc(1, res_bytes);
    c->h_result_pinned = false;
  }
  *out = c;
  return FIRP_OK;
}

firp_status firp_reset(firp_ctx* c) {
  if (!c) return FIRP_EINVAL;
  c->prefilled = false;
  c->batch = 0;
  c->last_rows = 0;
  std::fill(c->p0.begin(), c->p0.end(), 0);
  std::fill(c->drafts_valid.begin(), c->drafts_valid.end(), 0);
  return FIRP_OK;
}

void firp_destroy(firp_ctx* c) {
  if (!c) return;
  for (auto& e : c->ev) (void)hipEventDestroy(e);
  for (auto& e : c->ev_empty)
    if (e) (void)hipEventDestroy(e);
  for (auto& sl : c->slot)
    for (auto& ex : sl.exec)
      if (ex) (void)hipGraphExecDestroy(ex);
  if (c->h_result) {
    if (c->h_result_pinned)
      (void)hipHostFree(c->h_result);
    else
      free(c->h_result);
  }
  delete c;
}

const char* firp_last_error(const firp_ctx* c) { return c ? c->err.c_str() : g_init_error.c_str(); }

firp_status firp_prefill(firp_ctx* c, int32_t batch, const int32_t* tokens, const int32_t* lens,
                         int32_t* first_token) {
  if (!c) return FIRP_EINVAL;
  if (!tokens || !lens || !first_token) return c->fail(FIRP_EINVAL, "argument pointer is NULL");
  if (batch < 1 || batch > c->d.max_batch) return c->fail(FIRP_ECAPACITY, "batch %d outside [1, %d]", batch, c->d.max_batch);
  size_t total = 0;
  int longest = 0;
  for (int b = 0; b < batch; ++b) {
    if (lens[b] < 1) return c->fail(FIRP_EINVAL, "prompt %d is empty", b);
    if (lens[b] > c->d.max_ctx) return c->fail(FIRP_ECAPACITY, "prompt %d has %d tokens, max_ctx is %d", b, lens[b], c->d.max_ctx);
    longest = std::max(longest, lens[b]);
    total += lens[b];
  }
  for (size_t i = 0; i < total; ++i)
    if (tokens[i] < 0 || tokens[i] >= c->d.vocab) return c->fail(FIRP_EINVAL, "token %zu = %d outside the vocabulary", i, tokens[i]);
  int C = c->d.max_rows;
  if (!(c->attn_kind == 1 && c->split) && (size_t)(c->d.head_dim + longest + C) * sizeof(float) > 64 * 1024)
    return c->fail(FIRP_ECAPACITY, "prompt of %d tokens exceeds the plain attention kernel's limit", longest);
  hipStream_t s = c->stream;
  c->prefilled = false;
  c->tables_valid = false;
  firp_status cst = ensure_cache_clean(c);
  if (cst != FIRP_OK) return cst;
  // prompt[:-1] through the decoder in chunks: a chunk is a chain whose mask is lower-triangular
  std::vector<int> seq(C), local(C), pos(C);
  std::vector<unsigned long long> mask((size_t)C * FIRP_MASK_WORDS, 0);
  for (int j = 0; j < C; ++j) {
    local[j] = pos[j] = j;
    for (int i = 0; i <= j; ++i) mask[(size_t)j * FIRP_MASK_WORDS + (i >> 6)] |= 1ull << (i & 63);
  }
  select_slot(c, FIRP_TOPO_SLOTS);   // the chunk tables live in the slot that is never cached
  HIPCHK(hipStreamSynchronize(s));
  HIPCHK(hipMemcpy(c->rt_local, local.data(), C * sizeof(int), hipMemcpyHostToDevice));
  HIPCHK(hipMemcpy(c->rt_pos, pos.data(), C * sizeof(int), hipMemcpyHostToDevice));
  HIPCHK(hipMemcpy(c->rt_mask, mask.data(), mask.size() * sizeof(unsigned long long), hipMemcpyHostToDevice));
  const int32_t* tk = tokens;
  for (int b = 0; b < batch; ++b) {
    std::fill(seq.begin(), seq.end(), b);
    HIPCHK(hipStreamSynchronize(s));
    HIPCHK(hipMemcpy(c->rt_seq, seq.data(), C * sizeof(int), hipMemcpyHostToDevice));
    launch_set_root(c->st, b, tk[lens[b] - 1], 0, s);
    int done = 0, todo = lens[b] - 1;
    while (done < todo) {
      int n = std::min(C, todo - done);
      HIPCHK(hipMemcpyAsync(c->st.tok, tk + done, n * sizeof(int), hipMemcpyHostToDevice, s));
      firp_status st = forward(c, 1, n, 0, false, done, b, 0, 0);
      if (st != FIRP_OK) return st;
      launch_advance_by(c->st.p0, b, n, s);
      HIPCHK(hipStreamSynchronize(s));  // the token staging buffer is reused by the next chunk
      done += n;
    }
    c->p0[b] = todo;
    c->drafts_valid[b] = 0;
    tk += lens[b];
  }
  c->batch = batch;
  c->prefilled = true;
  // root-only step on the last prompt token: first generated token and first drafts
  int32_t par = -1, rk = 0;
  uint8_t an = 1;
  firp_tree root{1, &par, &rk, &an};
  std::vector<int32_t> acc((size_t)batch * (FIRP_MAX_K + 1)), nacc(batch);
  firp_status st = run_step(c, &root, nullptr, acc.data(), nacc.data());
  if (st != FIRP_OK) {
    c->prefilled = false;
    return st;
  }
  for (int b = 0; b < batch; ++b) first_token[b] = acc[(size_t)b * (FIRP_MAX_K + 1)];
  return FIRP_OK;
}

firp_status firp_train_forward(firp_ctx* c, const int32_t* tokens, int32_t n, int32_t step, double* loss,
                               float* kl) {
  if (!c) return FIRP_EINVAL;
  if (!tokens || !loss) return c->fail(FIRP_EINVAL, "argument pointer is NULL");
  if (step < 1 || step > c->k) return c->fail(FIRP_EINVAL, "step %d outside [1, k = %d]", step, c->k);
  if (n <= step) return c->fail(FIRP_EINVAL, "the sequence must be longer than the prediction step");
  if (2 * n > c->d.max_rows) return c->fail(FIRP_ECAPACITY, "2n = %d rows exceed max_rows %d", 2 * n, c->d.max_rows);
  if (c->prefilled) return c->fail(FIRP_ESTATE, "the training forward needs a context without sequences (firp_reset)");
  for (int i = 0; i < n; ++i)
    if (tokens[i] < 0 || tokens[i] >= c->d.vocab) return c->fail(FIRP_EINVAL, "token %d = %d outside the vocabulary", i, tokens[i]);
  if (!(c->attn_kind == 1 && c->split) && (size_t)(c->d.head_dim + 2 * n) * sizeof(float) > 64 * 1024)
    return c->fail(FIRP_ECAPACITY, "sequence exceeds the plain attention kernel's limit");
  hipStream_t s = c->stream;
  firp_status st = ensure_cache_clean(c);
  if (st != FIRP_OK) return st;
  // rows [h_1..h_n, h~_1..h~_n] of sequence 0 on an empty cache: the real rows are a chain; pseudo
  // row j (0-based) stands for position j + step, sees real rows 0 .. j + step - 1 and itself
  const int R = 2 * n;
  std::vector<int> seq(R, 0), local(R), pos(R), psrc(n);
  std::vector<unsigned long long> mask((size_t)R * FIRP_MASK_WORDS, 0);
  auto set = [&](int r, int bit) { mask[(size_t)r * FIRP_MASK_WORDS + (bit >> 6)] |= 1ull << (bit & 63); };
  for (int v = 0; v < n; ++v) {
    local[v] = pos[v] = v;
    for (int i = 0; i <= v; ++i) set(v, i);
    const int r = n + v;
    local[r] = r;
    pos[r] = v + step;
    for (int i = 0; i < std::min(v + step, n); ++i) set(r, i);
    set(r, r);
    psrc[v] = v;
  }
  c->tables_valid = false;
  select_slot(c, FIRP_TOPO_SLOTS);
  HIPCHK(hipStreamSynchronize(s));
  HIPCHK(hipMemcpy(c->rt_seq, seq.data(), R * sizeof(int), hipMemcpyHostToDevice));
  HIPCHK(hipMemcpy(c->rt_local, local.data(), R * sizeof(int), hipMemcpyHostToDevice));
  HIPCHK(hipMemcpy(c->rt_pos, pos.data(), R * sizeof(int), hipMemcpyHostToDevice));
  HIPCHK(hipMemcpy(c->rt_mask, mask.data(), mask.size() * sizeof(unsigned long long), hipMemcpyHostToDevice));
  HIPCHK(hipMemcpy(c->pseudo_src, psrc.data(), n * sizeof(int), hipMemcpyHostToDevice));
  HIPCHK(hipMemcpy(c->st.tok, tokens, n * sizeof(int), hipMemcpyHostToDevice));
  launch_set_root(c->st, 0, tokens[0], 0, s);   // cache length 0
  c->force_logits = true;   // the KL terms are formed from the logits
  st = forward(c, 1, n, n, true, 0, 0, step - 1, step);
  c->force_logits = false;
  if (st != FIRP_OK) return st;
  float* d_kl = (float*)c->attn_scratch;   // free again once the last attention has run
  launch_kl_rows(c->logits, c->d.vocab, n, step, d_kl, s);
  std::vector<float> h_kl(n - step);
  HIPCHK(hipMemcpyAsync(h_kl.data(), d_kl, (size_t)(n - step) * sizeof(float), hipMemcpyDeviceToHost, s));
  HIPCHK(hipStreamSynchronize(s));
  c->ev_used = 0;
  double total = 0.0;
  for (int q = 0; q < n - step; ++q) {
    total += (double)h_kl[q];
    if (kl) kl[q] = h_kl[q];
  }
  *loss = total;
  c->batch = 1;          // for the logits read-out; the context still holds no sequence
  c->last_rows = R;
  c->last_N = n;
  c->last_P = n;
  c->last_steps = 1;
  return FIRP_OK;
}

firp_status firp_step(firp_ctx* c, const firp_tree* tree, int32_t* accepted, int32_t* n_accepted) {
  return run_step(c, tree, nullptr, accepted, n_accepted);
}

firp_status firp_step_with_candidates(firp_ctx* c, const firp_tree* tree, const int32_t* node_tokens,
                                      int32_t* accepted, int32_t* n_accepted) {
  if (!c) return FIRP_EINVAL;
  if (!node_tokens) return c->fail(FIRP_EINVAL, "node_tokens is NULL");
  if (tree && tree->n_nodes >= 1 && tree->n_nodes <= c->d.max_nodes)
    for (int i = 0; i < c->batch * tree->n_nodes; ++i)
      if (i % tree->n_nodes && (node_tokens[i] < -1 || node_tokens[i] >= c->d.vocab))
        return c->fail(FIRP_EINVAL, "candidate %d = %d outside the vocabulary", i, node_tokens[i]);
  return run_step(c, tree, node_tokens, accepted, n_accepted);
}

firp_status firp_check_tree(firp_ctx* c, const firp_tree* tree, int32_t* n_rows) {
  if (!c) return FIRP_EINVAL;
  std::vector<int> parent, rank;
  std::vector<uint8_t> anchor;
  int max_depth = 0;
  firp_status st = check_tree(c, tree, false, parent, rank, anchor, max_depth);
  if (st != FIRP_OK) return st;
  int n_anchor = 0;
  for (auto a : anchor) n_anchor += a;
  if (n_rows) *n_rows = (int)parent.size() + c->k * n_anchor;
  return FIRP_OK;
}

firp_status firp_debug_last_logits(firp_ctx* c, float* logits, int32_t* n_rows) {
  if (!c) return FIRP_EINVAL;
  if (!logits || !n_rows) return c->fail(FIRP_EINVAL, "argument pointer is NULL");
  if (c->last_rows == 0) return c->fail(FIRP_ESTATE, "no step has run");
  if (!c->last_has_logits) return c->fail(FIRP_ESTATE, "the last step did not keep its logits (option \"keep_logits\")");
  int B = c->batch, N = c->last_N, P = c->last_P, T = N + P, V = c->d.vocab;
  HIPCHK(hipStreamSynchronize(c->stream));
  for (int b = 0; b < B; ++b) {
    HIPCHK(hipMemcpy(logits + ((size_t)b * T) * V, c->logits + ((size_t)b * N) * V, (size_t)N * V * sizeof(float), hipMemcpyDeviceToHost));
    // pseudo rows: step by step, inside a step sequence by sequence; handed out per sequence
    const int A = c->last_steps > 0 ? P / c->last_steps : 0;
    for (int i = 0; i < c->last_steps && A > 0; ++i)
      HIPCHK(hipMemcpy(logits + ((size_t)b * T + N + (size_t)i * A) * V,
                       c->logits + ((size_t)B * N + (size_t)i * B * A + (size_t)b * A) * V, (size_t)A * V * sizeof(float),
                       hipMemcpyDeviceToHost));
  }
  *n_rows = T;
  return FIRP_OK;
}

firp_status firp_debug_last_path(firp_ctx* c, int32_t* path_nodes) {
  if (!c) return FIRP_EINVAL;
  if (!path_nodes) return c->fail(FIRP_EINVAL, "argument pointer is NULL");
  if (!c->prefilled || c->last_rows == 0) return c->fail(FIRP_ESTATE, "no step has run");
  for (int b = 0; b < c->batch; ++b) {
    const int* r = c->h_result + b * FIRP_RESULT_STRIDE;
    for (int j = 0; j < r[0]; ++j) path_nodes[b * (FIRP_MAX_K + 1) + j] = r[3 + (FIRP_MAX_K + 1) + j];
  }
  return FIRP_OK;
}

firp_status firp_get_drafts(const firp_ctx* cc, int32_t* drafts, int32_t* valid) {
  firp_ctx* c = const_cast<firp_ctx*>(cc);
  if (!c) return FIRP_EINVAL;
  if (!valid) return c->fail(FIRP_EINVAL, "argument pointer is NULL");
  if (!c->prefilled) return c->fail(FIRP_ESTATE, "no sequence is running");
  if (drafts) {   // (without it only the flags are wanted: they are mirrored on the host)
    HIPCHK(hipStreamSynchronize(c->stream));
    if (c->k > 0)
      HIPCHK(hipMemcpy(drafts, c->st.drafts, (size_t)c->batch * c->k * c->d.b_max * sizeof(int), hipMemcpyDeviceToHost));
  }
  for (int b = 0; b < c->batch; ++b) valid[b] = c->drafts_valid[b];
  return FIRP_OK;
}

firp_status firp_get_ctx_len(const firp_ctx* cc, int32_t* len) {
  firp_ctx* c = const_cast<firp_ctx*>(cc);
  if (!c) return FIRP_EINVAL;
  if (!len) return c->fail(FIRP_EINVAL, "argument pointer is NULL");
  for (int b = 0; b < c->batch; ++b) len[b] = c->p0[b];
  return FIRP_OK;
}

firp_status firp_debug_read_cache(firp_ctx* c, int32_t seq, int32_t layer, float* k_out, float* v_out) {
  if (!c) return FIRP_EINVAL;
  if (!k_out || !v_out) return c->fail(FIRP_EINVAL, "argument pointer is NULL");
  if (!c->prefilled) return c->fail(FIRP_ESTATE, "no sequence is running");
  if (seq < 0 || seq >= c->batch || layer < 0 || layer >= c->d.n_layers) return c->fail(FIRP_EINVAL, "sequence or layer out of range");
  HIPCHK(hipStreamSynchronize(c->stream));
  int len = c->p0[seq], H = c->d.n_kv_heads, dh = c->d.head_dim, S = c->slots, es = c->esize;
  std::vector<char> hk((size_t)H * S * dh * es), hv((size_t)H * S * dh * es);
  size_t off = ((size_t)seq * c->kv_seq_stride + (size_t)layer * c->kv_layer_stride) * es;
  HIPCHK(hipMemcpy(hk.data(), (char*)c->kcache + off, hk.size(), hipMemcpyDeviceToHost));
  HIPCHK(hipMemcpy(hv.data(), (char*)c->vcache + off, hv.size(), hipMemcpyDeviceToHost));
  auto get = [&](const std::vector<char>& buf, size_t idx) -> float {
    if (es == 4) return ((const float*)buf.data())[idx];
    uint32_t u = ((uint32_t)((const uint16_t*)buf.data())[idx]) << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
  };
  for (int t = 0; t < len; ++t)
    for (int h = 0; h < H; ++h)
      for (int e = 0; e < dh; ++e) {
        k_out[((size_t)t * H + h) * dh + e] = get(hk, ((size_t)h * S + t) * dh + e);
        v_out[((size_t)t * H + h) * dh + e] = get(hv, ((size_t)h * dh + e) * S + t);
      }
  return FIRP_OK;
}

firp_status firp_set_option(firp_ctx* c, const char* name, int32_t value) {
  if (!c) return FIRP_EINVAL;
  if (!name) return c->fail(FIRP_EINVAL, "option name is NULL");
  if (!strcmp(name, "gemm")) {
    if (value == 0) {
      c->gemm_kind = 0;
      c->split = false;
      c->attn_kind = 0;
      return FIRP_OK;
    }
    if (value == 1 && c->dtype == FIRP_BF16 && mfma_shapes_ok(c->d, c->qkv_ld)) {
      c->gemm_kind = 1;
      c->split = true;
      c->attn_kind = attention_mfma_supported(c->d.head_dim, c->dtype) ? 1 : 0;
      return FIRP_OK;
    }
    return c->fail(FIRP_EINVAL, "gemm kind %d is not available for this model", value);
  }
  if (!strcmp(name, "attn")) {
    if (value == 0) {
      c->attn_kind = 0;
      return FIRP_OK;
    }
    if (value == 1 && c->split && attention_mfma_supported(c->d.head_dim, c->dtype)) {
      c->attn_kind = 1;
      return FIRP_OK;
    }
    return c->fail(FIRP_EINVAL, "attention kind %d is not available for this model", value);
  }
  if (!strcmp(name, "graph")) {
    if (value < 0 || value > 2) return c->fail(FIRP_EINVAL, "graph takes 0 (never), 1 (whenever possible) or 2 (where it pays)");
    c->graph_mode = value;
    c->use_graph = value == 1 || (value == 2 && step_weight_bytes(c) <= 8e9);
    return FIRP_OK;
  }
  if (!strcmp(name, "keep_logits")) {
    if (value != 0 && value != 1) return c->fail(FIRP_EINVAL, "keep_logits takes 0 or 1");
    c->keep_logits = value != 0;
    return FIRP_OK;
  }
  if (!strcmp(name, "time_gemm")) {
    if (value != 0 && value != 1) return c->fail(FIRP_EINVAL, "time_gemm takes 0 or 1");
    if (value && c->ev.empty()) {
      c->ev.resize(2 * (size_t)(8 * c->d.n_layers + 16));
      for (auto& e : c->ev)
        if (hipEventCreate(&e) != hipSuccess) {
          c->ev.clear();
          return c->fail(FIRP_EDEVICE, "hipEventCreate failed");
        }
    }
    if (value && !c->ev_empty[0])
      for (auto& e : c->ev_empty)
        if (hipEventCreate(&e) != hipSuccess) return c->fail(FIRP_EDEVICE, "hipEventCreate failed");
    c->time_gemm = value != 0;
    c->gemm_ms = c->gemm_bytes = 0.0;
    c->gemm_launches = 0;
    c->empty_ms = 0.0;
    c->empty_n = 0;
    c->ev_used = 0;
    return FIRP_OK;
  }
  return c->fail(FIRP_EINVAL, "unknown option '%s'", name);
}

firp_status firp_get_gemm_timing(const firp_ctx* c, int64_t* launches, double* total_ms, double* weight_bytes) {
  if (!c) return FIRP_EINVAL;
  if (launches) *launches = c->gemm_launches;
  if (total_ms) *total_ms = c->gemm_ms;
  if (weight_bytes) *weight_bytes = c->gemm_bytes;
  return FIRP_OK;
}

firp_status firp_get_stat(const firp_ctx* cc, const char* name, int64_t* value) {
  firp_ctx* c = const_cast<firp_ctx*>(cc);
  if (!c) return FIRP_EINVAL;
  if (!name || !value) return c->fail(FIRP_EINVAL, "argument pointer is NULL");
  if (!strcmp(name, "topo_uploads")) {
    *value = c->topo_uploads;
    return FIRP_OK;
  }
  if (!strcmp(name, "graph_launches")) {
    *value = c->graph_launches;
    return FIRP_OK;
  }
  if (!strcmp(name, "graph_captures")) {
    *value = c->graph_captures;
    return FIRP_OK;
  }
  return c->fail(FIRP_EINVAL, "unknown statistic '%s'", name);
}

firp_status firp_get_event_overhead(const firp_ctx* c, double* bracket_ms) {
  if (!c || !bracket_ms) return FIRP_EINVAL;
  *bracket_ms = c->empty_n > 0 ? c->empty_ms / (double)c->empty_n : 0.0;
  return FIRP_OK;
}

size_t firp_gemm_workspace_bytes(int32_t rows, int32_t n, int32_t k_dim) {
  if (rows < 1 || n < 1 || k_dim < 1) return 0;
  size_t rp = align_up(rows, 16);
  // activation planes, partial sums of up to 16 splits, the fragment-major copy of W
  return align_up(rp * k_dim * 2 * 2, 256) + align_up(rp * (size_t)n * 4 * 16, 256) +
         align_up(gemm_packed_bytes(n, k_dim), 256) + 512;
}

// the MFMA projection of the standalone entries: operand planes, split-K partial sums and the
// fragment-major copy of w live in `workspace` (>= firp_gemm_workspace_bytes)
static void gemm_in_workspace(const float* x, const void* w, float* y, int rows, int n, int k_dim, void* workspace,
                              hipStream_t s) {
  size_t rp = align_up(rows, 16);
  Act a{};
  a.ld = k_dim;
  a.hi = (bf16*)workspace;
  a.lo = a.hi + rp * k_dim;
  float* part = (float*)((char*)workspace + align_up(rp * k_dim * 2 * 2, 256));
  void* wpk = (char*)part + align_up(rp * (size_t)n * 4 * 16, 256);
  launch_split_act(x, rows, k_dim, a, s);
  launch_pack_weights(wseg1(w, n), n, k_dim, wpk, s);
  GemmPlan plan = gemm_mfma_plan(rows, n, k_dim, 0);
  launch_gemm_mfma(a, wpk, part, n, rp * n, rows, n, k_dim, plan, s);
  launch_reduce_partials(Partial{part, plan.S, rp * (size_t)n, n}, y, rows, s);
}

firp_status firp_debug_gemm(const float* x, const void* w, float* y, int32_t rows, int32_t n, int32_t k_dim,
                            int32_t dtype, int32_t kind, void* workspace, size_t workspace_bytes,
                            void* hip_stream) {
  if (!x || !w || !y || rows < 1 || n < 1 || k_dim < 1) return FIRP_EINVAL;
  if (dtype != FIRP_F32 && dtype != FIRP_BF16) return FIRP_EINVAL;
  hipStream_t s = (hipStream_t)hip_stream;
  if (kind == 0) {
    launch_gemm_simple(x, k_dim, w, dtype, y, n, rows, n, k_dim, s);
  } else if (kind == 1) {
    if (dtype != FIRP_BF16 || !gemm_mfma_supported(rows, n, k_dim)) return FIRP_EINVAL;
    if (!workspace || (((uintptr_t)workspace) & 255) || workspace_bytes < firp_gemm_workspace_bytes(rows, n, k_dim))
      return FIRP_ECAPACITY;
    gemm_in_workspace(x, w, y, rows, n, k_dim, workspace, s);
  } else {
    return FIRP_EINVAL;
  }
  return hipGetLastError() == hipSuccess ? FIRP_OK : FIRP_EDEVICE;
}

// ---- the projection entry that allocates nothing -------------------------------------------------
// Its scratch (operand planes, split-K partial sums, the fragment-major copy of w) is a fixed
// array in device memory that every GPU the library runs on holds until the process ends.  In
// host code the array's name is only a handle: its device address is looked up once per device
// and that pointer is what the kernels get.
#define FIRP_STATIC_SCRATCH_BYTES ((size_t)32 << 20)
#define FIRP_MAX_DEVICES 64
static __device__ __align__(256) unsigned char scratch[FIRP_STATIC_SCRATCH_BYTES];
static void* g_scratch_ptr[FIRP_MAX_DEVICES];

size_t firp_gemm_static_capacity(void) { return FIRP_STATIC_SCRATCH_BYTES; }

firp_status firp_debug_gemm_static(const float* x, const void* w, float* y, int32_t rows, int32_t n, int32_t k_dim,
                                   void* hip_stream) {
  auto bad = [&](firp_status code, const std::string& m) {
    g_init_error = m;
    return code;
  };
  if (!x || !w || !y || rows < 1 || n < 1 || k_dim < 1) return bad(FIRP_EINVAL, "firp_debug_gemm_static: NULL pointer or non-positive size");
  if (!gemm_mfma_supported(rows, n, k_dim)) return bad(FIRP_EINVAL, "firp_debug_gemm_static: n must be a multiple of 4 and K a multiple of 8");
  const size_t need = firp_gemm_workspace_bytes(rows, n, k_dim);
  if (need > FIRP_STATIC_SCRATCH_BYTES) {
    char buf[256];
    snprintf(buf, sizeof buf, "firp_debug_gemm_static: %d x %d x %d needs %zu bytes of scratch, the fixed buffer holds %zu",
             rows, n, k_dim, need, (size_t)FIRP_STATIC_SCRATCH_BYTES);
    return bad(FIRP_ECAPACITY, buf);
  }
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= FIRP_MAX_DEVICES) return bad(FIRP_EDEVICE, "firp_debug_gemm_static: no current device");
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) return bad(FIRP_EDEVICE, std::string("firp_debug_gemm_static: hipGetSymbolAddress failed: ") + hipGetErrorString(e));
    g_scratch_ptr[dev] = p;
  }
  gemm_in_workspace(x, w, y, rows, n, k_dim, g_scratch_ptr[dev], (hipStream_t)hip_stream);
  return hipGetLastError() == hipSuccess ? FIRP_OK : bad(FIRP_EDEVICE, "firp_debug_gemm_static: kernel launch failed");
}

firp_status firp_debug_stream_read(const void* src, size_t bytes, void* sink, void* hip_stream) {
  if (!src || !sink || bytes < 16 || (((uintptr_t)src) & 15)) return FIRP_EINVAL;
  launch_stream_read(src, bytes, (unsigned*)sink, (hipStream_t)hip_stream);
  return hipGetLastError() == hipSuccess ? FIRP_OK : FIRP_EDEVICE;
}

firp_status firp_debug_gemm_plan(int32_t rows, int32_t n, int32_t k_dim, int32_t* splits, int32_t* k_per_split,
                                 int32_t* waves, int32_t* grid, int32_t* row_block) {
  if (!gemm_mfma_supported(rows, n, k_dim)) return FIRP_EINVAL;
  const GemmPlan p = gemm_mfma_plan(rows, n, k_dim, 0);
  if (splits) *splits = p.S;
  if (k_per_split) *k_per_split = p.k_per;
  if (waves) *waves = p.nw;
  if (grid) *grid = p.grid;
  if (row_block) *row_block = p.row_block;
  return FIRP_OK;
}

}  // extern "C"
