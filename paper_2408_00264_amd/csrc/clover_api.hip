// C-ABI layer of libclover.so: context, validation, workspace carving and the kernel sequences of
// the three calls of a speculative step.  All arithmetic runs in the kernels this file launches.
#include "../../include/clover.h"
#include "clover_internal.h"

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <string>
#include <vector>

using namespace clv;

#ifdef CLOVER_ABLATE
#include <cstdlib>
#include <map>
namespace clv {
int tune_int(const char* name, int dflt) {
  static std::map<std::string, int> seen;   // read once per process
  auto it = seen.find(name);
  if (it != seen.end()) return it->second;
  const char* v = getenv(name);
  return seen[name] = v ? atoi(v) : dflt;
}
}  // namespace clv
#endif

namespace {

thread_local std::string g_err;

int op_gemm_impl(int32_t path, int32_t dtype, const float* X, const void* W, float* Y, int32_t ldy, int32_t M,
                 int32_t N, int32_t K, void* scratch, size_t scratch_bytes, void* hip_stream);

// Scratch of clover_op_gemm_static: one copy per GPU, held until the process ends.  In host code the name below is
// only a handle for hipGetSymbolAddress; every use goes through the per-device address looked up once.
__device__ __align__(256) unsigned char g_static_scratch[CLOVER_STATIC_SCRATCH_BYTES];
constexpr int kMaxDevices = 64;
void* g_static_scratch_ptr[kMaxDevices] = {};
int static_scratch_ptr(void** out);

const char* kClassNames[KC_COUNT] = {"embed",     "rmsnorm",     "gemm_qkv",   "rope_kv_write", "tree_attention", "gemm_wo",
                                     "gemm_gate_up", "gemm_down", "gemm_lm_head", "gemm_draft",  "ad_gate",        "topk",
                                     "draft_misc", "accept_walk", "compact_kv", "eltwise"};

size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

struct TreeHost {
  int n = 0, max_depth = 0;
  std::vector<int> parent, rank, depth, first_child, n_child;
  std::vector<int> lvl_nodes;           // internal nodes, grouped by depth
  std::vector<int> lvl_off;             // [max_depth+2]: internal nodes of depth j are lvl_nodes[lvl_off[j]..lvl_off[j+1])
  std::vector<int> par_row;             // per node: index of its parent within the parent's depth group
  std::vector<int> node_off;            // [max_depth+2]: nodes of depth j are [node_off[j], node_off[j+1])
  std::vector<int> kmax;                // per depth j: 1 + max rank among children of depth-j nodes
  std::vector<unsigned long long> anc;  // [n][2] (all zero for trees of more than 128 nodes: those use the labels)
  std::vector<int> iv;                  // [n][2] interval labels: enter, exit of a depth-first numbering
  bool is_chain = false;
};

struct ProfEvent {
  int cls;
  hipEvent_t a, b;
};

}  // namespace

struct clover_ctx {
  clover_config cfg;
  hipStream_t st;
  clover_weights w;
  std::vector<clover_layer_weights> layers, aug;
  std::vector<const void*> fc_w, fc_b;
  TreeHost tree;
  std::string err;
  // sizes
  int R, max_rows, H, QKVN, NQD;
  KVLayout kv;
  size_t k_layer_elems, v_layer_elems, esz, kv_esz;
  int kvdtype;  // 0: fp32 cache elements; 1: (hi, lo) bf16 planes, same bytes (a random-init 32-layer stack amplifies
                // plain bf16 cache rounding ~20x, so 16 mantissa bits are kept either way)
  size_t kv_layer_stride;  // cache elements (of the kvdtype's element type) per layer
  bool attn_fast;
  float *o_part, *ml_part;
  int attn_max_splits;
  // device regions
  int *d_seq_len, *d_aug_len, *d_err;
  int *d_depth, *d_parent, *d_rank, *d_first_child, *d_n_child, *d_lvl_nodes, *d_par_row;
  unsigned long long* d_anc;
  int* d_pages;            // page table [max_batch][max_seq / KV_PAGE] (used once clover_set_page_table was called)
  int* d_iv;               // interval labels of the static tree [R][2]
  bool interval;           // CLOVER_FLAG_INTERVAL_MASK: tree attention reads the labels instead of the bit sets
  char *kc, *vc, *aug_kc, *aug_vc;
  float *xd, *a_norm, *qkv, *q_rot, *attn_out, *h_ffn, *tmp_ffn, *cos_t, *sin_t;
  float *ad_q, *ad_k, *ad_v, *d_xs, *d_e, *d_cat, *d_g, *d_s, *d_state, *d_rootx, *z;
  void* cand;
  int* topk_ids;
  float* partial;          // split-K partial tiles / plain GEMM outputs of the MFMA path
  size_t partial_bytes;
  float* pl_y;             // planes of draft-side GEMM inputs that no fused producer writes
  char* packed;            // fragment-major copies of every linear weight (MFMA path)
  size_t packed_bytes;
  const void* lm_head_pk;
  bool fast;               // bf16 model on the MFMA path
  bool panel;              // full-K panel GEMM for the gate+up projection and the LM head
  int tile_min_kp = 65;    // narrow outputs over K ranges take the tiled GEMM's 128 x 256 form from this many rows on
  int tile_min = 129;      // passes of at least this many rows (up to 256) take the tiled GEMM: one weight pass
  int row_batch_max = 64;
  int row_batch = 64;      // rows per weight pass for passes of more than 64 rows: 128 when the panel kernel may take them  // passes of up to this many rows run through the <= 64-row GEMM kernels, in batches of 64
  // dynamic (score-pruned) tree: candidates, frontiers and the per-sequence topology tables
  bool dyn_on = false;
  DynTree dyn{};
  float *topk_vals, *topk_lse, *topk_aux;
  float* dyn_state;        // [B][DYN_MAX_CAND][H] draft states of the expanded candidates
  float* draft_capture = nullptr;   // test hook: device buffer that receives every depth's draft logits
  size_t draft_capture_floats = 0;
  // host-side bounds
  std::vector<int> len_ub, aug_ub;
  int m_upper;
  bool only_prefills;   // no accept call since init / reset: every pending hand-off has m = 1
  // profiling
  bool prof = false;
  std::vector<ProfEvent> prof_events;
  std::vector<ProfEvent> prof_pool;
};

namespace {

int fail(clover_ctx* ctx, int code, const std::string& msg) {
  if (ctx) ctx->err = msg; else g_err = msg;
  return code;
}

int check_config(const clover_config* c, std::string& why) {
  auto bad = [&](const char* m) { why = m; return CLOVER_E_CONFIG; };
  if (c->n_layers < 1 || c->hidden < 1 || c->n_q_heads < 1 || c->n_kv_heads < 1 || c->ffn < 1) return bad("non-positive model dimension");
  if (c->head_dim != 64 && c->head_dim != 128) return bad("head_dim must be 64 or 128");
  if (c->n_q_heads % c->n_kv_heads != 0) return bad("n_q_heads must be a multiple of n_kv_heads");
  if (c->ad_heads < 1 || c->hidden % c->ad_heads != 0) return bad("hidden must be a multiple of ad_heads");
  if (c->hidden % 4 != 0 || c->ffn % 4 != 0) return bad("hidden and ffn must be multiples of 4");
  if (c->vocab < 16 || c->vocab > 262144) return bad("vocab must be in [16, 262144]");
  if (c->dtype != CLOVER_DTYPE_F32 && c->dtype != CLOVER_DTYPE_BF16) return bad("unknown dtype");
  if (c->aug_layers < 1 || c->aug_layers > 8) return bad("aug_layers must be in [1, 8]");
  if (c->draft_depths < 1 || c->draft_depths > CLOVER_MAX_DEPTH) return bad("draft_depths out of range");
  if (c->max_batch < 1 || c->max_batch > 1024) return bad("max_batch out of range");
  if (c->max_seq % KV_PAGE != 0) return bad("max_seq must be a multiple of 32 (the page size of the caches)");
  if (c->max_nodes < 1 || c->max_nodes > ((c->flags & CLOVER_FLAG_INTERVAL_MASK) ? CLOVER_MAX_NODES_INTERVAL : CLOVER_MAX_NODES))
    return bad("max_nodes must be in [1, 128] (in [1, 256] with CLOVER_FLAG_INTERVAL_MASK)");
  if (c->prefill_rows < 0 || c->prefill_rows > CLOVER_MAX_PREFILL_ROWS) return bad("prefill_rows must be in [0, 256]");
  if (c->max_seq < c->max_nodes) return bad("max_seq smaller than max_nodes");
  if (!(c->rope_base > 1.f) || !(c->rms_eps > 0.f)) return bad("rope_base must be > 1 and rms_eps > 0");
  return CLOVER_OK;
}

int build_tree(const clover_config& cfg, const clover_tree* t, TreeHost& out, std::string& why) {
  auto bad = [&](const char* m) { why = m; return CLOVER_E_TREE; };
  if (!t->parent || !t->rank) { why = "tree arrays are null"; return CLOVER_E_NULL; }
  const int n = t->n_nodes;
  if (n < 1 || n > cfg.max_nodes) return bad("n_nodes outside [1, max_nodes]");
  if (t->parent[0] != -1) return bad("parent[0] must be -1");
  TreeHost h;
  h.n = n;
  h.parent.assign(t->parent, t->parent + n);
  h.rank.assign(t->rank, t->rank + n);
  h.depth.assign(n, 0);
  h.first_child.assign(n, 0);
  h.n_child.assign(n, 0);
  h.par_row.assign(n, 0);
  for (int u = 1; u < n; ++u) {
    const int p = h.parent[u];
    if (p < 0 || p >= u) return bad("parent index must satisfy 0 <= parent[u] < u");
    if (u >= 2 && p < h.parent[u - 1]) return bad("nodes must be in breadth-first order (parent non-decreasing)");
    if (h.rank[u] < 0 || h.rank[u] >= CLOVER_MAX_RANK) return bad("rank outside [0, 16)");
    h.depth[u] = h.depth[p] + 1;
    if (h.n_child[p] == 0) h.first_child[p] = u;
    h.n_child[p]++;
  }
  for (int u = 0; u < n; ++u) {
    unsigned seen = 0;
    for (int c = h.first_child[u]; c < h.first_child[u] + h.n_child[u]; ++c) {
      if (seen & (1u << h.rank[c])) return bad("siblings must have distinct ranks");
      seen |= 1u << h.rank[c];
    }
  }
  h.max_depth = h.depth[n - 1];
  h.is_chain = true;
  for (int u = 1; u < n; ++u) h.is_chain = h.is_chain && (h.parent[u] == u - 1);
  h.lvl_off.assign(h.max_depth + 2, 0);
  h.node_off.assign(h.max_depth + 2, 0);
  h.kmax.assign(h.max_depth + 1, 0);
  std::vector<int> row_in_level(n, -1);
  for (int j = 0; j <= h.max_depth; ++j) {
    h.lvl_off[j] = (int)h.lvl_nodes.size();
    for (int u = 0; u < n; ++u) {
      if (h.depth[u] != j) continue;
      if (h.n_child[u] > 0) {
        row_in_level[u] = (int)h.lvl_nodes.size() - h.lvl_off[j];
        h.lvl_nodes.push_back(u);
        for (int c = h.first_child[u]; c < h.first_child[u] + h.n_child[u]; ++c) h.kmax[j] = std::max(h.kmax[j], h.rank[c] + 1);
      }
    }
  }
  h.lvl_off[h.max_depth + 1] = (int)h.lvl_nodes.size();
  {
    int u = 0;
    for (int j = 0; j <= h.max_depth; ++j) {
      h.node_off[j] = u;
      while (u < n && h.depth[u] == j) ++u;
    }
    h.node_off[h.max_depth + 1] = n;
    if (u != n) return bad("depth must be non-decreasing");
  }
  for (int u = 1; u < n; ++u) h.par_row[u] = row_in_level[h.parent[u]];
  h.anc.assign((size_t)2 * n, 0ull);
  for (int u = 0; u < n && n <= CLOVER_MAX_NODES; ++u) {
    if (u > 0) { h.anc[2 * u] = h.anc[2 * h.parent[u]]; h.anc[2 * u + 1] = h.anc[2 * h.parent[u] + 1]; }
    h.anc[2 * u + (u >> 6)] |= 1ull << (u & 63);
  }
  // interval labels (Appendix A.1, linear-size mask): subtree sizes bottom-up (children have larger indices), then
  // enter[child] = enter[parent] + 1 + sizes of the earlier siblings; exit = enter + size - 1
  {
    std::vector<int> size(n, 1);
    for (int u = n - 1; u >= 1; --u) size[h.parent[u]] += size[u];
    h.iv.assign((size_t)2 * n, 0);
    for (int u = 0; u < n; ++u) {
      int e = h.iv[2 * u] + 1;
      for (int c = h.first_child[u]; c < h.first_child[u] + h.n_child[u]; ++c) { h.iv[2 * c] = e; e += size[c]; }
      h.iv[2 * u + 1] = h.iv[2 * u] + size[u] - 1;
    }
  }
  out = std::move(h);
  return CLOVER_OK;
}

// ---- workspace carving ---------------------------------------------------------------------
struct Carver {
  char* base;
  size_t off = 0;
  template <typename T>
  T* take(size_t count) {
    T* p = base ? (T*)(base + off) : nullptr;
    off = align256(off + count * sizeof(T));
    return p;
  }
};

struct GemmShape { int N, K, mode; };

void model_gemm_shapes(const clover_config& c, std::vector<GemmShape>& v) {
  const int H = c.hidden, nqd = c.n_q_heads * c.head_dim, qkvn = (c.n_q_heads + 2 * c.n_kv_heads) * c.head_dim;
  v = {{qkvn, H, 0}, {H, nqd, 1}, {c.ffn, H, 2}, {2 * c.ffn, H, 0}, {H, c.ffn, 1}, {c.vocab, H, 0}, {H, H, 0}, {H, 2 * H, 0}};
}

void carve(clover_ctx* x, char* base, size_t* total) {
  const clover_config& c = x->cfg;
  Carver cv{base};
  const int B = c.max_batch, R = c.max_nodes, H = c.hidden, d = c.head_dim;
  const int rows = std::max(B * R, c.prefill_rows);   // row capacity of every activation buffer
  const size_t esz = c.dtype == CLOVER_DTYPE_F32 ? 4 : 2;
  x->R = R; x->max_rows = rows; x->H = H; x->esz = esz;
  x->kv_esz = 4;  // bytes per cached value in both formats
  x->NQD = c.n_q_heads * d;
  x->QKVN = (c.n_q_heads + 2 * c.n_kv_heads) * d;
  x->k_layer_elems = (size_t)B * c.max_seq * c.n_kv_heads * d;
  x->d_pages = cv.take<int>((size_t)B * (c.max_seq / KV_PAGE));
  x->kv = KVLayout{B, c.max_seq, c.n_kv_heads, d, x->k_layer_elems, c.max_seq / KV_PAGE, 0, nullptr};
  x->v_layer_elems = x->k_layer_elems;
  x->d_seq_len = cv.take<int>(B);
  x->d_aug_len = cv.take<int>(B);
  x->d_err = cv.take<int>(1);
  x->d_depth = cv.take<int>(R);
  x->d_parent = cv.take<int>(R);
  x->d_rank = cv.take<int>(R);
  x->d_first_child = cv.take<int>(R);
  x->d_n_child = cv.take<int>(R);
  x->d_lvl_nodes = cv.take<int>(R);
  x->d_par_row = cv.take<int>(R);
  x->d_anc = cv.take<unsigned long long>(2 * R);
  x->d_iv = cv.take<int>(2 * R);
  x->kc = cv.take<char>(x->k_layer_elems * x->kv_esz * c.n_layers);
  x->vc = cv.take<char>(x->v_layer_elems * x->kv_esz * c.n_layers);
  x->aug_kc = cv.take<char>(x->k_layer_elems * x->kv_esz * c.aug_layers);
  x->aug_vc = cv.take<char>(x->v_layer_elems * x->kv_esz * c.aug_layers);
  x->xd = cv.take<float>((size_t)rows * H);
  x->a_norm = cv.take<float>((size_t)rows * 2 * H);
  x->qkv = cv.take<float>((size_t)rows * x->QKVN);
  x->q_rot = cv.take<float>((size_t)rows * x->NQD);
  x->attn_out = cv.take<float>((size_t)rows * x->NQD);
  x->h_ffn = cv.take<float>((size_t)rows * c.ffn);
  x->tmp_ffn = cv.take<float>((size_t)rows * c.ffn);
  x->cos_t = cv.take<float>((size_t)rows * d / 2);
  x->sin_t = cv.take<float>((size_t)rows * d / 2);
  x->ad_q = cv.take<float>((size_t)rows * H);
  x->ad_k = cv.take<float>((size_t)rows * H);
  x->ad_v = cv.take<float>((size_t)rows * H);
  x->d_xs = cv.take<float>((size_t)rows * H);
  x->d_e = cv.take<float>((size_t)rows * H);
  x->d_cat = cv.take<float>((size_t)rows * 2 * H);
  x->d_g = cv.take<float>((size_t)rows * H);
  x->d_s = cv.take<float>((size_t)rows * H);
  x->d_state = cv.take<float>((size_t)rows * H);
  x->d_rootx = cv.take<float>((size_t)B * H);
  x->z = cv.take<float>((size_t)rows * c.vocab);
  x->cand = cv.take<unsigned long long>((size_t)rows * topk_chunks(c.vocab) * 16);
  x->topk_ids = cv.take<int>((size_t)rows * 16);
  x->topk_vals = cv.take<float>((size_t)rows * 16);
  x->topk_lse = cv.take<float>((size_t)rows);
  x->topk_aux = cv.take<float>((size_t)rows * topk_chunks(c.vocab) * 2);
  x->dyn.cand_tok = cv.take<int>((size_t)B * DYN_MAX_CAND);
  x->dyn.cand_score = cv.take<float>((size_t)B * DYN_MAX_CAND);
  x->dyn.cand_par = cv.take<int>((size_t)B * DYN_MAX_CAND);
  x->dyn.frontier = cv.take<int>((size_t)B * CLOVER_MAX_DEPTH * DYN_MAX_FRONT);
  x->dyn.t_parent = cv.take<int>((size_t)rows);
  x->dyn.t_rank = cv.take<int>((size_t)rows);
  x->dyn.t_depth = cv.take<int>((size_t)rows);
  x->dyn.t_first_child = cv.take<int>((size_t)rows);
  x->dyn.t_n_child = cv.take<int>((size_t)rows);
  x->dyn.t_keep = cv.take<int>((size_t)rows);
  x->dyn.t_anc = cv.take<unsigned long long>((size_t)rows * 2);
  x->dyn.t_iv = cv.take<int>((size_t)rows * 2);
  x->dyn_state = cv.take<float>((size_t)B * DYN_MAX_CAND * H);
  // MFMA path: is every GEMM shape of this model supported, and how large can an output with its
  // split-K partials get?
  size_t pbytes = 256;
  bool fast = c.dtype == CLOVER_DTYPE_BF16 && !(c.flags & CLOVER_FLAG_GENERIC);
  if (fast) {
    std::vector<GemmShape> shapes;
    model_gemm_shapes(c, shapes);
    for (const GemmShape& s : shapes) fast = fast && mfma_gemm_supported(1, s.N, s.K, s.mode);
    fast = fast && (c.n_kv_heads * d) % 16 == 0;
  }
  size_t packed_bytes = 0;
  if (fast) {
    std::vector<GemmShape> shapes;
    model_gemm_shapes(c, shapes);
    for (const GemmShape& s : shapes) {
      if (s.mode == 2) continue;
      if (stream_gemm_supported(std::min(rows, 64), s.N, s.K))
        pbytes = std::max(pbytes, stream_gemm_out_bytes(std::min(rows, 64), s.N, s.K));
      for (int M = 65; M <= std::min(rows, 256); ++M) {
        const int sp = mfma_gemm_pick_splits(M, s.N, s.K, s.mode);
        const size_t mtot = rows <= 256 ? (size_t)M : (size_t)rows;
        pbytes = std::max(pbytes, (size_t)sp * mtot * s.N * sizeof(float));
      }
    }
    // 129..256 rows through the tiled kernel over K ranges: partial tiles of the whole pass
    if (rows > 64) {
      std::vector<GemmShape> shp;
      model_gemm_shapes(c, shp);
      const int rb = std::min(rows, 256);
      for (const GemmShape& g : shp)
        if (g.mode != 2 && tile_gemm_supported(rb, g.N, g.K, 0))
          pbytes = std::max(pbytes, (size_t)tile_gemm_pick_k_parts(rb, g.N, g.K) *
                                        rb * g.N * sizeof(float));
    }
    // 65..256 rows in batches of 64 through the K-slice kernel: partial tiles of the whole pass
    if (rows > 64 && !tune_int("CLOVER_NO_ROW_BATCH", 0)) {
      std::vector<GemmShape> shp;
      model_gemm_shapes(c, shp);
      const int rb = std::min(rows, 256);
      for (const GemmShape& g : shp)
        if (g.mode != 2 && g.N != c.vocab && g.N != 2 * c.ffn && stream_gemm_supported(64, g.N, g.K))
          pbytes = std::max(pbytes, stream_gemm_out_bytes(rb, g.N, g.K));
    }
    const size_t layer_elems = (size_t)x->QKVN * H + (size_t)H * x->NQD + (size_t)3 * c.ffn * H;
    packed_bytes = 2 * ((size_t)(c.n_layers + c.aug_layers) * layer_elems + (size_t)c.vocab * H + (size_t)7 * H * H +
                        (size_t)(c.draft_depths - 1) * 2 * H * H);
  }
  x->packed_bytes = packed_bytes;
  x->packed = cv.take<char>(packed_bytes ? packed_bytes : 256);
  x->fast = fast;
  x->panel = fast && !tune_int("CLOVER_NO_PANEL", 0);
  x->row_batch_max = (fast && !tune_int("CLOVER_NO_ROW_BATCH", 0)) ? 256 : 64;
  x->row_batch = (x->panel && !tune_int("CLOVER_ROW_BATCH_64", 0)) ? 128 : 64;
  x->tile_min = fast ? tune_int("CLOVER_TILE_MIN", 129) : 1 << 30;
  x->tile_min_kp = fast ? tune_int("CLOVER_TILE_MIN_KP", 65) : 1 << 30;
  x->kvdtype = fast ? 1 : 0;
  x->kv_layer_stride = fast ? 2 * x->k_layer_elems : x->k_layer_elems;
  x->attn_fast = fast && attn_mfma_supported(d, c.n_q_heads, c.n_kv_heads, c.max_seq);
  x->attn_max_splits = 16;
  x->o_part = cv.take<float>(x->attn_fast ? (size_t)x->attn_max_splits * rows * x->NQD : 64);
  x->ml_part = cv.take<float>(x->attn_fast ? (size_t)x->attn_max_splits * rows * c.n_q_heads * 2 : 64);
  x->partial_bytes = pbytes;
  x->partial = (float*)cv.take<char>(pbytes);
  x->pl_y = cv.take<float>((size_t)rows * 2 * H);
  *total = cv.off;
}

// ---- profiling ------------------------------------------------------------------------------
struct Scope {
  clover_ctx* x;
  ProfEvent ev;
  bool on;
  Scope(clover_ctx* ctx, int cls) : x(ctx), on(ctx->prof) {
    if (!on) return;
    if (!x->prof_pool.empty()) { ev = x->prof_pool.back(); x->prof_pool.pop_back(); }
    else { hipEventCreate(&ev.a); hipEventCreate(&ev.b); }
    ev.cls = cls;
    hipEventRecord(ev.a, x->st);
  }
  ~Scope() {
    if (!on) return;
    hipEventRecord(ev.b, x->st);
    x->prof_events.push_back(ev);
  }
};

// ---- GEMM dispatch ----------------------------------------------------------------------------
struct Planes {
  bf16_t *hi, *lo;
  int ld;
};
// planes view of an fp32 activation buffer of capacity max_rows x K floats (same bytes)
Planes planes_of(clover_ctx* x, float* buf, int K) {
  bf16_t* hi = (bf16_t*)buf;
  return Planes{hi, hi + (size_t)x->max_rows * K, K};
}

// MFMA path: out[s][M][N] = X * [W0; W1; W2]^T per split s.  Writes into `direct` (leading dimension
// ld_direct, no split) when given, else into x->partial as [splits][M][N].  Returns the split count.
int gemm_fast(clover_ctx* x, int cls, Planes X, int nseg, const void* const* W, const int* seg_n, int M, int N, int K,
              float* direct, int ld_direct, float* part = nullptr /* where the K-slice partials go (stream path) */) {
  Scope sc(x, cls);
  if (!part) part = x->partial;
  int segb[4] = {0, 0x7fffffff, 0x7fffffff, 0x7fffffff};
  const bf16_t* ws[3];
  {
    int off = 0;
    for (int s = 0; s < 3; ++s) {
      ws[s] = (const bf16_t*)(s < nseg ? W[s] : W[nseg - 1]);
      if (s < nseg) { segb[s] = off; off += seg_n[s]; }
    }
  }
  // Many rows (65..256: this route writes partials over K ranges, where the tiled kernel's 128-row form already beats
  // the panel kernel's K-range form from 65 rows on): one pass over the weights for all rows.
  if (!direct && M >= std::min(x->tile_min, x->tile_min_kp) && M <= 256 && tile_gemm_supported(M, N, K, 0)) {
    bool adjacent = true;
    for (int s = 1; s < nseg; ++s) adjacent = adjacent && ws[s] == ws[s - 1] + (size_t)seg_n[s - 1] * K;
    const int kp = tile_gemm_pick_k_parts(M, N, K);
    if (adjacent && (size_t)kp * M * N * sizeof(float) <= x->partial_bytes) {
      TileGemm g;
      memset(&g, 0, sizeof(g));
      g.Xhi = X.hi; g.Xlo = X.lo; g.ldx = X.ld;
      g.W[0] = g.W[1] = ws[0];
      g.Y = part; g.ldy = N; g.k_parts = kp; g.split_stride = (size_t)M * N;
      g.M = M; g.N = N; g.K = K; g.epi = 0;
      launch_gemm_tile(g, x->st);
      return kp;
    }
  }
  // Long K into a narrow output (the down projection): K ranges of the panel kernel, a few partials instead of
  // one per 512 columns.  Passes of more than 64 rows take this route for every GEMM it supports, in batches of
  // 128 rows (one weight pass per batch), including the three-segment QKV when the packed copies are adjacent.
  if (x->panel && !direct && M <= x->row_batch_max) {
    const int bm = M > 64 ? x->row_batch : 64;
    bool adjacent = true;
    for (int s = 1; s < nseg; ++s) adjacent = adjacent && ws[s] == ws[s - 1] + (size_t)seg_n[s - 1] * K;
    const int kp = (nseg == 1 || (bm > 64 && adjacent)) ? panel_gemm_pick_k_parts(std::min(M, bm), N, K) : 0;
    if (kp > 1 && (size_t)kp * M * N * sizeof(float) <= x->partial_bytes) {
      for (int m0 = 0; m0 < M; m0 += bm) {
        PanelGemm g;
        memset(&g, 0, sizeof(g));
        g.Xhi = X.hi + (size_t)m0 * X.ld; g.Xlo = X.lo + (size_t)m0 * X.ld; g.ldx = X.ld;
        g.W[0] = g.W[1] = ws[0];
        g.Y = part + (size_t)m0 * N; g.ldy = N; g.k_parts = kp; g.split_stride = (size_t)M * N;
        g.M = std::min(bm, M - m0); g.N = N; g.K = K; g.epi = 0;
        g.rows128 = bm > 64;   // a short last batch keeps the form the ranges were picked for
        launch_gemm_panel(g, x->st);
      }
      return kp;
    }
  }
  // Up to 64 rows: the K-slice kernel.  65..256 rows: the same kernel over batches of 64 rows -- the weights are
  // streamed once per batch, which still beats the tiled kernel (each of its wavefronts multiplies ALL rows and is
  // bound by the LDS reads of the activations).
  if (M <= x->row_batch_max && stream_gemm_supported(std::min(M, 64), N, K) &&
      stream_gemm_out_bytes(M, N, K) <= x->partial_bytes) {
    for (int m0 = 0; m0 < M; m0 += 64) {
      StreamGemm g;
      memset(&g, 0, sizeof(g));
      g.Xhi = X.hi + (size_t)m0 * X.ld; g.Xlo = X.lo + (size_t)m0 * X.ld; g.ldx = X.ld;
      for (int s = 0; s < 3; ++s) { g.W[s] = ws[s]; g.seg_begin[s] = segb[s]; }
      g.seg_begin[3] = 0x7fffffff;
      g.Y = part + (size_t)m0 * N; g.ldy = N; g.split_stride = (size_t)M * N;
      g.M = std::min(64, M - m0); g.N = N; g.K = K;
      g.tag = cls == KC_GEMM_GATEUP ? 1 : 0;
      launch_gemm_stream(g, x->st);
    }
    const int sp = stream_gemm_slices(K);
    if (direct) launch_reduce(part, sp, (size_t)M * N, N, nullptr, x->cfg.dtype, direct, ld_direct, M, N, 0, x->st);
    return direct ? 1 : sp;
  }
  int splits = 1;
  if (!direct) {
    splits = mfma_gemm_pick_splits(std::min(M, 256), N, K, 0);
    while (splits > 1 && (size_t)splits * M * N * sizeof(float) > x->partial_bytes) splits /= 2;
  }
  for (int m0 = 0; m0 < M; m0 += 256) {
    const int mm = std::min(256, M - m0);
    MfmaGemm g;
    memset(&g, 0, sizeof(g));
    g.Xhi = X.hi + (size_t)m0 * X.ld; g.Xlo = X.lo + (size_t)m0 * X.ld; g.ldx = X.ld;
    for (int s = 0; s < 3; ++s) { g.W[s] = ws[s]; g.seg_begin[s] = segb[s]; }
    g.seg_begin[3] = 0x7fffffff;
    if (direct) { g.Y = direct + (size_t)m0 * ld_direct; g.ldy = ld_direct; g.split_stride = 0; }
    else { g.Y = x->partial + (size_t)m0 * N; g.ldy = N; g.split_stride = (size_t)M * N; }
    g.M = mm; g.N = N; g.K = K; g.mode = 0; g.splits = splits;
    launch_gemm_mfma(g, x->st);
  }
  return splits;
}
int gemm_fast1(clover_ctx* x, int cls, Planes X, const void* W, int M, int N, int K, float* direct = nullptr,
               int ld_direct = 0) {
  const void* ws[1] = {W};
  const int sn[1] = {N};
  return gemm_fast(x, cls, X, 1, ws, sn, M, N, K, direct, ld_direct);
}
// Y = X W^T + bias through the MFMA path, for the small draft-side linears
void linear_fast(clover_ctx* x, Planes X, const void* W, const void* bias, float* Y, int ldy, int M, int N, int K) {
  const int sp = gemm_fast1(x, KC_GEMM_DRAFT, X, W, M, N, K);
  Scope sc(x, KC_ELTWISE);
  launch_reduce(x->partial, sp, (size_t)M * N, N, bias, x->cfg.dtype, Y, ldy, M, N, 0, x->st);
}
Planes split_to(clover_ctx* x, const float* src, int ld, float* planes_buf, int rows, int K) {
  Planes P = planes_of(x, planes_buf, K);
  Scope sc(x, KC_ELTWISE);
  launch_split_planes(src, ld, P.hi, P.lo, K, rows, K, x->st);
  return P;
}

// generic path: Y = X W^T (+bias), mode 1 adds into Y
void gemm_generic(clover_ctx* x, int cls, const float* X, int ldx, const void* W, const void* bias, float* Y, int ldy,
                  int M, int N, int K, int mode) {
  Scope sc(x, cls);
  launch_gemm_generic(X, ldx, W, bias, x->cfg.dtype, Y, ldy, M, N, K, mode, x->st);
}

// One LLaMA decoder layer over the rows of `rm` (residual stream xres, leading dimension H).
// MFMA path: on entry the planes of a_norm hold RMSNorm(xres) * attn_norm of this layer; on exit they
// hold RMSNorm(xres) * next_gain (skipped when next_gain is null).  Generic path: norms are computed here.
void run_layer(clover_ctx* x, const clover_layer_weights& lw, float* xres, RowMap rm, int M, char* kc_layer,
               char* vc_layer, const int* base_len, const unsigned long long* anc, const void* next_gain,
               int key_bound, int anc_stride = 0 /* nodes per sequence in a per-sequence mask table */,
               const int* iv = nullptr /* interval labels: decide visibility instead of anc */,
               int seq0 = 0 /* the rows belong to sequence seq0 + (their index in rm) */) {
  const clover_config& c = x->cfg;
  KVLayout kvl = x->kv;
  kvl.b0 = seq0;
  const int H = x->H, d = c.head_dim, F = c.ffn;
  const int sn[3] = {c.n_q_heads * d, c.n_kv_heads * d, c.n_kv_heads * d};
  const void* ws[3] = {lw.wq, lw.wk, lw.wv};
  if (x->fast) {
    Planes A = planes_of(x, x->a_norm, 2 * H);
    A.ld = H;
    Planes O = planes_of(x, x->attn_out, x->NQD);
    Planes Hf = planes_of(x, x->h_ffn, F);
    const int sq = gemm_fast(x, KC_GEMM_QKV, A, 3, ws, sn, M, x->QKVN, H, nullptr, 0);
    { Scope s(x, KC_ROPE_KV);
      Planes Q = planes_of(x, x->q_rot, x->NQD);
      launch_rope_kv_write(x->partial, x->QKVN, sq, (size_t)M * x->QKVN, x->cos_t, x->sin_t, x->q_rot, x->NQD, kc_layer,
                           vc_layer, x->kvdtype, kvl, base_len, c.n_q_heads, rm, x->d_err,
                           x->attn_fast ? Q.hi : nullptr, Q.lo, 1.0f / sqrtf((float)d), x->st); }
    { Scope s(x, KC_ATTN);
      if (x->attn_fast) {
        AttnParams ap;
        memset(&ap, 0, sizeof(ap));
        Planes Q = planes_of(x, x->q_rot, x->NQD);
        ap.q_hi = Q.hi; ap.q_lo = Q.lo; ap.ldq = x->NQD;
        ap.k_hi = (const bf16_t*)kc_layer; ap.k_plane = x->k_layer_elems;
        ap.v_hi = (const bf16_t*)vc_layer; ap.v_plane = x->v_layer_elems;
        ap.kv = kvl; ap.max_seq = c.max_seq; ap.n_kv = c.n_kv_heads; ap.n_q = c.n_q_heads;
        ap.base_len = base_len; ap.anc = anc; ap.iv = iv; ap.anc_stride = anc_stride; ap.rm = rm;
        ap.o_part = x->o_part; ap.ml_part = x->ml_part; ap.rows_total = x->max_rows; ap.max_splits = x->attn_max_splits;
        launch_attn_mfma(ap, key_bound, O.hi, O.lo, x->NQD, x->st);
      } else {
        launch_attn_generic(x->q_rot, x->NQD, kc_layer, vc_layer, x->kvdtype, kvl, base_len, anc, c.n_q_heads, nullptr,
                            x->NQD, O.hi, O.lo, rm, x->st, anc_stride, iv);
      } }
    const int sw = gemm_fast1(x, KC_GEMM_WO, O, lw.wo, M, H, x->NQD);
    { Scope s(x, KC_RMSNORM);
      launch_reduce_add_norm(xres, H, x->partial, sw, (size_t)M * H, H, lw.ffn_norm, c.dtype, c.rms_eps, A.hi, A.lo, H, M,
                             H, x->st); }
    if (M >= x->tile_min && M <= 256 && tile_gemm_supported(M, F, H, 1)) {
      Scope s(x, KC_GEMM_GATEUP);
      TileGemm g;
      memset(&g, 0, sizeof(g));
      g.Xhi = A.hi; g.Xlo = A.lo; g.ldx = H;
      g.W[0] = (const bf16_t*)lw.w_gate; g.W[1] = (const bf16_t*)lw.w_up;
      g.Yhi = Hf.hi; g.Ylo = Hf.lo; g.ldo = F;
      g.M = M; g.N = F; g.K = H; g.epi = 1; g.k_parts = 1;
      launch_gemm_tile(g, x->st);
    } else if (x->panel && M <= x->row_batch_max && panel_gemm_supported(std::min(M, 64), F, H, 1)) {
      Scope s(x, KC_GEMM_GATEUP);
      const int bm = (M > 64 && panel_gemm_supported(std::min(M, x->row_batch), F, H, 1)) ? x->row_batch : 64;
      for (int m0 = 0; m0 < M; m0 += bm) {  // (more than 64 rows: one weight pass per batch, see gemm_fast)
        PanelGemm g;
        memset(&g, 0, sizeof(g));
        g.Xhi = A.hi + (size_t)m0 * H; g.Xlo = A.lo + (size_t)m0 * H; g.ldx = H;
        g.W[0] = (const bf16_t*)lw.w_gate; g.W[1] = (const bf16_t*)lw.w_up;
        g.Yhi = Hf.hi + (size_t)m0 * F; g.Ylo = Hf.lo + (size_t)m0 * F; g.ldo = F;
        g.M = std::min(bm, M - m0); g.N = F; g.K = H; g.epi = 1;
        launch_gemm_panel(g, x->st);
      }
    } else if (M <= 64 && stream_gemm_supported(M, 2 * F, H) && stream_gemm_out_bytes(M, 2 * F, H) <= x->partial_bytes) {
      const void* wgu[2] = {lw.w_gate, lw.w_up};
      const int gun[2] = {F, F};
      const int sg = gemm_fast(x, KC_GEMM_GATEUP, A, 2, wgu, gun, M, 2 * F, H, nullptr, 0);
      Scope s(x, KC_ELTWISE);
      launch_reduce_swiglu(x->partial, sg, (size_t)M * 2 * F, 2 * F, F, Hf.hi, Hf.lo, F, M, x->st);
    } else {
      Scope s(x, KC_GEMM_GATEUP);
      for (int m0 = 0; m0 < M; m0 += 256) {
        MfmaGemm g;
        memset(&g, 0, sizeof(g));
        g.Xhi = A.hi + (size_t)m0 * H; g.Xlo = A.lo + (size_t)m0 * H; g.ldx = H;
        g.W[0] = g.W[1] = g.W[2] = (const bf16_t*)lw.w_gate;
        g.W_up = (const bf16_t*)lw.w_up;
        g.seg_begin[1] = g.seg_begin[2] = g.seg_begin[3] = 0x7fffffff;
        g.Yhi = Hf.hi + (size_t)m0 * F; g.Ylo = Hf.lo + (size_t)m0 * F; g.ldy = F;
        g.M = std::min(256, M - m0); g.N = F; g.K = H; g.mode = 2; g.splits = 1;
        launch_gemm_mfma(g, x->st);
      }
    }
    const int sd = gemm_fast1(x, KC_GEMM_DOWN, Hf, lw.w_down, M, H, F);
    { Scope s(x, KC_RMSNORM);
      launch_reduce_add_norm(xres, H, x->partial, sd, (size_t)M * H, H, next_gain, c.dtype, c.rms_eps, A.hi, A.lo, H, M,
                             H, x->st); }
    return;
  }
  { Scope s(x, KC_RMSNORM); launch_rmsnorm(xres, H, lw.attn_norm, c.dtype, c.rms_eps, x->a_norm, H, H, M, x->st); }
  { int off = 0;
    for (int sgm = 0; sgm < 3; ++sgm) {
      gemm_generic(x, KC_GEMM_QKV, x->a_norm, H, ws[sgm], nullptr, x->qkv + off, x->QKVN, M, sn[sgm], H, 0);
      off += sn[sgm];
    } }
  { Scope s(x, KC_ROPE_KV);
    launch_rope_kv_write(x->qkv, x->QKVN, 1, 0, x->cos_t, x->sin_t, x->q_rot, x->NQD, kc_layer, vc_layer, x->kvdtype,
                         kvl, base_len, c.n_q_heads, rm, x->d_err, nullptr, nullptr, 0.f, x->st); }
  { Scope s(x, KC_ATTN);
    launch_attn_generic(x->q_rot, x->NQD, kc_layer, vc_layer, x->kvdtype, kvl, base_len, anc, c.n_q_heads, x->attn_out,
                        x->NQD, nullptr, nullptr, rm, x->st, anc_stride, iv); }
  gemm_generic(x, KC_GEMM_WO, x->attn_out, x->NQD, lw.wo, nullptr, xres, H, M, H, x->NQD, 1);
  { Scope s(x, KC_RMSNORM); launch_rmsnorm(xres, H, lw.ffn_norm, c.dtype, c.rms_eps, x->a_norm, H, H, M, x->st); }
  gemm_generic(x, KC_GEMM_GATEUP, x->a_norm, H, lw.w_gate, nullptr, x->tmp_ffn, F, M, F, H, 0);
  gemm_generic(x, KC_GEMM_GATEUP, x->a_norm, H, lw.w_up, nullptr, x->h_ffn, F, M, F, H, 0);
  { Scope s(x, KC_ELTWISE); launch_swiglu(x->tmp_ffn, x->h_ffn, x->h_ffn, (size_t)M * F, x->st); }
  gemm_generic(x, KC_GEMM_DOWN, x->h_ffn, F, lw.w_down, nullptr, xres, H, M, H, F, 1);
}


// planes of RMSNorm(src) * gain in the a_norm buffer (MFMA path)
Planes norm_planes(clover_ctx* x, const float* src, const void* gain, int rows) {
  const clover_config& c = x->cfg;
  Planes A = planes_of(x, x->a_norm, 2 * x->H);
  A.ld = x->H;
  Scope s(x, KC_RMSNORM);
  launch_reduce_add_norm(const_cast<float*>(src), x->H, nullptr, 0, 0, 0, gain, c.dtype, c.rms_eps, A.hi, A.lo, x->H, rows,
                         x->H, x->st);
  return A;
}

// Attention Decoder on `rows` contiguous rows: out = x + gate(q(norm(x)), k(y)) * v(y)
void run_ad(clover_ctx* x, const clover_ad_weights& ad, const float* xin, const float* y, int rows, float* out) {
  const clover_config& c = x->cfg;
  const int H = x->H;
  if (x->fast) {
    Planes A = norm_planes(x, xin, ad.norm, rows);
    linear_fast(x, A, ad.wq, ad.bq, x->ad_q, H, rows, H, H);
    Planes Y = split_to(x, y, H, x->pl_y, rows, H);
    linear_fast(x, Y, ad.wk, ad.bk, x->ad_k, H, rows, H, H);
    linear_fast(x, Y, ad.wv, ad.bv, x->ad_v, H, rows, H, H);
  } else {
    { Scope s(x, KC_RMSNORM); launch_rmsnorm(xin, H, ad.norm, c.dtype, c.rms_eps, x->a_norm, H, H, rows, x->st); }
    gemm_generic(x, KC_GEMM_DRAFT, x->a_norm, H, ad.wq, ad.bq, x->ad_q, H, rows, H, H, 0);
    gemm_generic(x, KC_GEMM_DRAFT, y, H, ad.wk, ad.bk, x->ad_k, H, rows, H, H, 0);
    gemm_generic(x, KC_GEMM_DRAFT, y, H, ad.wv, ad.bv, x->ad_v, H, rows, H, H, 0);
  }
  { Scope s(x, KC_AD_GATE);
    launch_ad_gate(xin, H, x->ad_q, x->ad_k, x->ad_v, H, c.ad_heads, out, H, nullptr, 0, rows, x->st); }
}

// Y = X W^T + bias for a draft-side FC with fp32 input X [rows, K]
void run_fc(clover_ctx* x, const float* X, int K, const void* W, const void* bias, float* Y, int rows) {
  const int H = x->H;
  if (x->fast) {
    Planes P = split_to(x, X, K, x->pl_y, rows, K);
    linear_fast(x, P, W, bias, Y, H, rows, H, K);
  } else {
    gemm_generic(x, KC_GEMM_DRAFT, X, K, W, bias, Y, H, rows, H, K, 0);
  }
}

// out[rows, vocab] = A * lm_head^T (MFMA path)
void lm_head_fast(clover_ctx* x, Planes A, int rows, float* out) {
  const clover_config& c = x->cfg;
  if (rows >= x->tile_min && rows <= 256 && tile_gemm_supported(rows, c.vocab, x->H, 0)) {
    Scope s(x, KC_GEMM_LMHEAD);
    TileGemm g;
    memset(&g, 0, sizeof(g));
    g.Xhi = A.hi; g.Xlo = A.lo; g.ldx = A.ld;
    g.W[0] = g.W[1] = (const bf16_t*)x->lm_head_pk;
    g.Y = out; g.ldy = c.vocab; g.M = rows; g.N = c.vocab; g.K = x->H; g.epi = 0; g.k_parts = 1;
    launch_gemm_tile(g, x->st);
    return;
  }
  if (x->panel && rows <= x->row_batch_max && panel_gemm_supported(std::min(rows, 64), c.vocab, x->H, 0)) {
    Scope s(x, KC_GEMM_LMHEAD);
    const int bm = (rows > 64 && panel_gemm_supported(std::min(rows, x->row_batch), c.vocab, x->H, 0)) ? x->row_batch : 64;
    for (int m0 = 0; m0 < rows; m0 += bm) {  // (more than 64 rows: one weight pass per batch, see gemm_fast)
      PanelGemm g;
      memset(&g, 0, sizeof(g));
      g.Xhi = A.hi + (size_t)m0 * A.ld; g.Xlo = A.lo + (size_t)m0 * A.ld; g.ldx = A.ld;
      g.W[0] = g.W[1] = (const bf16_t*)x->lm_head_pk;
      g.Y = out + (size_t)m0 * c.vocab; g.ldy = c.vocab;
      g.M = std::min(bm, rows - m0); g.N = c.vocab; g.K = x->H; g.epi = 0;
      launch_gemm_panel(g, x->st);
    }
    return;
  }
  gemm_fast1(x, KC_GEMM_LMHEAD, A, x->lm_head_pk, rows, c.vocab, x->H, out, c.vocab);
}

// logits of `rows` contiguous rows of g through the head norm and the shared LM head, then top-k
void run_head(clover_ctx* x, const float* g, int rows, int k /* 0: logits only, left in x->z */) {
  const clover_config& c = x->cfg;
  const int H = x->H;
  if (x->fast) {
    Planes A = norm_planes(x, g, x->w.head_norm, rows);
    lm_head_fast(x, A, rows, x->z);
  } else {
    { Scope s(x, KC_RMSNORM); launch_rmsnorm(g, H, x->w.head_norm, c.dtype, c.rms_eps, x->a_norm, H, H, rows, x->st); }
    gemm_generic(x, KC_GEMM_LMHEAD, x->a_norm, H, x->w.lm_head, nullptr, x->z, c.vocab, rows, c.vocab, H, 0);
  }
  if (k > 0) { Scope s(x, KC_TOPK); launch_topk(x->z, c.vocab, c.vocab, rows, k, x->cand, x->topk_ids, x->st); }
}

// Can draft_tree take the fused route for `rows` GEMM rows?  (K-slice GEMMs for every draft linear, at most 8 slices
// for the Attention Decoder's projections, room for the q and the k|v partials side by side.)
bool draft_fused_ok(clover_ctx* x, int rows) {
  const int H = x->H;
  if (!x->fast || rows < 1 || rows > 64 || tune_int("CLOVER_DRAFT_UNFUSED", 0)) return false;
  if (!ad_gate_fused_supported(H, x->cfg.ad_heads)) return false;
  if (!stream_gemm_supported(rows, H, H) || !stream_gemm_supported(rows, 2 * H, H) || !stream_gemm_supported(rows, H, 2 * H) ||
      !stream_gemm_supported(rows, x->cfg.vocab, H))
    return false;
  const int sH = stream_gemm_slices(H);
  if (sH > 8) return false;
  const size_t need = std::max((size_t)sH * rows * 3 * H, std::max((size_t)stream_gemm_slices(2 * H) * rows * H,
                                                                    (size_t)sH * rows * x->cfg.vocab)) * sizeof(float);
  return need <= x->partial_bytes;
}

// Attention Decoder on the fused route: planes A = RMSNorm(x)*norm (rows, ld H), Y = y (rows, ld H) are in place;
// q and k|v projections leave their K-slice partials side by side, the gate kernel does the rest.
void run_ad_fused(clover_ctx* x, const clover_ad_weights& ad, Planes A, Planes Y, int rows, AdGateArgs g) {
  const int H = x->H, sH = stream_gemm_slices(H);
  float* Pq = x->partial;
  float* Pkv = x->partial + (size_t)sH * rows * H;
  gemm_fast1(x, KC_GEMM_DRAFT, A, ad.wq, rows, H, H, nullptr, 0);
  const void* wkv[2] = {ad.wk, ad.wv};
  const int nkv[2] = {H, H};
  gemm_fast(x, KC_GEMM_DRAFT, Y, 2, wkv, nkv, rows, 2 * H, H, nullptr, 0, Pkv);
  g.Pq = Pq; g.Sq = sH; g.sps_q = (size_t)rows * H;
  g.Pkv = Pkv; g.Skv = sH; g.sps_kv = (size_t)rows * 2 * H;
  g.bq = ad.bq; g.bk = ad.bk; g.bv = ad.bv;
  g.H = H; g.heads = x->cfg.ad_heads; g.eps = x->cfg.rms_eps;
  Scope sc(x, KC_AD_GATE);
  launch_ad_gate_fused(g, rows, x->st);
}

// test hook: copy the logits of the depth-j internal nodes (rows x vocab in x->z) behind those of the shallower depths
void capture_draft_logits(clover_ctx* x, int j, int rows) {
  if (!x->draft_capture) return;
  const size_t V = (size_t)x->cfg.vocab;
  size_t off;
  if (x->dyn_on) {   // rows of depth j start behind the rows of the shallower depths: batch * (F[0] + .. + F[j-1]) rows
    int before = 0;
    for (int i = 0; i < j; ++i) before += x->dyn.F[i];
    off = (size_t)(rows / std::max(1, x->dyn.F[j])) * before * V;
  } else {
    off = (size_t)(rows / std::max(1, x->tree.lvl_off[j + 1] - x->tree.lvl_off[j])) * x->tree.lvl_off[j] * V;
  }
  if (off + (size_t)rows * V > x->draft_capture_floats) return;
  hipMemcpyAsync(x->draft_capture + off, x->z, (size_t)rows * V * sizeof(float), hipMemcpyDeviceToDevice, x->st);
}

// Dynamic tree: expansion depth by depth (the root state and token are in candidate 0), then the selection.
// Depth j expands F[j] candidates per sequence; their logits go through a log-softmax so that scores add up
// along a path.
void draft_expand_dynamic(clover_ctx* x, int B, const int* m, int* tree_tokens, bool fused, Planes A, Planes Y, Planes Cc) {
  const clover_config& c = x->cfg;
  const DynTree& t = x->dyn;
  const int H = x->H, C = t.C, ns = CLOVER_MAX_DEPTH * DYN_MAX_FRONT;
  for (int j = 0; j < t.D; ++j) {
    const int n_lvl = t.F[j], rows = B * n_lvl;
    const int* nodes = t.frontier + (size_t)j * DYN_MAX_FRONT;
    if (fused) {
      int sp;
      if (j == 0) {
        sp = gemm_fast1(x, KC_GEMM_DRAFT, Y, x->w.fc0_w, rows, H, H);
      } else {
        { Scope s(x, KC_DRAFT_MISC);
          launch_draft_level(x->dyn_state, t.cand_tok, nodes, t.cand_par, n_lvl, B, C, H, x->w.lm_head, c.vocab,
                             x->w.ad2.norm, c.rms_eps, A.hi, A.lo, Y.hi, Y.lo, Cc.hi, Cc.lo, x->st, ns, C); }
        AdGateArgs g;
        memset(&g, 0, sizeof(g));
        g.x = x->dyn_state; g.ldx = H; g.out = x->dyn_state; g.ldo = H;
        g.nodes = nodes; g.parent = t.cand_par; g.n_lvl = n_lvl; g.R = C; g.m = m;
        g.nodes_stride = ns; g.parent_stride = C;
        g.c_hi = Cc.hi; g.c_lo = Cc.lo; g.ldc = 2 * H;
        run_ad_fused(x, x->w.ad2, A, Y, rows, g);
        Planes C2 = Cc;
        C2.ld = 2 * H;
        sp = gemm_fast1(x, KC_GEMM_DRAFT, C2, x->fc_w[j], rows, H, 2 * H);
      }
      { Scope s(x, KC_RMSNORM);
        launch_reduce_add_norm(x->d_g, H, x->partial, sp, (size_t)rows * H, H, x->w.head_norm, c.dtype, c.rms_eps, A.hi,
                               A.lo, H, rows, H, x->st, j == 0 ? x->w.fc0_b : x->fc_b[j]); }
      lm_head_fast(x, A, rows, x->z);
    } else {
      if (j == 0) {
        run_fc(x, x->d_rootx, H, x->w.fc0_w, x->w.fc0_b, x->d_g, rows);
      } else {
        { Scope s(x, KC_DRAFT_MISC);
          launch_draft_gather(x->dyn_state, t.cand_tok, nodes, t.cand_par, n_lvl, B, C, H, x->w.lm_head, c.dtype, c.vocab,
                              x->d_xs, x->d_e, x->d_cat, x->st, ns, C); }
        run_ad(x, x->w.ad2, x->d_xs, x->d_e, rows, x->d_s);
        { Scope s(x, KC_DRAFT_MISC);
          launch_draft_scatter_state(x->d_s, nodes, n_lvl, B, C, H, x->dyn_state, x->d_cat, x->st, ns); }
        run_fc(x, x->d_cat, 2 * H, x->fc_w[j], x->fc_b[j], x->d_g, rows);
      }
      run_head(x, x->d_g, rows, 0);
    }
    capture_draft_logits(x, j, rows);
    { Scope s(x, KC_TOPK);
      launch_topk_lse(x->z, c.vocab, c.vocab, rows, t.topk, x->cand, x->topk_aux, x->topk_ids, x->topk_vals, x->topk_lse, x->st); }
    { Scope s(x, KC_DRAFT_MISC);
      launch_dyn_assign(t, j, B, x->topk_ids, x->topk_vals, x->topk_lse, m, x->st);
      if (j + 1 < t.D) launch_dyn_frontier(t, j + 1, B, m, x->st); }
  }
  { Scope s(x, KC_DRAFT_MISC); launch_dyn_finalize(t, B, x->R, m, tree_tokens, x->st); }
}

int upload_tree(clover_ctx* x) {
  const TreeHost& t = x->tree;
  const int n = t.n;
  hipError_t e = hipSuccess;
  auto up = [&](void* dst, const void* src, size_t bytes) {
    if (bytes && e == hipSuccess) e = hipMemcpyAsync(dst, src, bytes, hipMemcpyHostToDevice, x->st);
  };
  up(x->d_depth, t.depth.data(), n * sizeof(int));
  up(x->d_parent, t.parent.data(), n * sizeof(int));
  up(x->d_rank, t.rank.data(), n * sizeof(int));
  up(x->d_first_child, t.first_child.data(), n * sizeof(int));
  up(x->d_n_child, t.n_child.data(), n * sizeof(int));
  up(x->d_lvl_nodes, t.lvl_nodes.data(), t.lvl_nodes.size() * sizeof(int));
  up(x->d_par_row, t.par_row.data(), n * sizeof(int));
  up(x->d_anc, t.anc.data(), 2 * n * sizeof(unsigned long long));
  up(x->d_iv, t.iv.data(), 2 * n * sizeof(int));
  if (e == hipSuccess) e = hipStreamSynchronize(x->st);  // the host vectors may change after return
  if (e != hipSuccess) return fail(x, CLOVER_E_HIP, std::string("tree upload: ") + hipGetErrorString(e));
  return CLOVER_OK;
}

int finish(clover_ctx* x, const char* what) {
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(x, CLOVER_E_HIP, std::string(what) + ": " + hipGetErrorString(e));
  return CLOVER_OK;
}

int check_batch(clover_ctx* x, int batch) {
  if (batch < 1 || batch > x->cfg.max_batch) return fail(x, CLOVER_E_SHAPE, "batch outside [1, max_batch]");
  return CLOVER_OK;
}

int accept_common(clover_ctx* x, int batch, const int* tree_tokens, const float* logits, const float* hidden,
                  const int* n_forced, const int* forced_next, int* m, int* acc_idx, int* new_tokens, float* hid_acc,
                  int* next_tok, float temperature = 0.f, const float* uniforms = nullptr) {
  const clover_config& c = x->cfg;
  const TreeHost& t = x->tree;
  const int n_nodes = x->dyn_on ? x->dyn.N : t.n;
  const int R = x->R, M = (batch - 1) * R + n_nodes;
  x->only_prefills = false;
  const int* fc_tab = x->dyn_on ? x->dyn.t_first_child : x->d_first_child;
  const int* nc_tab = x->dyn_on ? x->dyn.t_n_child : x->d_n_child;
  if (uniforms) {
    // temperature > 0: per-row log-sum-exp of logits / T, then the sampled walk
    const float inv_t = 1.0f / temperature;
    { Scope s(x, KC_TOPK);
      launch_topk_lse(logits, c.vocab, c.vocab, M, 1, x->cand, x->topk_aux, x->topk_ids, x->topk_vals, x->topk_lse, x->st, inv_t); }
    { Scope s(x, KC_ACCEPT);
      launch_accept_sample(logits, c.vocab, x->topk_lse, inv_t, tree_tokens, fc_tab, nc_tab, x->dyn_on ? R : 0, batch, R,
                           uniforms, m, acc_idx, new_tokens, next_tok, x->st); }
  } else {
  { Scope s(x, KC_TOPK); launch_topk(logits, c.vocab, c.vocab, M, 1, x->cand, x->topk_ids, x->st); }
  { Scope s(x, KC_ACCEPT);
    launch_accept_walk(x->topk_ids, tree_tokens, x->dyn_on ? x->dyn.t_first_child : x->d_first_child,
                       x->dyn_on ? x->dyn.t_n_child : x->d_n_child, n_nodes, batch, R, n_forced, forced_next,
                       m, acc_idx, new_tokens, next_tok, x->st, x->dyn_on ? R : 0); }
  }
  { Scope s(x, KC_COMPACT);
    launch_compact_kv(x->kc, x->vc, x->kvdtype, x->kv, c.n_layers, x->kv_layer_stride, x->kv_layer_stride, x->d_seq_len, m,
                      acc_idx, batch, R, x->st);
    launch_gather_hidden(hidden, acc_idx, m, batch, R, x->H, hid_acc, x->st);
    launch_add_len(x->d_seq_len, m, batch, x->st); }
  return finish(x, "accept");
}

int static_scratch_ptr(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) { g_err = std::string("hipGetDevice: ") + hipGetErrorString(e); return CLOVER_E_HIP; }
  if (dev < 0 || dev >= kMaxDevices) { g_err = "device index beyond the static scratch table"; return CLOVER_E_SHAPE; }
  if (!g_static_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(g_static_scratch));
    if (e != hipSuccess || !p) {
      g_err = std::string("hipGetSymbolAddress(static scratch): ") + hipGetErrorString(e);
      return CLOVER_E_HIP;
    }
    g_static_scratch_ptr[dev] = p;
  }
  *out = g_static_scratch_ptr[dev];
  return CLOVER_OK;
}

}  // namespace

// ================================================================================================
extern "C" {

int clover_workspace_bytes(const clover_config* cfg, size_t* bytes_out) {
  if (!cfg || !bytes_out) return fail(nullptr, CLOVER_E_NULL, "null argument");
  std::string why;
  const int rc = check_config(cfg, why);
  if (rc) return fail(nullptr, rc, why);
  clover_ctx tmp{};
  tmp.cfg = *cfg;
  size_t total = 0;
  carve(&tmp, nullptr, &total);
  *bytes_out = total;
  return CLOVER_OK;
}

int clover_init(const clover_config* cfg, const clover_weights* w, const clover_tree* tree, void* workspace,
                size_t workspace_bytes, void* hip_stream, clover_ctx** ctx_out) {
  if (!cfg || !w || !tree || !workspace || !ctx_out) return fail(nullptr, CLOVER_E_NULL, "null argument");
  std::string why;
  int rc = check_config(cfg, why);
  if (rc) return fail(nullptr, rc, why);
  if (((uintptr_t)workspace & 255) != 0) return fail(nullptr, CLOVER_E_CONFIG, "workspace must be 256-byte aligned");
  if (!w->embed || !w->layers || !w->final_norm || !w->lm_head || !w->aug || !w->fc0_w || !w->fc0_b || !w->fc_w ||
      !w->fc_b || !w->head_norm)
    return fail(nullptr, CLOVER_E_NULL, "null weight pointer");
  const clover_ad_weights* ads[2] = {&w->ad1, &w->ad2};
  for (const clover_ad_weights* a : ads)
    if (!a->norm || !a->wq || !a->bq || !a->wk || !a->bk || !a->wv || !a->bv) return fail(nullptr, CLOVER_E_NULL, "null Attention-Decoder weight");
  auto layer_ok = [](const clover_layer_weights& l) {
    return l.attn_norm && l.wq && l.wk && l.wv && l.wo && l.ffn_norm && l.w_gate && l.w_up && l.w_down;
  };
  for (int i = 0; i < cfg->n_layers; ++i) if (!layer_ok(w->layers[i])) return fail(nullptr, CLOVER_E_NULL, "null target layer weight");
  for (int i = 0; i < cfg->aug_layers; ++i) if (!layer_ok(w->aug[i])) return fail(nullptr, CLOVER_E_NULL, "null augmenting layer weight");
  for (int j = 1; j < cfg->draft_depths; ++j) if (!w->fc_w[j] || !w->fc_b[j]) return fail(nullptr, CLOVER_E_NULL, "null FC weight");
  TreeHost th;
  rc = build_tree(*cfg, tree, th, why);
  if (rc) return fail(nullptr, rc, why);

  clover_ctx* x = new clover_ctx{};
  x->cfg = *cfg;
  x->st = (hipStream_t)hip_stream;
  x->w = *w;
  x->layers.assign(w->layers, w->layers + cfg->n_layers);
  x->aug.assign(w->aug, w->aug + cfg->aug_layers);
  x->fc_w.assign(w->fc_w, w->fc_w + cfg->draft_depths);
  x->fc_b.assign(w->fc_b, w->fc_b + cfg->draft_depths);
  x->tree = std::move(th);
  size_t total = 0;
  carve(x, (char*)workspace, &total);
  if (total > workspace_bytes) { delete x; return fail(nullptr, CLOVER_E_CAPACITY, "workspace too small"); }
  x->len_ub.assign(cfg->max_batch, 0);
  x->aug_ub.assign(cfg->max_batch, 0);
  x->m_upper = cfg->max_nodes;
  x->only_prefills = true;
  x->interval = (cfg->flags & CLOVER_FLAG_INTERVAL_MASK) != 0;
  launch_fill_i32(x->d_seq_len, 0, cfg->max_batch, x->st);
  launch_fill_i32(x->d_aug_len, 0, cfg->max_batch, x->st);
  launch_fill_i32(x->d_err, 0, 1, x->st);
  if (x->fast) {
    // the MFMA attention multiplies masked probabilities (exact zeros) with whatever the cache rows of a
    // tile hold, so the caches must never contain non-finite garbage
    hipMemsetAsync(x->kc, 0, x->k_layer_elems * x->kv_esz * cfg->n_layers, x->st);
    hipMemsetAsync(x->vc, 0, x->v_layer_elems * x->kv_esz * cfg->n_layers, x->st);
    hipMemsetAsync(x->aug_kc, 0, x->k_layer_elems * x->kv_esz * cfg->aug_layers, x->st);
    hipMemsetAsync(x->aug_vc, 0, x->v_layer_elems * x->kv_esz * cfg->aug_layers, x->st);
    // private fragment-major copies of every linear weight; the originals are only read here
    // (and, for the LM head, by the draft's embedding gathers)
    char* cur = x->packed;
    auto pack = [&](const void*& w, int N, int K) {
      launch_pack_weight(w, cur, N, K, x->st);
      w = cur;
      cur += (size_t)N * K * 2;
    };
    const int H = x->H, d = cfg->head_dim, F = cfg->ffn;
    auto pack_layer = [&](clover_layer_weights& l) {
      pack(l.wq, cfg->n_q_heads * d, H); pack(l.wk, cfg->n_kv_heads * d, H); pack(l.wv, cfg->n_kv_heads * d, H);
      pack(l.wo, H, x->NQD); pack(l.w_gate, F, H); pack(l.w_up, F, H); pack(l.w_down, H, F);
    };
    for (auto& l : x->layers) pack_layer(l);
    for (auto& l : x->aug) pack_layer(l);
    x->lm_head_pk = x->w.lm_head;
    pack(x->lm_head_pk, cfg->vocab, H);
    for (clover_ad_weights* a : {&x->w.ad1, &x->w.ad2}) { pack(a->wq, H, H); pack(a->wk, H, H); pack(a->wv, H, H); }
    pack(x->w.fc0_w, H, H);
    for (int j = 1; j < cfg->draft_depths; ++j) pack(x->fc_w[j], H, 2 * H);
    if ((size_t)(cur - x->packed) > x->packed_bytes) { delete x; return fail(nullptr, CLOVER_E_CAPACITY, "internal: packed weights overflow"); }
  }
  rc = upload_tree(x);
  if (rc == CLOVER_OK) rc = finish(x, "init");
  if (rc) { g_err = x->err; delete x; return rc; }
  *ctx_out = x;
  return CLOVER_OK;
}

int clover_destroy(clover_ctx* x) {
  if (!x) return CLOVER_E_NULL;
  hipStreamSynchronize(x->st);
  for (ProfEvent& ev : x->prof_events) { hipEventDestroy(ev.a); hipEventDestroy(ev.b); }
  for (ProfEvent& ev : x->prof_pool) { hipEventDestroy(ev.a); hipEventDestroy(ev.b); }
  delete x;
  return CLOVER_OK;
}

int clover_reset(clover_ctx* x) {
  if (!x) return CLOVER_E_NULL;
  launch_fill_i32(x->d_seq_len, 0, x->cfg.max_batch, x->st);
  launch_fill_i32(x->d_aug_len, 0, x->cfg.max_batch, x->st);
  launch_fill_i32(x->d_err, 0, 1, x->st);
  std::fill(x->len_ub.begin(), x->len_ub.end(), 0);
  std::fill(x->aug_ub.begin(), x->aug_ub.end(), 0);
  x->m_upper = x->cfg.max_nodes;
  x->only_prefills = true;
  return finish(x, "reset");
}

int clover_set_tree(clover_ctx* x, const clover_tree* tree) {
  if (!x || !tree) return fail(x, CLOVER_E_NULL, "null argument");
  TreeHost th;
  std::string why;
  const int rc = build_tree(x->cfg, tree, th, why);
  if (rc) return fail(x, rc, why);
  hipError_t e = hipStreamSynchronize(x->st);  // kernels in flight still read the old tables
  if (e != hipSuccess) return fail(x, CLOVER_E_HIP, hipGetErrorString(e));
  x->tree = std::move(th);
  x->dyn_on = false;
  return upload_tree(x);
}

int clover_set_dynamic_tree(clover_ctx* x, int32_t n_nodes, int32_t topk, int32_t frontier) {
  if (!x) return CLOVER_E_NULL;
  const clover_config& c = x->cfg;
  if (n_nodes < 1 || n_nodes > c.max_nodes) return fail(x, CLOVER_E_TREE, "n_nodes outside [1, max_nodes]");
  if (n_nodes > CLOVER_MAX_NODES) return fail(x, CLOVER_E_TREE, "a dynamic tree has at most 128 nodes");
  if (topk < 1 || topk > CLOVER_MAX_RANK) return fail(x, CLOVER_E_TREE, "topk outside [1, 16]");
  if (frontier < 1 || frontier > DYN_MAX_FRONT || frontier > c.max_nodes)
    return fail(x, CLOVER_E_TREE, "frontier outside [1, min(64, max_nodes)]");
  DynTree t = x->dyn;   // keeps the workspace pointers
  t.D = c.draft_depths; t.topk = topk; t.N = n_nodes;
  t.off[0] = 0; t.off[1] = 1; t.F[0] = 1;
  int n_cand = topk;                               // candidates of depth 1
  for (int j = 1; j <= t.D; ++j) {
    t.off[j + 1] = t.off[j] + n_cand;
    if (n_cand > DYN_MAX_CAND) return fail(x, CLOVER_E_TREE, "more than 256 candidates in one depth");
    t.F[j] = std::min(frontier, n_cand);
    n_cand = t.F[j] * topk;
  }
  t.C = t.off[t.D + 1];
  if (t.C > DYN_MAX_CAND) return fail(x, CLOVER_E_TREE, "more than 256 candidates: lower topk, frontier or draft_depths");
  if (t.C < n_nodes) return fail(x, CLOVER_E_TREE, "fewer candidates than tree nodes");
  hipError_t e = hipStreamSynchronize(x->st);  // kernels in flight still read the old tables
  if (e != hipSuccess) return fail(x, CLOVER_E_HIP, hipGetErrorString(e));
  x->dyn = t;
  x->dyn_on = true;
  return CLOVER_OK;
}

int clover_read_dynamic_tree(clover_ctx* x, int32_t b, int32_t* parent_out, int32_t* rank_out, int32_t* keep_out,
                             int32_t* cand_token_out, float* cand_score_out, int32_t* cand_parent_out,
                             int32_t* frontier_out) {
  if (!x || !parent_out || !rank_out || !keep_out || !cand_token_out || !cand_score_out || !cand_parent_out || !frontier_out)
    return fail(x, CLOVER_E_NULL, "null argument");
  if (!x->dyn_on) return fail(x, CLOVER_E_TREE, "no dynamic tree is set");
  if (b < 0 || b >= x->cfg.max_batch) return fail(x, CLOVER_E_SHAPE, "sequence index out of range");
  const DynTree& t = x->dyn;
  const size_t ro = (size_t)b * x->R, co = (size_t)b * t.C;
  hipError_t e = hipSuccess;
  auto down = [&](void* dst, const void* src, size_t bytes) {
    if (e == hipSuccess) e = hipMemcpyAsync(dst, src, bytes, hipMemcpyDeviceToHost, x->st);
  };
  down(parent_out, t.t_parent + ro, t.N * sizeof(int));
  down(rank_out, t.t_rank + ro, t.N * sizeof(int));
  down(keep_out, t.t_keep + ro, t.N * sizeof(int));
  down(cand_token_out, t.cand_tok + co, t.C * sizeof(int));
  down(cand_score_out, t.cand_score + co, t.C * sizeof(float));
  down(cand_parent_out, t.cand_par + co, t.C * sizeof(int));
  down(frontier_out, t.frontier + (size_t)b * CLOVER_MAX_DEPTH * DYN_MAX_FRONT, CLOVER_MAX_DEPTH * DYN_MAX_FRONT * sizeof(int));
  if (e == hipSuccess) e = hipStreamSynchronize(x->st);
  if (e != hipSuccess) return fail(x, CLOVER_E_HIP, std::string("clover_read_dynamic_tree: ") + hipGetErrorString(e));
  return CLOVER_OK;
}

int draft_tree(clover_ctx* x, int32_t batch, const float* hid_acc, const int32_t* next_tok, const int32_t* m,
               int32_t* tree_tokens) {
  if (!x || !hid_acc || !next_tok || !m || !tree_tokens) return fail(x, CLOVER_E_NULL, "null argument");
  int rc = check_batch(x, batch);
  if (rc) return rc;
  const clover_config& c = x->cfg;
  const TreeHost& t = x->tree;
  const int B = batch, R = x->R, H = x->H, n = std::min(x->m_upper, R);
  for (int b = 0; b < B; ++b)
    if (x->aug_ub[b] + n > c.max_seq) return fail(x, CLOVER_E_CAPACITY, "augmenting-block cache could exceed max_seq");
  const RowMap rm{B, R, n, m};
  const int M = (B - 1) * R + n;
  int aug_bound = 0;
  for (int b = 0; b < B; ++b) aug_bound = std::max(aug_bound, x->aug_ub[b] + n);
  int max_lvl_rows = B;
  if (x->dyn_on)
    for (int j = 0; j < x->dyn.D; ++j) max_lvl_rows = std::max(max_lvl_rows, B * x->dyn.F[j]);
  else if (t.max_depth <= c.draft_depths)
    for (int j = 0; j < t.max_depth; ++j) max_lvl_rows = std::max(max_lvl_rows, B * (t.lvl_off[j + 1] - t.lvl_off[j]));
  const bool fused = draft_fused_ok(x, M) && draft_fused_ok(x, max_lvl_rows);
  Planes A = planes_of(x, x->a_norm, 2 * H);
  A.ld = H;
  Planes Y = planes_of(x, x->pl_y, 2 * H);
  Y.ld = H;
  Planes Cc = planes_of(x, x->d_cat, 2 * H);   // [state ; embedding] rows of the per-depth FC
  if (fused) {
    // embeddings of the follow-up tokens come from the LM-head rows; AD1 over (hidden state, embedding)
    { Scope s(x, KC_DRAFT_MISC);
      launch_draft_pre(hid_acc, next_tok, x->w.ad1.norm, c.rms_eps, x->w.lm_head, c.vocab, H, rm, A.hi, A.lo, Y.hi, Y.lo, x->st); }
    AdGateArgs g;
    memset(&g, 0, sizeof(g));
    g.x = hid_acc; g.ldx = H; g.out = x->xd; g.ldo = H;
    g.gain = x->aug[0].attn_norm; g.n_hi = A.hi; g.n_lo = A.lo;   // planes for the Augmenting Block's first layer
    run_ad_fused(x, x->w.ad1, A, Y, M, g);
    { Scope s(x, KC_ROPE_KV); launch_rope_table(x->d_aug_len, nullptr, c.rope_base, c.head_dim, x->cos_t, x->sin_t, rm, x->st); }
  } else {
  // embeddings of the follow-up tokens come from the LM-head rows
  { Scope s(x, KC_EMBED); launch_embed(x->w.lm_head, c.dtype, next_tok, c.vocab, x->d_e, H, H, rm, x->st); }
  run_ad(x, x->w.ad1, hid_acc, x->d_e, M, x->xd);
  { Scope s(x, KC_ROPE_KV); launch_rope_table(x->d_aug_len, nullptr, c.rope_base, c.head_dim, x->cos_t, x->sin_t, rm, x->st); }
  if (x->fast) norm_planes(x, x->xd, x->aug[0].attn_norm, M);
  }
  for (int l = 0; l < c.aug_layers; ++l)
    run_layer(x, x->aug[l], x->xd, rm, M, x->aug_kc + (size_t)l * x->k_layer_elems * x->kv_esz,
              x->aug_vc + (size_t)l * x->v_layer_elems * x->kv_esz, x->d_aug_len, nullptr /* the new rows form a chain */,
              l + 1 < c.aug_layers ? x->aug[l + 1].attn_norm : nullptr, aug_bound);
  {
    // root state and token: node 0 of the static tree, candidate 0 of the dynamic one
    float* root_state = x->dyn_on ? x->dyn_state : x->d_state;
    int* root_tok = x->dyn_on ? x->dyn.cand_tok : tree_tokens;
    const int Rs = x->dyn_on ? x->dyn.C : R;
    Scope s(x, KC_DRAFT_MISC);
    if (fused) {
      launch_draft_root_fused(x->xd, next_tok, m, B, R, H, root_state, root_tok, Y.hi, Y.lo, x->d_aug_len, x->st, Rs);
    } else {
      launch_draft_root(x->xd, next_tok, m, B, R, H, x->d_rootx, root_state, root_tok, x->st, Rs);
      launch_add_len(x->d_aug_len, m, B, x->st);
    }
  }
  for (int b = 0; b < B; ++b) x->aug_ub[b] += n;
  if (x->dyn_on) {
    draft_expand_dynamic(x, B, m, tree_tokens, fused, A, Y, Cc);
    return finish(x, "draft_tree");
  }
  // expansion, level by level; a tree deeper than the head (e.g. a prompt chain) is not expanded
  if (t.max_depth <= c.draft_depths) {
    for (int j = 0; j < t.max_depth; ++j) {
      const int n_lvl = t.lvl_off[j + 1] - t.lvl_off[j];
      if (n_lvl == 0) break;
      const int rows = B * n_lvl;
      if (fused) {
        // depth j: (AD2 over the parent's state and the node's token embedding, then) FC_j; the FC's K-slice partials
        // and bias go straight into the head norm; the LM head's partials go straight into the ranking
        int sp;
        if (j == 0) {
          sp = gemm_fast1(x, KC_GEMM_DRAFT, Y, x->w.fc0_w, rows, H, H);
        } else {
          const int* nodes = x->d_lvl_nodes + t.lvl_off[j];
          { Scope s(x, KC_DRAFT_MISC);
            launch_draft_level(x->d_state, tree_tokens, nodes, x->d_parent, n_lvl, B, R, H, x->w.lm_head, c.vocab,
                               x->w.ad2.norm, c.rms_eps, A.hi, A.lo, Y.hi, Y.lo, Cc.hi, Cc.lo, x->st); }
          AdGateArgs g;
          memset(&g, 0, sizeof(g));
          g.x = x->d_state; g.ldx = H; g.out = x->d_state; g.ldo = H;
          g.nodes = nodes; g.parent = x->d_parent; g.n_lvl = n_lvl; g.R = R; g.m = m;
          g.c_hi = Cc.hi; g.c_lo = Cc.lo; g.ldc = 2 * H;
          run_ad_fused(x, x->w.ad2, A, Y, rows, g);
          Planes C2 = Cc;
          C2.ld = 2 * H;
          sp = gemm_fast1(x, KC_GEMM_DRAFT, C2, x->fc_w[j], rows, H, 2 * H);
        }
        { Scope s(x, KC_RMSNORM);
          launch_reduce_add_norm(x->d_g, H, x->partial, sp, (size_t)rows * H, H, x->w.head_norm, c.dtype, c.rms_eps, A.hi,
                                 A.lo, H, rows, H, x->st, j == 0 ? x->w.fc0_b : x->fc_b[j]); }
        if (x->panel && panel_gemm_supported(std::min(rows, 64), c.vocab, H, 0)) {
          lm_head_fast(x, A, rows, x->z);
          capture_draft_logits(x, j, rows);
          Scope s(x, KC_TOPK);
          launch_topk(x->z, c.vocab, c.vocab, rows, t.kmax[j], x->cand, x->topk_ids, x->st);
        } else {
          const int spv = gemm_fast1(x, KC_GEMM_LMHEAD, A, x->lm_head_pk, rows, c.vocab, H);
          if (x->draft_capture) {
            launch_reduce(x->partial, spv, (size_t)rows * c.vocab, c.vocab, nullptr, c.dtype, x->z, c.vocab, rows, c.vocab, 0, x->st);
            capture_draft_logits(x, j, rows);
          }
          Scope s(x, KC_TOPK);
          launch_topk(x->partial, c.vocab, c.vocab, rows, t.kmax[j], x->cand, x->topk_ids, x->st, spv, (size_t)rows * c.vocab);
        }
        { Scope s(x, KC_DRAFT_MISC);
          launch_draft_assign(x->topk_ids, x->d_par_row, x->d_rank, t.node_off[j + 1], t.node_off[j + 2], n_lvl, B, R, m,
                              tree_tokens, x->st); }
        continue;
      }
      if (j == 0) {
        run_fc(x, x->d_rootx, H, x->w.fc0_w, x->w.fc0_b, x->d_g, rows);
      } else {
        const int* nodes = x->d_lvl_nodes + t.lvl_off[j];
        { Scope s(x, KC_DRAFT_MISC);
          launch_draft_gather(x->d_state, tree_tokens, nodes, x->d_parent, n_lvl, B, R, H, x->w.lm_head, c.dtype,
                              c.vocab, x->d_xs, x->d_e, x->d_cat, x->st); }
        run_ad(x, x->w.ad2, x->d_xs, x->d_e, rows, x->d_s);
        { Scope s(x, KC_DRAFT_MISC);
          launch_draft_scatter_state(x->d_s, nodes, n_lvl, B, R, H, x->d_state, x->d_cat, x->st); }
        run_fc(x, x->d_cat, 2 * H, x->fc_w[j], x->fc_b[j], x->d_g, rows);
      }
      run_head(x, x->d_g, rows, t.kmax[j]);
      capture_draft_logits(x, j, rows);
      { Scope s(x, KC_DRAFT_MISC);
        launch_draft_assign(x->topk_ids, x->d_par_row, x->d_rank, t.node_off[j + 1], t.node_off[j + 2], n_lvl, B, R, m,
                            tree_tokens, x->st); }
    }
  }
  return finish(x, "draft_tree");
}

int verify_tree(clover_ctx* x, int32_t batch, const int32_t* tree_tokens, float* logits, float* hidden) {
  if (!x || !tree_tokens || !logits || !hidden) return fail(x, CLOVER_E_NULL, "null argument");
  int rc = check_batch(x, batch);
  if (rc) return rc;
  const clover_config& c = x->cfg;
  const TreeHost& t = x->tree;
  const int B = batch, R = x->R, H = x->H;
  const int n_nodes = x->dyn_on ? x->dyn.N : t.n;
  // topology tables: one static tree for all sequences, or the tables draft_tree wrote per sequence
  const int* depth_tab = x->dyn_on ? x->dyn.t_depth : x->d_depth;
  const unsigned long long* anc_tab = x->dyn_on ? x->dyn.t_anc : x->d_anc;
  const int* iv_tab = !x->interval ? nullptr : x->dyn_on ? x->dyn.t_iv : x->d_iv;
  const int topo_stride = x->dyn_on ? R : 0;
  for (int b = 0; b < B; ++b)
    if (x->len_ub[b] + n_nodes > c.max_seq) return fail(x, CLOVER_E_CAPACITY, "sequence could exceed max_seq (call clover_seq_len to refresh the bound)");
  const RowMap rm{B, R, n_nodes, nullptr};
  const int M = (B - 1) * R + n_nodes;
  int key_bound = 0;
  for (int b = 0; b < B; ++b) key_bound = std::max(key_bound, x->len_ub[b] + n_nodes);
  { Scope s(x, KC_EMBED); launch_embed(x->w.embed, c.dtype, tree_tokens, c.vocab, hidden, H, H, rm, x->st); }
  { Scope s(x, KC_ROPE_KV);
    launch_rope_table(x->d_seq_len, depth_tab, c.rope_base, c.head_dim, x->cos_t, x->sin_t, rm, x->st, topo_stride); }
  if (x->fast) norm_planes(x, hidden, x->layers[0].attn_norm, M);
  for (int l = 0; l < c.n_layers; ++l)
    run_layer(x, x->layers[l], hidden, rm, M, x->kc + (size_t)l * x->k_layer_elems * x->kv_esz,
              x->vc + (size_t)l * x->v_layer_elems * x->kv_esz, x->d_seq_len, anc_tab,
              l + 1 < c.n_layers ? x->layers[l + 1].attn_norm : x->w.final_norm, key_bound, topo_stride, iv_tab);
  if (x->fast) {
    Planes A = planes_of(x, x->a_norm, 2 * H);
    A.ld = H;
    lm_head_fast(x, A, M, logits);
  } else {
    { Scope s(x, KC_RMSNORM); launch_rmsnorm(hidden, H, x->w.final_norm, c.dtype, c.rms_eps, x->a_norm, H, H, M, x->st); }
    gemm_generic(x, KC_GEMM_LMHEAD, x->a_norm, H, x->w.lm_head, nullptr, logits, c.vocab, M, c.vocab, H, 0);
  }
  return finish(x, "verify_tree");
}

int accept_and_compact(clover_ctx* x, int32_t batch, const int32_t* tree_tokens, const float* logits,
                       const float* hidden, int32_t* m, int32_t* acc_idx, int32_t* new_tokens, float* hid_acc,
                       int32_t* next_tok) {
  if (!x || !tree_tokens || !logits || !hidden || !m || !acc_idx || !new_tokens || !hid_acc || !next_tok)
    return fail(x, CLOVER_E_NULL, "null argument");
  int rc = check_batch(x, batch);
  if (rc) return rc;
  rc = accept_common(x, batch, tree_tokens, logits, hidden, nullptr, nullptr, m, acc_idx, new_tokens, hid_acc, next_tok);
  if (rc) return rc;
  x->m_upper = std::min((x->dyn_on ? x->dyn.D : x->tree.max_depth) + 1, x->R);
  for (int b = 0; b < batch; ++b) x->len_ub[b] += x->m_upper;
  return CLOVER_OK;
}

int accept_and_compact_sampled(clover_ctx* x, int32_t batch, const int32_t* tree_tokens, const float* logits,
                               const float* hidden, float temperature, const float* uniforms, int32_t* m,
                               int32_t* acc_idx, int32_t* new_tokens, float* hid_acc, int32_t* next_tok) {
  if (!x || !tree_tokens || !logits || !hidden || !uniforms || !m || !acc_idx || !new_tokens || !hid_acc || !next_tok)
    return fail(x, CLOVER_E_NULL, "null argument");
  int rc = check_batch(x, batch);
  if (rc) return rc;
  if (!(temperature > 0.f) || !(temperature < 1e6f)) return fail(x, CLOVER_E_SHAPE, "temperature must be positive (use accept_and_compact for temperature 0)");
  rc = accept_common(x, batch, tree_tokens, logits, hidden, nullptr, nullptr, m, acc_idx, new_tokens, hid_acc, next_tok,
                     temperature, uniforms);
  if (rc) return rc;
  x->m_upper = std::min((x->dyn_on ? x->dyn.D : x->tree.max_depth) + 1, x->R);
  for (int b = 0; b < batch; ++b) x->len_ub[b] += x->m_upper;
  return CLOVER_OK;
}

int clover_accept_forced(clover_ctx* x, int32_t batch, const int32_t* tree_tokens, const float* logits,
                         const float* hidden, const int32_t* n_rows, const int32_t* forced_next, int32_t* m,
                         int32_t* acc_idx, int32_t* new_tokens, float* hid_acc, int32_t* next_tok) {
  if (!x || !tree_tokens || !logits || !hidden || !n_rows || !forced_next || !m || !acc_idx || !new_tokens ||
      !hid_acc || !next_tok)
    return fail(x, CLOVER_E_NULL, "null argument");
  int rc = check_batch(x, batch);
  if (rc) return rc;
  if (x->dyn_on || !x->tree.is_chain) return fail(x, CLOVER_E_TREE, "clover_accept_forced needs a chain-shaped tree");
  rc = accept_common(x, batch, tree_tokens, logits, hidden, n_rows, forced_next, m, acc_idx, new_tokens, hid_acc, next_tok);
  if (rc) return rc;
  x->m_upper = x->tree.n;
  for (int b = 0; b < batch; ++b) x->len_ub[b] += x->tree.n;
  return CLOVER_OK;
}

int clover_prefill(clover_ctx* x, int32_t b, const int32_t* tokens, int32_t n, float* logits_last, float* hid_last,
                   int32_t* next_tok_out) {
  if (!x || !tokens || !logits_last || !hid_last) return fail(x, CLOVER_E_NULL, "null argument");
  const clover_config& c = x->cfg;
  if (b < 0 || b >= c.max_batch) return fail(x, CLOVER_E_SHAPE, "sequence index out of range");
  if (n < 1) return fail(x, CLOVER_E_SHAPE, "a prompt has at least one token");
  if (x->len_ub[b] + n > c.max_seq || x->aug_ub[b] + n - 1 > c.max_seq)
    return fail(x, CLOVER_E_CAPACITY, "prompt would exceed max_seq (call clover_seq_len to refresh the bound)");
  const int H = x->H;
  const int P = std::min(x->max_rows, CLOVER_MAX_PREFILL_ROWS);   // rows per pass
  int* len_b = x->d_seq_len + b;
  int* aug_len_b = x->d_aug_len + b;
  float* xres = x->d_xs;   // residual stream of the pass (the draft head's staging buffers are idle here)
  for (int c0 = 0; c0 < n; c0 += P) {
    const int M = std::min(P, n - c0);
    const bool last = c0 + M == n;
    const RowMap rm{1, P, M, nullptr};
    // ---- target: embedding, layers with causal attention (no mask table: a chain), K/V in place ----
    { Scope s(x, KC_EMBED); launch_embed(x->w.embed, c.dtype, tokens + c0, c.vocab, xres, H, H, rm, x->st); }
    { Scope s(x, KC_ROPE_KV); launch_rope_table(len_b, nullptr, c.rope_base, c.head_dim, x->cos_t, x->sin_t, rm, x->st); }
    if (x->fast) norm_planes(x, xres, x->layers[0].attn_norm, M);
    const int key_bound = x->len_ub[b] + M;
    for (int l = 0; l < c.n_layers; ++l)
      run_layer(x, x->layers[l], xres, rm, M, x->kc + (size_t)l * x->k_layer_elems * x->kv_esz,
                x->vc + (size_t)l * x->v_layer_elems * x->kv_esz, len_b, nullptr,
                l + 1 < c.n_layers ? x->layers[l + 1].attn_norm : x->w.final_norm, key_bound, 0, nullptr, b);
    { Scope s(x, KC_DRAFT_MISC); launch_add_scalar(len_b, M, x->st); }
    x->len_ub[b] += M;
    if (last) {
      // LM head on the last row only; its hidden state is the hand-off row
      if (x->fast) {
        Planes A = planes_of(x, x->a_norm, 2 * H);
        A.ld = H;
        A.hi += (size_t)(M - 1) * H;
        A.lo += (size_t)(M - 1) * H;
        lm_head_fast(x, A, 1, logits_last);
      } else {
        { Scope s(x, KC_RMSNORM);
          launch_rmsnorm(xres + (size_t)(M - 1) * H, H, x->w.final_norm, c.dtype, c.rms_eps, x->a_norm, H, H, 1, x->st); }
        gemm_generic(x, KC_GEMM_LMHEAD, x->a_norm, H, x->w.lm_head, nullptr, logits_last, c.vocab, 1, c.vocab, H, 0);
      }
      hipMemcpyAsync(hid_last, xres + (size_t)(M - 1) * H, (size_t)H * sizeof(float), hipMemcpyDeviceToDevice, x->st);
      if (next_tok_out) {
        { Scope s(x, KC_TOPK); launch_topk(logits_last, c.vocab, c.vocab, 1, 1, x->cand, x->topk_ids, x->st); }
        hipMemcpyAsync(next_tok_out, x->topk_ids, sizeof(int), hipMemcpyDeviceToDevice, x->st);
      }
    }
    // ---- draft side: position i pairs with token i+1 (all but the prompt's last position, whose follow-up token
    // does not exist yet): Attention Decoder 1, then the Augmenting Block over its own cache ----
    const int Md = last ? M - 1 : M;
    if (Md > 0) {
      const RowMap rd{1, P, Md, nullptr};
      { Scope s(x, KC_EMBED); launch_embed(x->w.lm_head, c.dtype, tokens + c0 + 1, c.vocab, x->d_e, H, H, rd, x->st); }
      run_ad(x, x->w.ad1, xres, x->d_e, Md, x->xd);
      { Scope s(x, KC_ROPE_KV); launch_rope_table(aug_len_b, nullptr, c.rope_base, c.head_dim, x->cos_t, x->sin_t, rd, x->st); }
      if (x->fast) norm_planes(x, x->xd, x->aug[0].attn_norm, Md);
      const int aug_bound = x->aug_ub[b] + Md;
      for (int l = 0; l < c.aug_layers; ++l)
        run_layer(x, x->aug[l], x->xd, rd, Md, x->aug_kc + (size_t)l * x->k_layer_elems * x->kv_esz,
                  x->aug_vc + (size_t)l * x->v_layer_elems * x->kv_esz, aug_len_b, nullptr,
                  l + 1 < c.aug_layers ? x->aug[l + 1].attn_norm : nullptr, aug_bound, 0, nullptr, b);
      { Scope s(x, KC_DRAFT_MISC); launch_add_scalar(aug_len_b, Md, x->st); }
      x->aug_ub[b] += Md;
    }
  }
  if (x->only_prefills) x->m_upper = 1;
  return finish(x, "clover_prefill");
}

int clover_set_page_table(clover_ctx* x, const int32_t* table_host) {
  if (!x) return fail(x, CLOVER_E_NULL, "null argument");
  if (!table_host) {   // back to the identity mapping
    x->kv.pages = nullptr;
    return CLOVER_OK;
  }
  const int n = x->cfg.max_batch * x->kv.T;
  std::vector<char> seen((size_t)n, 0);
  for (int i = 0; i < n; ++i) {
    const int pg = table_host[i];
    if (pg < 0 || pg >= n || seen[pg]) return fail(x, CLOVER_E_SHAPE, "page table must be a permutation of 0 .. max_batch * max_seq / 32 - 1");
    seen[pg] = 1;
  }
  hipError_t e = hipMemcpyAsync(x->d_pages, table_host, (size_t)n * sizeof(int), hipMemcpyHostToDevice, x->st);
  if (e == hipSuccess) e = hipStreamSynchronize(x->st);
  if (e != hipSuccess) return fail(x, CLOVER_E_HIP, std::string("page table upload: ") + hipGetErrorString(e));
  x->kv.pages = x->d_pages;
  return CLOVER_OK;
}

int clover_seq_len(clover_ctx* x, int32_t* out_host) {
  if (!x || !out_host) return fail(x, CLOVER_E_NULL, "null argument");
  const int B = x->cfg.max_batch;
  std::vector<int> aug(B);
  int err = 0;
  hipError_t e = hipMemcpyAsync(out_host, x->d_seq_len, B * sizeof(int), hipMemcpyDeviceToHost, x->st);
  if (e == hipSuccess) e = hipMemcpyAsync(aug.data(), x->d_aug_len, B * sizeof(int), hipMemcpyDeviceToHost, x->st);
  if (e == hipSuccess) e = hipMemcpyAsync(&err, x->d_err, sizeof(int), hipMemcpyDeviceToHost, x->st);
  if (e == hipSuccess) e = hipStreamSynchronize(x->st);
  if (e != hipSuccess) return fail(x, CLOVER_E_HIP, std::string("clover_seq_len: ") + hipGetErrorString(e));
  for (int b = 0; b < B; ++b) { x->len_ub[b] = out_host[b]; x->aug_ub[b] = aug[b]; }
  if (err) return fail(x, CLOVER_E_STATE, "a kernel refused to write past max_seq");
  return CLOVER_OK;
}

int clover_read_kv(clover_ctx* x, int32_t stack, int32_t layer, int32_t b, int32_t slot0, int32_t n_slots,
                   float* k_out_host, float* v_out_host) {
  if (!x || !k_out_host || !v_out_host) return fail(x, CLOVER_E_NULL, "null argument");
  const clover_config& c = x->cfg;
  const int nl = stack == 0 ? c.n_layers : c.aug_layers;
  if (stack < 0 || stack > 1 || layer < 0 || layer >= nl || b < 0 || b >= c.max_batch || slot0 < 0 || n_slots < 0 ||
      slot0 + n_slots > c.max_seq)
    return fail(x, CLOVER_E_SHAPE, "clover_read_kv: index out of range");
  const size_t n = (size_t)n_slots * c.n_kv_heads * c.head_dim;
  if (2 * n > (size_t)x->max_rows * c.vocab) return fail(x, CLOVER_E_SHAPE, "clover_read_kv: too many slots at once");
  if (n == 0) return CLOVER_OK;
  const char* kbase = (stack == 0 ? x->kc : x->aug_kc) + (size_t)layer * x->k_layer_elems * x->kv_esz;
  const char* vbase = (stack == 0 ? x->vc : x->aug_vc) + (size_t)layer * x->v_layer_elems * x->kv_esz;
  launch_read_kv(kbase, vbase, x->kvdtype, x->kv, b, slot0, n_slots, x->z, x->z + n, x->st);
  hipError_t e = hipMemcpyAsync(k_out_host, x->z, n * sizeof(float), hipMemcpyDeviceToHost, x->st);
  if (e == hipSuccess) e = hipMemcpyAsync(v_out_host, x->z + n, n * sizeof(float), hipMemcpyDeviceToHost, x->st);
  if (e == hipSuccess) e = hipStreamSynchronize(x->st);
  if (e != hipSuccess) return fail(x, CLOVER_E_HIP, std::string("clover_read_kv: ") + hipGetErrorString(e));
  return CLOVER_OK;
}

int clover_write_kv(clover_ctx* x, int32_t stack, int32_t layer, int32_t b, int32_t slot0, int32_t n_slots,
                    const float* k_in_host, const float* v_in_host) {
  if (!x || !k_in_host || !v_in_host) return fail(x, CLOVER_E_NULL, "null argument");
  const clover_config& c = x->cfg;
  const int nl = stack == 0 ? c.n_layers : c.aug_layers;
  if (stack < 0 || stack > 1 || layer < 0 || layer >= nl || b < 0 || b >= c.max_batch || slot0 < 0 || n_slots < 0 ||
      slot0 + n_slots > c.max_seq)
    return fail(x, CLOVER_E_SHAPE, "clover_write_kv: index out of range");
  const size_t n = (size_t)n_slots * c.n_kv_heads * c.head_dim;
  if (2 * n > (size_t)x->max_rows * c.vocab) return fail(x, CLOVER_E_SHAPE, "clover_write_kv: too many slots at once");
  if (n == 0) return CLOVER_OK;
  char* kbase = (stack == 0 ? x->kc : x->aug_kc) + (size_t)layer * x->k_layer_elems * x->kv_esz;
  char* vbase = (stack == 0 ? x->vc : x->aug_vc) + (size_t)layer * x->v_layer_elems * x->kv_esz;
  hipError_t e = hipMemcpyAsync(x->z, k_in_host, n * sizeof(float), hipMemcpyHostToDevice, x->st);
  if (e == hipSuccess) e = hipMemcpyAsync(x->z + n, v_in_host, n * sizeof(float), hipMemcpyHostToDevice, x->st);
  if (e == hipSuccess) {
    launch_write_kv(kbase, vbase, x->kvdtype, x->kv, b, slot0, n_slots, x->z, x->z + n, x->st);
    e = hipStreamSynchronize(x->st);   // the host arrays and the staging area are free again on return
  }
  if (e != hipSuccess) return fail(x, CLOVER_E_HIP, std::string("clover_write_kv: ") + hipGetErrorString(e));
  return CLOVER_OK;
}

int clover_set_seq_len(clover_ctx* x, const int32_t* len_host, const int32_t* aug_len_host) {
  if (!x || !len_host || !aug_len_host) return fail(x, CLOVER_E_NULL, "null argument");
  const int B = x->cfg.max_batch;
  for (int b = 0; b < B; ++b)
    if (len_host[b] < 0 || len_host[b] > x->cfg.max_seq || aug_len_host[b] < 0 || aug_len_host[b] > x->cfg.max_seq)
      return fail(x, CLOVER_E_CAPACITY, "clover_set_seq_len: length outside [0, max_seq]");
  hipError_t e = hipMemcpyAsync(x->d_seq_len, len_host, B * sizeof(int), hipMemcpyHostToDevice, x->st);
  if (e == hipSuccess) e = hipMemcpyAsync(x->d_aug_len, aug_len_host, B * sizeof(int), hipMemcpyHostToDevice, x->st);
  if (e == hipSuccess) e = hipStreamSynchronize(x->st);
  if (e != hipSuccess) return fail(x, CLOVER_E_HIP, std::string("clover_set_seq_len: ") + hipGetErrorString(e));
  for (int b = 0; b < B; ++b) { x->len_ub[b] = len_host[b]; x->aug_ub[b] = aug_len_host[b]; }
  return CLOVER_OK;
}

int clover_capture_draft_logits(clover_ctx* x, float* dev_out, size_t capacity_floats) {
  if (!x) return CLOVER_E_NULL;
  x->draft_capture = dev_out;
  x->draft_capture_floats = dev_out ? capacity_floats : 0;
  return CLOVER_OK;
}

int clover_profile_enable(clover_ctx* x, int32_t on) {
  if (!x) return CLOVER_E_NULL;
  x->prof = on != 0;
  return CLOVER_OK;
}

int clover_profile_collect(clover_ctx* x, double* ms, int64_t* launches, int32_t n_classes) {
  if (!x || !ms || !launches) return fail(x, CLOVER_E_NULL, "null argument");
  if (n_classes < KC_COUNT) return fail(x, CLOVER_E_SHAPE, "n_classes too small");
  for (int i = 0; i < n_classes; ++i) { ms[i] = 0.0; launches[i] = 0; }
  hipError_t e = hipStreamSynchronize(x->st);
  if (e != hipSuccess) return fail(x, CLOVER_E_HIP, hipGetErrorString(e));
  for (ProfEvent& ev : x->prof_events) {
    float t = 0.f;
    if (hipEventElapsedTime(&t, ev.a, ev.b) == hipSuccess) { ms[ev.cls] += t; launches[ev.cls] += 1; }
    x->prof_pool.push_back(ev);
  }
  x->prof_events.clear();
  return CLOVER_OK;
}

int clover_path_info(clover_ctx* x) {
  if (!x) return CLOVER_E_NULL;
  return (x->fast ? 1 : 0) | (x->attn_fast ? 2 : 0);
}

int clover_kernel_class_count(void) { return KC_COUNT; }
const char* clover_kernel_class_name(int32_t cls) { return (cls >= 0 && cls < KC_COUNT) ? kClassNames[cls] : ""; }

const char* clover_last_error(clover_ctx* x) { return x ? x->err.c_str() : ""; }
const char* clover_last_global_error(void) { return g_err.c_str(); }

size_t clover_op_gemm_scratch_bytes(int32_t M, int32_t N, int32_t K) {
  if (M < 1 || N < 1 || K < 1) return 256;
  size_t bytes = 256;
  if (M <= 256 && mfma_gemm_supported(M, N, K, 0)) {
    size_t out = mfma_gemm_out_bytes(M, N, mfma_gemm_pick_splits(M, N, K, 0));
    if (stream_gemm_supported(M, N, K)) out = std::max(out, stream_gemm_out_bytes(M, N, K));
    out = std::max(out, (size_t)std::max(panel_gemm_pick_k_parts(M, N, K), 0) * M * N * sizeof(float));
    if (tile_gemm_supported(M, N, K, 0))
      out = std::max(out, (size_t)tile_gemm_pick_k_parts(M, N, K) * M * N * sizeof(float));
    bytes += align256((size_t)M * K * 4) + align256(out) + align256((size_t)N * K * 2);
  }
  return bytes;
}

int clover_op_gemm(int32_t path, int32_t dtype, const float* X, const void* W, float* Y, int32_t ldy, int32_t M,
                   int32_t N, int32_t K, void* scratch, size_t scratch_bytes, void* hip_stream) {
  return op_gemm_impl(path, dtype, X, W, Y, ldy, M, N, K, scratch, scratch_bytes, hip_stream);
}

int clover_op_gemm_static(int32_t path, int32_t dtype, const float* X, const void* W, float* Y, int32_t ldy, int32_t M,
                          int32_t N, int32_t K, void* hip_stream) {
  if (path != 0 && path != 1 && path != 3 && path != 5)
    return fail(nullptr, CLOVER_E_SHAPE, "clover_op_gemm_static: path must be 0, 1, 3 or 5 (the shared buffer keeps no copy between calls)");
  if (M >= 1 && N >= 1 && K >= 1 && clover_op_gemm_scratch_bytes(M, N, K) > CLOVER_STATIC_SCRATCH_BYTES)
    return fail(nullptr, CLOVER_E_CAPACITY, "clover_op_gemm_static: M, N, K need more than CLOVER_STATIC_SCRATCH_BYTES of scratch");
  void* ptr = nullptr;
  const int rc = static_scratch_ptr(&ptr);
  if (rc) return rc;
  return op_gemm_impl(path, dtype, X, W, Y, ldy, M, N, K, ptr, CLOVER_STATIC_SCRATCH_BYTES, hip_stream);
}

}  // extern "C"

namespace {
int op_gemm_impl(int32_t path, int32_t dtype, const float* X, const void* W, float* Y, int32_t ldy, int32_t M,
                 int32_t N, int32_t K, void* scratch, size_t scratch_bytes, void* hip_stream) {
  if (!X || !W || !Y || !scratch) return fail(nullptr, CLOVER_E_NULL, "null argument");
  if (M < 1 || N < 1 || K < 1 || ldy < N) return fail(nullptr, CLOVER_E_SHAPE, "bad GEMM shape");
  hipStream_t st = (hipStream_t)hip_stream;
  if (path == 0) {
    launch_gemm_generic(X, K, W, nullptr, dtype, Y, ldy, M, N, K, 0, st);
  } else {
    if (dtype != CLOVER_DTYPE_BF16 || M > 256 || !mfma_gemm_supported(M, N, K, 0))
      return fail(nullptr, CLOVER_E_SHAPE, "shape not supported by the MFMA GEMM");
    if (scratch_bytes < clover_op_gemm_scratch_bytes(M, N, K)) return fail(nullptr, CLOVER_E_CAPACITY, "scratch too small");
    // scratch: [packed weight copy][activation planes][partials]; the copy is made once per scratch
    // buffer contents, so repeated calls with the same W measure the GEMM alone (path 2 skips it)
    bf16_t* wp = (bf16_t*)scratch;
    bf16_t* hi = (bf16_t*)((char*)scratch + align256((size_t)N * K * 2));
    bf16_t* lo = hi + (size_t)M * K;
    float* part = (float*)((char*)hi + align256((size_t)M * K * 4));
    if (path & 1) launch_pack_weight(W, wp, N, K, st);
    launch_split_planes(X, K, hi, lo, K, M, K, st);
    int splits;
    if (path == 7) {   // tiled kernel over K ranges, then the sum of the ranges
      if (!tile_gemm_supported(M, N, K, 0)) return fail(nullptr, CLOVER_E_SHAPE, "shape not supported by the tiled GEMM");
      const int kp = tile_gemm_pick_k_parts(M, N, K);
      TileGemm g;
      memset(&g, 0, sizeof(g));
      g.Xhi = hi; g.Xlo = lo; g.ldx = K;
      g.W[0] = g.W[1] = wp;
      g.Y = part; g.ldy = N; g.k_parts = kp; g.split_stride = (size_t)M * N;
      g.M = M; g.N = N; g.K = K; g.epi = 0;
      launch_gemm_tile(g, st);
      launch_reduce(part, kp, (size_t)M * N, N, nullptr, dtype, Y, ldy, M, N, 0, st);
      const hipError_t e = hipGetLastError();
      if (e != hipSuccess) return fail(nullptr, CLOVER_E_HIP, hipGetErrorString(e));
      return CLOVER_OK;
    }
    if (path >= 3) {
      if (!panel_gemm_supported(M, N, K, 0) || ldy % 4 != 0)
        return fail(nullptr, CLOVER_E_SHAPE, "shape not supported by the panel GEMM");
      PanelGemm g;
      memset(&g, 0, sizeof(g));
      g.Xhi = hi; g.Xlo = lo; g.ldx = K;
      g.W[0] = g.W[1] = wp;
      g.Y = Y; g.ldy = ldy; g.M = M; g.N = N; g.K = K; g.epi = 0;
      if (path >= 5) {  // K ranges into partials, then the reduction every consumer of partials performs
        const int kp = panel_gemm_pick_k_parts(M, N, K);
        if (kp < 2) return fail(nullptr, CLOVER_E_SHAPE, "shape not supported by the K-range panel GEMM");
        g.Y = part; g.ldy = N; g.k_parts = kp; g.split_stride = (size_t)M * N;
        launch_gemm_panel(g, st);
        launch_reduce(part, kp, (size_t)M * N, N, nullptr, dtype, Y, ldy, M, N, 0, st);
      } else {
        launch_gemm_panel(g, st);
      }
      const hipError_t e = hipGetLastError();
      if (e != hipSuccess) return fail(nullptr, CLOVER_E_HIP, hipGetErrorString(e));
      return CLOVER_OK;
    }
    if (M <= 64 && stream_gemm_supported(M, N, K)) {
      StreamGemm g;
      memset(&g, 0, sizeof(g));
      g.Xhi = hi; g.Xlo = lo; g.ldx = K;
      g.W[0] = g.W[1] = g.W[2] = wp;
      g.seg_begin[1] = g.seg_begin[2] = g.seg_begin[3] = 0x7fffffff;
      g.Y = part; g.ldy = N; g.split_stride = (size_t)M * N; g.M = M; g.N = N; g.K = K;
      launch_gemm_stream(g, st);
      splits = stream_gemm_slices(K);
    } else {
      MfmaGemm g;
      memset(&g, 0, sizeof(g));
      g.Xhi = hi; g.Xlo = lo; g.ldx = K;
      g.W[0] = g.W[1] = g.W[2] = wp;
      g.seg_begin[0] = 0; g.seg_begin[1] = g.seg_begin[2] = g.seg_begin[3] = 0x7fffffff;
      g.Y = part; g.ldy = N; g.split_stride = (size_t)M * N;
      g.M = M; g.N = N; g.K = K; g.mode = 0;
      g.splits = splits = mfma_gemm_pick_splits(M, N, K, 0);
      launch_gemm_mfma(g, st);
    }
    launch_reduce(part, splits, (size_t)M * N, N, nullptr, dtype, Y, ldy, M, N, 0, st);
  }
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(nullptr, CLOVER_E_HIP, hipGetErrorString(e));
  return CLOVER_OK;
}

}  // namespace
