// Internal declarations shared by the translation units of libclover.so.
// Host-side launch wrappers only: every wrapper validates nothing (the C-ABI layer does) and
// enqueues on the given stream.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "../../include/clover.h"

namespace clv {

typedef unsigned short bf16_t;  // raw bfloat16 bit pattern

enum KernelClass {
  KC_EMBED = 0, KC_RMSNORM, KC_GEMM_QKV, KC_ROPE_KV, KC_ATTN, KC_GEMM_WO, KC_GEMM_GATEUP, KC_GEMM_DOWN,
  KC_GEMM_LMHEAD, KC_GEMM_DRAFT, KC_AD_GATE, KC_TOPK, KC_DRAFT_MISC, KC_ACCEPT, KC_COMPACT, KC_ELTWISE,
  KC_COUNT
};

// Rows are laid out [B, R]; row (b,i) exists for i < n and is valid iff i < (n_valid ? n_valid[b] : n).
struct RowMap {
  int B, R, n;
  const int* n_valid;  // dev [B] or null
};

constexpr int KV_PAGE = 32;   // cached positions per page (= the key tile of the MFMA attention)
struct KVLayout {
  // Paged caches, one pair per layer.  A page holds KV_PAGE consecutive positions of one sequence for all KV heads:
  //   K page:  [n_kv][KV_PAGE][d]      V page (transposed):  [n_kv][d][KV_PAGE]
  // so the K rows and the V^T columns of one (page, head) -- one key tile of the attention -- are one contiguous
  // block each.  Position `slot` of sequence b lives in page pages[(b + b0) * T + slot / KV_PAGE] (identity when
  // pages is null), at row slot % KV_PAGE.
  // kvdtype 0: fp32 elements.  kvdtype 1: each cache is two bf16 planes (hi, then lo `plane` elements
  // later) with hi + lo == value to 16 mantissa bits -- the operand format of the MFMA attention.
  int max_batch, max_seq, n_kv, d;
  size_t plane;
  int T;               // pages per sequence = max_seq / KV_PAGE
  int b0;              // added to every sequence index (a call that works on one sequence of the batch)
  const int* pages;    // dev [max_batch * T] page table, or null
};
#ifdef __HIPCC__
__device__ __forceinline__ size_t kv_page_of(const KVLayout& kv, int b, int slot) {
  const int lp = (b + kv.b0) * kv.T + slot / KV_PAGE;
  return (size_t)(kv.pages ? kv.pages[lp] : lp);
}
// element index of K[b][slot][head][0] (d contiguous elements follow)
__device__ __forceinline__ size_t kv_k_at(const KVLayout& kv, int b, int slot, int head) {
  return ((kv_page_of(kv, b, slot) * kv.n_kv + head) * KV_PAGE + slot % KV_PAGE) * kv.d;
}
// element index of V^T[b][head][dim][slot] (the rest of the page's positions follow contiguously)
__device__ __forceinline__ size_t kv_v_at(const KVLayout& kv, int b, int head, int dim, int slot) {
  return ((kv_page_of(kv, b, slot) * kv.n_kv + head) * kv.d + dim) * KV_PAGE + slot % KV_PAGE;
}
#endif

// ---- generic (fp32 ALU) kernels; wdtype: 0 fp32, 1 bf16 ---------------------------------------
void launch_embed(const void* table, int wdtype, const int* tok, int vocab, float* out, int ldo, int H,
                  RowMap rm, hipStream_t st);
void launch_rmsnorm(const float* x, int ldx, const void* gain, int wdtype, float eps, float* out, int ldo, int H,
                    int rows, hipStream_t st);
// depth_stride: 0 when all sequences share one tree, else the per-sequence stride of the depth table
void launch_rope_table(const int* base_len, const int* depth /*null: row index*/, float rope_base, int d,
                       float* cos_t, float* sin_t, RowMap rm, hipStream_t st, int depth_stride = 0);
void launch_rope_kv_write(const float* qkv, int ldqkv, int qkv_splits, size_t qkv_split_stride, const float* cos_t, const float* sin_t, float* q_out, int ldq,
                          void* k_cache, void* v_cache, int kvdtype, KVLayout kv, const int* base_len, int n_q,
                          RowMap rm, int* err_flag, bf16_t* q_hi /*null: fp32 q_out*/, bf16_t* q_lo, float q_scale,
                          hipStream_t st);
void launch_attn_generic(const float* q, int ldq, const void* k_cache, const void* v_cache, int kvdtype, KVLayout kv,
                         const int* base_len, const unsigned long long* anc /*[n][2]*/, int n_q, float* out, int ldo,
                         bf16_t* out_hi, bf16_t* out_lo /*planes instead of fp32 when non-null*/, RowMap rm,
                         hipStream_t st, int anc_stride = 0 /*nodes per sequence in a per-sequence mask table, 0: shared*/,
                         const int* iv = nullptr /*[n][2] interval labels: decide visibility instead of anc when given*/);
// mode 0: Y = X W^T (+bias); mode 1: Y += X W^T (+bias)
void launch_gemm_generic(const float* X, int ldx, const void* W, const void* bias, int wdtype, float* Y, int ldy,
                         int M, int N, int K, int mode, hipStream_t st);
void launch_swiglu(const float* g, const float* u, float* h, size_t n, hipStream_t st);
void launch_ad_gate(const float* x, int ldx, const float* q, const float* k, const float* v, int H, int heads,
                    float* out, int ldo, float* out2, int ldo2, int rows, hipStream_t st);

// top-k of each row of z[rows, V] by (value desc, id asc); k <= CLOVER_MAX_RANK.
// cand: scratch [rows][chunks][16] of (float,int) pairs; out_ids [rows][16]; chunks = topk_chunks(V).
int topk_chunks(int V);
// z may be given as `splits` partial tiles z[s*split_stride + row*ldz + id] that are summed on the fly (1: plain)
void launch_topk(const float* z, int ldz, int V, int rows, int k, void* cand, int* out_ids, hipStream_t st, int splits = 1,
                 size_t split_stride = 0);

// ---- draft-tree bookkeeping -------------------------------------------------------------------
// gather for level rows: row (b,r) <- node u = lvl_nodes[r]; xs = state[b][parent(u)], e = lm_head[token[b][u]]
// (nodes_stride / parent_stride: per-sequence strides of the index tables, 0 when all sequences share them)
void launch_draft_gather(const float* state, const int* tokens, const int* lvl_nodes, const int* parent, int n_lvl,
                         int B, int R, int H, const void* lm_head, int wdtype, int vocab, float* xs, float* e,
                         float* cat /*[rows,2H], second half <- e*/, hipStream_t st, int nodes_stride = 0,
                         int parent_stride = 0);
// state[b][u] <- s rows (also first half of cat)
void launch_draft_scatter_state(const float* s, const int* lvl_nodes, int n_lvl, int B, int R, int H, float* state,
                                float* cat, hipStream_t st, int nodes_stride = 0);
// root rows: xs_root[b] = a[b][m[b]-1]; state[b][0] = same; tokens[b][0] = next_tok[b][m[b]-1]
// (Rs: row stride of state and tokens when it differs from R, the stride of a and next_tok)
void launch_draft_root(const float* a, const int* next_tok, const int* m, int B, int R, int H, float* root_x,
                       float* state, int* tokens, hipStream_t st, int Rs = 0);
// tokens[b][c] = ids[(b*n_par + par_row[c])*16 + rank[c]] for children c in [c0,c1); skipped when m[b] < 1
void launch_draft_assign(const int* ids, const int* par_row, const int* rank, int c0, int c1, int n_par, int B, int R,
                         const int* m, int* tokens, hipStream_t st);
void launch_add_len(int* len, const int* m, int B, hipStream_t st);
void launch_add_scalar(int* p, int v, hipStream_t st);   // *p += v

// ---- accept / compact -------------------------------------------------------------------------
void launch_accept_walk(const int* argmax, const int* tokens, const int* first_child, const int* n_child, int n_nodes,
                        int B, int R, const int* n_forced, const int* forced_next, int* m, int* acc_idx,
                        int* new_tokens, int* next_tok, hipStream_t st, int child_stride = 0);
void launch_compact_kv(void* k_cache, void* v_cache, int kvdtype, KVLayout kv, int n_layers, size_t k_layer_elems,
                       size_t v_layer_elems, const int* len, const int* m, const int* acc_idx, int B, int R,
                       hipStream_t st);
void launch_gather_hidden(const float* hidden, const int* acc_idx, const int* m, int B, int R, int H, float* hid_acc,
                          hipStream_t st);
void launch_read_kv(const void* k_cache, const void* v_cache, int kvdtype, KVLayout kv, int b, int slot0, int n_slots,
                    float* k_out, float* v_out, hipStream_t st);
void launch_write_kv(void* k_cache, void* v_cache, int kvdtype, KVLayout kv, int b, int slot0, int n_slots,
                     const float* k_in, const float* v_in, hipStream_t st);
void launch_fill_i32(int* p, int v, int n, hipStream_t st);

// ---- split-bf16 activation planes and partial-sum consumers ------------------------------------
// An activation matrix that feeds the MFMA GEMM is stored as two bf16 planes (hi, lo) with
// hi + lo == x to 16 mantissa bits.
void launch_split_planes(const float* x, int ldx, bf16_t* hi, bf16_t* lo, int ldo, int rows, int K, hipStream_t st);
// Y[m,n] (=|+=) sum_s P[s*split_stride + m*ldp + n] (+ bias[n]);  mode 0 store, 1 add
void launch_reduce(const float* P, int splits, size_t split_stride, int ldp, const void* bias, int wdtype, float* Y,
                   int ldy, int M, int N, int mode, hipStream_t st);
// x[m,:] += sum_s P[s][m][:]  (splits may be 0); then, if gain: (hi, lo)[m,:] = split(rmsnorm(x[m,:]) * gain)
// bias non-null: x[m,:] = bias + sum_s P[s][m][:] (the old x is not read)
void launch_reduce_add_norm(float* x, int ldx, const float* P, int splits, size_t split_stride, int ldp,
                            const void* gain, int wdtype, float eps, bf16_t* hi, bf16_t* lo, int ldo, int rows, int H,
                            hipStream_t st, const void* bias = nullptr);

// ---- MFMA weight-streaming GEMM (bf16 weights, split-bf16 activations in, fp32 out) -------------
struct MfmaGemm {
  const bf16_t *Xhi, *Xlo; int ldx;   // activation planes [M, K]
  const bf16_t* W[3];      // up to three fragment-major row-segments (fused QKV); plain GEMM uses W[0]
  int seg_begin[4];        // segment s covers output columns [seg_begin[s], seg_begin[s+1])
  const bf16_t* W_up;      // mode 2: second matrix (W[0] = gate)
  float* Y; int ldy;       // mode 0: split s writes Y[s*split_stride + m*ldy + n]
  size_t split_stride;
  bf16_t *Yhi, *Ylo;       // mode 2: silu(X Wg^T) * (X Wu^T) as planes, leading dimension ldy
  int M, N, K;
  int mode;                // 0 partial/plain fp32 store, 2 SwiGLU
  int splits;              // split-K factor (>=1; 1 for mode 2)
  int dbg;                 // ablation builds only: 1 no MFMA, 2 no weight loads, 4 no activation loads
};
bool mfma_gemm_supported(int M, int N, int K, int mode);
int mfma_gemm_pick_splits(int M, int N, int K, int mode);
size_t mfma_gemm_out_bytes(int M, int N, int splits);
void launch_gemm_mfma(const MfmaGemm& g, hipStream_t st);


// ---- MFMA tree attention (head_dim 128, caches as bf16 planes) ---------------------------------
struct AttnParams {
  const bf16_t *q_hi, *q_lo; int ldq;    // [rows, n_q*128] planes: RoPE applied, scaled by 1/sqrt(128)
  const bf16_t* k_hi; size_t k_plane;    // K planes of one layer (paged, see KVLayout); lo = hi + k_plane
  const bf16_t* v_hi; size_t v_plane;    // V^T planes
  KVLayout kv;
  int max_seq, n_kv, n_q;
  const int* base_len;                   // dev [B]
  const unsigned long long* anc;         // dev [n][2]; null (and no interval labels): the nodes form a chain
  const int* iv;                         // dev [n][2] interval labels (enter, exit) of a depth-first numbering, or null:
                                         //   when given they decide visibility instead of the bit sets
  int anc_stride;                        // nodes per sequence in a per-sequence mask table, 0: one table for all
  RowMap rm;
  float* o_part;                         // [max_splits][rows_total][n_q][128]
  float* ml_part;                        // [max_splits][rows_total][n_q][2]
  int rows_total, max_splits;
  int tiles_per_split, n_splits;         // filled in by launch_attn_mfma
};
bool attn_mfma_supported(int head_dim, int n_q, int n_kv, int max_seq);
// max_total_keys: host-side upper bound of base_len[b] + rm.n over the batch (sizes the key splits)
void launch_attn_mfma(AttnParams p, int max_total_keys, bf16_t* out_hi, bf16_t* out_lo, int ldo, hipStream_t st);

// ---- fragment-major weights and the K-slice-resident streaming GEMM (M <= 64) -------------------
// [N,K] row-major bf16 -> [N/16][K/32][64 lanes][8]: lane l of tile (nb, kt) holds row nb*16 + l%16,
// columns kt*32 + (l/16)*8 .. +7.  Both MFMA GEMMs read this layout.
void launch_pack_weight(const void* src, void* dst, int N, int K, hipStream_t st);
struct StreamGemm {
  const bf16_t *Xhi, *Xlo; int ldx;   // activation planes [M, K]
  const bf16_t* W[3];                 // fragment-major weight segments
  int seg_begin[4];                   // segment s covers output columns [seg_begin[s], seg_begin[s+1])
  float* Y; int ldy;                  // slice s writes Y[s*split_stride + m*ldy + n]
  size_t split_stride;
  int M, N, K;
  int n_slices, groups;               // filled in by launch_gemm_stream
  int tag;                            // 1: gate+up projection (selects a separately named instantiation)
  int dbg;                            // ablation builds only: 1 no activation loads, 2 no stores
};
bool stream_gemm_supported(int M, int N, int K);
int stream_gemm_slices(int K);
size_t stream_gemm_out_bytes(int M, int N, int K);
void launch_gemm_stream(StreamGemm g, hipStream_t st);
// (hi, lo)[m, c] = split(silu(sum_s P[s][m][c]) * sum_s P[s][m][F + c])
void launch_reduce_swiglu(const float* P, int splits, size_t split_stride, int ldp, int F, bf16_t* hi, bf16_t* lo,
                          int ldo, int rows, hipStream_t st);


// ---- full-K panel GEMM (M <= 64, many output columns): finished results, no K-slice partials ----
struct PanelGemm {
  const bf16_t *Xhi, *Xlo; int ldx;   // activation planes [M, K]
  const bf16_t* W[2];                 // fragment-major; epi 1: W[0] = gate, W[1] = up, each [N, K]
  float* Y; int ldy;                  // epi 0: fp32 [M, N]
  bf16_t *Yhi, *Ylo; int ldo;         // epi 1: planes of silu(X W0^T) * (X W1^T), [M, N]
  int M, N, K;
  int epi;                            // 0 plain, 1 SwiGLU
  int k_parts; size_t split_stride;   // epi 0 only: K is cut into k_parts ranges, range r writes Y + r * split_stride
  int rows128;                        // use the 65..128-row form whatever M is (k_parts was picked for its stage width)
  int dbg;                            // ablation builds only: 1 no activation loads, 2 no stage rotation
};
bool panel_gemm_supported(int M, int N, int K, int epi);
// how many K ranges make the plain panel GEMM fill the chip for a NARROW output (0: not worth it)
int panel_gemm_pick_k_parts(int M, int N, int K);
void launch_gemm_panel(const PanelGemm& g, hipStream_t st);

// ---- tiled GEMM for 65..256 rows: one weight pass, 128-row x 256-column workgroup tiles ------------------
struct TileGemm {
  const bf16_t *Xhi, *Xlo; int ldx;   // activation planes [M, K]
  const bf16_t* W[2];                 // fragment-major; epi 1: W[0] = gate, W[1] = up, each [N, K]
  float* Y; int ldy;                  // epi 0: fp32 [M, N]; range r of K writes Y + r * split_stride
  bf16_t *Yhi, *Ylo; int ldo;         // epi 1: planes of silu(X W0^T) * (X W1^T), [M, N]
  int M, N, K;
  int epi;                            // 0 plain, 1 SwiGLU
  int k_parts; size_t split_stride;   // epi 0 only
  int n_units;                        // filled in by launch_gemm_tile: column tiles x K ranges
};
bool tile_gemm_supported(int M, int N, int K, int epi);
int tile_gemm_pick_k_parts(int M, int N, int K);
void launch_gemm_tile(const TileGemm& g, hipStream_t st);

// ---- fused bookkeeping kernels of the draft head (MFMA path, bf16 weights) ----------------------
// planes of RMSNorm(hid[row]) * gain -> (a_hi, a_lo) and of the embedding of tok[row] -> (y_hi, y_lo), rows of `rm`
void launch_draft_pre(const float* hid, const int* tok, const void* gain, float eps, const void* table, int vocab, int H,
                      RowMap rm, bf16_t* a_hi, bf16_t* a_lo, bf16_t* y_hi, bf16_t* y_lo, hipStream_t st);
// Attention-Decoder gate reading the q and (k|v) GEMMs' K-slice partials and adding the biases itself
struct AdGateArgs {
  const float* x; int ldx;                    // residual input rows
  const float* Pq; int Sq; size_t sps_q;      // [Sq][M][H], Sq <= 8
  const float* Pkv; int Skv; size_t sps_kv;   // [Skv][M][2H]: k columns, then v columns, Skv <= 8
  const void *bq, *bk, *bv;                   // bf16 [H]
  int H, heads;
  const int *nodes, *parent; int n_lvl, R;    // nodes null: row g -> row g; else g = b*n_lvl + r, u = nodes[r]: row b*R+parent[u] -> row b*R+u
  int nodes_stride, parent_stride;            // per-sequence strides of nodes / parent (0: shared by all sequences)
  const int* m;                               // with nodes: sequences with m[b] < 1 are skipped (null: none)
  float* out; int ldo;
  const void* gain; float eps; bf16_t *n_hi, *n_lo;   // gain non-null: planes of RMSNorm(result)*gain, row g, ld H
  bf16_t *c_hi, *c_lo; int ldc;               // non-null: planes of the result, row g
};
bool ad_gate_fused_supported(int H, int heads);
void launch_ad_gate_fused(const AdGateArgs& a, int rows, hipStream_t st);
// root state/token from the last accepted row, its planes (row b, ld H), aug_len[b] += m[b]
void launch_draft_root_fused(const float* a, const int* next_tok, const int* m, int B, int R, int H, float* state,
                             int* tokens, bf16_t* y_hi, bf16_t* y_lo, int* aug_len, hipStream_t st, int Rs = 0);
// per internal node r of one depth (u = nodes[r]): planes of RMSNorm(state[parent(u)]) * gain (row b*n_lvl + r, ld H),
// planes of the embedding of tokens[u] in (y_hi, y_lo) (ld H) and in the second half of (c_hi, c_lo) (ld 2H)
void launch_draft_level(const float* state, const int* tokens, const int* nodes, const int* parent, int n_lvl, int B,
                        int R, int H, const void* table, int vocab, const void* gain, float eps, bf16_t* a_hi,
                        bf16_t* a_lo, bf16_t* y_hi, bf16_t* y_lo, bf16_t* c_hi, bf16_t* c_lo, hipStream_t st,
                        int nodes_stride = 0, int parent_stride = 0);

// ---- dynamic (score-pruned) draft tree ----------------------------------------------------------
constexpr int DYN_MAX_CAND = 256;    // candidates per sequence, the root included
constexpr int DYN_MAX_FRONT = 64;    // candidates expanded per depth
struct DynTree {
  int C, D, topk, N;                       // candidates, depths, children per expansion, tree nodes
  int off[CLOVER_MAX_DEPTH + 2];           // candidates of depth j are [off[j], off[j + 1])
  int F[CLOVER_MAX_DEPTH + 1];             // candidates expanded at depth j (F[0] = 1: the root)
  int* cand_tok; float* cand_score; int* cand_par;   // dev [B][C]
  int* frontier;                           // dev [B][CLOVER_MAX_DEPTH][DYN_MAX_FRONT]: expanded candidates, best first
  int *t_parent, *t_rank, *t_depth, *t_first_child, *t_n_child, *t_keep;   // dev [B][R]: the tree as verified
  unsigned long long* t_anc;               // dev [B][R][2]
  int* t_iv;                               // dev [B][R][2]: interval labels (enter, exit) of the tree as verified
};
// per row of z[rows, V]: ids and values of the k best entries (value descending, id ascending) and the row's
// log-sum-exp.  cand: [rows][chunks][16] 64-bit keys, aux: [rows][chunks][2] floats, chunks = ceil(V / 2048)
// (scale: every value is multiplied by it first -- an inverse temperature)
void launch_topk_lse(const float* z, int ldz, int V, int rows, int k, void* cand, float* aux, int* out_ids,
                     float* out_vals, float* out_lse, hipStream_t st, float scale = 1.0f);
// verification at a temperature > 0: lse[row] = log-sum-exp of logits[row] * inv_temp; uniforms [B][R][17]
void launch_accept_sample(const float* logits, int V, const float* lse, float inv_temp, const int* tokens,
                          const int* first_child, const int* n_child, int child_stride, int B, int R,
                          const float* uniforms, int* m, int* acc_idx, int* new_tokens, int* next_tok, hipStream_t st);
void launch_dyn_assign(const DynTree& t, int j, int B, const int* ids, const float* vals, const float* lse, const int* m,
                       hipStream_t st);
void launch_dyn_frontier(const DynTree& t, int j, int B, const int* m, hipStream_t st);
void launch_dyn_finalize(const DynTree& t, int B, int R, const int* m, int* tree_tokens, hipStream_t st);   // (also t.t_iv when set)

// ---- tuning knobs -------------------------------------------------------------------------------
// The shipped library reads no environment variable: every knob is its default.  A build with
// -DCLOVER_ABLATE (kernel-tuning experiments only) reads CLOVER_<NAME> once per process instead, and only
// such a build honours the `dbg` fields of the GEMM descriptors (ablations that skip loads or stores).
#ifdef CLOVER_ABLATE
int tune_int(const char* name, int dflt);
#define CLV_DBG(p, bit) ((p).dbg & (bit))
#else
inline int tune_int(const char*, int dflt) { return dflt; }
#define CLV_DBG(p, bit) 0
#endif

}  // namespace clv
