// Internal declarations shared by the translation units of libclover.so.
// Host-side launch wrappers only: every wrapper validates nothing (the C-ABI layer does) and
// enqueues on the given stream.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

namespace clv {

typedef unsigned short bf16_t;  // raw bfloat16 bit pattern

enum KernelClass {
  KC_EMBED = 0, KC_RMSNORM, KC_GEMM_QKV, KC_ROPE_KV, KC_ATTN, KC_GEMM_WO, KC_GEMM_GATEUP, KC_GEMM_DOWN,
  KC_GEMM_LMHEAD, KC_GEMM_DRAFT, KC_AD_GATE, KC_TOPK, KC_DRAFT_MISC, KC_ACCEPT, KC_COMPACT, KC_ELTWISE, KC_MEGA,
  KC_COUNT
};

// Rows are laid out [B, R]; row (b,i) exists for i < n and is valid iff i < (n_valid ? n_valid[b] : n).
struct RowMap {
  int B, R, n;
  const int* n_valid;  // dev [B] or null
};

struct KVLayout {
  // K: [max_batch][max_seq][n_kv][d]; V (transposed): [max_batch][n_kv][d][max_seq]; one such pair per layer.
  // kvdtype 0: fp32 elements.  kvdtype 1: each cache is two bf16 planes (hi, then lo `plane` elements
  // later) with hi + lo == value to 16 mantissa bits -- the operand format of the MFMA attention.
  int max_batch, max_seq, n_kv, d;
  size_t plane;
};

// ---- generic (fp32 ALU) kernels; wdtype: 0 fp32, 1 bf16 ---------------------------------------
void launch_embed(const void* table, int wdtype, const int* tok, int vocab, float* out, int ldo, int H,
                  RowMap rm, hipStream_t st);
void launch_rmsnorm(const float* x, int ldx, const void* gain, int wdtype, float eps, float* out, int ldo, int H,
                    int rows, hipStream_t st);
void launch_rope_table(const int* base_len, const int* depth /*null: row index*/, float rope_base, int d,
                       float* cos_t, float* sin_t, RowMap rm, hipStream_t st);
void launch_rope_kv_write(const float* qkv, int ldqkv, int qkv_splits, size_t qkv_split_stride, const float* cos_t, const float* sin_t, float* q_out, int ldq,
                          void* k_cache, void* v_cache, int kvdtype, KVLayout kv, const int* base_len, int n_q,
                          RowMap rm, int* err_flag, bf16_t* q_hi /*null: fp32 q_out*/, bf16_t* q_lo, float q_scale,
                          hipStream_t st);
void launch_attn_generic(const float* q, int ldq, const void* k_cache, const void* v_cache, int kvdtype, KVLayout kv,
                         const int* base_len, const unsigned long long* anc /*[n][2]*/, int n_q, float* out, int ldo,
                         bf16_t* out_hi, bf16_t* out_lo /*planes instead of fp32 when non-null*/, RowMap rm,
                         hipStream_t st);
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
void launch_draft_gather(const float* state, const int* tokens, const int* lvl_nodes, const int* parent, int n_lvl,
                         int B, int R, int H, const void* lm_head, int wdtype, int vocab, float* xs, float* e,
                         float* cat /*[rows,2H], second half <- e*/, hipStream_t st);
// state[b][u] <- s rows (also first half of cat)
void launch_draft_scatter_state(const float* s, const int* lvl_nodes, int n_lvl, int B, int R, int H, float* state,
                                float* cat, hipStream_t st);
// root rows: xs_root[b] = a[b][m[b]-1]; state[b][0] = same; tokens[b][0] = next_tok[b][m[b]-1]
void launch_draft_root(const float* a, const int* next_tok, const int* m, int B, int R, int H, float* root_x,
                       float* state, int* tokens, hipStream_t st);
// tokens[b][c] = ids[(b*n_par + par_row[c])*16 + rank[c]] for children c in [c0,c1); skipped when m[b] < 1
void launch_draft_assign(const int* ids, const int* par_row, const int* rank, int c0, int c1, int n_par, int B, int R,
                         const int* m, int* tokens, hipStream_t st);
void launch_add_len(int* len, const int* m, int B, hipStream_t st);

// ---- accept / compact -------------------------------------------------------------------------
void launch_accept_walk(const int* argmax, const int* tokens, const int* first_child, const int* n_child, int n_nodes,
                        int B, int R, const int* n_forced, const int* forced_next, int* m, int* acc_idx,
                        int* new_tokens, int* next_tok, hipStream_t st);
void launch_compact_kv(void* k_cache, void* v_cache, int kvdtype, KVLayout kv, int n_layers, size_t k_layer_elems,
                       size_t v_layer_elems, const int* len, const int* m, const int* acc_idx, int B, int R,
                       hipStream_t st);
void launch_gather_hidden(const float* hidden, const int* acc_idx, const int* m, int B, int R, int H, float* hid_acc,
                          hipStream_t st);
void launch_read_kv(const void* k_cache, const void* v_cache, int kvdtype, KVLayout kv, int b, int slot0, int n_slots,
                    float* k_out, float* v_out, hipStream_t st);
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
  int dbg;                 // timing experiments only (CLOVER_GEMM_DBG): 1 no MFMA, 2 no weight loads, 4 no activation loads
};
bool mfma_gemm_supported(int M, int N, int K, int mode);
int mfma_gemm_pick_splits(int M, int N, int K, int mode);
size_t mfma_gemm_out_bytes(int M, int N, int splits);
void launch_gemm_mfma(const MfmaGemm& g, hipStream_t st);


// ---- MFMA tree attention (head_dim 128, caches as bf16 planes) ---------------------------------
struct AttnParams {
  const bf16_t *q_hi, *q_lo; int ldq;    // [rows, n_q*128] planes: RoPE applied, scaled by 1/sqrt(128)
  const bf16_t* k_hi; size_t k_plane;    // K planes [B][max_seq][n_kv][128]; lo = hi + k_plane
  const bf16_t* v_hi; size_t v_plane;    // V^T planes [B][n_kv][128][max_seq]
  int max_seq, n_kv, n_q;
  const int* base_len;                   // dev [B]
  const unsigned long long* anc;         // dev [n][2]
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
  int dbg;                            // timing experiments only (CLOVER_STREAM_DBG): 1 no activation loads, 2 no stores
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
  int dbg;                            // timing experiments only (CLOVER_PANEL_DBG): 1 no activation loads
};
bool panel_gemm_supported(int M, int N, int K, int epi);
// how many K ranges make the plain panel GEMM fill the chip for a NARROW output (0: not worth it)
int panel_gemm_pick_k_parts(int M, int N, int K);
void launch_gemm_panel(const PanelGemm& g, hipStream_t st);

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
  const int* m;                               // with nodes: sequences with m[b] < 1 are skipped (null: none)
  float* out; int ldo;
  const void* gain; float eps; bf16_t *n_hi, *n_lo;   // gain non-null: planes of RMSNorm(result)*gain, row g, ld H
  bf16_t *c_hi, *c_lo; int ldc;               // non-null: planes of the result, row g
};
bool ad_gate_fused_supported(int H, int heads);
void launch_ad_gate_fused(const AdGateArgs& a, int rows, hipStream_t st);
// root state/token from the last accepted row, its planes (row b, ld H), aug_len[b] += m[b]
void launch_draft_root_fused(const float* a, const int* next_tok, const int* m, int B, int R, int H, float* state,
                             int* tokens, bf16_t* y_hi, bf16_t* y_lo, int* aug_len, hipStream_t st);
// per internal node r of one depth (u = nodes[r]): planes of RMSNorm(state[parent(u)]) * gain (row b*n_lvl + r, ld H),
// planes of the embedding of tokens[u] in (y_hi, y_lo) (ld H) and in the second half of (c_hi, c_lo) (ld 2H)
void launch_draft_level(const float* state, const int* tokens, const int* nodes, const int* parent, int n_lvl, int B,
                        int R, int H, const void* table, int vocab, const void* gain, float eps, bf16_t* a_hi,
                        bf16_t* a_lo, bf16_t* y_hi, bf16_t* y_lo, bf16_t* c_hi, bf16_t* c_lo, hipStream_t st);

// ---- persistent phase-program kernel (M <= 64 rows, bf16 weights, head_dim 128) -------------------
// One cooperative launch walks phases [p_begin, p_end) of a program with a barrier before each phase
// after the first.  Every pointer is a device pointer; buffers written in one phase and read in a later
// one must not be touched by anything else while the launch runs.
//
// XCD sharding (shard != 0).  Workgroups with the same index modulo 8 run on the same XCD and share its
// L2.  When the head and FFN counts divide by 8, XCD x owns head group x and FFN slice x for the whole
// layer: QKV columns -> RoPE -> attention -> merge -> its K slice of the output projection, and gate/up
// columns -> SwiGLU -> its K slice of the down projection.  Inside such a chain data passes through the
// XCD's own L2 (plain stores, an L1 invalidate, an XCD-local barrier of ~1 us); only the two residual
// sums per layer cross XCDs (write-through stores, L2 invalidate, grid barrier of ~4 us).
enum MegaOp { MG_OP_GEMM = 1, MG_OP_REDUCE, MG_OP_ROPE, MG_OP_ATTN, MG_OP_MERGE };
struct MegaSync {
  unsigned xcount[8 * 64];  // grid barrier: arrivals per XCD group (workgroup % 8), one counter per 256 bytes
  unsigned lcount[8 * 64];  // XCD-local barriers: arrivals per XCD group
  unsigned top;             // grid barrier: XCD groups that have completed it
  unsigned abort;           // sticky: a barrier timed out
  unsigned off_tag;         // (launch tag << 3) | (XCC id - workgroup index) mod 8 of workgroup 0: must hold for every workgroup
  unsigned pad[61];
};
struct MegaPhase {
  int op, M;                                   // M: rows b*R + i of the row map, <= 64
  int sync;                                    // barrier before this phase: 0 grid-wide, 1 XCD-local
  int bar_ord;                                 // 1-based ordinal of that barrier among the program's barriers of its kind
  int wt;                                      // 1: outputs are written through (read on other XCDs), 0: plain stores
  int shard;                                   // 0: work spread over all workgroups; GEMM 1: column-sharded, 2: K-sharded;
                                               // ROPE / ATTN / MERGE 1: XCD x handles head group x
  // GEMM: out = X[M,K] * W[N,K]^T
  int N, K, KG, epi;                           // KG K-groups (shard 0: 1, 2, 4, 8 over the XCDs; shard 1: local groups);
                                               // epi 0: fp32 partial per K-group, 1: SwiGLU planes (N = F; W = gate rows,
                                               // then up rows), 2: fp32 out
  const bf16_t *Xhi, *Xlo; int ldx;            // activation planes
  const bf16_t* W; unsigned w_bytes;           // fragment-major weights
  float* Y; int ldy; size_t split_stride;      // GEMM out (epi 0: K-group g at Y + g*split_stride); partials in for REDUCE / ROPE
  bf16_t *Yhi, *Ylo; int ldo;                  // planes out (GEMM epi 1, REDUCE, MERGE)
  const float* ss; int H; float eps;           // [row][4] sums of squares of the row the input planes came from:
                                               // epi 1 / 2 and ROPE scale by rsqrt(sum / H + eps) (the RMSNorm scale)
  int seg_base[3], seg_bnd[3][9];              // shard 1: XCD x owns the 16-column blocks seg_base[s] + [seg_bnd[s][x], seg_bnd[s][x+1])
  int ks_bnd[9];                               // shard 2: XCD x owns the 256-column K stages [ks_bnd[x], ks_bnd[x+1])
  float* lbuf; size_t lbuf_stride;             // shard 1: XCD x's private scratch = lbuf + x*lbuf_stride (floats): QKV partials
                                               // [KG][M][ldy] with LOCAL column indices, then the attention partials
  size_t lo_off, lml_off;                      // float offsets of the attention partial outputs / (max, sum) pairs in it
  // REDUCE: x[g,:] = (tok ? table[tok[g]] : x[g,:]) + sum of KG partials; planes of x*gain; ss_out
  float* x; const bf16_t* gain; float* ss_out; const int* tok; const bf16_t* table; int vocab;
  // ROPE / ATTN / MERGE
  RowMap rm; int n_q, n_kv, max_seq; const int* base_len; int* err_flag;
  const float *cos_t, *sin_t; float q_scale;
  bf16_t *q_hi, *q_lo; int ldq;
  bf16_t* k_hi; size_t k_plane; bf16_t* v_hi; size_t v_plane;   // caches of this layer (lo plane = hi + plane)
  const unsigned long long* anc;
  float *o_part, *ml_part; int rows_total, n_splits;            // shard 0 partial outputs; n_splits in both modes
  int dbg;                                     // timing experiments only (CLOVER_MEGA_DBG), 0 in normal use
};
int mega_grid_size();   // workgroups of a launch on the current device; 0: cooperative launch not available
int mega_barrier_timeout_ticks(long long* out);
int mega_pick_kg(int N, int K, int epi, int grid);
bool mega_gemm_supported(int M, int N, int K);
// stamps: null, or dev [n_phases + 1] wall-clock ticks (phase starts as seen by workgroup 0, then the end)
// gseq_base / lseq_base: grid-wide / XCD-local barriers executed since the counters were zeroed
// check_xcd: compare every workgroup's XCD placement with workgroup 0's at the end (needs a grid barrier in the range)
hipError_t launch_mega(const MegaPhase* prog_dev, int p_begin, int p_end, MegaSync* sync, unsigned gseq_base,
                       unsigned lseq_base, long long limit_ticks, int* err_flag, long long* stamps, int check_xcd,
                       int grid, hipStream_t st);

}  // namespace clv
