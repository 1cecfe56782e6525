// Dynamic (score-pruned) draft tree: the kernels between the draft head's LM-head passes.
//
// Candidates of one sequence are numbered in creation order: 0 = root, then the depth-1 candidates in rank
// order, then for every depth the children of the expanded candidates in (expansion slot, rank) order, so the
// id of a candidate encodes its depth, the slot of its parent in that depth's frontier and its rank.  A
// candidate's score is the sum of the draft log-probabilities along its root path.  Per depth the best
// candidates (score descending, lower id first) are expanded; at the end the best n_nodes - 1 candidates
// (score descending, shallower first, lower id first) become the tree, numbered breadth-first (depth, parent's
// number, rank), and the per-sequence topology tables the verification pass reads are written.
#include "clover_internal.h"

#include <climits>

namespace clv {

namespace {

__device__ __forceinline__ float d_wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
__device__ __forceinline__ float d_wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ unsigned long long d_wave_max_u64(unsigned long long v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    unsigned lo = __shfl_xor((unsigned)(v & 0xFFFFFFFFull), o, 64);
    unsigned hi = __shfl_xor((unsigned)(v >> 32), o, 64);
    unsigned long long w = ((unsigned long long)hi << 32) | lo;
    v = w > v ? w : v;
  }
  return v;
}
// order-preserving 64-bit key of (value, id): larger value first, then the smaller id
__device__ __forceinline__ unsigned long long d_key(float v, int id) {
  v = v + 0.0f;
  unsigned u = __float_as_uint(v);
  u = (u & 0x80000000u) ? ~u : (u | 0x80000000u);
  return ((unsigned long long)u << 32) | (unsigned long long)(0xFFFFFFFFu - (unsigned)id);
}
__device__ __forceinline__ float d_key_value(unsigned long long key) {
  const unsigned u = (unsigned)(key >> 32);
  return __uint_as_float((u & 0x80000000u) ? (u & 0x7FFFFFFFu) : ~u);
}
__device__ __forceinline__ unsigned long long d_block_max_u64(unsigned long long v, unsigned long long* red) {
  v = d_wave_max_u64(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  unsigned long long r = red[0];
  r = red[1] > r ? red[1] : r;
  r = red[2] > r ? red[2] : r;
  r = red[3] > r ? red[3] : r;
  return r;
}

constexpr int DY_CHUNK = 2048;
constexpr int DY_EPT = DY_CHUNK / 256;

// stage 1: per 2048-wide chunk of a row of logits, its k best (value, id) keys, its maximum and the sum of
// exp(value - maximum) (the pieces of the row's log-sum-exp)
__global__ __launch_bounds__(256) void topk_lse_stage1_kernel(const float* __restrict__ z, int ldz, int V, int k,
                                                              unsigned long long* __restrict__ cand,
                                                              float* __restrict__ aux, float scale) {
  __shared__ unsigned long long red[4];
  __shared__ float fred[4];
  const int chunk = blockIdx.x, row = blockIdx.y, chunks = gridDim.x;
  unsigned long long key[DY_EPT];
  float val[DY_EPT];
  float mx = -INFINITY;
#pragma unroll
  for (int e = 0; e < DY_EPT; ++e) {
    const int id = chunk * DY_CHUNK + e * 256 + threadIdx.x;
    val[e] = id < V ? z[(size_t)row * ldz + id] * scale : -INFINITY;
    key[e] = id < V ? d_key(val[e], id) : 0ull;
    mx = fmaxf(mx, val[e]);
  }
  mx = d_wave_max(mx);
  if ((threadIdx.x & 63) == 0) fred[threadIdx.x >> 6] = mx;
  __syncthreads();
  mx = fmaxf(fmaxf(fred[0], fred[1]), fmaxf(fred[2], fred[3]));
  __syncthreads();
  float sm = 0.f;
#pragma unroll
  for (int e = 0; e < DY_EPT; ++e) sm += val[e] == -INFINITY ? 0.f : expf(val[e] - mx);
  sm = d_wave_sum(sm);
  if ((threadIdx.x & 63) == 0) fred[threadIdx.x >> 6] = sm;
  __syncthreads();
  if (threadIdx.x == 0) {
    aux[((size_t)row * chunks + chunk) * 2] = mx;
    aux[((size_t)row * chunks + chunk) * 2 + 1] = fred[0] + fred[1] + fred[2] + fred[3];
  }
  for (int r = 0; r < k; ++r) {
    unsigned long long best = 0ull;
#pragma unroll
    for (int e = 0; e < DY_EPT; ++e) best = key[e] > best ? key[e] : best;
    best = d_block_max_u64(best, red);
#pragma unroll
    for (int e = 0; e < DY_EPT; ++e)
      if (key[e] == best) key[e] = 0ull;
    if (threadIdx.x == 0) cand[((size_t)row * chunks + chunk) * 16 + r] = best;
  }
}

// stage 2: the row's k best ids and values, and its log-sum-exp (chunks merged in chunk order by one thread,
// so the sum does not depend on the launch shape)
__global__ __launch_bounds__(256) void topk_lse_stage2_kernel(const unsigned long long* __restrict__ cand,
                                                              const float* __restrict__ aux, int chunks, int k,
                                                              int* __restrict__ out_ids, float* __restrict__ out_vals,
                                                              float* __restrict__ out_lse) {
  __shared__ unsigned long long red[4];
  const int row = blockIdx.x;
  const int total = chunks * k;
  unsigned long long key[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const int idx = e * 256 + threadIdx.x;
    key[e] = idx < total ? cand[((size_t)row * chunks + idx / k) * 16 + idx % k] : 0ull;
  }
  if (threadIdx.x == 0) {
    float M = -INFINITY;
    for (int c = 0; c < chunks; ++c) M = fmaxf(M, aux[((size_t)row * chunks + c) * 2]);
    float S = 0.f;
    for (int c = 0; c < chunks; ++c) S += aux[((size_t)row * chunks + c) * 2 + 1] * expf(aux[((size_t)row * chunks + c) * 2] - M);
    out_lse[row] = M + logf(S);
  }
  for (int r = 0; r < k; ++r) {
    unsigned long long best = 0ull;
#pragma unroll
    for (int e = 0; e < 8; ++e) best = key[e] > best ? key[e] : best;
    best = d_block_max_u64(best, red);
#pragma unroll
    for (int e = 0; e < 8; ++e)
      if (key[e] == best) key[e] = 0ull;
    if (threadIdx.x == 0) {
      out_ids[row * 16 + r] = (int)(0xFFFFFFFFu - (unsigned)(best & 0xFFFFFFFFull));
      out_vals[row * 16 + r] = d_key_value(best);
    }
  }
}

// children of the candidates expanded at depth j: token, cumulative score, parent
__global__ void dyn_assign_kernel(DynTree t, int j, const int* __restrict__ ids, const float* __restrict__ vals,
                                  const float* __restrict__ lse, const int* __restrict__ m) {
  const int r = blockIdx.x, b = blockIdx.y, i = threadIdx.x;
  if (i >= t.topk || m[b] < 1) return;
  const int row = b * t.F[j] + r;
  const int par = j == 0 ? 0 : t.frontier[((size_t)b * CLOVER_MAX_DEPTH + j) * DYN_MAX_FRONT + r];
  const int cid = t.off[j + 1] + r * t.topk + i;
  const size_t o = (size_t)b * t.C;
  t.cand_tok[o + cid] = ids[row * 16 + i];
  t.cand_score[o + cid] = (j == 0 ? 0.f : t.cand_score[o + par]) + (vals[row * 16 + i] - lse[row]);
  t.cand_par[o + cid] = par;
}

// frontier of depth j: the F[j] best of its candidates (score descending, lower id first), in that order
__global__ __launch_bounds__(256) void dyn_frontier_kernel(DynTree t, int j, const int* __restrict__ m) {
  __shared__ float sc[DYN_MAX_CAND];
  const int b = blockIdx.x, tid = threadIdx.x;
  if (m[b] < 1) return;
  const int n = t.off[j + 1] - t.off[j];
  const size_t o = (size_t)b * t.C;
  if (tid < n) sc[tid] = t.cand_score[o + t.off[j] + tid];
  __syncthreads();
  if (tid >= n) return;
  int better = 0;
  for (int u = 0; u < n; ++u) better += (sc[u] > sc[tid] || (sc[u] == sc[tid] && u < tid)) ? 1 : 0;
  if (better < t.F[j]) t.frontier[((size_t)b * CLOVER_MAX_DEPTH + j) * DYN_MAX_FRONT + better] = t.off[j] + tid;
}

// selection of the tree and its breadth-first numbering; per-sequence topology tables
__global__ __launch_bounds__(DYN_MAX_CAND) void dyn_finalize_kernel(DynTree t, int R, const int* __restrict__ m,
                                                                   int* __restrict__ tree_tokens) {
  __shared__ float sc[DYN_MAX_CAND];
  __shared__ int dep[DYN_MAX_CAND], par[DYN_MAX_CAND], sel[DYN_MAX_CAND], nid[DYN_MAX_CAND];
  __shared__ int n_child[CLOVER_MAX_NODES], first_child[CLOVER_MAX_NODES];
  __shared__ unsigned long long anc[CLOVER_MAX_NODES][2];
  __shared__ int pnode[CLOVER_MAX_NODES], sub[CLOVER_MAX_NODES], ent[CLOVER_MAX_NODES];   // parent, subtree size, enter label
  __shared__ int level_count;
  const int b = blockIdx.x, c = threadIdx.x;
  if (m[b] < 1) return;
  const size_t o = (size_t)b * t.C;
  const bool live = c < t.C;
  int my_dep = 0;
  if (live) {
    for (int j = 1; j <= t.D; ++j) my_dep += c >= t.off[j] ? 1 : 0;
    sc[c] = c == 0 ? INFINITY : t.cand_score[o + c];
    dep[c] = my_dep;
    par[c] = c == 0 ? 0 : t.cand_par[o + c];
  }
  if (c < CLOVER_MAX_NODES) { n_child[c] = 0; first_child[c] = INT_MAX; anc[c][0] = anc[c][1] = 0ull; }
  __syncthreads();
  int keep = 0;
  if (live) {
    int better = 0;   // candidates (the root included) that come before this one
    for (int u = 0; u < t.C; ++u) {
      if (u == c) continue;
      const bool first = sc[u] > sc[c] || (sc[u] == sc[c] && (dep[u] < dep[c] || (dep[u] == dep[c] && u < c)));
      better += first ? 1 : 0;
    }
    keep = better < t.N ? 1 : 0;
    sel[c] = keep;
    if (c == 0) nid[0] = 0;
  }
  int base = 1;
  for (int j = 1; j <= t.D; ++j) {
    if (c == 0) level_count = 0;
    __syncthreads();
    if (live && keep && my_dep == j) {
      const int rk = (c - t.off[j]) % t.topk;
      const int key = nid[par[c]] * 16 + rk;
      int pos = 0;
      for (int u = t.off[j]; u < t.off[j + 1]; ++u)
        if (sel[u] && u != c) pos += (nid[par[u]] * 16 + (u - t.off[j]) % t.topk) < key ? 1 : 0;
      nid[c] = base + pos;
      atomicAdd(&level_count, 1);
    }
    __syncthreads();
    base += level_count;
    __syncthreads();
  }
  // tables
  const size_t ro = (size_t)b * R;
  if (live && keep) {
    const int node = nid[c];
    const int pn = c == 0 ? -1 : nid[par[c]];
    tree_tokens[ro + node] = t.cand_tok[o + c];
    t.t_parent[ro + node] = pn;
    t.t_rank[ro + node] = c == 0 ? 0 : (c - t.off[my_dep]) % t.topk;
    t.t_depth[ro + node] = my_dep;
    t.t_keep[ro + node] = c;
    pnode[node] = pn;
    if (c > 0) { atomicAdd(&n_child[pn], 1); atomicMin(&first_child[pn], node); }
  }
  if (c == 0) anc[0][0] = 1ull;
  for (int j = 1; j <= t.D; ++j) {
    __syncthreads();
    if (live && keep && my_dep == j) {
      const int node = nid[c], pn = nid[par[c]];
      anc[node][0] = anc[pn][0];
      anc[node][1] = anc[pn][1];
      anc[node][node >> 6] |= 1ull << (node & 63);
    }
  }
  __syncthreads();
  // interval labels of a depth-first numbering (the linear-size form of the mask): subtree sizes bottom-up (children
  // have larger numbers than their parents and are numbered consecutively), then enter labels top-down
  if (c == 0) {
    for (int u = 0; u < t.N; ++u) sub[u] = 1;
    for (int u = t.N - 1; u >= 1; --u) sub[pnode[u]] += sub[u];
    ent[0] = 0;
    for (int u = 0; u < t.N; ++u) {
      int e = ent[u] + 1;
      for (int k = 0; k < n_child[u]; ++k) { ent[first_child[u] + k] = e; e += sub[first_child[u] + k]; }
    }
  }
  __syncthreads();
  if (c < t.N) {
    t.t_n_child[ro + c] = n_child[c];
    t.t_first_child[ro + c] = n_child[c] ? first_child[c] : 0;
    t.t_anc[(ro + c) * 2] = anc[c][0];
    t.t_anc[(ro + c) * 2 + 1] = anc[c][1];
    t.t_iv[(ro + c) * 2] = ent[c];
    t.t_iv[(ro + c) * 2 + 1] = ent[c] + sub[c] - 1;
  }
}

// Verification at a temperature > 0 (one 1024-thread workgroup per sequence).  Thread 0 walks the tree: at node u
// with p = softmax(logits[u] / T), the children are tried in index order, child i accepted when
// uniforms[u][i] < p(token) / (1 - mass of the children already refused).  When none is accepted (or u is a leaf)
// the whole workgroup draws the next token from what is left of p (refused tokens removed) by inverting its
// cumulative sum in token order with uniforms[u][16]; sums are carried in double precision.
constexpr int SAMPLE_THREADS = 1024;
__global__ __launch_bounds__(SAMPLE_THREADS) void accept_sample_kernel(
    const float* __restrict__ logits, int V, const float* __restrict__ lse, float inv_temp, const int* __restrict__ tokens,
    const int* __restrict__ first_child, const int* __restrict__ n_child, int child_stride, int R,
    const float* __restrict__ uniforms, int* __restrict__ m, int* __restrict__ acc_idx, int* __restrict__ new_tokens,
    int* __restrict__ next_tok) {
  __shared__ int s_u, s_len, s_nk, s_kid_tok[CLOVER_MAX_RANK], s_pick;
  __shared__ double s_part[SAMPLE_THREADS / 64], s_total;
  const int b = blockIdx.x, tid = threadIdx.x;
  const size_t o = (size_t)b * R;
  first_child += (size_t)b * child_stride;
  n_child += (size_t)b * child_stride;
  if (tid == 0) {
    int u = 0, len = 1;
    acc_idx[o] = 0;
    for (;;) {
      const float* zr = logits + (o + u) * (size_t)V;
      const float l = lse[o + u];
      const int c0 = first_child[u], nk = min(n_child[u], CLOVER_MAX_RANK);
      double refused = 0.0;
      int accepted = -1;
      for (int i = 0; i < nk; ++i) {
        const int x = tokens[o + c0 + i];
        const double px = (x >= 0 && x < V) ? exp((double)(zr[x] * inv_temp) - (double)l) : 0.0;
        const double a = px / fmax(1.0 - refused, 1e-300);
        if ((double)uniforms[(o + u) * 17 + i] < a) { accepted = c0 + i; break; }
        refused += px;
      }
      if (accepted < 0 || len >= R) break;
      u = accepted;
      acc_idx[o + len++] = u;
    }
    s_u = u; s_len = len;
    const int nk = min(n_child[u], CLOVER_MAX_RANK);
    s_nk = nk;
    for (int i = 0; i < nk; ++i) s_kid_tok[i] = tokens[o + first_child[u] + i];
    s_pick = V - 1;
  }
  __syncthreads();
  const int u = s_u, nk = s_nk;
  const float* zr = logits + (o + u) * (size_t)V;
  const double l = (double)lse[o + u];
  // each thread owns a contiguous range of token ids
  const int per = (V + SAMPLE_THREADS - 1) / SAMPLE_THREADS;
  const int t0 = tid * per, t1 = min(V, t0 + per);
  auto rest = [&](int t) -> double {
    for (int i = 0; i < nk; ++i)
      if (s_kid_tok[i] == t) return 0.0;
    return exp((double)(zr[t] * inv_temp) - l);
  };
  double mine = 0.0;
  for (int t = t0; t < t1; ++t) mine += rest(t);
  // inclusive scan over the threads: wavefront scan, then the wavefront totals
  double incl = mine;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const double v = __shfl_up(incl, d, 64);
    if ((tid & 63) >= d) incl += v;
  }
  if ((tid & 63) == 63) s_part[tid >> 6] = incl;
  __syncthreads();
  if (tid == 0) {
    double run = 0.0;
    for (int w = 0; w < SAMPLE_THREADS / 64; ++w) { const double v = s_part[w]; s_part[w] = run; run += v; }
    s_total = run;
  }
  __syncthreads();
  const double before = s_part[tid >> 6] + incl - mine;      // mass of all smaller token ids
  const double target = (double)uniforms[(o + u) * 17 + 16] * s_total;
  if (mine > 0.0 && before <= target && target < before + mine) {
    double run = before;
    int pick = t1 - 1;
    for (int t = t0; t < t1; ++t) {
      run += rest(t);
      if (run > target) { pick = t; break; }
    }
    s_pick = pick;   // exactly one thread's range contains the target
  }
  __syncthreads();
  if (tid == 0) {
    const int len = s_len, bonus = s_pick;
    for (int j = 1; j < len; ++j) {
      const int t = tokens[o + acc_idx[o + j]];
      new_tokens[o + j - 1] = t;
      next_tok[o + j - 1] = t;
    }
    new_tokens[o + len - 1] = bonus;
    next_tok[o + len - 1] = bonus;
    m[b] = len;
  }
}

}  // namespace

void launch_accept_sample(const float* logits, int V, const float* lse, float inv_temp, const int* tokens,
                          const int* first_child, const int* n_child, int child_stride, int B, int R,
                          const float* uniforms, int* m, int* acc_idx, int* new_tokens, int* next_tok, hipStream_t st) {
  accept_sample_kernel<<<B, SAMPLE_THREADS, 0, st>>>(logits, V, lse, inv_temp, tokens, first_child, n_child, child_stride, R,
                                                     uniforms, m, acc_idx, new_tokens, next_tok);
}

void launch_topk_lse(const float* z, int ldz, int V, int rows, int k, void* cand, float* aux, int* out_ids,
                     float* out_vals, float* out_lse, hipStream_t st, float scale) {
  if (rows <= 0) return;
  const int chunks = (V + DY_CHUNK - 1) / DY_CHUNK;
  topk_lse_stage1_kernel<<<dim3(chunks, rows), 256, 0, st>>>(z, ldz, V, k, (unsigned long long*)cand, aux, scale);
  topk_lse_stage2_kernel<<<rows, 256, 0, st>>>((const unsigned long long*)cand, aux, chunks, k, out_ids, out_vals, out_lse);
}
void launch_dyn_assign(const DynTree& t, int j, int B, const int* ids, const float* vals, const float* lse, const int* m,
                       hipStream_t st) {
  dyn_assign_kernel<<<dim3(t.F[j], B), 16, 0, st>>>(t, j, ids, vals, lse, m);
}
void launch_dyn_frontier(const DynTree& t, int j, int B, const int* m, hipStream_t st) {
  dyn_frontier_kernel<<<B, 256, 0, st>>>(t, j, m);
}
void launch_dyn_finalize(const DynTree& t, int B, int R, const int* m, int* tree_tokens, hipStream_t st) {
  dyn_finalize_kernel<<<B, DYN_MAX_CAND, 0, st>>>(t, R, m, tree_tokens);
}

}  // namespace clv
