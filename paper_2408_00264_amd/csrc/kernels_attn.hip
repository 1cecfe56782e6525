// Tree-masked decode attention on the gfx950 matrix cores (head_dim 128).
//
// For one sequence and one KV head, the G query heads that share it and the N tree nodes form
// G*N query rows; they attend to the L cached keys (all visible) and to the N tree keys, of which
// node u sees exactly those on its own root path (one bit per tree node in anc[u]).  Without a mask table
// (anc == null) the nodes form a chain of any length -- a prompt chunk: node u sees tree keys 0..u, and the key tiles
// behind a node group's last row are skipped.  With interval labels (iv: enter and exit of a depth-first numbering,
// two integers per node) tree key w is visible to node u iff enter[w] <= enter[u] <= exit[w]; the labels of the tree
// keys sit in the LDS behind the stage buffers, so the test is two integer compares against LDS values.
//
// Work split: a workgroup = (sequence, KV head, group of 32 nodes, range of 32-key tiles); its G
// wavefronts are the G query heads.  K and V^T tiles are staged once per workgroup in LDS and
// shared by the heads; every split writes an un-normalised partial (O, running max, running sum)
// and a small kernel merges the splits with the usual log-sum-exp weights.
//
// MFMA mapping (v_mfma_f32_16x16x32_bf16, D[i][j] += sum_k A[i][k] B[j][k]):
//   scores   S^T[key][row] : A = K tile  (16 keys x 32 d),  B = Q (16 rows x 32 d)
//   output   O^T[d][row]   : A = V^T tile (16 d x 32 keys), B = P (16 rows x 32 keys)
// A lane owns one query row in both products (j = lane%16), so the soft-max statistics and the
// rescaling of O never leave the lane, and the eight probabilities a lane computes for the keys
// 8*(lane/16)..+7 of a tile are exactly the B fragment of the second product.
//
// Precision: a random-init stack amplifies bf16 rounding ~20x over 32 layers, so Q, K, V and P are
// all carried as hi + lo bf16 pairs and each product takes three MFMAs (hi*hi, hi*lo, lo*hi).  The
// caches already hold K and V^T as (hi, lo) planes.
#include "clover_internal.h"

#include <algorithm>
#include <cstdlib>
#include <type_traits>

namespace clv {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

union Frag {
  u32x4 u;
  bf16x8 v;
};

// float -> bf16 (round to nearest even) through the hardware conversion (v_cvt_pk_bf16_f32)
__device__ __forceinline__ unsigned a_rn(float a) { return (unsigned)__builtin_bit_cast(unsigned short, (__bf16)a); }
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
// (a, b) -> packed hi pair and packed lo pair, hi + lo == value to 16 mantissa bits: six instructions per pair
__device__ __forceinline__ void a_split2(float a, float b, unsigned& hi, unsigned& lo) {
  const f32x2_t v = {a, b};
  const bf16x2_t h = __builtin_convertvector(v, bf16x2_t);
  const bf16x2_t l = __builtin_convertvector(v - __builtin_convertvector(h, f32x2_t), bf16x2_t);
  hi = __builtin_bit_cast(unsigned, h);
  lo = __builtin_bit_cast(unsigned, l);
}

constexpr int AT_D = 128;         // head dim
constexpr int AT_TK = KV_PAGE;    // keys per tile = one page of the caches
// (WM, a template parameter: wavefronts per query head; a workgroup always covers 32 nodes, a wavefront 32 / WM)
// LDS row strides (bf16).  +32 B: measured on gfx950, ds_read_b128 fragment reads (row = lane % 16, 16-byte piece = lane / 16) run at the full 256 B/clk when the row stride is 32 mod 64 bytes and at half of it with a 16-byte pad.
constexpr int AT_KLD = AT_D + 16;
constexpr int AT_VLD = AT_TK + 16;
constexpr int AT_KPLANE = AT_TK * AT_KLD;
constexpr int AT_VPLANE = AT_D * AT_VLD;
constexpr int AT_KSTAGE = 2 * AT_KPLANE, AT_VSTAGE = 2 * AT_VPLANE;   // one staged tile: K hi, K lo / V^T hi, V^T lo
constexpr int AT_LDS_EL = 2 * AT_KSTAGE + 3 * AT_VSTAGE;              // two K buffers, three V^T buffers
constexpr int AT_MAX_IV = CLOVER_MAX_NODES_INTERVAL;   // interval labels of the tree keys kept in the LDS

template <int G, int WM>
__global__ __launch_bounds__(64 * G * WM) void attn_mfma_kernel(AttnParams p) {
  constexpr int AT_MB = 2 / WM;     // 16-row blocks of nodes per wavefront
  extern __shared__ __attribute__((aligned(16))) bf16_t sm[];  // [2][AT_KSTAGE] [3][AT_VSTAGE] [AT_MAX_IV] labels
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int l16 = lane & 15, g4 = lane >> 4;
  const int split = blockIdx.x, ng = blockIdx.y / p.n_kv, kvh = blockIdx.y % p.n_kv, b = blockIdx.z;
  const RowMap& rm = p.rm;
  const int t0 = split * p.tiles_per_split;
  const int head = kvh * G + wave % G;
  const int nsub = (wave / G) * AT_MB * 16;   // this wavefront's first node within the workgroup's 32

  // ---- staging: 16-byte pieces; K rows are stored in the order the score MFMA consumes them ----
  constexpr int NT = 64 * G * WM;
  constexpr int KSLOTS = 2 * AT_TK * 16, VSLOTS = 2 * AT_D * 4;  // both 1024
  constexpr int KIT = KSLOTS / NT, VIT = VSLOTS / NT;
  // two register sets: while a tile is multiplied, the next one sits in LDS or lands in one set and
  // the one after it is in flight into the other
  u32x4 krA[KIT], vrA[VIT], krB[KIT], vrB[VIT];
  // Key tile t of this sequence is page pages[b * T + t] of the paged caches: the K rows and the V^T columns of
  // (page, KV head) are one contiguous 8 KB block each per plane.  The page number is a scalar that is fetched one
  // load ahead of its use (page_of), and a thread's piece of a block is tid * 16 bytes behind a uniform base, so the
  // loads of a tile need no vector address arithmetic (address registers that alias a staging set would make every
  // new load wait for the ones in flight).
  const KVLayout& kv = p.kv;
  auto page_of = [&](int t) __attribute__((always_inline)) -> int {
    const int lp = (b + kv.b0) * kv.T + min(t, kv.T - 1);
    return kv.pages ? kv.pages[lp] : lp;
  };
  auto load_tile = [&](u32x4 (&kr)[KIT], u32x4 (&vr)[VIT], int page) __attribute__((always_inline)) {
    const size_t blk = ((size_t)page * kv.n_kv + kvh) * (size_t)(KV_PAGE * AT_D);   // elements; K and V^T blocks are equal
    const bf16_t* kb = p.k_hi + blk;
    const bf16_t* vb = p.v_hi + blk;
#pragma unroll
    for (int it = 0; it < KIT; ++it) {
      const int plane = (it * NT) >> 9, first = (it * NT) & 511;   // uniform: NT divides 512
      kr[it] = *(const u32x4*)(kb + plane * p.k_plane + (first + tid) * 8);
    }
#pragma unroll
    for (int it = 0; it < VIT; ++it) {
      const int plane = (it * NT) >> 9, first = (it * NT) & 511;
      vr[it] = *(const u32x4*)(vb + plane * p.v_plane + (first + tid) * 8);
    }
  };
  // The first key tile is requested before anything else is waited for (its address needs the page table only:
  // keys past the cache are clamped and masked later), so its HBM latency overlaps the loads of the lengths,
  // the masks and Q.
  load_tile(krA, vrA, page_of(t0));
  int pg_next = page_of(t0 + 1);   // page of the tile the next load_tile call fetches
  const int nv = rm.n_valid ? min(rm.n_valid[b], rm.n) : rm.n;
  const int L = p.base_len[b];
  if (ng * 32 >= nv || L + nv > p.max_seq) return;  // whole workgroup
  const int total = L + nv;
  const bool chain = p.anc == nullptr && p.iv == nullptr;
  int2* kiv = (int2*)(sm + AT_LDS_EL);   // [AT_MAX_IV] (enter, exit) of the tree keys; published by the first barrier
  if (p.iv)
    for (int w = tid; w < nv; w += NT) kiv[w] = *(const int2*)(p.iv + 2 * ((size_t)b * p.anc_stride + w));
  const int n_tiles = ((chain ? min(total, L + ng * 32 + 32) : total) + AT_TK - 1) / AT_TK;
  const int t1 = min(n_tiles, t0 + p.tiles_per_split);

  // ---- Q fragments (already scaled and split by the RoPE kernel), ancestor masks ----
  Frag qh[AT_MB][4], ql[AT_MB][4];
  unsigned long long a0[AT_MB], a1[AT_MB];
  int my_enter[AT_MB];
#pragma unroll
  for (int mb = 0; mb < AT_MB; ++mb) {
    const int node = ng * 32 + nsub + mb * 16 + l16;
    const bool ok = node < nv;
    const bool bits = !chain && !p.iv;
    a0[mb] = !ok ? 0ull : bits ? p.anc[2 * ((size_t)b * p.anc_stride + node)] : ~0ull;
    a1[mb] = !ok ? 0ull : bits ? p.anc[2 * ((size_t)b * p.anc_stride + node) + 1] : ~0ull;
    my_enter[mb] = ok && p.iv ? p.iv[2 * ((size_t)b * p.anc_stride + node)] : 0;
    const size_t qo = ((size_t)b * rm.R + (ok ? node : 0)) * p.ldq + head * AT_D + g4 * 8;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      qh[mb][ks].u = (u32x4){0u, 0u, 0u, 0u};
      ql[mb][ks].u = (u32x4){0u, 0u, 0u, 0u};
      if (ok) {
        qh[mb][ks].u = *(const u32x4*)(p.q_hi + qo + ks * 32);
        ql[mb][ks].u = *(const u32x4*)(p.q_lo + qo + ks * 32);
      }
    }
  }

  f32x4 O[8][AT_MB];
#pragma unroll
  for (int db = 0; db < 8; ++db)
#pragma unroll
    for (int mb = 0; mb < AT_MB; ++mb) O[db][mb] = (f32x4){0.f, 0.f, 0.f, 0.f};
  float m_run[AT_MB], l_run[AT_MB];
#pragma unroll
  for (int mb = 0; mb < AT_MB; ++mb) { m_run[mb] = -INFINITY; l_run[mb] = 0.f; }

  // LDS: two K buffers (tile i in buffer i % 2) and three V^T buffers (tile i in buffer i % 3): the output product of
  // tile i - 1 runs one iteration behind its scores (see the loop), so V^T of tile i - 1 is still read while tile i + 1
  // is staged.
  bf16_t* const k_lds = sm;
  bf16_t* const v_lds = sm + 2 * AT_KSTAGE;
  auto store_tile = [&](const u32x4 (&kr)[KIT], const u32x4 (&vr)[VIT], int kbuf, int vbuf) __attribute__((always_inline)) {
    bf16_t* kbase = k_lds + kbuf * AT_KSTAGE;
    bf16_t* vbase = v_lds + vbuf * AT_VSTAGE;
#pragma unroll
    for (int it = 0; it < KIT; ++it) {
      const int idx = it * NT + tid, plane = idx >> 9, rem = idx & 511, key = rem >> 4, sl = rem & 15;
      // key k of the tile is row ((k/4)%2)*16 + (k/8)*4 + k%4: sub-tile tt holds keys 8g + 4tt + r at row 4g + r
      const int row = ((key >> 2) & 1) * 16 + (key >> 3) * 4 + (key & 3);
      *(u32x4*)(kbase + plane * AT_KPLANE + row * AT_KLD + sl * 8) = kr[it];
    }
#pragma unroll
    for (int it = 0; it < VIT; ++it) {
      const int idx = it * NT + tid, plane = idx >> 9, rem = idx & 511, dr = rem >> 2, sl = rem & 3;
      *(u32x4*)(vbase + plane * AT_VPLANE + dr * AT_VLD + sl * 8) = vr[it];
    }
  };

  // ---- the three steps of a key tile.  scores: S^T = K Q^T (matrix pipe); soft_max: running statistics, the
  // probabilities as hi/lo fragments and the factor the output so far has to be scaled by (vector ALU);
  // output: O^T += V^T P (matrix pipe). ----
  auto scores = [&](int kbuf, f32x4 (&sc)[2][AT_MB]) __attribute__((always_inline)) {
    const bf16_t* kb = k_lds + kbuf * AT_KSTAGE + l16 * AT_KLD + g4 * 8;
#pragma unroll
    for (int tt = 0; tt < 2; ++tt)
#pragma unroll
      for (int mb = 0; mb < AT_MB; ++mb) sc[tt][mb] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int tt = 0; tt < 2; ++tt)
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        Frag kh, kl;
        kh.u = *(const u32x4*)(kb + tt * 16 * AT_KLD + ks * 32);
        kl.u = *(const u32x4*)(kb + AT_KPLANE + tt * 16 * AT_KLD + ks * 32);
#pragma unroll
        for (int mb = 0; mb < AT_MB; ++mb) {
          sc[tt][mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kl.v, qh[mb][ks].v, sc[tt][mb], 0, 0, 0);
          sc[tt][mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kh.v, ql[mb][ks].v, sc[tt][mb], 0, 0, 0);
          sc[tt][mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kh.v, qh[mb][ks].v, sc[tt][mb], 0, 0, 0);
        }
      }
  };
  auto soft_max_t = [&](int t, const f32x4 (&sc)[2][AT_MB], Frag (&ph)[AT_MB], Frag (&pl)[AT_MB], auto cachedc)
                        __attribute__((always_inline)) {
    constexpr bool CACHED = decltype(cachedc)::value;  // every key of the tile is a cached token: no tree mask
#pragma unroll
    for (int mb = 0; mb < AT_MB; ++mb) {
      float sv[8];
      float tmax = -INFINITY;
#pragma unroll
      for (int e = 0; e < 8; ++e) {  // e-th key of this lane: slot t*32 + 8*g4 + e
        const int j = t * AT_TK + 8 * g4 + e;
        bool vis = CACHED || j < L;
        if (!CACHED && !vis && j < total) {
          const int wn = j - L;
          if (chain) vis = wn <= ng * 32 + nsub + mb * 16 + l16;
          else if (p.iv) { const int2 ke = kiv[wn]; vis = ke.x <= my_enter[mb] && my_enter[mb] <= ke.y; }
          else vis = ((wn < 64 ? (a0[mb] >> wn) : (a1[mb] >> (wn - 64))) & 1ull) != 0ull;
        }
        if (a0[mb] == 0ull && a1[mb] == 0ull) vis = false;  // padding row
        sv[e] = vis ? sc[e >> 2][mb][e & 3] : -INFINITY;
        tmax = fmaxf(tmax, sv[e]);
      }
      tmax = fmaxf(tmax, __shfl_xor(tmax, 16, 64));
      tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
      const float m_new = fmaxf(m_run[mb], tmax);
      const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
      const float corr = __expf(m_run[mb] - m_safe);  // exp(-inf) = 0 on the first visible tile
      float pe[8], psum = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) { pe[e] = __expf(sv[e] - m_safe); psum += pe[e]; }
      l_run[mb] = l_run[mb] * corr + psum;
      m_run[mb] = m_new;
      // the running maximum rarely moves after the first tiles: rescale only when some row of the wavefront needs it
      // (every output product issued before this point has been accumulated by the time the scaling reads O)
      if (__builtin_amdgcn_ballot_w64(corr != 1.0f) != 0ull) {
#pragma unroll
        for (int db = 0; db < 8; ++db) O[db][mb] *= corr;
      }
      unsigned h, l;
      a_split2(pe[0], pe[1], h, l); ph[mb].u.x = h; pl[mb].u.x = l;
      a_split2(pe[2], pe[3], h, l); ph[mb].u.y = h; pl[mb].u.y = l;
      a_split2(pe[4], pe[5], h, l); ph[mb].u.z = h; pl[mb].u.z = l;
      a_split2(pe[6], pe[7], h, l); ph[mb].u.w = h; pl[mb].u.w = l;
    }
  };
  auto soft_max = [&](int t, const f32x4 (&sc)[2][AT_MB], Frag (&ph)[AT_MB], Frag (&pl)[AT_MB]) __attribute__((always_inline)) {
    // (specialised only where the register file has room for both versions)
    if ((G == 2 || G == 4 || WM == 2) && (t + 1) * AT_TK <= L) soft_max_t(t, sc, ph, pl, std::true_type{});  // uniform
    else soft_max_t(t, sc, ph, pl, std::false_type{});
  };
  auto output = [&](int vbuf, const Frag (&ph)[AT_MB], const Frag (&pl)[AT_MB]) __attribute__((always_inline)) {
    const bf16_t* vb = v_lds + vbuf * AT_VSTAGE + l16 * AT_VLD + g4 * 8;
#pragma unroll
    for (int db = 0; db < 8; ++db) {
      Frag vh, vl;
      vh.u = *(const u32x4*)(vb + db * 16 * AT_VLD);
      vl.u = *(const u32x4*)(vb + AT_VPLANE + db * 16 * AT_VLD);
#pragma unroll
      for (int mb = 0; mb < AT_MB; ++mb) {
        O[db][mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vl.v, ph[mb].v, O[db][mb], 0, 0, 0);
        O[db][mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vh.v, pl[mb].v, O[db][mb], 0, 0, 0);
        O[db][mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vh.v, ph[mb].v, O[db][mb], 0, 0, 0);
      }
    }
  };

  // ---- the loop over this split's key tiles.  Staging: with two register sets the tile after next is in flight
  // while the next one waits in the other set; with one set (few threads per workgroup: all the register file holds)
  // the next tile is in flight.  One barrier per tile: tile i + 1 is written to the LDS at the end of iteration i.
  //
  // Order of the steps (two wavefronts per query head): scores of tile i, output product of tile i - 1, soft-max of
  // tile i.  The fragment reads of the output product are then in flight behind the score products instead of
  // behind the soft-max, on whose result they do not depend; measured 4 % faster over 8192 keys than scores,
  // soft-max, output of the same tile.  Running the second four wavefronts of a workgroup one step out of phase
  // with the first four, so that one of a SIMD's pair multiplies while the other exponentiates, was measured too
  // and gains nothing: on this chip a SIMD's matrix and vector instructions hardly overlap, whichever wavefront
  // they come from (24 MFMA in one wavefront and 96 fma in the other take 86-100 % of the sum of their times;
  // probes/mfma_valu_overlap.hip).  Every accumulator sees the same operations in the same order in all of these
  // variants. ----
  if (t0 < t1) {  // uniform over the workgroup
    const int n = t1 - t0;
    constexpr bool TWO_SETS = G * WM >= 4;
    // (one wavefront per query head covers 32 nodes and has no registers left to carry a tile's probabilities
    // into the next iteration: it runs scores, soft-max and output of tile i back to back)
    constexpr bool PIPELINED = WM == 2;
    f32x4 sc[2][AT_MB];
    Frag ph[AT_MB], pl[AT_MB];
    auto iteration = [&](int i, int kb, int vcur, int vprev) __attribute__((always_inline)) {
      scores(kb, sc);
      if constexpr (PIPELINED) {
        if (i > 0) output(vprev, ph, pl);
        soft_max(t0 + i, sc, ph, pl);
      } else {
        soft_max(t0 + i, sc, ph, pl);
        output(vcur, ph, pl);
      }
    };
    if constexpr (TWO_SETS) {
      if (n > 1) { load_tile(krB, vrB, pg_next); pg_next = page_of(t0 + 2); }
    }
    store_tile(krA, vrA, 0, 0);
    __syncthreads();
    int vcur = 0, vprev = 2;   // V^T buffers of tiles i and i - 1
    for (int i = 0; i < n; i += 2) {
      if constexpr (TWO_SETS) {
        if (i + 2 < n) { load_tile(krA, vrA, pg_next); pg_next = page_of(t0 + i + 3); }
      } else {
        if (i + 1 < n) { load_tile(krA, vrA, pg_next); pg_next = page_of(t0 + i + 2); }
      }
      iteration(i, 0, vcur, vprev);
      vprev = vcur; vcur = vcur == 2 ? 0 : vcur + 1;
      if (i + 1 >= n) break;
      if constexpr (TWO_SETS) store_tile(krB, vrB, 1, vcur); else store_tile(krA, vrA, 1, vcur);
      __syncthreads();
      if constexpr (TWO_SETS) {
        if (i + 3 < n) { load_tile(krB, vrB, pg_next); pg_next = page_of(t0 + i + 4); }
      } else {
        if (i + 2 < n) { load_tile(krA, vrA, pg_next); pg_next = page_of(t0 + i + 3); }
      }
      iteration(i + 1, 1, vcur, vprev);
      vprev = vcur; vcur = vcur == 2 ? 0 : vcur + 1;
      if (i + 2 < n) store_tile(krA, vrA, 0, vcur);
      __syncthreads();
    }
    // the output product still owed for the last tile (its V^T buffer is vprev after the final rotation)
    if constexpr (PIPELINED) output(vprev, ph, pl);
  }

  // ---- partial result of this split ----
#pragma unroll
  for (int mb = 0; mb < AT_MB; ++mb) {
    const int node = ng * 32 + nsub + mb * 16 + l16;
    float lsum = l_run[mb];
    lsum += __shfl_xor(lsum, 16, 64);
    lsum += __shfl_xor(lsum, 32, 64);
    if (node >= nv) continue;
    const size_t prow = ((size_t)split * p.rows_total + (size_t)b * rm.R + node) * p.n_q + head;
#pragma unroll
    for (int db = 0; db < 8; ++db) {
      const f32x4 v = O[db][mb];
      *(float4*)(p.o_part + prow * AT_D + db * 16 + 4 * g4) = make_float4(v[0], v[1], v[2], v[3]);
    }
    if (g4 == 0) {
      p.ml_part[prow * 2] = m_run[mb];
      p.ml_part[prow * 2 + 1] = lsum;
    }
  }
}

// merge the splits of one (row, head): out = sum_s e^{m_s - M} O_s / sum_s e^{m_s - M} l_s, as planes.
// One thread owns four adjacent channels of one head; the (m, l) pairs and then the partial rows of
// all splits are loaded as one batch each, so a thread waits for memory twice, not once per split.
constexpr int MG_HEADS = 8;   // heads per workgroup (32 threads each)
constexpr int MG_MAXS = 16;   // >= the largest split count the launcher picks
__global__ __launch_bounds__(MG_HEADS * 32) void attn_merge_kernel(const float* __restrict__ o_part,
                                                                    const float* __restrict__ ml_part, int n_splits,
                                                                    int rows_total, int n_q, bf16_t* __restrict__ out_hi,
                                                                    bf16_t* __restrict__ out_lo, int ldo, RowMap rm) {
  const int i = blockIdx.x, b = blockIdx.y;
  const int head = blockIdx.z * MG_HEADS + (threadIdx.x >> 5), d4 = (threadIdx.x & 31) * 4;
  const int nv = rm.n_valid ? min(rm.n_valid[b], rm.n) : rm.n;
  if (i >= nv || head >= n_q) return;
  const size_t row = (size_t)b * rm.R + i;
  const size_t sstride = (size_t)rows_total * n_q;   // (row, head) pairs per split
  const size_t pr0 = row * n_q + head;
  float2 ml[MG_MAXS];
#pragma unroll
  for (int s = 0; s < MG_MAXS; ++s)
    ml[s] = s < n_splits ? *(const float2*)(ml_part + (pr0 + s * sstride) * 2) : make_float2(-INFINITY, 0.f);
  float4 o[MG_MAXS];
#pragma unroll
  for (int s = 0; s < MG_MAXS; ++s)
    o[s] = s < n_splits ? *(const float4*)(o_part + (pr0 + s * sstride) * AT_D + d4) : make_float4(0.f, 0.f, 0.f, 0.f);
  float M = -INFINITY;
#pragma unroll
  for (int s = 0; s < MG_MAXS; ++s) M = fmaxf(M, ml[s].x);
  float4 num = make_float4(0.f, 0.f, 0.f, 0.f);
  float den = 0.f;
#pragma unroll
  for (int s = 0; s < MG_MAXS; ++s) {  // split order: the sum does not depend on how the loads were batched
    const float wgt = ml[s].x == -INFINITY ? 0.f : __expf(ml[s].x - M);
    den += wgt * ml[s].y;
    num.x += wgt * o[s].x; num.y += wgt * o[s].y; num.z += wgt * o[s].z; num.w += wgt * o[s].w;
  }
  const float v[4] = {num.x / den, num.y / den, num.z / den, num.w / den};
  unsigned h[4], l[4];
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    h[r] = a_rn(v[r]);
    l[r] = a_rn(v[r] - __uint_as_float(h[r] << 16));
  }
  *(uint2*)(out_hi + row * ldo + head * AT_D + d4) = make_uint2(h[0] | (h[1] << 16), h[2] | (h[3] << 16));
  *(uint2*)(out_lo + row * ldo + head * AT_D + d4) = make_uint2(l[0] | (l[1] << 16), l[2] | (l[3] << 16));
}

bool attn_mfma_supported(int head_dim, int n_q, int n_kv, int max_seq) {
  const int g = n_q / n_kv;
  return head_dim == AT_D && (g == 1 || g == 2 || g == 4 || g == 8) && max_seq % KV_PAGE == 0 && max_seq >= KV_PAGE;
}

template <int G, int WM>
static void launch_attn_one(const AttnParams& p, dim3 grid, hipStream_t st) {
  constexpr size_t lds = (size_t)AT_LDS_EL * sizeof(bf16_t) + AT_MAX_IV * sizeof(int2);
  static bool attr_done = false;
  if (!attr_done) {
    hipFuncSetAttribute((const void*)attn_mfma_kernel<G, WM>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    attr_done = true;
  }
  attn_mfma_kernel<G, WM><<<grid, 64 * G * WM, lds, st>>>(p);
}

void launch_attn_mfma(AttnParams p, int max_total_keys, bf16_t* out_hi, bf16_t* out_lo, int ldo, hipStream_t st) {
  const int g = p.n_q / p.n_kv;
  const int node_groups = (p.rm.n + 31) / 32;
  const int n_tiles = (max_total_keys + AT_TK - 1) / AT_TK;
  // about one workgroup per CU (two on a CU do not overlap: a CU finishes one key tile per ~4 us either way, so a
  // launch of 1.5 workgroups per CU takes as long as one of 2), at least two tiles per split, within the partial buffer
  const int target = tune_int("CLOVER_ATTN_WGS", 256);
  int splits = std::max(1, target / (p.rm.B * p.n_kv * node_groups));
  splits = std::max(1, std::min(std::min(splits, std::min(p.max_splits, MG_MAXS)), (n_tiles + 1) / 2));
  p.tiles_per_split = (n_tiles + splits - 1) / splits;
  p.n_splits = (n_tiles + p.tiles_per_split - 1) / p.tiles_per_split;
  dim3 grid(p.n_splits, node_groups * p.n_kv, p.rm.B);
  // Two wavefronts per head (16 nodes each) share a SIMD, so one's matrix products overlap the other's soft-max
  // arithmetic, and both share the staged K / V^T tile.
  const int wm1 = tune_int("CLOVER_ATTN_WM1", 0);
  switch (g) {
    case 1: if (wm1) launch_attn_one<1, 1>(p, grid, st); else launch_attn_one<1, 2>(p, grid, st); break;
    case 2: if (wm1) launch_attn_one<2, 1>(p, grid, st); else launch_attn_one<2, 2>(p, grid, st); break;
    case 4: if (wm1) launch_attn_one<4, 1>(p, grid, st); else launch_attn_one<4, 2>(p, grid, st); break;
    default: launch_attn_one<8, 1>(p, grid, st); break;
  }
  attn_merge_kernel<<<dim3(p.rm.n, p.rm.B, (p.n_q + MG_HEADS - 1) / MG_HEADS), MG_HEADS * 32, 0, st>>>(
      p.o_part, p.ml_part, p.n_splits, p.rows_total, p.n_q, out_hi, out_lo, ldo, p.rm);
}

}  // namespace clv
