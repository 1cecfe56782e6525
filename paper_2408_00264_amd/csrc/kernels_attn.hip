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
// A staged tile lies in the LDS fragment by fragment: 1 KB blocks in which lane l's 16 bytes sit at l * 16, exactly what
// one 16x32 MFMA operand read takes (a contiguous KB: the LDS's full 256 B/clk).  K: blocks [plane][tt][ks] (16 keys of
// sub-tile tt, head-dim columns 32 ks ..), V^T: blocks [plane][db] (head-dim rows 16 db .., the 32 keys).
constexpr int AT_FRAG = 512;                  // bf16 elements of a fragment block
constexpr int AT_KSTAGE = 16 * AT_FRAG, AT_VSTAGE = 16 * AT_FRAG;   // one staged tile: 16 KB of K, 16 KB of V^T
constexpr int AT_PGR = 4;                    // page-number registers: at most 64 * AT_PGR tiles per split
constexpr int AT_NKB = 2, AT_NVB = 2;         // K and V^T buffers: tile i in buffers i % 2
constexpr int AT_LDS_EL = AT_NKB * AT_KSTAGE + AT_NVB * AT_VSTAGE;
constexpr int AT_MAX_IV = CLOVER_MAX_NODES_INTERVAL;   // interval labels of the tree keys kept in the LDS

// One staging load: 64 lanes x 16 bytes from (uniform base) + (lane offset) in global memory to the KB at `dst` in
// the LDS (the hardware adds lane * 16 to dst).  dst is the same for all lanes.  (No memory clobber: the staged data is
// read only behind a later barrier, which is a fence for the compiler, and a clobber would turn the scalar loads of the
// page table into vector loads that wait for every staging load in flight.)
__device__ __forceinline__ void lds_dma16(const __attribute__((address_space(1))) char* base, unsigned lane_off,
                                          unsigned dst /* LDS byte address */) {
  const unsigned m0 = __builtin_amdgcn_readfirstlane(dst);
  asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2" : : "s"(m0), "v"(lane_off), "s"(base) : "m0");
}
// Wait until at most N of this wavefront's vector-memory loads are outstanding (the vmcnt field of s_waitcnt: bits 3:0
// and 15:14; the other counters are left alone).
template <int N>
__device__ __forceinline__ void wait_staging() {
  static_assert(N >= 0 && N < 64, "vmcnt has six bits");
  __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | (15 << 8) | ((N >> 4) << 14));
}

template <int G, int WM>
__global__ __launch_bounds__(64 * G * WM) void attn_mfma_kernel(AttnParams p) {
  constexpr int AT_MB = 2 / WM;     // 16-row blocks of nodes per wavefront
  extern __shared__ __attribute__((aligned(16))) bf16_t sm[];  // [2][AT_KSTAGE] [2][AT_VSTAGE] [AT_MAX_IV] labels
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int l16 = lane & 15, g4 = lane >> 4;
  const int split = blockIdx.x, ng = blockIdx.y / p.n_kv, kvh = blockIdx.y % p.n_kv, b = blockIdx.z;
  const RowMap& rm = p.rm;
  const int t0 = split * p.tiles_per_split;
  const int head = kvh * G + wave % G;
  const int nsub = (wave / G) * AT_MB * 16;   // this wavefront's first node within the workgroup's 32

  // ---- staging: global -> LDS without a stop in registers.  A wavefront instruction moves one fragment block: lane l
  // fetches the 16 bytes the MFMA operand layout wants at l * 16 (K: key 8 (l%16 / 4) + 4 tt + l%16 % 4, columns
  // 32 ks + 8 (l / 16) ..; V^T: row 16 db + l % 16, keys 8 (l / 16) ..) and the hardware writes them to
  // (LDS base of the block) + l * 16.  The 32 blocks of a tile are dealt to the workgroup's wavefronts.
  // Key tile t of this sequence is page pages[b * T + t] of the paged caches: the K rows and the V^T columns of
  // (page, KV head) are one contiguous 8 KB block each per plane.  An address is a uniform base plus the lane's 32-bit
  // offset, so staging costs no vector-ALU instruction.  The compiler is not told that these loads write the LDS (it would wait for all of
  // them before every LDS read that follows): the waits before the barriers below are written by hand.
  constexpr int NT = 64 * G * WM, NW = G * WM;
  constexpr int FPW = 16 / NW;          // K blocks and V^T blocks per wavefront and tile
  constexpr int DPT = 2 * FPW;          // staging loads per wavefront and tile
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);
  const unsigned k_lane = (unsigned)((((l16 >> 2) * 8 + (l16 & 3)) * AT_D + g4 * 8) * 2);   // bytes
  const unsigned v_lane = (unsigned)((l16 * AT_TK + g4 * 8) * 2);
  bf16_t* const k_lds = sm;
  bf16_t* const v_lds = sm + AT_NKB * AT_KSTAGE;
  const KVLayout& kv = p.kv;
  // Page numbers of this split's tiles: lane l of register r holds the page of tile t0 + 64 r + l, read from the page
  // table once, before the first staging load (a table read inside the loop would have to be a vector load -- the
  // compiler must assume that the staging statements write memory -- and its wait would drain the staging loads in
  // flight).  page_of(i) then is a lane read: no memory, no wait.
  int pgv[AT_PGR];
#pragma unroll
  for (int r = 0; r < AT_PGR; ++r) {
    const int lp = (b + kv.b0) * kv.T + min(t0 + 64 * r + lane, kv.T - 1);
    pgv[r] = kv.pages ? kv.pages[lp] : lp;
  }
  auto page_of = [&](int i) __attribute__((always_inline)) -> int {   // i: tile index within the split, < 64 AT_PGR
    int pg = __builtin_amdgcn_readlane(pgv[0], i & 63);              // (one lane read per register and a scalar
#pragma unroll                                                       //  select: a select between the registers
    for (int r = 1; r < AT_PGR; ++r) {                               //  would be turned into an indexed array)
      const int q = __builtin_amdgcn_readlane(pgv[r], i & 63);
      pg = (i >> 6) == r ? q : pg;
    }
    return pg;
  };
  typedef const __attribute__((address_space(1))) char* gbyte_ptr;
  const unsigned lds0 = (unsigned)(size_t)(__attribute__((address_space(3))) char*)sm;   // LDS byte address of sm
  auto stage_tile = [&](int kbuf, int vbuf, int page) __attribute__((always_inline)) {
    const size_t blk = ((size_t)page * kv.n_kv + kvh) * (size_t)(KV_PAGE * AT_D);   // elements; K and V^T blocks are equal
#pragma unroll
    for (int j = 0; j < FPW; ++j) {
      const int f = wave_u * FPW + j, plane = f >> 3;
      const bf16_t* ksrc = p.k_hi + blk + (size_t)plane * p.k_plane + ((f >> 2) & 1) * 4 * AT_D + (f & 3) * 32;
      const bf16_t* vsrc = p.v_hi + blk + (size_t)plane * p.v_plane + (f & 7) * 16 * AT_TK;
      lds_dma16((gbyte_ptr)ksrc, k_lane, lds0 + 2u * (unsigned)(kbuf * AT_KSTAGE + f * AT_FRAG));
      lds_dma16((gbyte_ptr)vsrc, v_lane, lds0 + 2u * (unsigned)(AT_NKB * AT_KSTAGE + vbuf * AT_VSTAGE + f * AT_FRAG));
    }
  };
  // The first key tile is requested before anything else is waited for (its address needs the page table only:
  // keys past the cache are clamped and masked later), so its HBM latency overlaps the loads of the lengths,
  // the masks and Q.
  stage_tile(0, 0, page_of(0));
  const int nv = rm.n_valid ? min(rm.n_valid[b], rm.n) : rm.n;
  const int L = p.base_len[b];
  if (ng * 32 >= nv || L + nv > p.max_seq) {  // whole workgroup
    wait_staging<0>();   // no staging load may land in the LDS after the workgroup has given it back
    return;
  }
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

  // ---- the three steps of a key tile.  scores: S^T = K Q^T (matrix pipe); soft_max: running statistics, the
  // probabilities as hi/lo fragments and the factor the output so far has to be scaled by (vector ALU);
  // output: O^T += V^T P (matrix pipe). ----
  auto scores = [&](int kbuf, f32x4 (&sc)[2][AT_MB]) __attribute__((always_inline)) {
    const bf16_t* kb = k_lds + kbuf * AT_KSTAGE + lane * 8;
#pragma unroll
    for (int tt = 0; tt < 2; ++tt)
#pragma unroll
      for (int mb = 0; mb < AT_MB; ++mb) sc[tt][mb] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int tt = 0; tt < 2; ++tt)
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        Frag kh, kl;
        kh.u = *(const u32x4*)(kb + (tt * 4 + ks) * AT_FRAG);
        kl.u = *(const u32x4*)(kb + (8 + tt * 4 + ks) * AT_FRAG);
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
    const bf16_t* vb = v_lds + vbuf * AT_VSTAGE + lane * 8;
#pragma unroll
    for (int db = 0; db < 8; ++db) {
      Frag vh, vl;
      vh.u = *(const u32x4*)(vb + db * AT_FRAG);
      vl.u = *(const u32x4*)(vb + (8 + db) * AT_FRAG);
#pragma unroll
      for (int mb = 0; mb < AT_MB; ++mb) {
        O[db][mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vl.v, ph[mb].v, O[db][mb], 0, 0, 0);
        O[db][mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vh.v, pl[mb].v, O[db][mb], 0, 0, 0);
        O[db][mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vh.v, ph[mb].v, O[db][mb], 0, 0, 0);
      }
    }
  };

  // ---- the loop over this split's key tiles.  Tile i + 1 is requested at the top of iteration i into the buffers
  // tile i - 1 has left (every wavefront is past the barrier of iteration i - 1) and has to be complete, and visible
  // to every wavefront, at the barrier that ends iteration i: each wavefront waits for its own staging loads first.
  // Measured on the same machine, 8192 + 96 keys (attention + merge, us): this form 58.9; the tile after next in
  // flight as well (three K and four V^T buffers, output product one tile behind the scores) 62.2; tiles staged
  // through registers and padded LDS rows, two in flight, 61.3.  Two workgroups of this kernel fit a CU (114
  // registers, 66 KB of LDS) and a launch of two per CU is no faster than one per CU: per key tile a workgroup costs
  // the CU ~1.5 us however the work is arranged -- scores 0.29, soft-max 0.40, output 0.23 (each timed by leaving
  // it out), the rest barriers, waits and the parts of the staging latency that the products do not cover -- and on
  // this chip a SIMD's matrix and vector instructions hardly overlap, whichever wavefronts they come from (24 MFMA
  // in one wavefront and 96 fma in another take 86-100 % of the sum of their times: probes/mfma_valu_overlap.hip),
  // so running half of the wavefronts one step out of phase with the others gains nothing either. ----
  if (t0 < t1) {  // uniform over the workgroup
    const int n = t1 - t0;
    f32x4 sc[2][AT_MB];
    Frag ph[AT_MB], pl[AT_MB];
    wait_staging<0>();
    __syncthreads();
    for (int i = 0; i < n; ++i) {
      const int cur = i & 1;
      if (i + 1 < n) stage_tile(cur ^ 1, cur ^ 1, page_of(i + 1));
      scores(cur, sc);
      soft_max(t0 + i, sc, ph, pl);
      output(cur, ph, pl);
      wait_staging<0>();
      __syncthreads();
    }
  }

  wait_staging<0>();   // (a split without tiles still has its first staging loads in flight)
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
  // (a split keeps the page numbers of at most 64 * AT_PGR tiles in registers, and there are at most MG_MAXS splits)
  return head_dim == AT_D && (g == 1 || g == 2 || g == 4 || g == 8) && max_seq % KV_PAGE == 0 && max_seq >= KV_PAGE &&
         max_seq / KV_PAGE <= 64 * AT_PGR * MG_MAXS;
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
  // about one workgroup per CU (two fit and do not overlap: a key tile costs the CU ~1.5 us of a workgroup's time
  // whether the workgroup shares the CU or not, so a launch of 1.5 workgroups per CU takes as long as one of 2), at
  // least two tiles per split, within the partial buffer
  const int target = tune_int("CLOVER_ATTN_WGS", 256);
  int splits = std::max(1, target / (p.rm.B * p.n_kv * node_groups));
  splits = std::max(1, std::min(std::min(splits, std::min(p.max_splits, MG_MAXS)), (n_tiles + 1) / 2));
  splits = std::max(splits, (n_tiles + 64 * AT_PGR - 1) / (64 * AT_PGR));   // <= MG_MAXS: attn_mfma_supported
  p.tiles_per_split = (n_tiles + splits - 1) / splits;
  p.n_splits = (n_tiles + p.tiles_per_split - 1) / p.tiles_per_split;
  dim3 grid(p.n_splits, node_groups * p.n_kv, p.rm.B);
  // Two wavefronts per head (16 nodes each, two per SIMD): while one waits for fragments, a shuffle or the
  // barrier the other issues, and both share the staged K / V^T tile (one wavefront per head with 32 nodes measured
  // slower at every launch size).
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
