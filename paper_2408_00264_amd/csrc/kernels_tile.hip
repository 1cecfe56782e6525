// Tiled MFMA GEMM for MANY activation rows (65..256) on gfx950: one pass over the weights for all rows.
//
//   EPI 0:  Y[M,N]       = X[M,K] * W[N,K]^T                   (fp32; over k_parts ranges of K: partial tiles)
//   EPI 1:  (hi,lo)[M,F]  = split(silu(X Wg^T) * (X Wu^T))      (the SwiGLU projection)
//
// Why a third GEMM shape.  With 64 rows the weight stream bounds the time and every wavefront multiplies its
// weight fragments against ALL rows (kernels_stream / kernels_panel).  With 128..256 rows that layout reads
// 16 KB of activation fragments from the LDS per 32 matrix instructions of a wavefront -- the whole LDS
// bandwidth of the CU -- so the 128-row form of the panel kernel sits at ~30 % of the matrix peak and 256 rows
// need two weight passes.  Here the wavefronts of a workgroup tile the output in two dimensions; activations are
// hi + lo bf16 planes (two matrix instructions per fragment pair), accumulation in fp32.
#include "clover_internal.h"

#include <algorithm>
#include <type_traits>

namespace clv {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

namespace {

union Frag {
  u32x4 u;
  bf16x8 v;
};

constexpr int TL_KST = 64;            // K columns per activation stage (2 k-tiles of 32)
constexpr int TL_LDK = TL_KST + 16;   // LDS row stride (bf16): 32 mod 64 bytes, the stride at which fragment reads run at the full LDS rate

template <int I, int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (I < N) {
    f(std::integral_constant<int, I>{});
    static_for<I + 1, N>(f);
  }
}

__device__ __forceinline__ unsigned t_rn(float a) { return (unsigned)__builtin_bit_cast(unsigned short, (__bf16)a); }

// ------------------------------------------------------------------------------------------
// Workgroup tile 128 rows x 256 columns, four wavefronts (one per SIMD), wavefront tile 128 x 64.
//
// Why this shape.  A first version (256 x 128 tiles, 4 x 2 wavefronts of 64 x 64, two per SIMD) moved, per 64-column
// K stage, 64 KB of activations and 64 KB of weight fragments through a compute unit's vector L1 (every weight
// fragment fetched by the four wavefronts of the four row quarters): at 64 B/clk exactly as long as the stage's 2048
// matrix-pipe cycles, so nothing overlapped for free, and it ran at 0.30 of the matrix peak.  A 128 x 256 tile
// needs half the activation rows per column and lets every wavefront own its columns:
// per stage 32 KB of activations + 32 KB of weight fragments (each fetched once) pass the L1, the LDS serves 128 KB of
// fragment reads and takes 32 KB of stores (62 % of the stage).  One wavefront per SIMD has the 512-register budget
// that the software pipeline needs: 128 accumulators, two sets of 16 activation fragments (the next k-tile's
// fragments are read from the LDS while this one is multiplied), a ring of four k-tiles of weight fragments in
// flight, one stage of activations on its way from global memory to the LDS.  Three stage buffers: the stage two
// ahead is stored while the next one is already being read, one barrier per stage.
// Rows beyond 128 are a second workgroup on the same columns; it is placed next to the first one on the same XCD
// (workgroup ids 8 apart) so that one of the two finds the weight fragments in that XCD's L2.
// ------------------------------------------------------------------------------------------
constexpr int TW_ROWS = 128;          // rows per workgroup
constexpr int TW_NW = 4;              // wavefronts, 64 output columns each
constexpr int TW_PLANE = TW_ROWS * TL_LDK;
constexpr int TW_BUF = 2 * TW_PLANE;  // hi and lo plane of one stage
constexpr int TW_NBUF = 3;
// Ablation bits, compile time only (a tuning build compiled with -DCLOVER_TILE_ABLATE=<bits>; 0 in every library that
// computes): 1 no activation loads after the third stage, 16 no activation stores to the LDS, 2 no LDS fragment
// reads, 4 no weight loads after the first four k-tiles, 8 no barrier.  Run-time switches would put branches between
// the hand-placed instructions of a stage and break the schedule they are meant to measure.
#ifdef CLOVER_TILE_ABLATE
constexpr int TW_ABLATE = CLOVER_TILE_ABLATE;
#else
constexpr int TW_ABLATE = 0;
#endif
constexpr int TW_XIT = 2 * TW_ROWS * (TL_KST / 8) / (TW_NW * 64);   // 16-byte pieces per thread and stage (= 8)

// acc += A B^T with the accumulator tied to one accumulation-register tuple for the whole kernel.  (Written through the
// builtin, the register allocator gives a fifth of the 256 products of a loop trip a destination that differs from its
// source and moves ~190 registers per trip back; those moves are vector-ALU instructions and do not overlap the
// matrix pipe.)
__device__ __forceinline__ void mfma_acc(f32x4& acc, const bf16x8& a, const bf16x8& b) {
  asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(acc) : "v"(a), "v"(b));
}

template <int EPI>
__global__ __launch_bounds__(TW_NW * 64) void gemm_tile_wide_kernel(TileGemm p) {
  extern __shared__ __attribute__((aligned(16))) bf16_t xs[];   // [3 buffers][hi, lo][128][TL_LDK]
  constexpr int NT = TW_NW * 64;
  const int tid = threadIdx.x, wn = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
  const int l16 = lane & 15, g4 = lane >> 4;
  const int KT = p.K / 32;
  // workgroup id -> (row half, column tile, K range): ids 8 apart share an XCD, so the two row halves of a tile are
  // the neighbours (2j, 2j + 1) in that XCD's own order
  const int halves = p.M > TW_ROWS ? 2 : 1;
  int rh = 0, unit = (int)blockIdx.x;
  if (halves == 2) {
    const int xcd = (int)blockIdx.x & 7, j = (int)blockIdx.x >> 3;
    rh = j & 1;
    unit = (j >> 1) * 8 + xcd;
  }
  if (unit >= p.n_units) return;   // (grid rounded up to whole XCD rows; uniform over the workgroup)
  const int part = unit % p.k_parts, tile = unit / p.k_parts;
  const int NS = p.K / TL_KST / p.k_parts;             // stages of this workgroup's K range
  const int ks0 = part * NS;
  const int row0 = rh * TW_ROWS;

  // Every load below is (uniform base) + (32-bit offset of the lane): the bases live in scalar registers and advance
  // with scalar arithmetic, so a load costs no vector-ALU instruction (those do not overlap the matrix pipe).
  const bf16_t* wbase[4];   // uniform: first fragment of this wavefront's four column blocks
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    int nb;
    if (EPI == 1) {   // 32 columns of F per wavefront: blocks 0,1 gate rows, blocks 2,3 the up rows of the same columns
      nb = min((tile * TW_NW + wn) * 2 + (c & 1), p.N / 16 - 1);
      wbase[c] = p.W[c >> 1] + (size_t)nb * KT * 512;
    } else {
      nb = min((tile * TW_NW + wn) * 4 + c, p.N / 16 - 1);
      wbase[c] = p.W[0] + (size_t)nb * KT * 512;
    }
  }

  f32x4 acc[4][8];   // [column block][row block]
#pragma unroll
  for (int c = 0; c < 4; ++c)
#pragma unroll
    for (int rb = 0; rb < 8; ++rb) acc[c][rb] = (f32x4){0.f, 0.f, 0.f, 0.f};
  asm volatile("s_nop 7" ::: "memory");   // (as below: write of an accumulator register -> matrix instruction)

  constexpr int RING = 4;
  Frag w[RING][4];      // [k-tile modulo 4][column block]
  Frag xa[8], xb[8];    // activation fragments of row blocks 0..3 / 4..7 of a k-tile: [row block][hi, lo]
  u32x4 xv[TW_XIT];
  const int n_kt = NS * 2;

  const unsigned lane_off = (unsigned)lane * 8u;
  // (the empty statements pin the uniform part of an address in a scalar register pair and keep the widening of the
  // lane's 32-bit offset next to the load -- `fresh`, once per stage: otherwise the optimiser folds the offset into a
  // per-lane 64-bit pointer outside the loop and adds the moving part with vector instructions)
  auto fresh = [](unsigned v) __attribute__((always_inline)) { asm("" : "+v"(v)); return v; };
  typedef const __attribute__((address_space(1))) char* gbyte_ptr;
  typedef const __attribute__((address_space(1))) u32x4* gvec_ptr;
  auto at = [](const bf16_t* uniform, unsigned lane_el) __attribute__((always_inline)) -> gvec_ptr {
    gbyte_ptr g = (gbyte_ptr)uniform;
    asm("" : "+s"(g));
    return (gvec_ptr)(g + lane_el * 2u);
  };
  // ---- the pieces a stage is made of: one instruction each, so that the stage can place them between the matrix
  // instructions by hand (the scheduler neither moves memory operations across the asm statements nor knows that
  // they are matrix instructions) ----
  auto load_w1 = [&](auto tc, int kt, int c, unsigned lo) __attribute__((always_inline)) {
    constexpr int t = decltype(tc)::value;
    const size_t off = (size_t)(ks0 * 2 + kt) * 512;
    if ((TW_ABLATE & 4) && kt > 3) return;
    w[t][c].u = __builtin_nontemporal_load(at(wbase[c] + off, lo));
  };
  auto load_w = [&](auto tc, int kt) __attribute__((always_inline)) {
    const unsigned lo = fresh(lane_off);
#pragma unroll
    for (int c = 0; c < 4; ++c) load_w1(tc, kt, c, lo);
  };
  // rows past M read row M - 1 again: an output row depends on its own activation row only, and the epilogue
  // never stores rows >= M, so their accumulators may hold anything
  // (piece it of a thread: plane it / 4, and the same row and 16-byte slot in both planes)
  unsigned xoff[TW_XIT / 2];
  int xdst[TW_XIT / 2];     // LDS element offset of the piece inside a plane
#pragma unroll
  for (int it = 0; it < TW_XIT / 2; ++it) {
    const int idx = it * NT + tid;
    const int r = idx / (TL_KST / 8), sl = idx % (TL_KST / 8);
    xoff[it] = (unsigned)(min(row0 + r, p.M - 1) * p.ldx + sl * 8);
    xdst[it] = r * TL_LDK + sl * 8;
  }
  const bf16_t* const xhi0 = p.Xhi + (size_t)ks0 * TL_KST;
  const bf16_t* const xlo0 = p.Xlo + (size_t)ks0 * TL_KST;
  auto x_load1 = [&](int s, int it, unsigned xo) __attribute__((always_inline)) {   // xo: this thread's xoff[it % 4]
    if ((TW_ABLATE & 1) && s > 2) return;
    xv[it] = *at((it < TW_XIT / 2 ? xhi0 : xlo0) + (size_t)s * TL_KST, xo);
  };
  auto x_store1 = [&](int b, int it) __attribute__((always_inline)) {
    if (TW_ABLATE & 16) return;
    *(u32x4*)(xs + b * TW_BUF + (it / (TW_XIT / 2)) * TW_PLANE + xdst[it % (TW_XIT / 2)]) = xv[it];
  };
  auto x_load = [&](int s) __attribute__((always_inline)) {
    unsigned xo[TW_XIT / 2];
#pragma unroll
    for (int it = 0; it < TW_XIT / 2; ++it) xo[it] = fresh(xoff[it]);
#pragma unroll
    for (int it = 0; it < TW_XIT; ++it) x_load1(s, it, xo[it % (TW_XIT / 2)]);
  };
  auto x_store = [&](int b) __attribute__((always_inline)) {
#pragma unroll
    for (int it = 0; it < TW_XIT; ++it) x_store1(b, it);
  };
  // fragment j (row block j / 2, plane j % 2) of row blocks 4 q .. 4 q + 3 of k-tile `half` of the stage in buffer b
  auto frag1 = [&](Frag (&xf)[8], int b, int half, int q, int j) __attribute__((always_inline)) {
    if (TW_ABLATE & 2) return;
    xf[j].u = *(const u32x4*)(xs + b * TW_BUF + (j & 1) * TW_PLANE + (q * 64 + (j >> 1) * 16 + l16) * TL_LDK + g4 * 8 + half * 32);
  };
  auto frag_load = [&](Frag (&xf)[8], int b, int half, int q) __attribute__((always_inline)) {
#pragma unroll
    for (int j = 0; j < 8; ++j) frag1(xf, b, half, q, j);
  };
  // matrix instruction m (0..31) of a group: row blocks 4 q .. 4 q + 3 (fragments xf) against the four weight
  // fragments of ring slot t; per row block the lo plane against the four column blocks, then the hi plane
  auto mm = [&](auto tc, auto qc, const Frag (&xf)[8], int m) __attribute__((always_inline)) {
    constexpr int t = decltype(tc)::value, q = decltype(qc)::value;
    const int rb = m >> 3, c = m & 3, lo = ((m >> 2) & 1) ^ 1;
    mfma_acc(acc[c][4 * q + rb], w[t][c].v, xf[2 * rb + lo].v);
  };

  // ---- prologue: weight ring, stages 0 and 1 in the LDS, stage 2 in registers, the first fragments ----
  load_w(std::integral_constant<int, 0>{}, 0);
  if (n_kt > 1) load_w(std::integral_constant<int, 1>{}, 1);
  if (n_kt > 2) load_w(std::integral_constant<int, 2>{}, 2);
  x_load(0);
  x_store(0);
  if (NS > 1) { x_load(1); x_store(1); }
  if (NS > 2) x_load(2);
  __syncthreads();
  frag_load(xa, 0, 0, 0);

  // One stage = two k-tiles = four groups of 32 matrix instructions (row blocks 0..3 / 4..7 of each k-tile); while
  // one group is multiplied the next group's fragments are read from the LDS into the other fragment set.  Around
  // them: the activations of stage st + 2 (in registers since the previous stage) go to the LDS and stage st + 3 is
  // requested (first group), the weights of k-tiles 2 st + 3 and 2 st + 4 are requested (second and third group).
  // With one wavefront per SIMD nothing else hides the issue of these instructions, so each of them is placed
  // between two matrix instructions, where it issues while the matrix pipe is busy.
  using Q0 = std::integral_constant<int, 0>;
  using Q1 = std::integral_constant<int, 1>;
  auto stage = [&](auto w0, auto w1, auto w3, auto fullc, int st, int b /* st % 3 */) {
    // w0, w1: ring slots of this stage's k-tiles; w3: slot of k-tile 2 st + 3; k-tile 2 st + 4 reuses w0
    constexpr bool FULL = decltype(fullc)::value;
    const int b1 = b == TW_NBUF - 1 ? 0 : b + 1, b2 = b1 == TW_NBUF - 1 ? 0 : b1 + 1;
    const bool do_store = FULL || st + 2 < NS, do_xload = FULL || st + 3 < NS;
    const bool do_w3 = FULL || 2 * st + 3 < n_kt, do_w4 = FULL || 2 * st + 4 < n_kt, do_next = FULL || st + 1 < NS;
    const unsigned lo = fresh(lane_off);
    unsigned xo[TW_XIT / 2];
#pragma unroll
    for (int it = 0; it < TW_XIT / 2; ++it) xo[it] = fresh(xoff[it]);
    // group 0: 8 x (product, LDS store, product, fragment read, product, activation load), 8 products
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      mm(w0, Q0{}, xa, 3 * i);
      if (do_store) x_store1(b2, i);
      mm(w0, Q0{}, xa, 3 * i + 1);
      frag1(xb, b, 0, 1, i);
      mm(w0, Q0{}, xa, 3 * i + 2);
      if (do_xload) x_load1(st + 3, i, xo[i % (TW_XIT / 2)]);
    }
#pragma unroll
    for (int m = 24; m < 32; ++m) mm(w0, Q0{}, xa, m);
    // group 1: 4 x (2 products, fragment read, 2 products, fragment read, product, weight load), 12 products
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      mm(w0, Q1{}, xb, 5 * i); mm(w0, Q1{}, xb, 5 * i + 1);
      frag1(xa, b, 1, 0, 2 * i);
      mm(w0, Q1{}, xb, 5 * i + 2); mm(w0, Q1{}, xb, 5 * i + 3);
      frag1(xa, b, 1, 0, 2 * i + 1);
      mm(w0, Q1{}, xb, 5 * i + 4);
      if (do_w3) load_w1(w3, 2 * st + 3, i, lo);
    }
#pragma unroll
    for (int m = 20; m < 32; ++m) mm(w0, Q1{}, xb, m);
    // group 2: the same with the other k-tile; the weight slot of k-tile 2 st is free now and takes k-tile 2 st + 4
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      mm(w1, Q0{}, xa, 5 * i); mm(w1, Q0{}, xa, 5 * i + 1);
      frag1(xb, b, 1, 1, 2 * i);
      mm(w1, Q0{}, xa, 5 * i + 2); mm(w1, Q0{}, xa, 5 * i + 3);
      frag1(xb, b, 1, 1, 2 * i + 1);
      mm(w1, Q0{}, xa, 5 * i + 4);
      if (do_w4) load_w1(w0, 2 * st + 4, i, lo);
    }
#pragma unroll
    for (int m = 20; m < 32; ++m) mm(w1, Q0{}, xa, m);
    // group 3: 8 x (3 products, fragment read of the next stage's first group), 8 products
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      mm(w1, Q1{}, xb, 3 * i); mm(w1, Q1{}, xb, 3 * i + 1); mm(w1, Q1{}, xb, 3 * i + 2);
      if (do_next) frag1(xa, b1, 0, 0, i);
    }
#pragma unroll
    for (int m = 24; m < 32; ++m) mm(w1, Q1{}, xb, m);
    if (!(TW_ABLATE & 8)) __syncthreads();
  };
  using I0 = std::integral_constant<int, 0>;
  using I1 = std::integral_constant<int, 1>;
  using I2 = std::integral_constant<int, 2>;
  using I3 = std::integral_constant<int, 3>;
  int st = 0, b = 0;
  for (; st + 4 < NS; st += 2) {   // two stages = four k-tiles per iteration: static ring slots
    stage(I0{}, I1{}, I3{}, std::true_type{}, st, b);
    b = b == TW_NBUF - 1 ? 0 : b + 1;
    stage(I2{}, I3{}, I1{}, std::true_type{}, st + 1, b);
    b = b == TW_NBUF - 1 ? 0 : b + 1;
  }
  for (; st < NS; st += 2) {
    stage(I0{}, I1{}, I3{}, std::false_type{}, st, b);
    b = b == TW_NBUF - 1 ? 0 : b + 1;
    if (st + 1 < NS) stage(I2{}, I3{}, I1{}, std::false_type{}, st + 1, b);
    b = b == TW_NBUF - 1 ? 0 : b + 1;
  }

  // (the compiler does not know that the asm statements are matrix instructions, so the wait states between the last
  // of them and the first read of an accumulator are spelled out: two no-ops of 16 cover the longest one)
  asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
  // ---- epilogue: lane holds rows rb*16 + l16 of the tile, columns 4*g4 .. 4*g4+3 of each block ----
  if (EPI == 1) {
    const int fblock = (tile * TW_NW + wn) * 2;
#pragma unroll
    for (int c = 0; c < 2; ++c) {
      if ((fblock + c) * 16 >= p.N) continue;
      const int col = (fblock + c) * 16 + 4 * g4;
#pragma unroll
      for (int rb = 0; rb < 8; ++rb) {
        const int m = row0 + rb * 16 + l16;
        if (m >= p.M) continue;
        unsigned h[4], l[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const float g = acc[c][rb][r], u = acc[c + 2][rb][r];
          const float o = g / (1.0f + expf(-g)) * u;
          h[r] = t_rn(o);
          l[r] = t_rn(o - __uint_as_float(h[r] << 16));
        }
        *(uint2*)(p.Yhi + (size_t)m * p.ldo + col) = make_uint2(h[0] | (h[1] << 16), h[2] | (h[3] << 16));
        *(uint2*)(p.Ylo + (size_t)m * p.ldo + col) = make_uint2(l[0] | (l[1] << 16), l[2] | (l[3] << 16));
      }
    }
  } else {
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const int blk = (tile * TW_NW + wn) * 4 + c;
      if (blk * 16 >= p.N) continue;
      const int col = blk * 16 + 4 * g4;
#pragma unroll
      for (int rb = 0; rb < 8; ++rb) {
        const int m = row0 + rb * 16 + l16;
        const f32x4 v = acc[c][rb];
        if (m < p.M) *(float4*)(p.Y + part * p.split_stride + (size_t)m * p.ldy + col) = make_float4(v[0], v[1], v[2], v[3]);
      }
    }
  }
}

template <int EPI>
void launch_tile_wide(const TileGemm& g, int wgs, hipStream_t st) {
  constexpr size_t lds = (size_t)TW_NBUF * TW_BUF * sizeof(bf16_t);
  static_assert(lds <= 160 * 1024, "stage buffers exceed the LDS");
  static bool attr_done = false;
  if (!attr_done) {
    hipFuncSetAttribute((const void*)gemm_tile_wide_kernel<EPI>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    attr_done = true;
  }
  gemm_tile_wide_kernel<EPI><<<wgs, TW_NW * 64, lds, st>>>(g);
}

}  // namespace

// N: output columns (EPI 1: the FFN width F with W[0] = gate, W[1] = up, each [F, K]); k_parts divides K / 64
bool tile_gemm_supported(int M, int N, int K, int epi) {
  if (M < 1 || M > 256 || K % TL_KST != 0 || N % 16 != 0) return false;
  return epi == 1 || N % 4 == 0;
}
// K ranges for an output too narrow to give every CU a workgroup: the largest divisor of the stage count that keeps
// the grid within one workgroup per CU and at least 8 stages per range; column tiles of 256 (epi 1: 128 columns of
// F), one or two row halves
int tile_gemm_pick_k_parts(int M, int N, int K) {
  const int tiles = (N / 16 + 15) / 16 * (M > TW_ROWS ? 2 : 1), NS = K / TL_KST;
  int best = 1;
  for (int d = 1; d <= NS; ++d)
    if (NS % d == 0 && tiles * d <= 256 && NS / d >= 8) best = d;
  return best;
}

void launch_gemm_tile(const TileGemm& g_in, hipStream_t st) {
  TileGemm g = g_in;
  if (g.k_parts < 1 || g.epi == 1) g.k_parts = 1;
  const int blocks = g.N / 16;
  const int tiles = g.epi == 1 ? (blocks + 7) / 8 : (blocks + 15) / 16;
  g.n_units = tiles * g.k_parts;
  const int wgs = g.M > TW_ROWS ? (g.n_units + 7) / 8 * 8 * 2 : g.n_units;
  if (g.epi == 1) launch_tile_wide<1>(g, wgs, st);
  else launch_tile_wide<0>(g, wgs, st);
}

}  // namespace clv
