// Full-K "panel" GEMM for few activation rows (M <= 64) and MANY output columns on gfx950:
//
//   EPI 0:  Y[M,N]      = X[M,K] * W[N,K]^T                               (fp32, e.g. the LM head)
//   EPI 1:  (hi,lo)[M,F] = split(silu(X Wg^T) * (X Wu^T))                  (the SwiGLU projection)
//
// Why a second M <= 64 kernel.  The K-slice-resident kernel keeps its activation slice in LDS and
// pays for that with one fp32 partial tile per K slice: S * M * N * 4 bytes written and read back.
// For N = 28672 (gate+up) or N = 128256 (LM head) that is 25..50 % on top of the weight bytes, plus a
// consumer kernel whose only job is to add the slices.  Here a workgroup owns a narrow range of
// output columns over ALL of K, so results leave the kernel finished (and the SwiGLU is applied in
// registers).  The price is that every workgroup walks the whole activation matrix: it is staged
// through LDS in 256-column stages, double buffered (global -> registers -> LDS while the previous
// stage is multiplied), one barrier per stage.  That traffic is L2 hits (the matrix is 1 MB); it is
// affordable only because few workgroups share the weights' columns, which is why the narrow
// GEMMs (N <= 6144) stay with the K-slice kernel.
//
// A third use cuts K into ranges (k_parts > 1, EPI 0): a narrow output with a long K (the down projection)
// has too few column blocks for full-K panels on every CU, so each range writes a partial [M,N] tile that the
// consumer adds -- a few partials of several thousand columns each instead of one per 512 columns.
//
// Work split inside a workgroup of 8 wavefronts: UW = 8 / KW column units x KW parts of each
// stage's 8 k-tiles.  A wavefront keeps NFW = 2 weight fragments (16 output columns each; for EPI 1
// the gate and the up fragment of the same columns) against all 64 rows, streams its weights
// global -> registers one stage ahead (NBUF = 2 register buffers), and reads the activation fragments from LDS.
// With KW = 2 the two k-parts are added through LDS once, after the last stage.
#include "clover_internal.h"

#include <algorithm>
#include <cstdlib>
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

constexpr int PN_WAVES = 8;
constexpr int PN_KST = 256;           // K columns per activation stage (8 k-tiles of 32)
constexpr int PN_NFW = 2;

// float -> bf16 (round to nearest even) through the hardware conversion (v_cvt_pk_bf16_f32)
__device__ __forceinline__ unsigned rn_bf16(float a) { return (unsigned)__builtin_bit_cast(unsigned short, (__bf16)a); }

template <int I, int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (I < N) {
    f(std::integral_constant<int, I>{});
    static_for<I + 1, N>(f);
  }
}

// NOPAD: the launch has exactly MT * 16 rows (no padding rows in the tile).
template <int MT, int KW, int EPI, int NBUF, int KST, bool NOPAD>
__global__ __launch_bounds__(PN_WAVES * 64) void gemm_panel_kernel(PanelGemm p) {
  constexpr int ROWS = MT * 16;
  constexpr int PN_LDK = KST + 16;              // LDS row stride (bf16): 32 mod 64 bytes, the stride at which fragment reads run at the full LDS rate
  constexpr int TILES = KST / 32;               // k-tiles per stage
  constexpr int SL = KST / 8;                   // 16-byte pieces per row and stage
  constexpr int PLANE = ROWS * PN_LDK;          // bf16 elements per plane of one stage buffer
  constexpr int BUF = 2 * PLANE;                // hi and lo
  constexpr int UW = PN_WAVES / KW;             // column units per workgroup
  constexpr int CH = TILES / KW;                   // k-tiles per wavefront and stage
  constexpr int XIT = 2 * ROWS * SL / (PN_WAVES * 64);  // 16-byte pieces per thread and stage
  extern __shared__ __attribute__((aligned(16))) bf16_t xs[];      // [2 buffers][hi, lo][ROWS][PN_LDK]

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int l16 = lane & 15, g4 = lane >> 4;
  const int uw = wave / KW, kp = wave % KW;
  const int KT = p.K / 32;
  const int NS = p.K / KST / p.k_parts;      // stages of this workgroup's K range
  // K range = workgroup id % k_parts: workgroups are dealt to the 8 XCDs round-robin, so with 8 ranges
  // every XCD's L2 holds ONE range of the activations instead of all of them (K = 14336: the whole
  // 3.7 MB matrix would not stay in a 4 MB L2 beside the weight stream and was fetched again and again)
  const int part = p.k_parts > 1 ? (int)blockIdx.x % p.k_parts : 0;
  const int wg = p.k_parts > 1 ? (int)blockIdx.x / p.k_parts : (int)blockIdx.x;
  const int ks0 = part * NS;                    // its first stage
  // Workgroups start at different K stages: all weight blocks have the same power-of-two size, and
  // walking them in lock-step would keep every workgroup on the same few HBM channels.
  // (a launch of more than one workgroup per CU staggers by itself, and measured faster unrotated)
  const int rot = (CLV_DBG(p, 2) || gridDim.x > 256) ? 0 : wg % NS;
  const int n_blocks = p.N / 16;                // 16-column blocks of the output
  // EPI 1: unit = one 16-column block (fragments: gate rows, up rows); EPI 0: unit = two adjacent blocks
  const int unit = wg * UW + uw;
  int nb[PN_NFW];
  const bf16_t* wbase[PN_NFW];
  bool live;
  if (EPI == 1) {
    live = unit < n_blocks;
    nb[0] = nb[1] = live ? unit : 0;
    wbase[0] = p.W[0] + (size_t)nb[0] * KT * 512 + lane * 8;
    wbase[1] = p.W[1] + (size_t)nb[1] * KT * 512 + lane * 8;
  } else {
    live = unit * 2 < n_blocks;
    nb[0] = live ? unit * 2 : 0;
    nb[1] = min(nb[0] + 1, n_blocks - 1);       // an odd tail block is computed twice and stored once
    wbase[0] = p.W[0] + (size_t)nb[0] * KT * 512 + lane * 8;
    wbase[1] = p.W[0] + (size_t)nb[1] * KT * 512 + lane * 8;
  }

  Frag w[NBUF][PN_NFW][CH];
  f32x4 acc[PN_NFW][MT];
#pragma unroll
  for (int f = 0; f < PN_NFW; ++f)
#pragma unroll
    for (int mb = 0; mb < MT; ++mb) acc[f][mb] = (f32x4){0.f, 0.f, 0.f, 0.f};

  auto load_w = [&](auto bufc, int s) {
    constexpr int buf = decltype(bufc)::value;
    const int ks = ks0 + (s + rot) % NS;
    const size_t off = (size_t)(ks * TILES + kp * CH) * 512;
#pragma unroll
    for (int f = 0; f < PN_NFW; ++f)
#pragma unroll
      for (int t = 0; t < CH; ++t) w[buf][f][t].u = __builtin_nontemporal_load((const u32x4*)(wbase[f] + off + t * 512));
  };
  u32x4 xv[XIT];
  auto x_load = [&](int s) {
    const int ks = ks0 + (s + rot) % NS;
#pragma unroll
    for (int it = 0; it < XIT; ++it) {
      const int idx = it * (PN_WAVES * 64) + tid;
      const int rp = idx / SL, sl = idx % SL, plane = rp / ROWS, r = rp % ROWS;
      // Rows past M read row M - 1 again and are then zeroed by a predicate, which the compiler turns into a branch
      // around every load: good when M is well below the tile's rows (the padding rows' loads are skipped: the LM
      // head at 17..32 rows is 8 us faster with it), 0.7 % of the verify pass lost at exactly 64 rows -- hence the
      // NOPAD form without predicate for a tile with no padding rows.  (Choosing between the two at run time inside
      // one kernel loses the gain again; the 128-row form without its branches measured 5 % slower.)
      const bf16_t* src = (plane ? p.Xlo : p.Xhi) + (size_t)(NOPAD ? r : min(r, p.M - 1)) * p.ldx + ks * KST + sl * 8;
      u32x4 v = (u32x4){0u, 0u, 0u, 0u};
      if (!CLV_DBG(p, 1)) v = *(const u32x4*)src;
      if constexpr (NOPAD) xv[it] = v;
      else xv[it] = r < p.M ? v : (u32x4){0u, 0u, 0u, 0u};
    }
  };
  auto x_store = [&](int b) {
#pragma unroll
    for (int it = 0; it < XIT; ++it) {
      const int idx = it * (PN_WAVES * 64) + tid;
      const int rp = idx / SL, sl = idx % SL, plane = rp / ROWS, r = rp % ROWS;
      *(u32x4*)(xs + b * BUF + plane * PLANE + r * PN_LDK + sl * 8) = xv[it];
    }
  };
  auto compute = [&](auto bufc, int b) {
    constexpr int buf = decltype(bufc)::value;
    if (CLV_DBG(p, 4)) {  // keep the weight loads alive without LDS reads and matrix work
#pragma unroll
      for (int f = 0; f < PN_NFW; ++f)
#pragma unroll
        for (int t = 0; t < CH; ++t) acc[f][0][0] += __uint_as_float(w[buf][f][t].u.x & 0x3f800000u);
      return;
    }
    const bf16_t* hi = xs + b * BUF + l16 * PN_LDK + g4 * 8 + kp * CH * 32;
    const bf16_t* lo = hi + PLANE;
#pragma unroll
    for (int t = 0; t < CH; ++t) {
#pragma unroll
      for (int mb = 0; mb < MT; ++mb) {
        Frag bh, bl;
        bh.u = *(const u32x4*)(hi + mb * 16 * PN_LDK + t * 32);
        bl.u = *(const u32x4*)(lo + mb * 16 * PN_LDK + t * 32);
#pragma unroll
        for (int f = 0; f < PN_NFW; ++f)
          acc[f][mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w[buf][f][t].v, bl.v, acc[f][mb], 0, 0, 0);
#pragma unroll
        for (int f = 0; f < PN_NFW; ++f)
          acc[f][mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w[buf][f][t].v, bh.v, acc[f][mb], 0, 0, 0);
      }
    }
  };

  // ---- prologue: the weight stream starts before the first activation stage is staged ----
  static_for<0, NBUF - 1>([&](auto ic) {
    if (decltype(ic)::value < NS) load_w(ic, decltype(ic)::value);
  });
  x_load(0);
  x_store(0);
  __syncthreads();

  // One stage: prefetch the next activation stage and the weights NBUF - 1 stages ahead, multiply.
  // FULL stages issue every load unconditionally, so the compiler's wait before the multiply counts
  // exactly the younger loads and leaves them in flight; the scheduling barriers keep it from
  // sinking the loads below the MFMAs they are meant to overlap.
  auto stage = [&](auto ic, auto fullc, int s) {
    constexpr int I = decltype(ic)::value;
    constexpr bool FULL = decltype(fullc)::value;
    if (FULL || s + 1 < NS) x_load(s + 1);
    if (FULL || s + NBUF - 1 < NS) load_w(std::integral_constant<int, (I + NBUF - 1) % NBUF>{}, s + NBUF - 1);
    __builtin_amdgcn_sched_barrier(0);
    compute(std::integral_constant<int, I>{}, s & 1);
    __builtin_amdgcn_sched_barrier(0);
    if (FULL || s + 1 < NS) x_store((s + 1) & 1);
    if (!CLV_DBG(p, 8)) __syncthreads();
  };
  int s0 = 0;
  for (; s0 + 2 * NBUF - 2 < NS; s0 += NBUF)
    static_for<0, NBUF>([&](auto ic) { stage(ic, std::true_type{}, s0 + decltype(ic)::value); });
  for (; s0 < NS; s0 += NBUF)
    static_for<0, NBUF>([&](auto ic) {
      if (s0 + decltype(ic)::value < NS) stage(ic, std::false_type{}, s0 + decltype(ic)::value);
    });

  // ---- add the k-parts (KW == 2): part 1 hands its accumulators to part 0 through LDS ----
  if (KW == 2) {
    f32x4* red = (f32x4*)xs + (size_t)uw * PN_NFW * MT * 64 + lane;  // the stage buffers are free now
    if (kp == 1) {
#pragma unroll
      for (int f = 0; f < PN_NFW; ++f)
#pragma unroll
        for (int mb = 0; mb < MT; ++mb) red[(f * MT + mb) * 64] = acc[f][mb];
    }
    __syncthreads();
    if (kp == 0) {
#pragma unroll
      for (int f = 0; f < PN_NFW; ++f)
#pragma unroll
        for (int mb = 0; mb < MT; ++mb) acc[f][mb] += red[(f * MT + mb) * 64];
    }
  }
  if (kp != 0 || !live) return;

  // ---- epilogue: lane holds rows mb*16 + l16, columns 4*g4 .. 4*g4+3 of each fragment ----
  if (EPI == 1) {
    const int col = nb[0] * 16 + 4 * g4;
#pragma unroll
    for (int mb = 0; mb < MT; ++mb) {
      const int m = mb * 16 + l16;
      if (m >= p.M) continue;
      unsigned h[4], l[4];
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const float g = acc[0][mb][r], u = acc[1][mb][r];
        const float o = g / (1.0f + expf(-g)) * u;
        h[r] = rn_bf16(o);
        l[r] = rn_bf16(o - __uint_as_float(h[r] << 16));
      }
      *(uint2*)(p.Yhi + (size_t)m * p.ldo + col) = make_uint2(h[0] | (h[1] << 16), h[2] | (h[3] << 16));
      *(uint2*)(p.Ylo + (size_t)m * p.ldo + col) = make_uint2(l[0] | (l[1] << 16), l[2] | (l[3] << 16));
    }
  } else {
#pragma unroll
    for (int f = 0; f < PN_NFW; ++f) {
      if (f == 1 && nb[1] == nb[0]) continue;  // odd tail
      const int col = nb[f] * 16 + 4 * g4;
#pragma unroll
      for (int mb = 0; mb < MT; ++mb) {
        const int m = mb * 16 + l16;
        const f32x4 v = acc[f][mb];
        if (m < p.M) {
          float4* dst = (float4*)(p.Y + part * p.split_stride + (size_t)m * p.ldy + col);
          if (CLV_DBG(p, 16)) __builtin_nontemporal_store(v, (f32x4*)dst);
          else *dst = make_float4(v[0], v[1], v[2], v[3]);
        }
      }
    }
  }
}

template <int MT, int KW, int EPI, int NBUF, int KST, bool NOPAD>
void launch_panel_kernel(const PanelGemm& g, int wgs, hipStream_t st) {
  constexpr size_t lds = (size_t)2 * 2 * MT * 16 * (KST + 16) * sizeof(bf16_t);
  static_assert(lds <= 160 * 1024, "stage buffers exceed the LDS");
  static bool attr_done = false;
  if (!attr_done) {
    hipFuncSetAttribute((const void*)gemm_panel_kernel<MT, KW, EPI, NBUF, KST, NOPAD>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    attr_done = true;
  }
  gemm_panel_kernel<MT, KW, EPI, NBUF, KST, NOPAD><<<wgs * g.k_parts, PN_WAVES * 64, lds, st>>>(g);
}
template <int MT, int KW, int EPI, int NBUF, int KST = PN_KST>
void launch_panel_one(const PanelGemm& g, int wgs, hipStream_t st) {
  if (MT == 4 && g.M == MT * 16) launch_panel_kernel<MT, KW, EPI, NBUF, KST, MT == 4>(g, wgs, st);   // (only the 64-row form has a NOPAD kernel)
  else launch_panel_kernel<MT, KW, EPI, NBUF, KST, false>(g, wgs, st);
}

}  // namespace

// N: output columns (EPI 1: the FFN width F, with W[0] = gate and W[1] = up, each [F, K]).
// Up to 64 rows: 256-column stages.  65..128 rows: eight row blocks per wavefront and 128-column stages (the two stage
// buffers of 128 rows would not fit the LDS otherwise); twice the matrix work per weight byte, still one pass over W.
bool panel_gemm_supported(int M, int N, int K, int epi) {
  if (M < 1 || M > 128 || K % (M > 64 ? 128 : PN_KST) != 0 || N % 16 != 0) return false;
  if (epi == 0) return N % 4 == 0;
  return true;
}

// Narrow outputs (N = hidden) have too few 16-column blocks to give every CU a full-K panel, so K
// is cut into ranges and each range writes its own fp32 partial, as the K-slice kernel does -- but
// with 4 blocks x 2 k-parts per workgroup a range is several thousand columns long, i.e. a handful
// of partials instead of one per 512 columns (K = 14336: 8 instead of 28, 21 MB less to write and
// read back per call).  Picks the largest divisor of the stage count that keeps the grid within
// one workgroup per CU; 0 when that leaves CUs idle or ranges shorter than 4 stages.  (More than 64 rows:
// there is no K-slice kernel to fall back to, so three quarters of the CUs are accepted.)
int panel_gemm_pick_k_parts(int M, int N, int K) {
  if (!panel_gemm_supported(M, N, K, 0) || N % 32 != 0) return 0;
  const int wgs_n = (N / 32 + 3) / 4, NS = K / (M > 64 ? 128 : PN_KST);
  int best = 0;
  for (int d = 1; d <= NS; ++d)
    if (NS % d == 0 && wgs_n * d <= 256 && NS / d >= 4) best = d;
  return (best > 1 && wgs_n * best >= (M > 64 ? 160 : 224)) ? best : 0;
}

void launch_gemm_panel(const PanelGemm& g_in, hipStream_t st) {
  PanelGemm g = g_in;
  g.dbg = tune_int("CLOVER_PANEL_DBG", 0);
  const int n_blocks = g.N / 16;
  const bool big = g.M > 64 || g.rows128, small = g.M <= 16 && !big;
  if (g.epi == 0 && g.k_parts > 1) {
    // K ranges: 4 units of two blocks x 2 k-parts per workgroup
    const int wgs = ((n_blocks + 1) / 2 + 3) / 4;
    if (small) launch_panel_one<1, 2, 0, 2>(g, wgs, st);
    else if (big) launch_panel_one<8, 2, 0, 3, 128>(g, wgs, st);  // (4 KB stages: a third buffer in flight measured 8 % faster)
    else launch_panel_one<4, 2, 0, 2>(g, wgs, st);
    return;
  }
  g.k_parts = 1; g.split_stride = 0;
  if (g.epi == 1) {
    // gate+up: 4 units x 2 k-parts per workgroup (896 blocks -> 224 workgroups for F = 14336)
    const int wgs = (n_blocks + 3) / 4;
    if (small) launch_panel_one<1, 2, 1, 2>(g, wgs, st);
    else if (big) launch_panel_one<8, 2, 1, 3, 128>(g, wgs, st);
    else launch_panel_one<4, 2, 1, 2>(g, wgs, st);
  } else {
    // plain: 8 units of two blocks per workgroup
    const int units = (n_blocks + 1) / 2;
    const int wgs = (units + 7) / 8;
    if (small) launch_panel_one<1, 1, 0, 2>(g, wgs, st);
    else if (big) launch_panel_one<8, 1, 0, 2, 128>(g, wgs, st);
    else launch_panel_one<4, 1, 0, 2>(g, wgs, st);
  }
}

}  // namespace clv
