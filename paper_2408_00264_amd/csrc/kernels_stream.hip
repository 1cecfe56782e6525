// K-slice-resident weight-streaming GEMM for few activation rows (M <= 64) on gfx950, and the
// fragment-major weight layout both MFMA GEMMs read.
//
//   P[s][M,N] = X[M, slice s of K] * W[N, slice s of K]^T        (fp32 partial per K slice)
//
// Why this shape.  With M <= 64 the GEMM is bound by streaming W from HBM, and what has to be kept
// small is everything else that crosses the L2 fabric.  A workgroup is therefore tied to ONE slice of
// K (512 columns): its activation slice (hi and lo bf16 planes, 64 x 512 x 4 B = 128 KB) is copied
// into LDS once (global -> LDS directly, a row per instruction), and from then on its eight wavefronts do nothing but stream weight fragments
// (global -> registers, 16 KB in flight per wavefront) and multiply them against the resident slice:
// no barrier and no activation traffic in the steady state.  Each workgroup walks a contiguous range
// of 16-row weight blocks; the per-slice partial tiles are summed, in slice order, by whichever
// kernel consumes the result (RoPE, residual add + RMSNorm, SwiGLU, bias add).
//
// Weight layout.  A 16x16x32 MFMA A-fragment takes, per lane, 8 consecutive k of row lane%16 at
// k-offset 8*(lane/16).  Read from a row-major matrix that is 16 rows x 64 B per load instruction,
// i.e. every 128-byte line is requested by two different instructions and crosses the L2->L1 fabric
// twice.  The weights are therefore re-laid out once (at init, into the library's own copy) as
// [N/16][K/32][64 lanes][8] so that one load instruction reads one contiguous KB.
#include "clover_internal.h"

#include <algorithm>
#include <cstdlib>
#include <type_traits>

namespace clv {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef const u32x4 __attribute__((address_space(1)))* gvec_ptr;  // global (not flat) address: vmcnt only

union Frag {
  u32x4 u;
  bf16x8 v;
};

// ------------------------------------------------------------------------------------------
// row-major [N,K] -> fragment-major [N/16][K/32][64][8]
// ------------------------------------------------------------------------------------------
__global__ void pack_weight_kernel(const bf16_t* __restrict__ src, bf16_t* __restrict__ dst, int N, int K) {
  const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;  // one 16-byte piece each
  const size_t total = (size_t)N * K / 8;
  if (idx >= total) return;
  const int lane = (int)(idx & 63);
  const size_t tile = idx >> 6;
  const int KT = K / 32;
  const size_t nb = tile / KT;
  const int kt = (int)(tile % KT);
  const size_t row = nb * 16 + (lane & 15);
  const int k = kt * 32 + (lane >> 4) * 8;
  *(u32x4*)(dst + idx * 8) = *(const u32x4*)(src + row * K + k);
}
void launch_pack_weight(const void* src, void* dst, int N, int K, hipStream_t st) {
  const size_t total = (size_t)N * K / 8;
  pack_weight_kernel<<<(unsigned)((total + 255) / 256), 256, 0, st>>>((const bf16_t*)src, (bf16_t*)dst, N, K);
}

// ------------------------------------------------------------------------------------------
// the streaming kernel
// ------------------------------------------------------------------------------------------
constexpr int ST_WAVES = 8;
constexpr int ST_KSL = 512;          // K columns per slice
constexpr int ST_LDK = ST_KSL + 16;  // LDS row stride (bf16): 32 mod 64 bytes, the stride at which fragment reads run at the full LDS rate
constexpr int ST_STAGE = 4;          // 32-column weight tiles per pipeline stage (4 KB per fragment, contiguous); deeper
                                     // stages (8) measured 4 % slower over the verify pass: longer queues, no more bandwidth

// TAG only names the instantiation (1: the gate+up projection) so that a kernel trace lists the
// dominant launch under its own name.
template <int MT, int NF, int TAG>
__global__ __launch_bounds__(ST_WAVES * 64) void gemm_stream_kernel(StreamGemm p) {
  constexpr int ROWS = MT * 16;
  constexpr int PLANE = ROWS * ST_LDK;
  extern __shared__ __attribute__((aligned(16))) bf16_t xs[];  // [hi, lo][ROWS][ST_LDK]

  const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
  const int l16 = lane & 15, g4 = lane >> 4;
  const int slice = blockIdx.x % p.n_slices, grp = blockIdx.x / p.n_slices;
  const int k0 = slice * ST_KSL;
  const int kt_n = min(ST_KSL, p.K - k0) / 32;  // 32-column tiles in this slice (multiple of ST_STAGE)
  const int n_st = kt_n / ST_STAGE;
  const int KT = p.K / 32;

  // units of NF 16-row blocks; this workgroup owns units [u0, u1)
  const int n_units = p.N / (16 * NF);
  const int per = (n_units + p.groups - 1) / p.groups;
  const int u0 = grp * per, u1 = min(n_units, u0 + per);
  if (u0 >= u1) return;  // whole workgroup

  // ---- this wavefront's units: u0 + wave, u0 + wave + 8, ...; one item = one stage of one unit ----
  const int my_units = (u1 - u0 - wave + ST_WAVES - 1) / ST_WAVES;
  const int n_items = max(my_units, 0) * n_st;

  Frag w[2][NF][ST_STAGE];
  f32x4 acc[NF][MT];
#pragma unroll
  for (int f = 0; f < NF; ++f)
#pragma unroll
    for (int mb = 0; mb < MT; ++mb) acc[f][mb] = (f32x4){0.f, 0.f, 0.f, 0.f};

  // Segment lookup by arithmetic on scalars held in registers: base = W0 + [n >= b1] * d1 + [n >= b2] * d2
  // with d1, d2 the pointer differences corrected for the segments' first rows.  (Indexing the
  // by-value argument struct with a runtime index, or a chain of pointer selects, ends up as a
  // memory load whose wait also drains the weight loads in flight.)
  const long long KT512 = (long long)KT * 512;
  const long long seg_w0 = (long long)p.W[0];
  const long long seg_d1 = (long long)p.W[1] - (long long)p.W[0] - (long long)(p.seg_begin[1] / 16) * KT512 * 2;
  const long long seg_d2 = (long long)p.W[2] - (long long)p.W[1] - (long long)((p.seg_begin[2] - p.seg_begin[1]) / 16) * KT512 * 2;
  const int seg_b1 = p.seg_begin[1], seg_b2 = p.seg_begin[2];
  auto frag_base = [&](int unit, int f) -> const bf16_t* {
    const int n = (unit * NF + f) * 16;
    const long long b = seg_w0 + (seg_d1 & -(long long)(n >= seg_b1)) + (seg_d2 & -(long long)(n >= seg_b2));
    return (const bf16_t*)b + ((size_t)(n / 16) * KT + k0 / 32) * 512 + lane * 8;
  };
  auto load = [&](auto bufc, int item) {
    constexpr int buf = decltype(bufc)::value;
    const int unit = u0 + wave + (item / n_st) * ST_WAVES, st = item % n_st;
#pragma unroll
    for (int f = 0; f < NF; ++f) {
      const bf16_t* b = frag_base(unit, f) + (size_t)st * ST_STAGE * 512;
#pragma unroll
      for (int t = 0; t < ST_STAGE; ++t) w[buf][f][t].u = __builtin_nontemporal_load((gvec_ptr)(b + t * 512));
    }
  };
  constexpr std::integral_constant<int, 0> B0{};
  constexpr std::integral_constant<int, 1> B1{};
  if (n_items > 0) load(B0, 0);  // the HBM stream starts before the activation slice is staged

  // ---- activation slice -> LDS, without a stop in registers: one wavefront instruction moves one row of one plane
  // (64 lanes x 16 B = 512 columns) from global memory to the row's place in the LDS (the hardware writes lane l's 16
  // bytes at row base + 16 l).  Rows >= M read row M - 1 again: an output row depends on its own activation row only
  // and rows >= M are never stored.  In a last slice shorter than 512 columns the lanes past it re-read its last
  // piece (the products never touch those LDS columns).  The compiler is not told that these loads write the LDS;
  // the wait before the barrier is written by hand. ----
  {
    const int slots = kt_n * 4;  // 16-byte pieces per row and plane (<= 64)
    const unsigned lane_off = (unsigned)(min(lane, slots - 1) * 16);
    const unsigned lds0 = (unsigned)(size_t)(__attribute__((address_space(3))) char*)xs;
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    constexpr int XIT = 2 * ROWS / ST_WAVES;
#pragma unroll
    for (int it = 0; it < XIT; ++it) {
      const int rp = it * ST_WAVES + wave_u, plane = rp / ROWS, r = rp % ROWS;
      if (CLV_DBG(p, 1)) continue;
      const bf16_t* src = (plane ? p.Xlo : p.Xhi) + (size_t)min(r, p.M - 1) * p.ldx + k0;
      const unsigned m0 = __builtin_amdgcn_readfirstlane(lds0 + 2u * (unsigned)(plane * PLANE + r * ST_LDK));
      asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2" : : "s"(m0), "v"(lane_off),
                   "s"((const __attribute__((address_space(1))) char*)src) : "m0");
    }
    __builtin_amdgcn_s_waitcnt(0 | (7 << 4) | (15 << 8));   // vmcnt(0): this wavefront's rows are in the LDS
  }
  __syncthreads();
  if (n_items == 0) return;

  auto compute = [&](auto bufc, int item) {
    constexpr int buf = decltype(bufc)::value;
    const int st = item % n_st;
    const bf16_t* hi = xs + l16 * ST_LDK + g4 * 8 + st * ST_STAGE * 32;
    const bf16_t* lo = hi + PLANE;
#pragma unroll
    for (int t = 0; t < ST_STAGE; ++t) {
#pragma unroll
      for (int mb = 0; mb < MT; ++mb) {
        Frag bh, bl;
        bh.u = *(const u32x4*)(hi + mb * 16 * ST_LDK + t * 32);
        bl.u = *(const u32x4*)(lo + mb * 16 * ST_LDK + t * 32);
#pragma unroll
        for (int f = 0; f < NF; ++f) {
          acc[f][mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w[buf][f][t].v, bl.v, acc[f][mb], 0, 0, 0);
          acc[f][mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w[buf][f][t].v, bh.v, acc[f][mb], 0, 0, 0);
        }
      }
    }
    if (st == n_st - 1) {  // unit complete: write this slice's partial tile and start over
      const int unit = u0 + wave + (item / n_st) * ST_WAVES;
      float* ybase = p.Y + (size_t)slice * p.split_stride;
#pragma unroll
      for (int f = 0; f < NF; ++f) {
        const int col = (unit * NF + f) * 16 + 4 * g4;
#pragma unroll
        for (int mb = 0; mb < MT; ++mb) {
          const int m = mb * 16 + l16;
          const f32x4 v = acc[f][mb];
          if (m < p.M && !CLV_DBG(p, 2)) {
            float4* dst = (float4*)(ybase + (size_t)m * p.ldy + col);
            if (CLV_DBG(p, 4)) __builtin_nontemporal_store(v, (f32x4*)dst);
            else *dst = make_float4(v[0], v[1], v[2], v[3]);
          }
          acc[f][mb] = (f32x4){0.f, 0.f, 0.f, 0.f};
        }
      }
    }
  };

  // Steady state without conditions around the loads, so that the wait before a compute step
  // counts exactly the loads issued after its buffer and leaves them in flight.
  int i = 0;
  // (the scheduling barriers keep the compiler from sinking a buffer's loads below the compute step
  // they are meant to overlap)
  for (; i + 2 < n_items; i += 2) {
    load(B1, i + 1);
    __builtin_amdgcn_sched_barrier(0);
    compute(B0, i);
    __builtin_amdgcn_sched_barrier(0);
    load(B0, i + 2);
    __builtin_amdgcn_sched_barrier(0);
    compute(B1, i + 1);
    __builtin_amdgcn_sched_barrier(0);
  }
  if (i + 1 < n_items) {
    load(B1, i + 1);
    __builtin_amdgcn_sched_barrier(0);
    compute(B0, i);
    compute(B1, i + 1);
  } else {
    compute(B0, i);
  }
}

// ------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------
bool stream_gemm_supported(int M, int N, int K) {
  return M >= 1 && M <= 64 && K % (ST_STAGE * 32) == 0 && N % 32 == 0;
}
int stream_gemm_slices(int K) { return (K + ST_KSL - 1) / ST_KSL; }
size_t stream_gemm_out_bytes(int M, int N, int K) { return (size_t)stream_gemm_slices(K) * M * N * sizeof(float); }

template <int MT, int NF, int TAG>
static void launch_stream_one(const StreamGemm& g, int wgs, hipStream_t st) {
  constexpr size_t lds = (size_t)2 * MT * 16 * ST_LDK * sizeof(bf16_t);
  static bool attr_done = false;
  if (!attr_done) {
    hipFuncSetAttribute((const void*)gemm_stream_kernel<MT, NF, TAG>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    attr_done = true;
  }
  gemm_stream_kernel<MT, NF, TAG><<<wgs, ST_WAVES * 64, lds, st>>>(g);
}

void launch_gemm_stream(StreamGemm g, hipStream_t st) {
  g.n_slices = stream_gemm_slices(g.K);
  g.dbg = tune_int("CLOVER_STREAM_DBG", 0);
  const int mt = g.M <= 16 ? 1 : 4;  // 17..32 rows run as 64 (zero rows cost MFMA time only, the kernel is HBM-bound)
  // one workgroup per CU: a 64-row slice fills most of the LDS.  Pair fragments (halves the LDS
  // reads per weight byte) when that still leaves every wavefront a unit.
  const int target = tune_int("CLOVER_STREAM_WGS", 256);
  int groups = std::max(1, target / g.n_slices);
  int nf = 2;
  if (g.N / 32 < groups * ST_WAVES) nf = 1;
  const int n_units = g.N / (16 * nf);
  groups = std::min(groups, std::max(1, (n_units + ST_WAVES - 1) / ST_WAVES));
  g.groups = groups;
  const int wgs = groups * g.n_slices;
#define CLV_ST(MT_)                                                   \
  if (nf == 2 && g.tag == 1) launch_stream_one<MT_, 2, 1>(g, wgs, st); \
  else if (nf == 2) launch_stream_one<MT_, 2, 0>(g, wgs, st);          \
  else launch_stream_one<MT_, 1, 0>(g, wgs, st);
  if (mt == 1) { CLV_ST(1) } else { CLV_ST(4) }
#undef CLV_ST
}

// ------------------------------------------------------------------------------------------
// consumer of the fused gate/up projection: h = silu(sum_s P[s][m][c]) * (sum_s P[s][m][F + c]), as planes
// ------------------------------------------------------------------------------------------
// float -> bf16 (round to nearest even) through the hardware conversion (v_cvt_pk_bf16_f32)
__device__ __forceinline__ unsigned rn_bf16(float a) { return (unsigned)__builtin_bit_cast(unsigned short, (__bf16)a); }
__global__ void reduce_swiglu_kernel(const float* __restrict__ P, int splits, size_t sps, int ldp, int F,
                                     bf16_t* __restrict__ hi, bf16_t* __restrict__ lo, int ldo) {
  const size_t row = blockIdx.y;
  const int c = (blockIdx.x * blockDim.x + threadIdx.x) * 4;
  if (c >= F) return;
  float4 g = {0.f, 0.f, 0.f, 0.f}, u = {0.f, 0.f, 0.f, 0.f};
  for (int s = 0; s < splits; ++s) {
    const float4 a = *(const float4*)(P + s * sps + row * ldp + c);
    const float4 b = *(const float4*)(P + s * sps + row * ldp + F + c);
    g.x += a.x; g.y += a.y; g.z += a.z; g.w += a.w;
    u.x += b.x; u.y += b.y; u.z += b.z; u.w += b.w;
  }
  const float o[4] = {g.x / (1.0f + expf(-g.x)) * u.x, g.y / (1.0f + expf(-g.y)) * u.y,
                      g.z / (1.0f + expf(-g.z)) * u.z, g.w / (1.0f + expf(-g.w)) * u.w};
  unsigned h[4], l[4];
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    h[r] = rn_bf16(o[r]);
    l[r] = rn_bf16(o[r] - __uint_as_float(h[r] << 16));
  }
  *(uint2*)(hi + row * ldo + c) = make_uint2(h[0] | (h[1] << 16), h[2] | (h[3] << 16));
  *(uint2*)(lo + row * ldo + c) = make_uint2(l[0] | (l[1] << 16), l[2] | (l[3] << 16));
}
void launch_reduce_swiglu(const float* P, int splits, size_t split_stride, int ldp, int F, bf16_t* hi, bf16_t* lo,
                          int ldo, int rows, hipStream_t st) {
  if (rows <= 0) return;
  reduce_swiglu_kernel<<<dim3((F / 4 + 255) / 256, rows), 256, 0, st>>>(P, splits, split_stride, ldp, F, hi, lo, ldo);
}

}  // namespace clv
