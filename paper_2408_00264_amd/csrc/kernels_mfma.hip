// Weight-streaming skinny GEMM on the gfx950 matrix cores.
//
//   Y[M,N] = X[M,K] * W[N,K]^T     W bf16 (streamed once from HBM), X as split-bf16 planes, fp32 accumulate
//
// M is the number of tree rows (tens to a few hundred), so the kernel is bound by reading W.
//
// * v_mfma_f32_16x16x32_bf16 with the WEIGHT rows as the A operand and the activation rows as the
//   B operand.  A wavefront owns NF 16-row weight blocks and all M activation rows; each lane loads
//   its 16-byte A fragments straight from global memory into registers.  The weights are stored
//   fragment-major ([N/16][K/32][64 lanes][8]), so a load instruction reads one contiguous KB and
//   every weight byte is read exactly once.  This tiled kernel serves M > 64; up to 64 rows the
//   K-slice-resident kernel is used.
// * A random-init 32-layer stack amplifies a bf16 rounding of the activations about twenty-fold by
//   the last layer, so each activation x arrives as two bf16 planes, hi = bf16(x) and
//   lo = bf16(x - hi), and both halves are multiplied (two MFMAs per fragment): 16 mantissa bits,
//   at no cost in HBM traffic.  The planes are written once by the kernel that produces x.
// * Two producer wavefronts copy the activation chunk of step i+1 into LDS while four consumer
//   wavefronts multiply step i.  The consumers' memory queue holds nothing but the weight stream,
//   three chunks deep (registers), so they never wait behind a short-latency activation load.
// * Weight rows are K*2 bytes apart, a power of two: workgroups that walk K in the same order all
//   hit the same few HBM channels at the same time.  Each workgroup therefore starts at a different
//   (rotated) K chunk.
// * Split-K: every split writes its own fp32 partial tile; the kernel that consumes the result
//   (RoPE, residual add + RMSNorm, bias add) sums the partials in a fixed order.  No atomics, no
//   in-kernel fences, results independent of scheduling.
#include "clover_internal.h"

#include <cstdlib>

namespace clv {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ unsigned bf16_rn_bits(float a) {  // bf16 bits in the low half
  unsigned u = __float_as_uint(a);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return u >> 16;
}
// split two floats into packed (hi, hi) and (lo, lo) bf16 pairs
__device__ __forceinline__ void split2(float a, float b, unsigned& hi, unsigned& lo) {
  const unsigned ha = bf16_rn_bits(a), hb = bf16_rn_bits(b);
  const float ra = a - __uint_as_float(ha << 16), rb = b - __uint_as_float(hb << 16);
  hi = ha | (hb << 16);
  lo = bf16_rn_bits(ra) | (bf16_rn_bits(rb) << 16);
}

union Frag {
  u32x4 u;
  bf16x8 v;
};

constexpr int GEMM_CW = 4;                          // consumer wavefronts: stream weights, MFMA
constexpr int GEMM_PW = 2;                          // producer wavefronts: stage the activation chunks
constexpr int GEMM_THREADS = 64 * (GEMM_CW + GEMM_PW);

template <int MT, int NF, int KC>
__global__ __launch_bounds__(GEMM_THREADS) void gemm_mfma_kernel(MfmaGemm p) {
  constexpr int LDK = KC + 16;     // LDS row stride in bf16 (+32 B: a stride of 32 mod 64 bytes lets the fragment reads run at the full LDS rate)
  constexpr int KS = KC / 32;      // MFMA k-steps per chunk
  constexpr int ROWS = MT * 16;
  constexpr int PLANE = ROWS * LDK;  // one bf16 plane (hi or lo) of one buffer
  extern __shared__ __attribute__((aligned(16))) bf16_t smem[];  // [2 buffers][hi, lo][ROWS][LDK]

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int l16 = lane & 15, g4 = lane >> 4;
  const int K = p.K, M = p.M;
  const bool producer = wave >= GEMM_CW;
  const int grp = blockIdx.x * GEMM_CW + wave;
  const int n_groups = (p.mode == 2) ? p.N / (8 * NF) : p.N / (16 * NF);
  const bool active = !producer && grp < n_groups;

  const int n_chunks = K / KC;
  const int per = (n_chunks + p.splits - 1) / p.splits;
  const int c0 = blockIdx.y * per;
  const int n_it = max(0, min(c0 + per, n_chunks) - c0);
  const int rot = n_it > 0 ? (int)((blockIdx.x * 5u + blockIdx.y * 3u) % (unsigned)n_it) : 0;
  auto chunk_k = [&](int i) {
    int j = i + rot;
    if (j >= n_it) j -= n_it;
    return (c0 + j) * KC;
  };

  f32x4 acc[NF][MT];
#pragma unroll
  for (int f = 0; f < NF; ++f)
#pragma unroll
    for (int mb = 0; mb < MT; ++mb) acc[f][mb] = (f32x4){0.f, 0.f, 0.f, 0.f};
  int col[NF];
#pragma unroll
  for (int f = 0; f < NF; ++f) col[f] = 0;

  if (producer) {
    // ---------------- producer wavefronts: X[:, chunk] -> (hi, lo) bf16 planes in LDS ----------------
    // Their memory queue holds only these short-latency (L2) loads, so they never wait behind the
    // long HBM weight stream of the consumers.
    constexpr int SLOTS = KC / 8;                  // 16-byte slots per row and plane
    constexpr int NIT = (2 * ROWS * SLOTS) / (64 * GEMM_PW);
    static_assert((2 * ROWS * SLOTS) % (64 * GEMM_PW) == 0, "chunk must divide among the producer lanes");
    const int ptid = tid - 64 * GEMM_CW;
    auto stage_x = [&](int kc, int buf) {
      u32x4 v[NIT];
#pragma unroll
      for (int it = 0; it < NIT; ++it) {
        const int idx = it * (64 * GEMM_PW) + ptid;
        const int plane = idx / (ROWS * SLOTS), rem = idx % (ROWS * SLOTS);
        const int r = rem / SLOTS, sl = rem % SLOTS;
        v[it] = (u32x4){0u, 0u, 0u, 0u};
        if (r < M && !CLV_DBG(p, 4)) v[it] = *(const u32x4*)((plane ? p.Xlo : p.Xhi) + (size_t)r * p.ldx + kc + sl * 8);
      }
#pragma unroll
      for (int it = 0; it < NIT; ++it) {
        const int idx = it * (64 * GEMM_PW) + ptid;
        const int plane = idx / (ROWS * SLOTS), rem = idx % (ROWS * SLOTS);
        const int r = rem / SLOTS, sl = rem % SLOTS;
        *(u32x4*)(smem + (size_t)(buf * 2 + plane) * PLANE + r * LDK + sl * 8) = v[it];
      }
    };
    if (n_it > 0) {
      stage_x(chunk_k(0), 0);
      __syncthreads();
      for (int i = 0; i < n_it; ++i) {
        if (i + 1 < n_it) stage_x(chunk_k(i + 1), (i + 1) & 1);
        __syncthreads();
      }
    }
  } else {
    // ---------------- consumer wavefronts: weight stream + MFMA ----------------
    // weight row pointer and first output column of each fragment
    const bf16_t* wrow[NF];
#pragma unroll
    for (int f = 0; f < NF; ++f) {
      wrow[f] = p.W[0];
      if (active) {
        if (p.mode == 2) {
          constexpr int HF = NF / 2 > 0 ? NF / 2 : 1;
          const int r0 = grp * (8 * NF) + (f % HF) * 16;
          wrow[f] = ((f < HF) ? p.W[0] : p.W_up) + (size_t)(r0 / 16) * (K / 32) * 512 + lane * 8;
          col[f] = r0;
        } else {
          const int n = grp * (16 * NF) + f * 16;
          int s = 0;
          if (n >= p.seg_begin[1]) s = 1;
          if (n >= p.seg_begin[2]) s = 2;
          wrow[f] = p.W[s] + (size_t)((n - p.seg_begin[s]) / 16) * (K / 32) * 512 + lane * 8;
          col[f] = n;
        }
      }
    }
    constexpr int RING = 4;        // weight fragments of up to three future chunks are in flight
    Frag w[RING][NF][KS];
    auto load_w = [&](int slot, int kc) {
      if (!active || CLV_DBG(p, 2)) return;
#pragma unroll
      for (int f = 0; f < NF; ++f)
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
          w[slot][f][ks].u = __builtin_nontemporal_load((const u32x4*)(wrow[f] + (size_t)(kc / 32 + ks) * 512));
    };
    auto compute = [&](int slot, int buf) {
      if (!active) return;
      if (CLV_DBG(p, 1)) {  // keep the loads alive without the matrix work
#pragma unroll
        for (int f = 0; f < NF; ++f)
#pragma unroll
          for (int ks = 0; ks < KS; ++ks) acc[f][0][0] += __uint_as_float(w[slot][f][ks].u.x & 0x3f800000u);
        return;
      }
      const bf16_t* hi = smem + (size_t)buf * 2 * PLANE + l16 * LDK + g4 * 8;
      const bf16_t* lo = hi + PLANE;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
#pragma unroll
        for (int mb = 0; mb < MT; ++mb) {
          Frag bh, bl;
          bh.u = *(const u32x4*)(hi + mb * 16 * LDK + ks * 32);
          bl.u = *(const u32x4*)(lo + mb * 16 * LDK + ks * 32);
#pragma unroll
          for (int f = 0; f < NF; ++f) {
            acc[f][mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w[slot][f][ks].v, bl.v, acc[f][mb], 0, 0, 0);
            acc[f][mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w[slot][f][ks].v, bh.v, acc[f][mb], 0, 0, 0);
          }
        }
      }
    };
    // stage(r, i): multiply chunk i (weights in ring slot r, activations in LDS buffer i&1) while the
    // weights of chunk i+3 are fetched
    auto stage = [&](int r, int i) {
      if (i + 3 < n_it) load_w((r + 3) & 3, chunk_k(i + 3));
      compute(r, r & 1);
      __syncthreads();
    };
    if (n_it > 0) {
      load_w(0, chunk_k(0));
      if (n_it > 1) load_w(1, chunk_k(1));
      if (n_it > 2) load_w(2, chunk_k(2));
      __syncthreads();
      for (int i = 0; i < n_it; i += 4) {
        stage(0, i);
        if (i + 1 >= n_it) break;
        stage(1, i + 1);
        if (i + 2 >= n_it) break;
        stage(2, i + 2);
        if (i + 3 >= n_it) break;
        stage(3, i + 3);
      }
    }
  }

  if (!active) return;

  // ---- epilogue: lane holds rows m = mb*16 + l16, columns col + 4*g4 + 0..3 ----
#pragma unroll
  for (int mb = 0; mb < MT; ++mb) {
    const int m = mb * 16 + l16;
    if (m >= M) continue;
    if (p.mode == 2) {
      constexpr int HF = NF / 2 > 0 ? NF / 2 : 1;
#pragma unroll
      for (int f = 0; f < HF; ++f) {
        const f32x4 g = acc[f][mb], u = acc[(f + HF) % NF][mb];
        float o[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) o[r] = g[r] / (1.0f + expf(-g[r])) * u[r];
        unsigned h0, l0, h1, l1;
        split2(o[0], o[1], h0, l0);
        split2(o[2], o[3], h1, l1);
        const size_t off = (size_t)m * p.ldy + col[f] + 4 * g4;
        *(uint2*)(p.Yhi + off) = make_uint2(h0, h1);
        *(uint2*)(p.Ylo + off) = make_uint2(l0, l1);
      }
    } else {
      float* yrow = p.Y + (size_t)blockIdx.y * p.split_stride + (size_t)m * p.ldy;
#pragma unroll
      for (int f = 0; f < NF; ++f) {
        const f32x4 v = acc[f][mb];
        *(float4*)(yrow + col[f] + 4 * g4) = make_float4(v[0], v[1], v[2], v[3]);
      }
    }
  }
}

// ------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------
static int mt_for(int M) { return M <= 16 ? 1 : M <= 32 ? 2 : M <= 64 ? 4 : M <= 128 ? 8 : 16; }
static int kc_for(int mt) { return mt <= 4 ? 128 : mt == 8 ? 64 : 32; }

bool mfma_gemm_supported(int M, int N, int K, int mode) {
  if (M < 1 || M > 256) return false;
  if (K % 128 != 0) return false;
  return N % 16 == 0;
}

// fragments per wavefront: 2 when the column count allows it, else 1 (mode 2 always pairs gate/up)
static int nf_for(int N, int mode) {
  if (mode == 2) return 2;
  const int forced = tune_int("CLOVER_GEMM_NF", 0);
  if (forced == 1 || forced == 2) return (N % (16 * forced) == 0) ? forced : 1;
  return (N % 32 == 0 && N >= 8192) ? 2 : 1;
}
static int tiles_for(int N, int mode) {
  const int nf = nf_for(N, mode);
  const int groups = (mode == 2) ? N / (8 * nf) : N / (16 * nf);
  return (groups + 3) / 4;
}

int mfma_gemm_pick_splits(int M, int N, int K, int mode) {
  const int forced = tune_int("CLOVER_GEMM_SPLITS", 0);
  const int mt = mt_for(M);
  const int chunks = K / kc_for(mt);
  if (forced > 0) return std::min(forced, chunks);
  const int tiles = tiles_for(N, mode);
  int s = 1;
  if (mode == 2) return 1;  // the SwiGLU epilogue needs complete sums
  // fill the chip (>= 256 workgroups), keep >= 4 chunks per split for the pipeline, and keep the
  // fp32 partial tiles (splits * M * 4 bytes per column) below a quarter of the weight bytes (K * 2)
  while (tiles * s < 256 && (s * 2) * 4 <= chunks && (size_t)(s * 2) * M * 4 * 4 <= (size_t)K * 2) s *= 2;
  return s;
}

size_t mfma_gemm_out_bytes(int M, int N, int splits) { return (size_t)std::max(splits, 1) * M * N * sizeof(float); }

template <int MT, int NF, int KC>
static void launch_one(const MfmaGemm& g, dim3 grid, hipStream_t st) {
  constexpr size_t lds = (size_t)2 * 2 * MT * 16 * (KC + 16) * sizeof(bf16_t);
  static bool attr_done = false;
  if (!attr_done) {
    hipFuncSetAttribute((const void*)gemm_mfma_kernel<MT, NF, KC>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    attr_done = true;
  }
  gemm_mfma_kernel<MT, NF, KC><<<grid, GEMM_THREADS, lds, st>>>(g);
}

void launch_gemm_mfma(const MfmaGemm& g, hipStream_t st) {
  const int mt = mt_for(g.M), nf = nf_for(g.N, g.mode);
  dim3 grid(tiles_for(g.N, g.mode), g.splits);
  MfmaGemm g2 = g;
  g2.dbg = tune_int("CLOVER_GEMM_DBG", 0);
#define CLV_CASE(MT_, KC_)                                              \
  if (nf == 2) launch_one<MT_, 2, KC_>(g2, grid, st);                   \
  else launch_one<MT_, 1, KC_>(g2, grid, st);
  switch (mt) {
    case 1: CLV_CASE(1, 128) break;
    case 2: CLV_CASE(2, 128) break;
    case 4: CLV_CASE(4, 128) break;
    case 8: CLV_CASE(8, 64) break;
    default: CLV_CASE(16, 32) break;
  }
#undef CLV_CASE
}

}  // namespace clv
