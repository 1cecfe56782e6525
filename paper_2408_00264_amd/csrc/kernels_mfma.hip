// Weight-streaming skinny GEMM on the gfx950 matrix cores.
//
//   Y[M,N] = X[M,K] * W[N,K]^T     W bf16 row-major (streamed once from HBM), X fp32, fp32 accumulate
//
// M is the number of tree rows (tens to a few hundred), so the kernel is bound by reading W.
// Mapping: v_mfma_f32_16x16x32_bf16 with the WEIGHT rows as the A operand and the activation rows as
// the B operand.  A wavefront owns two 16-row weight blocks and all M activation rows; each lane
// loads its 16-byte A fragment straight from global memory (row = lane%16, k = 8*(lane/16)..+7),
// i.e. every weight byte is read exactly once and goes directly to registers.  The activation
// chunk is converted to bf16 and staged once per workgroup in LDS, from which every wavefront
// reads its B fragments.  Split-K partial tiles are combined by the last workgroup to arrive
// (fixed summation order, so results do not depend on scheduling).
#include "clover_internal.h"

namespace clv {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ unsigned pack_bf16x2(float a, float b) {
  unsigned ua = __float_as_uint(a), ub = __float_as_uint(b);
  ua += 0x7FFFu + ((ua >> 16) & 1u);
  ub += 0x7FFFu + ((ub >> 16) & 1u);
  return (ua >> 16) | (ub & 0xFFFF0000u);
}

union Frag {
  u32x4 u;
  bf16x8 v;
};

template <int MT, int KC>
__global__ __launch_bounds__(256) void gemm_mfma_kernel(MfmaGemm p) {
  constexpr int LDK = KC + 8;  // row stride in bf16: +16 bytes keeps the 16 lanes of a fragment read on distinct banks
  constexpr int KS = KC / 32;  // MFMA k-steps per chunk
  __shared__ __attribute__((aligned(16))) bf16_t xs[MT * 16 * LDK];
  __shared__ int s_last;

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int l16 = lane & 15, g4 = lane >> 4;
  const int K = p.K, M = p.M;
  const int pair = blockIdx.x * 4 + wave;
  const int n_pairs = (p.mode == 2) ? p.N / 16 : p.N / 32;
  const bool active = pair < n_pairs;

  // weight row pointers of this lane's two A fragments, and the output columns they produce
  const bf16_t *wa = p.W[0], *wb = p.W[0];
  int colA = 0, colB = 0;
  if (active) {
    if (p.mode == 2) {
      wa = p.W[0] + (size_t)(pair * 16 + l16) * K;
      wb = p.W_up + (size_t)(pair * 16 + l16) * K;
      colA = colB = pair * 16;
    } else {
      const int n = pair * 32;
      int s = 0;
      if (n >= p.seg_begin[1]) s = 1;
      if (n >= p.seg_begin[2]) s = 2;
      wa = p.W[s] + (size_t)(n - p.seg_begin[s] + l16) * K;
      wb = wa + (size_t)16 * K;
      colA = n;
      colB = n + 16;
    }
  }
  wa += g4 * 8;
  wb += g4 * 8;

  f32x4 acc[2][MT];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int mb = 0; mb < MT; ++mb) acc[i][mb] = (f32x4){0.f, 0.f, 0.f, 0.f};

  const int n_chunks = K / KC;
  const int per = (n_chunks + p.splits - 1) / p.splits;
  const int c0 = blockIdx.y * per;
  const int c1 = min(c0 + per, n_chunks);

  for (int c = c0; c < c1; ++c) {
    const int kc = c * KC;
    // issue this chunk's weight loads first: they are the long-latency HBM stream
    Frag fa[KS], fb[KS];
    if (active) {
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        fa[ks].u = __builtin_nontemporal_load((const u32x4*)(wa + kc + ks * 32));
        fb[ks].u = __builtin_nontemporal_load((const u32x4*)(wb + kc + ks * 32));
      }
    }
    // stage X[:, kc:kc+KC] as bf16: a thread converts 8 consecutive k of one row per pass
    constexpr int TPR = KC / 8;         // threads per row
    constexpr int RPP = 256 / TPR;      // rows per pass
#pragma unroll
    for (int r0 = 0; r0 < MT * 16; r0 += RPP) {
      const int r = r0 + tid / TPR, kk = (tid % TPR) * 8;
      u32x4 o = {0u, 0u, 0u, 0u};
      if (r < M) {
        const float4* src = (const float4*)(p.X + (size_t)r * p.ldx + kc + kk);
        const float4 v0 = src[0], v1 = src[1];
        o.x = pack_bf16x2(v0.x, v0.y);
        o.y = pack_bf16x2(v0.z, v0.w);
        o.z = pack_bf16x2(v1.x, v1.y);
        o.w = pack_bf16x2(v1.z, v1.w);
      }
      *(u32x4*)(&xs[r * LDK + kk]) = o;
    }
    __syncthreads();
    if (active) {
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
#pragma unroll
        for (int mb = 0; mb < MT; ++mb) {
          Frag b;
          b.u = *(const u32x4*)(&xs[(mb * 16 + l16) * LDK + ks * 32 + g4 * 8]);
          acc[0][mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa[ks].v, b.v, acc[0][mb], 0, 0, 0);
          acc[1][mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fb[ks].v, b.v, acc[1][mb], 0, 0, 0);
        }
      }
    }
    __syncthreads();
  }

  // ---- split-K: publish the partial tile; the last workgroup of this column sums all of them ----
  if (p.splits > 1) {
    // layout [tile][split][wave][i][mb][lane] of f32x4: a lane re-reads exactly its own positions
    f32x4* part = (f32x4*)p.partial;
    const size_t tile_stride = (size_t)p.splits * 4 * 2 * MT * 64;
    const size_t base = (size_t)blockIdx.x * tile_stride;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int mb = 0; mb < MT; ++mb)
        part[base + ((((size_t)blockIdx.y * 4 + wave) * 2 + i) * MT + mb) * 64 + lane] = acc[i][mb];
    __threadfence();
    __syncthreads();
    if (tid == 0) {
      const int prev = atomicAdd(&p.counters[blockIdx.x], 1);
      s_last = (prev == p.splits - 1) ? 1 : 0;
    }
    __syncthreads();
    if (!s_last) return;
    __threadfence();
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int mb = 0; mb < MT; ++mb) {
        f32x4 sum = (f32x4){0.f, 0.f, 0.f, 0.f};
        for (int s = 0; s < p.splits; ++s) {
          const f32x4 v = __builtin_nontemporal_load(
              &part[base + ((((size_t)s * 4 + wave) * 2 + i) * MT + mb) * 64 + lane]);
          sum += v;
        }
        acc[i][mb] = sum;
      }
    if (tid == 0) p.counters[blockIdx.x] = 0;  // ready for the next launch on this stream
  }
  if (!active) return;

  // ---- epilogue: lane holds Y[m = mb*16 + l16][col + 4*g4 + 0..3] ----
#pragma unroll
  for (int mb = 0; mb < MT; ++mb) {
    const int m = mb * 16 + l16;
    if (m >= M) continue;
    float* yrow = p.Y + (size_t)m * p.ldy;
    if (p.mode == 2) {
      const f32x4 g = acc[0][mb], u = acc[1][mb];
      float4 o;
      o.x = g[0] / (1.0f + __expf(-g[0])) * u[0];
      o.y = g[1] / (1.0f + __expf(-g[1])) * u[1];
      o.z = g[2] / (1.0f + __expf(-g[2])) * u[2];
      o.w = g[3] / (1.0f + __expf(-g[3])) * u[3];
      *(float4*)(yrow + colA + 4 * g4) = o;
    } else {
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const int col = (i == 0 ? colA : colB) + 4 * g4;
        f32x4 v = acc[i][mb];
        if (p.bias) {
          const bf16_t* bp = p.bias + col;
#pragma unroll
          for (int r = 0; r < 4; ++r) v[r] += __uint_as_float(((unsigned)bp[r]) << 16);
        }
        float4* dst = (float4*)(yrow + col);
        float4 o = {v[0], v[1], v[2], v[3]};
        if (p.mode == 1) {
          const float4 old = *dst;
          o.x += old.x; o.y += old.y; o.z += old.z; o.w += old.w;
        }
        *dst = o;
      }
    }
  }
}

// ------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------
static int mt_for(int M) { return M <= 16 ? 1 : M <= 32 ? 2 : M <= 64 ? 4 : M <= 128 ? 8 : 16; }
static int kc_for(int mt) { return mt <= 4 ? 256 : mt == 8 ? 128 : 64; }

bool mfma_gemm_supported(int M, int N, int K, int mode) {
  if (M < 1 || M > 256) return false;
  if (K % 256 != 0) return false;
  if (mode == 2) return N % 16 == 0;
  return N % 32 == 0;
}

static int tiles_for(int N, int mode) {
  const int pairs = (mode == 2) ? N / 16 : N / 32;
  return (pairs + 3) / 4;
}

int mfma_gemm_pick_splits(int M, int N, int K, int mode) {
  const int tiles = tiles_for(N, mode);
  const int chunks = K / kc_for(mt_for(M));
  int s = 1;
  // aim at >= 512 workgroups (two per CU) while keeping at least two chunks per split
  while (tiles * s < 512 && s * 2 <= chunks / 2 && s < 32) s *= 2;
  return s;
}

size_t mfma_gemm_partial_bytes(int M, int N, int K, int mode, int splits) {
  if (splits <= 1) return 0;
  return (size_t)tiles_for(N, mode) * splits * 4 * 2 * mt_for(M) * 64 * sizeof(float) * 4;
}

int mfma_gemm_counters(int N, int mode) { return tiles_for(N, mode); }

void launch_gemm_mfma(const MfmaGemm& g, hipStream_t st) {
  const int mt = mt_for(g.M);
  dim3 grid(tiles_for(g.N, g.mode), g.splits);
  switch (mt) {
    case 1: gemm_mfma_kernel<1, 256><<<grid, 256, 0, st>>>(g); break;
    case 2: gemm_mfma_kernel<2, 256><<<grid, 256, 0, st>>>(g); break;
    case 4: gemm_mfma_kernel<4, 256><<<grid, 256, 0, st>>>(g); break;
    case 8: gemm_mfma_kernel<8, 128><<<grid, 256, 0, st>>>(g); break;
    default: gemm_mfma_kernel<16, 64><<<grid, 256, 0, st>>>(g); break;
  }
}

}  // namespace clv
