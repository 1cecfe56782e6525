// Fused bookkeeping kernels of the draft head on the MFMA path (bf16 weights).
//
// The draft head (Clover-2 Sec. 3.1-3.3) is a chain of small dependent steps: token embedding,
// RMSNorm, the Attention Decoder's three projections and its cosine gate, the per-depth FC and the
// shared LM head with its ranking.  At one to sixteen rows each of these is launch-bound, so the
// element-wise steps between two GEMMs are folded into ONE kernel each, and those kernels read the
// GEMMs' K-slice partial sums (and add the bias) themselves instead of waiting for a reduce pass:
//
//   draft_pre      rows of (hidden state, follow-up token)  -> planes of RMSNorm(x)*gain, planes of the embedding
//   ad_gate_fused  q/k/v partials + biases -> per-head cosine gate, residual; writes the result where the next
//                  step wants it (fp32 row, normalised planes for the Augmenting Block, or the
//                  regressive state of a tree node plus the first half of the FC input planes)
//   draft_root     last accepted row -> root state, root token, FC_0 input planes; advances the
//                  Augmenting Block's cache length
//   draft_level    per internal node of one tree depth: the parent's state -> normalised planes, the node's token's
//                  embedding -> planes (AD input and second half of the FC input)
//
// Activation planes: hi = bf16(x), lo = bf16(x - hi).  An embedding row is bf16 already: hi = its bits, lo = 0.
#include "clover_internal.h"

namespace clv {

namespace {

// float -> bf16 (round to nearest even) through the hardware conversion (v_cvt_pk_bf16_f32)
__device__ __forceinline__ unsigned rn_bf16(float a) { return (unsigned)__builtin_bit_cast(unsigned short, (__bf16)a); }
__device__ __forceinline__ float bf16f(bf16_t b) { return __uint_as_float((unsigned)b << 16); }
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
// sum over a block of NW wavefronts; `red` has NW floats; every thread gets the total
template <int NW>
__device__ __forceinline__ float block_sum(float v, float* red) {
  v = wave_sum(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  float t = 0.f;
#pragma unroll
  for (int w = 0; w < NW; ++w) t += red[w];
  return t;
}
__device__ __forceinline__ void store_planes4(bf16_t* hi, bf16_t* lo, size_t off, float o0, float o1, float o2, float o3) {
  const unsigned h0 = rn_bf16(o0), h1 = rn_bf16(o1), h2 = rn_bf16(o2), h3 = rn_bf16(o3);
  const unsigned l0 = rn_bf16(o0 - __uint_as_float(h0 << 16)), l1 = rn_bf16(o1 - __uint_as_float(h1 << 16));
  const unsigned l2 = rn_bf16(o2 - __uint_as_float(h2 << 16)), l3 = rn_bf16(o3 - __uint_as_float(h3 << 16));
  *(uint2*)(hi + off) = make_uint2(h0 | (h1 << 16), h2 | (h3 << 16));
  *(uint2*)(lo + off) = make_uint2(l0 | (l1 << 16), l2 | (l3 << 16));
}
// planes of RMSNorm(x[0..H)) * gain at (hi, lo) + off; 256 threads; x is read twice (L1/L2 hit)
__device__ __forceinline__ void norm_row_planes(const float* __restrict__ x, const bf16_t* __restrict__ gain, float eps,
                                                int H, bf16_t* hi, bf16_t* lo, size_t off, float* red) {
  float ss = 0.f;
  for (int c = threadIdx.x * 4; c < H; c += 1024) {
    const float4 v = *(const float4*)(x + c);
    ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
  }
  const float tot = block_sum<4>(ss, red);
  const float scale = 1.0f / sqrtf(tot / (float)H + eps);
  for (int c = threadIdx.x * 4; c < H; c += 1024) {
    const float4 v = *(const float4*)(x + c);
    store_planes4(hi, lo, off + c, v.x * scale * bf16f(gain[c]), v.y * scale * bf16f(gain[c + 1]),
                  v.z * scale * bf16f(gain[c + 2]), v.w * scale * bf16f(gain[c + 3]));
  }
}
// planes of one embedding row (bf16 bits): hi = bits, lo = 0
__device__ __forceinline__ void embed_row_planes(const bf16_t* __restrict__ table, int t, int H, bf16_t* hi, bf16_t* lo,
                                                 size_t off) {
  for (int c = threadIdx.x * 4; c < H; c += 1024) {
    *(uint2*)(hi + off + c) = *(const uint2*)(table + (size_t)t * H + c);
    *(uint2*)(lo + off + c) = make_uint2(0u, 0u);
  }
}

// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void draft_pre_kernel(const float* __restrict__ hid, const int* __restrict__ tok,
                                                        const bf16_t* __restrict__ gain, float eps,
                                                        const bf16_t* __restrict__ table, int vocab, int H, RowMap rm,
                                                        bf16_t* a_hi, bf16_t* a_lo, bf16_t* y_hi, bf16_t* y_lo) {
  __shared__ float red[4];
  const int i = blockIdx.x, b = blockIdx.y;
  const int nv = rm.n_valid ? min(rm.n_valid[b], rm.n) : rm.n;
  if (i >= nv) return;
  const size_t row = (size_t)b * rm.R + i;
  norm_row_planes(hid + row * H, gain, eps, H, a_hi, a_lo, row * H, red);
  int t = tok[row];
  t = t < 0 ? 0 : (t >= vocab ? vocab - 1 : t);
  embed_row_planes(table, t, H, y_hi, y_lo, row * H);
}

// ------------------------------------------------------------------------------------------
// One 512-thread block per GEMM row, a thread takes four adjacent columns at a time (a head spans H/heads/4 adjacent
// lanes).
// q = bq + sum_s Pq[s][row], (k | v) = (bk | bv) + sum_s Pkv[s][row]; per head h:
// r_h = x_h + cos(q_h, k_h) * v_h  (Sec. 3.1 and the Attention-Decoder listing of Appendix A.3; each norm
// clamped at 1e-8).  Every partial sum is loaded before the first one is used: one memory round trip.
struct AdGate {
  const float* x; int ldx;
  const float* Pq; int Sq; size_t sps_q;
  const float* Pkv; int Skv; size_t sps_kv;
  const bf16_t *bq, *bk, *bv;
  int H, heads;
  const int *nodes, *parent; int n_lvl, R;
  int nodes_stride, parent_stride;
  const int* m;
  float* out; int ldo;
  const bf16_t* gain; float eps;
  bf16_t *n_hi, *n_lo;
  bf16_t *c_hi, *c_lo; int ldc;
};
constexpr int AG_MAXS = 8;
__device__ __forceinline__ float4 ld_bias4(const bf16_t* b, int c) {
  const uint2 u = *(const uint2*)(b + c);
  return make_float4(__uint_as_float(u.x << 16), __uint_as_float(u.x & 0xFFFF0000u), __uint_as_float(u.y << 16),
                     __uint_as_float(u.y & 0xFFFF0000u));
}
__global__ __launch_bounds__(512) void ad_gate_fused_kernel(AdGate p) {
  __shared__ float red[8];
  const int g = blockIdx.x;
  size_t xin = g, xout = g;
  if (p.nodes) {
    const int r = g % p.n_lvl, b = g / p.n_lvl, u = p.nodes[(size_t)b * p.nodes_stride + r];
    if (p.m && p.m[b] < 1) return;  // whole block
    xin = (size_t)b * p.R + p.parent[(size_t)b * p.parent_stride + u];
    xout = (size_t)b * p.R + u;
  }
  const int H = p.H, lanes_per_head = H / p.heads / 4;  // power of two, <= 64
  const float* xr = p.x + xin * p.ldx;
  float* orow = p.out + xout * p.ldo;
  const float* pq = p.Pq + (size_t)g * H;
  const float* pkv = p.Pkv + (size_t)g * 2 * H;
  float ss = 0.f;
  for (int c0 = 0; c0 < H; c0 += 2048) {  // (uniform trip count; threads past H idle but keep the shuffles in step)
    const int c = c0 + threadIdx.x * 4;
    const bool in = c < H;
    float4 q = {0.f, 0.f, 0.f, 0.f}, k = q, v = q, xv = q;
    // every load is unconditional (a clamped address, the value zeroed afterwards): no branch around a load, so
    // all of them are in flight together
    const int cc = in ? c : 0;
    float4 tq[AG_MAXS], tk[AG_MAXS], tv[AG_MAXS];
#pragma unroll
    for (int s = 0; s < AG_MAXS; ++s) {
      const int sq = min(s, p.Sq - 1), sk = min(s, p.Skv - 1);
      tq[s] = *(const float4*)(pq + sq * p.sps_q + cc);
      tk[s] = *(const float4*)(pkv + sk * p.sps_kv + cc);
      tv[s] = *(const float4*)(pkv + sk * p.sps_kv + H + cc);
    }
    q = ld_bias4(p.bq, cc); k = ld_bias4(p.bk, cc); v = ld_bias4(p.bv, cc);
    xv = *(const float4*)(xr + cc);
#pragma unroll
    for (int s = 0; s < AG_MAXS; ++s) {  // slice order
      const float fq = s < p.Sq ? 1.f : 0.f, fk = s < p.Skv ? 1.f : 0.f;
      tq[s].x *= fq; tq[s].y *= fq; tq[s].z *= fq; tq[s].w *= fq;
      tk[s].x *= fk; tk[s].y *= fk; tk[s].z *= fk; tk[s].w *= fk;
      tv[s].x *= fk; tv[s].y *= fk; tv[s].z *= fk; tv[s].w *= fk;
      q.x += tq[s].x; q.y += tq[s].y; q.z += tq[s].z; q.w += tq[s].w;
      k.x += tk[s].x; k.y += tk[s].y; k.z += tk[s].z; k.w += tk[s].w;
      v.x += tv[s].x; v.y += tv[s].y; v.z += tv[s].z; v.w += tv[s].w;
    }
    float qq = q.x * q.x + q.y * q.y + q.z * q.z + q.w * q.w;
    float kk = k.x * k.x + k.y * k.y + k.z * k.z + k.w * k.w;
    float qk = q.x * k.x + q.y * k.y + q.z * k.z + q.w * k.w;
    for (int o = lanes_per_head >> 1; o > 0; o >>= 1) {
      qq += __shfl_xor(qq, o, 64); kk += __shfl_xor(kk, o, 64); qk += __shfl_xor(qk, o, 64);
    }
    const float att = qk / (fmaxf(sqrtf(qq), 1e-8f) * fmaxf(sqrtf(kk), 1e-8f));
    const float4 r = {xv.x + att * v.x, xv.y + att * v.y, xv.z + att * v.z, xv.w + att * v.w};
    if (in) {
      *(float4*)(orow + c) = r;
      ss += r.x * r.x + r.y * r.y + r.z * r.z + r.w * r.w;
      if (p.c_hi) store_planes4(p.c_hi, p.c_lo, (size_t)g * p.ldc + c, r.x, r.y, r.z, r.w);
    }
  }
  if (!p.gain) return;
  const float tot = block_sum<8>(ss, red);   // also orders this block's row stores before the reads below
  const float scale = 1.0f / sqrtf(tot / (float)H + p.eps);
  for (int c = threadIdx.x * 4; c < H; c += 2048) {
    const float4 v = *(const float4*)(orow + c);
    const float4 gn = ld_bias4(p.gain, c);
    store_planes4(p.n_hi, p.n_lo, (size_t)g * H + c, v.x * scale * gn.x, v.y * scale * gn.y, v.z * scale * gn.z, v.w * scale * gn.w);
  }
}

// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void draft_root_fused_kernel(const float* __restrict__ a, const int* __restrict__ next_tok,
                                                               const int* __restrict__ m, int R, int H,
                                                               float* __restrict__ state, int* __restrict__ tokens,
                                                               bf16_t* y_hi, bf16_t* y_lo, int* __restrict__ aug_len,
                                                               int Rs) {
  const int b = blockIdx.x;
  const int mb = min(m[b], R);
  for (int c = threadIdx.x * 4; c < H; c += 1024) {
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    if (mb >= 1) v = *(const float4*)(a + ((size_t)b * R + mb - 1) * H + c);
    *(float4*)(state + ((size_t)b * Rs) * H + c) = v;
    store_planes4(y_hi, y_lo, (size_t)b * H + c, v.x, v.y, v.z, v.w);
  }
  if (threadIdx.x == 0) {
    if (mb >= 1) tokens[(size_t)b * Rs] = next_tok[(size_t)b * R + mb - 1];
    aug_len[b] += max(m[b], 0);
  }
}

// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void draft_level_kernel(const float* __restrict__ state, const int* __restrict__ tokens,
                                                          const int* __restrict__ nodes, const int* __restrict__ parent,
                                                          int n_lvl, int R, int H, const bf16_t* __restrict__ table,
                                                          int vocab, const bf16_t* __restrict__ gain, float eps,
                                                          bf16_t* a_hi, bf16_t* a_lo, bf16_t* y_hi, bf16_t* y_lo,
                                                          bf16_t* c_hi, bf16_t* c_lo, int nodes_stride,
                                                          int parent_stride) {
  __shared__ float red[4];
  const int r = blockIdx.x, b = blockIdx.y;
  const int u = nodes[(size_t)b * nodes_stride + r], p = parent[(size_t)b * parent_stride + u];
  int t = tokens[(size_t)b * R + u];
  t = t < 0 ? 0 : (t >= vocab ? vocab - 1 : t);
  const size_t row = (size_t)b * n_lvl + r;
  norm_row_planes(state + ((size_t)b * R + p) * H, gain, eps, H, a_hi, a_lo, row * H, red);
  embed_row_planes(table, t, H, y_hi, y_lo, row * H);
  embed_row_planes(table, t, H, c_hi, c_lo, row * 2 * H + H);
}

}  // namespace

void launch_draft_pre(const float* hid, const int* tok, const void* gain, float eps, const void* table, int vocab, int H,
                      RowMap rm, bf16_t* a_hi, bf16_t* a_lo, bf16_t* y_hi, bf16_t* y_lo, hipStream_t st) {
  draft_pre_kernel<<<dim3(rm.n, rm.B), 256, 0, st>>>(hid, tok, (const bf16_t*)gain, eps, (const bf16_t*)table, vocab, H,
                                                     rm, a_hi, a_lo, y_hi, y_lo);
}

// a head must span a power-of-two number (<= 64) of four-column lanes
bool ad_gate_fused_supported(int H, int heads) {
  if (heads < 1 || H % (4 * heads) != 0) return false;
  const int l = H / heads / 4;
  return l >= 1 && l <= 64 && (l & (l - 1)) == 0;
}

void launch_ad_gate_fused(const AdGateArgs& a, int rows, hipStream_t st) {
  if (rows <= 0) return;
  AdGate p;
  p.x = a.x; p.ldx = a.ldx;
  p.Pq = a.Pq; p.Sq = a.Sq; p.sps_q = a.sps_q;
  p.Pkv = a.Pkv; p.Skv = a.Skv; p.sps_kv = a.sps_kv;
  p.bq = (const bf16_t*)a.bq; p.bk = (const bf16_t*)a.bk; p.bv = (const bf16_t*)a.bv;
  p.H = a.H; p.heads = a.heads;
  p.nodes = a.nodes; p.parent = a.parent; p.n_lvl = a.n_lvl; p.R = a.R; p.m = a.m;
  p.nodes_stride = a.nodes_stride; p.parent_stride = a.parent_stride;
  p.out = a.out; p.ldo = a.ldo;
  p.gain = (const bf16_t*)a.gain; p.eps = a.eps; p.n_hi = a.n_hi; p.n_lo = a.n_lo;
  p.c_hi = a.c_hi; p.c_lo = a.c_lo; p.ldc = a.ldc;
  ad_gate_fused_kernel<<<rows, 512, 0, st>>>(p);
}

void launch_draft_root_fused(const float* a, const int* next_tok, const int* m, int B, int R, int H, float* state,
                             int* tokens, bf16_t* y_hi, bf16_t* y_lo, int* aug_len, hipStream_t st, int Rs) {
  draft_root_fused_kernel<<<B, 256, 0, st>>>(a, next_tok, m, R, H, state, tokens, y_hi, y_lo, aug_len, Rs ? Rs : R);
}

void launch_draft_level(const float* state, const int* tokens, const int* nodes, const int* parent, int n_lvl, int B,
                        int R, int H, const void* table, int vocab, const void* gain, float eps, bf16_t* a_hi,
                        bf16_t* a_lo, bf16_t* y_hi, bf16_t* y_lo, bf16_t* c_hi, bf16_t* c_lo, hipStream_t st,
                        int nodes_stride, int parent_stride) {
  if (n_lvl <= 0) return;
  draft_level_kernel<<<dim3(n_lvl, B), 256, 0, st>>>(state, tokens, nodes, parent, n_lvl, R, H, (const bf16_t*)table, vocab,
                                                     (const bf16_t*)gain, eps, a_hi, a_lo, y_hi, y_lo, c_hi, c_lo,
                                                     nodes_stride, parent_stride);
}

}  // namespace clv
