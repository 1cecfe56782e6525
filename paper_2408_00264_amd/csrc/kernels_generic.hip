// Plain fp32-ALU kernels of the Clover-2 speculative step: every stage that is not a large
// contraction, plus simple (slow, shape-agnostic) GEMM and attention used for fp32 models and
// as the on-device cross-check of the MFMA path.
#include "clover_internal.h"

namespace clv {

// ------------------------------------------------------------------------------------------
// small device helpers
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ float bf16_to_f32(bf16_t u) { return __uint_as_float(((unsigned)u) << 16); }
// round to nearest even through the hardware conversion (v_cvt_pk_bf16_f32)
__device__ __forceinline__ bf16_t f32_to_bf16(float f) { return __builtin_bit_cast(unsigned short, (__bf16)f); }
__device__ __forceinline__ float ldf(const float* p, size_t i) { return p[i]; }
__device__ __forceinline__ float ldf(const bf16_t* p, size_t i) { return bf16_to_f32(p[i]); }
__device__ __forceinline__ void stf(float* p, size_t i, float v) { p[i] = v; }
__device__ __forceinline__ void stf(bf16_t* p, size_t i, float v) { p[i] = f32_to_bf16(v); }
// KV-cache elements: fp32, or a (hi, lo) pair of bf16 planes `plane` elements apart
__device__ __forceinline__ float ldkv(const float* p, size_t i, size_t) { return p[i]; }
__device__ __forceinline__ float ldkv(const bf16_t* p, size_t i, size_t plane) {
  return bf16_to_f32(p[i]) + bf16_to_f32(p[i + plane]);
}
__device__ __forceinline__ void stkv(float* p, size_t i, size_t, float v) { p[i] = v; }
__device__ __forceinline__ void stkv(bf16_t* p, size_t i, size_t plane, float v) {
  const bf16_t h = f32_to_bf16(v);
  p[i] = h;
  p[i + plane] = f32_to_bf16(v - bf16_to_f32(h));
}
__device__ __forceinline__ void mvkv(float* p, size_t dst, size_t src, size_t) { p[dst] = p[src]; }
__device__ __forceinline__ void mvkv(bf16_t* p, size_t dst, size_t src, size_t plane) {
  p[dst] = p[src];
  p[dst + plane] = p[src + plane];
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
__device__ __forceinline__ unsigned long long wave_max_u64(unsigned long long v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    unsigned lo = __shfl_xor((unsigned)(v & 0xFFFFFFFFull), o, 64);
    unsigned hi = __shfl_xor((unsigned)(v >> 32), o, 64);
    unsigned long long w = ((unsigned long long)hi << 32) | lo;
    v = w > v ? w : v;
  }
  return v;
}
// sum over a 256-thread block; `red` is 4 floats of LDS.  All threads get the result.
__device__ __forceinline__ float block_sum_256(float v, float* red) {
  v = wave_sum(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  return red[0] + red[1] + red[2] + red[3];
}

__device__ __forceinline__ int rows_valid(const RowMap& rm, int b) { return rm.n_valid ? min(rm.n_valid[b], rm.n) : rm.n; }

// ------------------------------------------------------------------------------------------
// embedding gather: out[row, 0:H] = table[tok[row], :]
// ------------------------------------------------------------------------------------------
template <typename WT>
__global__ void embed_kernel(const WT* __restrict__ table, const int* __restrict__ tok, int vocab,
                             float* __restrict__ out, int ldo, int H, RowMap rm) {
  const int b = blockIdx.y, i = blockIdx.x;
  if (i >= rows_valid(rm, b)) return;
  const size_t row = (size_t)b * rm.R + i;
  int t = tok[row];
  t = t < 0 ? 0 : (t >= vocab ? vocab - 1 : t);
  for (int c = threadIdx.x; c < H; c += blockDim.x) out[row * ldo + c] = ldf(table, (size_t)t * H + c);
}

void launch_embed(const void* table, int wdtype, const int* tok, int vocab, float* out, int ldo, int H, RowMap rm,
                  hipStream_t st) {
  dim3 grid(rm.n, rm.B);
  if (wdtype == 0)
    embed_kernel<float><<<grid, 256, 0, st>>>((const float*)table, tok, vocab, out, ldo, H, rm);
  else
    embed_kernel<bf16_t><<<grid, 256, 0, st>>>((const bf16_t*)table, tok, vocab, out, ldo, H, rm);
}

// ------------------------------------------------------------------------------------------
// RMSNorm: out = x * rsqrt(mean(x^2) + eps) * gain      (one block per row)
// ------------------------------------------------------------------------------------------
template <typename WT>
__global__ void rmsnorm_kernel(const float* __restrict__ x, int ldx, const WT* __restrict__ gain, float eps,
                               float* __restrict__ out, int ldo, int H) {
  __shared__ float red[4];
  const size_t row = blockIdx.x;
  const float* xr = x + row * ldx;
  float ss = 0.f;
  for (int c = threadIdx.x; c < H; c += 256) { float v = xr[c]; ss += v * v; }
  ss = block_sum_256(ss, red);
  const float scale = 1.0f / sqrtf(ss / (float)H + eps);
  for (int c = threadIdx.x; c < H; c += 256) out[row * ldo + c] = xr[c] * scale * ldf(gain, c);
}

void launch_rmsnorm(const float* x, int ldx, const void* gain, int wdtype, float eps, float* out, int ldo, int H,
                    int rows, hipStream_t st) {
  if (rows <= 0) return;
  if (wdtype == 0)
    rmsnorm_kernel<float><<<rows, 256, 0, st>>>(x, ldx, (const float*)gain, eps, out, ldo, H);
  else
    rmsnorm_kernel<bf16_t><<<rows, 256, 0, st>>>(x, ldx, (const bf16_t*)gain, eps, out, ldo, H);
}

// ------------------------------------------------------------------------------------------
// rotary tables: row (b,i) sits at position base_len[b] + (depth ? depth[i] : i)
// ------------------------------------------------------------------------------------------
__global__ void rope_table_kernel(const int* __restrict__ base_len, const int* __restrict__ depth, float rope_base,
                                  int d, float* __restrict__ cos_t, float* __restrict__ sin_t, RowMap rm,
                                  int depth_stride) {
  const int b = blockIdx.y, i = blockIdx.x, half = d / 2;
  const size_t row = (size_t)b * rm.R + i;
  const int pos = base_len[b] + (depth ? depth[(size_t)b * depth_stride + i] : i);
  for (int c = threadIdx.x; c < half; c += blockDim.x) {
    const double inv = pow((double)rope_base, -2.0 * (double)c / (double)d);
    const double ang = (double)pos * inv;
    cos_t[row * half + c] = (float)cos(ang);
    sin_t[row * half + c] = (float)sin(ang);
  }
}

void launch_rope_table(const int* base_len, const int* depth, float rope_base, int d, float* cos_t, float* sin_t,
                       RowMap rm, hipStream_t st, int depth_stride) {
  dim3 grid(rm.n, rm.B);
  rope_table_kernel<<<grid, 64, 0, st>>>(base_len, depth, rope_base, d, cos_t, sin_t, rm, depth_stride);
}

// ------------------------------------------------------------------------------------------
// RoPE on q and k (half-split pairing), K rows and transposed V columns into the cache; sums the
// split-K partials of the QKV projection on the way (fixed order, eight loads in flight).
// blocks [0, n*hc): 256 (head, pair) items of one row; then blocks of 8 (head,dim) lines of V^T
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ float sum_partials(const float* __restrict__ p, int nsp, size_t sps) {
  float v = 0.f;
  for (int s0 = 0; s0 < nsp; s0 += 8) {
    float q[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) q[j] = (s0 + j < nsp) ? p[(size_t)(s0 + j) * sps] : 0.f;
#pragma unroll
    for (int j = 0; j < 8; ++j) v += q[j];
  }
  return v;
}

template <typename KT>
__global__ void rope_kv_write_kernel(const float* __restrict__ qkv, int ldqkv, int nsp, size_t sps,
                                     const float* __restrict__ cos_t,
                                     const float* __restrict__ sin_t, float* __restrict__ q_out, int ldq,
                                     KT* __restrict__ kc, KT* __restrict__ vc, KVLayout kv,
                                     const int* __restrict__ base_len, int n_q, RowMap rm, int* err_flag, int hc,
                                     bf16_t* __restrict__ q_hi, bf16_t* __restrict__ q_lo, float q_scale) {
  const int b = blockIdx.y;
  const int nv = rows_valid(rm, b);
  const int L = base_len[b];
  const int d = kv.d, half = d / 2, n_kv = kv.n_kv;
  if (L + nv > kv.max_seq) {  // would overrun the cache: refuse, flag
    if (threadIdx.x == 0 && blockIdx.x == 0) atomicOr(err_flag, 1);
    return;
  }
  if ((int)blockIdx.x < rm.n * hc) {
    const int i = blockIdx.x / hc;
    if (i >= nv) return;
    const int idx = (blockIdx.x % hc) * 256 + threadIdx.x;
    if (idx >= (n_q + n_kv) * half) return;
    const size_t row = (size_t)b * rm.R + i;
    const int slot = L + i;
    const float* src = qkv + row * ldqkv;
    const int hh = idx / half, ii = idx - hh * half;
    const float c = cos_t[row * half + ii], s = sin_t[row * half + ii];
    const float x1 = sum_partials(src + hh * d + ii, nsp, sps);
    const float x2 = sum_partials(src + hh * d + ii + half, nsp, sps);
    const float o1 = x1 * c - x2 * s, o2 = x2 * c + x1 * s;
    if (hh < n_q) {
      if (q_hi) {  // operand format of the MFMA attention: pre-scaled (hi, lo) bf16 planes
        const float s1 = o1 * q_scale, s2 = o2 * q_scale;
        const bf16_t h1 = f32_to_bf16(s1), h2 = f32_to_bf16(s2);
        q_hi[row * ldq + hh * d + ii] = h1;
        q_hi[row * ldq + hh * d + ii + half] = h2;
        q_lo[row * ldq + hh * d + ii] = f32_to_bf16(s1 - bf16_to_f32(h1));
        q_lo[row * ldq + hh * d + ii + half] = f32_to_bf16(s2 - bf16_to_f32(h2));
      } else {
        q_out[row * ldq + hh * d + ii] = o1;
        q_out[row * ldq + hh * d + ii + half] = o2;
      }
    } else {
      const size_t base = kv_k_at(kv, b, slot, hh - n_q);
      stkv(kc, base + ii, kv.plane, o1);
      stkv(kc, base + ii + half, kv.plane, o2);
    }
  } else {
    const int vb = blockIdx.x - rm.n * hc;
    const int voff = (n_q + n_kv) * d;
    for (int idx = threadIdx.x; idx < 8 * rm.n; idx += blockDim.x) {
      const int node = idx % rm.n, e = vb * 8 + idx / rm.n;
      if (node >= nv || e >= n_kv * d) continue;
      const float v = sum_partials(qkv + ((size_t)b * rm.R + node) * ldqkv + voff + e, nsp, sps);
      stkv(vc, kv_v_at(kv, b, e / d, e % d, L + node), kv.plane, v);
    }
  }
}

// The same operation for the MFMA path's formats (q as pre-scaled bf16 planes, bf16-plane caches), vectorised:
// a thread of the first blocks rotates four adjacent pairs of one head (float4 loads of every partial, issued
// before anything else is waited for; 8-byte plane stores); the last blocks transpose 64 nodes x 32 channels of V
// through LDS so that the partials are read along the channels and V^T is written along the nodes.
__device__ __forceinline__ void planes4(bf16_t* hi, bf16_t* lo, size_t off, const float (&o)[4]) {
  unsigned h[4], l[4];
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const bf16_t hb = f32_to_bf16(o[r]);
    h[r] = hb;
    l[r] = f32_to_bf16(o[r] - bf16_to_f32(hb));
  }
  *(uint2*)(hi + off) = make_uint2(h[0] | (h[1] << 16), h[2] | (h[3] << 16));
  *(uint2*)(lo + off) = make_uint2(l[0] | (l[1] << 16), l[2] | (l[3] << 16));
}
__device__ __forceinline__ float4 sum_partials4(const float* __restrict__ p, int nsp, size_t sps) {
  float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int s0 = 0; s0 < nsp; s0 += 8) {
    float4 q[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) q[j] = (s0 + j < nsp) ? *(const float4*)(p + (size_t)(s0 + j) * sps) : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
    for (int j = 0; j < 8; ++j) { v.x += q[j].x; v.y += q[j].y; v.z += q[j].z; v.w += q[j].w; }
  }
  return v;
}
__global__ __launch_bounds__(256) void rope_kv_planes_kernel(const float* __restrict__ qkv, int ldqkv, int nsp, size_t sps,
                                                             const float* __restrict__ cos_t, const float* __restrict__ sin_t,
                                                             bf16_t* __restrict__ kc, bf16_t* __restrict__ vc, KVLayout kv,
                                                             const int* __restrict__ base_len, int n_q, RowMap rm,
                                                             int* err_flag, int qk_blocks, bf16_t* __restrict__ q_hi,
                                                             bf16_t* __restrict__ q_lo, int ldq, float q_scale) {
  __shared__ float tile[64][33];
  const int b = blockIdx.y, tid = threadIdx.x;
  const int d = kv.d, half = d / 2, n_kv = kv.n_kv;
  if ((int)blockIdx.x < qk_blocks) {
    const int quads = half / 4, per_row = (n_q + n_kv) * quads;
    const int idx = blockIdx.x * 256 + tid;
    const int i = idx / per_row, rem = idx - i * per_row, hh = rem / quads, ii = (rem - hh * quads) * 4;
    const size_t row = (size_t)b * rm.R + min(i, rm.n - 1);
    const float* src = qkv + row * ldqkv + hh * d + ii;
    const float4 x1 = sum_partials4(src, nsp, sps), x2 = sum_partials4(src + half, nsp, sps);
    const float4 c = *(const float4*)(cos_t + row * half + ii), s = *(const float4*)(sin_t + row * half + ii);
    const int nv = rows_valid(rm, b), L = base_len[b];
    if (L + nv > kv.max_seq) {  // would overrun the cache: refuse, flag
      if (tid == 0 && blockIdx.x == 0) atomicOr(err_flag, 1);
      return;
    }
    if (i >= nv) return;
    float o1[4] = {x1.x * c.x - x2.x * s.x, x1.y * c.y - x2.y * s.y, x1.z * c.z - x2.z * s.z, x1.w * c.w - x2.w * s.w};
    float o2[4] = {x2.x * c.x + x1.x * s.x, x2.y * c.y + x1.y * s.y, x2.z * c.z + x1.z * s.z, x2.w * c.w + x1.w * s.w};
    if (hh < n_q) {
#pragma unroll
      for (int r = 0; r < 4; ++r) { o1[r] *= q_scale; o2[r] *= q_scale; }
      planes4(q_hi, q_lo, row * ldq + hh * d + ii, o1);
      planes4(q_hi, q_lo, row * ldq + hh * d + ii + half, o2);
    } else {
      const size_t base = kv_k_at(kv, b, L + i, hh - n_q) + ii;
      planes4(kc, kc + kv.plane, base, o1);
      planes4(kc, kc + kv.plane, base + half, o2);
    }
  } else {
    const int n_eb = n_kv * d / 32;
    const int vblk = blockIdx.x - qk_blocks, eb = vblk % n_eb, nb0 = (vblk / n_eb) * 64;
    const int voff = (n_q + n_kv) * d + eb * 32;
    float4 v[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int f = tid + 256 * j, node = min(nb0 + f / 8, rm.n - 1), e4 = (f % 8) * 4;
      v[j] = sum_partials4(qkv + ((size_t)b * rm.R + node) * ldqkv + voff + e4, nsp, sps);
    }
    const int nv = rows_valid(rm, b), L = base_len[b];
    if (L + nv > kv.max_seq) return;  // (flagged by the first block)
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int f = tid + 256 * j, e4 = (f % 8) * 4;
      tile[f / 8][e4] = v[j].x; tile[f / 8][e4 + 1] = v[j].y; tile[f / 8][e4 + 2] = v[j].z; tile[f / 8][e4 + 3] = v[j].w;
    }
    __syncthreads();
    const int nl = tid % 64, node = nb0 + nl;
    if (node >= nv) return;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int e = tid / 64 + 4 * j;
      const float val = tile[nl][e];
      const size_t at = kv_v_at(kv, b, (eb * 32 + e) / d, (eb * 32 + e) % d, L + node);
      const bf16_t hb = f32_to_bf16(val);
      vc[at] = hb;
      vc[at + kv.plane] = f32_to_bf16(val - bf16_to_f32(hb));
    }
  }
}

void launch_rope_kv_write(const float* qkv, int ldqkv, int qkv_splits, size_t qkv_split_stride, const float* cos_t,
                          const float* sin_t, float* q_out, int ldq,
                          void* k_cache, void* v_cache, int kvdtype, KVLayout kv, const int* base_len, int n_q,
                          RowMap rm, int* err_flag, bf16_t* q_hi, bf16_t* q_lo, float q_scale, hipStream_t st) {
  if (kvdtype == 1 && q_hi && kv.d % 32 == 0 && ldqkv % 4 == 0 && qkv_split_stride % 4 == 0 && ldq % 4 == 0) {
    const int per_row = (n_q + kv.n_kv) * (kv.d / 8);
    const int qk_blocks = (rm.n * per_row + 255) / 256;
    const int v_blocks = (kv.n_kv * kv.d / 32) * ((rm.n + 63) / 64);
    rope_kv_planes_kernel<<<dim3(qk_blocks + v_blocks, rm.B), 256, 0, st>>>(
        qkv, ldqkv, qkv_splits, qkv_split_stride, cos_t, sin_t, (bf16_t*)k_cache, (bf16_t*)v_cache, kv, base_len, n_q, rm,
        err_flag, qk_blocks, q_hi, q_lo, ldq, q_scale);
    return;
  }
  const int vblocks = (kv.n_kv * kv.d + 7) / 8;
  const int hc = ((n_q + kv.n_kv) * (kv.d / 2) + 255) / 256;
  dim3 grid(rm.n * hc + vblocks, rm.B);
  if (kvdtype == 0)
    rope_kv_write_kernel<float><<<grid, 256, 0, st>>>(qkv, ldqkv, qkv_splits, qkv_split_stride, cos_t, sin_t, q_out, ldq, (float*)k_cache,
                                                      (float*)v_cache, kv, base_len, n_q, rm, err_flag, hc, q_hi, q_lo, q_scale);
  else
    rope_kv_write_kernel<bf16_t><<<grid, 256, 0, st>>>(qkv, ldqkv, qkv_splits, qkv_split_stride, cos_t, sin_t, q_out, ldq, (bf16_t*)k_cache,
                                                       (bf16_t*)v_cache, kv, base_len, n_q, rm, err_flag, hc, q_hi, q_lo, q_scale);
}

// ------------------------------------------------------------------------------------------
// tree-masked attention, one wavefront per (row, q head).  Keys: cached slots [0,L) all visible,
// then the rm.n new rows at slots L+w, visible iff bit w of the row's ancestor mask is set.
// anc == null: the rows form a chain (row i sees new rows 0..i), any number of rows.
// iv != null: new row w is visible to row i iff enter[w] <= enter[i] <= exit[w] (interval labels, two ints per node).
// ------------------------------------------------------------------------------------------
template <typename KT>
__global__ void attn_generic_kernel(const float* __restrict__ q, int ldq, const KT* __restrict__ kc,
                                    const KT* __restrict__ vc, KVLayout kv, const int* __restrict__ base_len,
                                    const unsigned long long* __restrict__ anc, int n_q, float* __restrict__ out,
                                    int ldo, bf16_t* __restrict__ out_hi, bf16_t* __restrict__ out_lo, RowMap rm,
                                    int anc_stride, const int* __restrict__ iv) {
  __shared__ float qs[128];
  __shared__ float ps[64];
  const int h = blockIdx.x, i = blockIdx.y, b = blockIdx.z, lane = threadIdx.x;
  const int nv = rows_valid(rm, b);
  if (i >= nv) return;
  const int d = kv.d, n_kv = kv.n_kv;
  const int L = base_len[b];
  if (L + nv > kv.max_seq) return;
  const size_t row = (size_t)b * rm.R + i;
  const bool chain = anc == nullptr && iv == nullptr;
  const bool bits = anc != nullptr && iv == nullptr;
  const unsigned long long a0 = bits ? anc[2 * ((size_t)b * anc_stride + i)] : 0ull;
  const unsigned long long a1 = bits ? anc[2 * ((size_t)b * anc_stride + i) + 1] : 0ull;
  const int my_enter = iv ? iv[2 * ((size_t)b * anc_stride + i)] : 0;
  const int g = h / (n_q / n_kv);
  const float scale = 1.0f / sqrtf((float)d);
  for (int c = lane; c < d; c += 64) qs[c] = q[row * ldq + h * d + c] * scale;
  __syncthreads();
  float mrun = -INFINITY, lrun = 0.f, o0 = 0.f, o1 = 0.f;
  const int total = L + rm.n;
  const int ntiles = (total + 63) / 64;
  for (int t = 0; t < ntiles; ++t) {
    const int s = t * 64 + lane;
    bool vis = s < L;
    if (!vis && s < total) {
      const int w = s - L;
      if (chain) vis = w <= i;
      else if (iv) vis = iv[2 * ((size_t)b * anc_stride + w)] <= my_enter && my_enter <= iv[2 * ((size_t)b * anc_stride + w) + 1];
      else vis = ((w < 64 ? (a0 >> w) : (a1 >> (w - 64))) & 1ull) != 0ull;
    }
    float sc = -INFINITY;
    if (vis) {
      const KT* kr = kc + kv_k_at(kv, b, s, g);
      float acc = 0.f;
      for (int c = 0; c < d; ++c) acc += qs[c] * ldkv(kr, c, kv.plane);
      sc = acc;
    }
    const float mnew = fmaxf(mrun, wave_max(sc));
    if (mnew == -INFINITY) continue;  // uniform across the wave
    const float p = vis ? expf(sc - mnew) : 0.f;
    const float corr = (mrun == -INFINITY) ? 0.f : expf(mrun - mnew);
    lrun = lrun * corr + wave_sum(p);
    o0 *= corr;
    o1 *= corr;
    mrun = mnew;
    __syncthreads();
    ps[lane] = p;
    __syncthreads();
    const int jmax = min(64, total - t * 64);
    for (int j = 0; j < jmax; ++j) {
      const float pj = ps[j];
      if (pj != 0.f) {
        o0 += pj * ldkv(vc, kv_v_at(kv, b, g, lane, t * 64 + j), kv.plane);
        if (d > 64) o1 += pj * ldkv(vc, kv_v_at(kv, b, g, lane + 64, t * 64 + j), kv.plane);
      }
    }
  }
  const float inv = 1.0f / lrun;
  if (out_hi) {
    const float r0 = o0 * inv, r1 = o1 * inv;
    const bf16_t h0 = f32_to_bf16(r0), h1 = f32_to_bf16(r1);
    out_hi[row * ldo + h * d + lane] = h0;
    out_lo[row * ldo + h * d + lane] = f32_to_bf16(r0 - bf16_to_f32(h0));
    if (d > 64) {
      out_hi[row * ldo + h * d + 64 + lane] = h1;
      out_lo[row * ldo + h * d + 64 + lane] = f32_to_bf16(r1 - bf16_to_f32(h1));
    }
    return;
  }
  out[row * ldo + h * d + lane] = o0 * inv;
  if (d > 64) out[row * ldo + h * d + 64 + lane] = o1 * inv;
}

void launch_attn_generic(const float* q, int ldq, const void* k_cache, const void* v_cache, int kvdtype, KVLayout kv,
                         const int* base_len, const unsigned long long* anc, int n_q, float* out, int ldo,
                         bf16_t* out_hi, bf16_t* out_lo, RowMap rm, hipStream_t st, int anc_stride, const int* iv) {
  dim3 grid(n_q, rm.n, rm.B);
  if (kvdtype == 0)
    attn_generic_kernel<float><<<grid, 64, 0, st>>>(q, ldq, (const float*)k_cache, (const float*)v_cache, kv, base_len,
                                                    anc, n_q, out, ldo, out_hi, out_lo, rm, anc_stride, iv);
  else
    attn_generic_kernel<bf16_t><<<grid, 64, 0, st>>>(q, ldq, (const bf16_t*)k_cache, (const bf16_t*)v_cache, kv,
                                                     base_len, anc, n_q, out, ldo, out_hi, out_lo, rm, anc_stride, iv);
}

// ------------------------------------------------------------------------------------------
// generic GEMM: Y[M,N] (+)= X[M,K] W[N,K]^T (+ bias), 64x64x16 LDS tiles, 4x4 per thread
// ------------------------------------------------------------------------------------------
template <typename WT>
__global__ __launch_bounds__(256) void gemm_generic_kernel(const float* __restrict__ X, int ldx,
                                                           const WT* __restrict__ W, const WT* __restrict__ bias,
                                                           float* __restrict__ Y, int ldy, int M, int N, int K,
                                                           int mode) {
  __shared__ float Xs[16][68];
  __shared__ float Ws[16][68];
  const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
  const int bm = blockIdx.y * 64, bn = blockIdx.x * 64;
  float acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;
  for (int k0 = 0; k0 < K; k0 += 16) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int idx = tid + j * 256, r = idx >> 4, kk = idx & 15;
      const bool kin = (k0 + kk) < K;
      Xs[kk][r] = (kin && bm + r < M) ? X[(size_t)(bm + r) * ldx + k0 + kk] : 0.f;
      Ws[kk][r] = (kin && bn + r < N) ? ldf(W, (size_t)(bn + r) * K + k0 + kk) : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < 16; ++kk) {
      float a[4], w[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = Xs[kk][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) w[j] = Ws[kk][tx * 4 + j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] += a[i] * w[j];
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int m = bm + ty * 4 + i;
    if (m >= M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int n = bn + tx * 4 + j;
      if (n >= N) continue;
      float v = acc[i][j];
      if (bias) v += ldf(bias, n);
      float* y = Y + (size_t)m * ldy + n;
      *y = (mode == 1) ? (*y + v) : v;
    }
  }
}

void launch_gemm_generic(const float* X, int ldx, const void* W, const void* bias, int wdtype, float* Y, int ldy,
                         int M, int N, int K, int mode, hipStream_t st) {
  if (M <= 0 || N <= 0) return;
  dim3 grid((N + 63) / 64, (M + 63) / 64);
  if (wdtype == 0)
    gemm_generic_kernel<float><<<grid, 256, 0, st>>>(X, ldx, (const float*)W, (const float*)bias, Y, ldy, M, N, K, mode);
  else
    gemm_generic_kernel<bf16_t><<<grid, 256, 0, st>>>(X, ldx, (const bf16_t*)W, (const bf16_t*)bias, Y, ldy, M, N, K,
                                                      mode);
}

__global__ void swiglu_kernel(const float* __restrict__ g, const float* __restrict__ u, float* __restrict__ h,
                              size_t n) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) {
    const float a = g[i];
    h[i] = a / (1.0f + expf(-a)) * u[i];
  }
}
void launch_swiglu(const float* g, const float* u, float* h, size_t n, hipStream_t st) {
  if (n == 0) return;
  swiglu_kernel<<<(unsigned)((n + 255) / 256), 256, 0, st>>>(g, u, h, n);
}

// ------------------------------------------------------------------------------------------
// Attention-Decoder gate: per head cos(q_h, k_h) scales v_h, residual add of x
// ------------------------------------------------------------------------------------------
__global__ void ad_gate_kernel(const float* __restrict__ x, int ldx, const float* __restrict__ q,
                               const float* __restrict__ k, const float* __restrict__ v, int H, int heads,
                               float* __restrict__ out, int ldo, float* __restrict__ out2, int ldo2) {
  const size_t row = blockIdx.x;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, hd = H / heads;
  for (int h = wave; h < heads; h += 4) {
    const size_t o = row * H + (size_t)h * hd;
    float qq = 0.f, kk = 0.f, qk = 0.f;
    for (int c = lane; c < hd; c += 64) {
      const float a = q[o + c], bb = k[o + c];
      qq += a * a; kk += bb * bb; qk += a * bb;
    }
    qq = wave_sum(qq); kk = wave_sum(kk); qk = wave_sum(qk);
    const float att = qk / (fmaxf(sqrtf(qq), 1e-8f) * fmaxf(sqrtf(kk), 1e-8f));
    for (int c = lane; c < hd; c += 64) {
      const float r = x[row * ldx + h * hd + c] + att * v[o + c];
      out[row * ldo + h * hd + c] = r;
      if (out2) out2[row * ldo2 + h * hd + c] = r;
    }
  }
}
void launch_ad_gate(const float* x, int ldx, const float* q, const float* k, const float* v, int H, int heads,
                    float* out, int ldo, float* out2, int ldo2, int rows, hipStream_t st) {
  if (rows <= 0) return;
  ad_gate_kernel<<<rows, 256, 0, st>>>(x, ldx, q, k, v, H, heads, out, ldo, out2, ldo2);
}

// ------------------------------------------------------------------------------------------
// top-k by (value desc, id asc).  Keys are 64-bit: order-preserving image of the float in the high
// word, ~id in the low word, so an unsigned max picks the larger value and, among equals, the
// smaller id.  Stage 1: one block per 2048-wide chunk; stage 2: one block per row merges.
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ unsigned long long topk_key(float v, int id) {
  v = v + 0.0f;  // -0 -> +0 so that equal values compare equal
  unsigned u = __float_as_uint(v);
  u = (u & 0x80000000u) ? ~u : (u | 0x80000000u);
  return ((unsigned long long)u << 32) | (unsigned long long)(0xFFFFFFFFu - (unsigned)id);
}
__device__ __forceinline__ unsigned long long block_max_u64_256(unsigned long long v, unsigned long long* red) {
  v = wave_max_u64(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  unsigned long long r = red[0];
  r = red[1] > r ? red[1] : r;
  r = red[2] > r ? red[2] : r;
  r = red[3] > r ? red[3] : r;
  return r;
}

constexpr int TOPK_CHUNK = 2048;
constexpr int TOPK_EPT = TOPK_CHUNK / 256;
int topk_chunks(int V) { return (V + TOPK_CHUNK - 1) / TOPK_CHUNK; }

__global__ __launch_bounds__(256) void topk_stage1_kernel(const float* __restrict__ z, int ldz, int V, int k,
                                                          unsigned long long* __restrict__ cand, int splits,
                                                          size_t sps) {
  __shared__ unsigned long long red[4];
  const int chunk = blockIdx.x, row = blockIdx.y, chunks = gridDim.x;
  unsigned long long key[TOPK_EPT];
#pragma unroll
  for (int e = 0; e < TOPK_EPT; ++e) {
    const int id = chunk * TOPK_CHUNK + e * 256 + threadIdx.x;
    float v = 0.f;
    if (id < V) {
      float q[8];
#pragma unroll
      for (int s = 0; s < 8; ++s) q[s] = s < splits ? z[s * sps + (size_t)row * ldz + id] : 0.f;  // one batch of loads
#pragma unroll
      for (int s = 0; s < 8; ++s) v += q[s];  // split order, as the reduce kernel
      for (int s = 8; s < splits; ++s) v += z[s * sps + (size_t)row * ldz + id];
    }
    key[e] = id < V ? topk_key(v, id) : 0ull;
  }
  for (int r = 0; r < k; ++r) {
    unsigned long long best = 0ull;
#pragma unroll
    for (int e = 0; e < TOPK_EPT; ++e) best = key[e] > best ? key[e] : best;
    best = block_max_u64_256(best, red);
#pragma unroll
    for (int e = 0; e < TOPK_EPT; ++e)
      if (key[e] == best) key[e] = 0ull;
    if (threadIdx.x == 0) cand[((size_t)row * chunks + chunk) * 16 + r] = best;
  }
}

__global__ __launch_bounds__(256) void topk_stage2_kernel(const unsigned long long* __restrict__ cand, int chunks,
                                                          int k, int* __restrict__ out_ids) {
  __shared__ unsigned long long red[4];
  const int row = blockIdx.x;
  const int total = chunks * k;  // <= 63*16 for V <= 129024; loop handles more
  unsigned long long key[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const int idx = e * 256 + threadIdx.x;
    key[e] = idx < total ? cand[((size_t)row * chunks + idx / k) * 16 + idx % k] : 0ull;
  }
  for (int r = 0; r < k; ++r) {
    unsigned long long best = 0ull;
#pragma unroll
    for (int e = 0; e < 8; ++e) best = key[e] > best ? key[e] : best;
    best = block_max_u64_256(best, red);
#pragma unroll
    for (int e = 0; e < 8; ++e)
      if (key[e] == best) key[e] = 0ull;
    if (threadIdx.x == 0) out_ids[row * 16 + r] = (int)(0xFFFFFFFFu - (unsigned)(best & 0xFFFFFFFFull));
  }
}

void launch_topk(const float* z, int ldz, int V, int rows, int k, void* cand, int* out_ids, hipStream_t st, int splits,
                 size_t split_stride) {
  if (rows <= 0) return;
  const int chunks = topk_chunks(V);  // chunks * k <= 2048 is checked at init (vocab <= 262144)
  topk_stage1_kernel<<<dim3(chunks, rows), 256, 0, st>>>(z, ldz, V, k, (unsigned long long*)cand, splits, split_stride);
  topk_stage2_kernel<<<rows, 256, 0, st>>>((const unsigned long long*)cand, chunks, k, out_ids);
}

// ------------------------------------------------------------------------------------------
// draft-tree bookkeeping
// ------------------------------------------------------------------------------------------
template <typename WT>
__global__ void draft_gather_kernel(const float* __restrict__ state, const int* __restrict__ tokens,
                                    const int* __restrict__ lvl_nodes, const int* __restrict__ parent, int n_lvl,
                                    int R, int H, const WT* __restrict__ lm_head, int vocab, float* __restrict__ xs,
                                    float* __restrict__ e, float* __restrict__ cat, int nodes_stride, int parent_stride) {
  const int r = blockIdx.x, b = blockIdx.y;
  const int u = lvl_nodes[(size_t)b * nodes_stride + r], p = parent[(size_t)b * parent_stride + u];
  int t = tokens[(size_t)b * R + u];
  t = t < 0 ? 0 : (t >= vocab ? vocab - 1 : t);
  const size_t row = (size_t)b * n_lvl + r;
  for (int c = threadIdx.x; c < H; c += blockDim.x) {
    xs[row * H + c] = state[((size_t)b * R + p) * H + c];
    const float ev = ldf(lm_head, (size_t)t * H + c);
    e[row * H + c] = ev;
    cat[row * 2 * H + H + c] = ev;
  }
}
void launch_draft_gather(const float* state, const int* tokens, const int* lvl_nodes, const int* parent, int n_lvl,
                         int B, int R, int H, const void* lm_head, int wdtype, int vocab, float* xs, float* e,
                         float* cat, hipStream_t st, int nodes_stride, int parent_stride) {
  if (n_lvl <= 0) return;
  dim3 grid(n_lvl, B);
  if (wdtype == 0)
    draft_gather_kernel<float><<<grid, 256, 0, st>>>(state, tokens, lvl_nodes, parent, n_lvl, R, H,
                                                     (const float*)lm_head, vocab, xs, e, cat, nodes_stride, parent_stride);
  else
    draft_gather_kernel<bf16_t><<<grid, 256, 0, st>>>(state, tokens, lvl_nodes, parent, n_lvl, R, H,
                                                      (const bf16_t*)lm_head, vocab, xs, e, cat, nodes_stride, parent_stride);
}

__global__ void draft_scatter_state_kernel(const float* __restrict__ s, const int* __restrict__ lvl_nodes, int n_lvl,
                                           int R, int H, float* __restrict__ state, float* __restrict__ cat,
                                           int nodes_stride) {
  const int r = blockIdx.x, b = blockIdx.y;
  const int u = lvl_nodes[(size_t)b * nodes_stride + r];
  const size_t row = (size_t)b * n_lvl + r;
  for (int c = threadIdx.x; c < H; c += blockDim.x) {
    const float v = s[row * H + c];
    state[((size_t)b * R + u) * H + c] = v;
    cat[row * 2 * H + c] = v;
  }
}
void launch_draft_scatter_state(const float* s, const int* lvl_nodes, int n_lvl, int B, int R, int H, float* state,
                                float* cat, hipStream_t st, int nodes_stride) {
  if (n_lvl <= 0) return;
  draft_scatter_state_kernel<<<dim3(n_lvl, B), 256, 0, st>>>(s, lvl_nodes, n_lvl, R, H, state, cat, nodes_stride);
}

__global__ void draft_root_kernel(const float* __restrict__ a, const int* __restrict__ next_tok,
                                  const int* __restrict__ m, int R, int H, float* __restrict__ root_x,
                                  float* __restrict__ state, int* __restrict__ tokens, int Rs) {
  const int b = blockIdx.x;
  const int mb = min(m[b], R);
  for (int c = threadIdx.x; c < H; c += blockDim.x) {
    const float v = mb >= 1 ? a[((size_t)b * R + mb - 1) * H + c] : 0.f;
    root_x[(size_t)b * H + c] = v;
    state[((size_t)b * Rs) * H + c] = v;
  }
  if (threadIdx.x == 0 && mb >= 1) tokens[(size_t)b * Rs] = next_tok[(size_t)b * R + mb - 1];
}
void launch_draft_root(const float* a, const int* next_tok, const int* m, int B, int R, int H, float* root_x,
                       float* state, int* tokens, hipStream_t st, int Rs) {
  draft_root_kernel<<<B, 256, 0, st>>>(a, next_tok, m, R, H, root_x, state, tokens, Rs ? Rs : R);
}

__global__ void draft_assign_kernel(const int* __restrict__ ids, const int* __restrict__ par_row,
                                    const int* __restrict__ rank, int c0, int c1, int n_par, int R,
                                    const int* __restrict__ m, int* __restrict__ tokens) {
  const int b = blockIdx.x;
  if (m[b] < 1) return;
  for (int c = c0 + threadIdx.x; c < c1; c += blockDim.x)
    tokens[(size_t)b * R + c] = ids[((size_t)b * n_par + par_row[c]) * 16 + rank[c]];
}
void launch_draft_assign(const int* ids, const int* par_row, const int* rank, int c0, int c1, int n_par, int B, int R,
                         const int* m, int* tokens, hipStream_t st) {
  if (c1 <= c0) return;
  draft_assign_kernel<<<B, 128, 0, st>>>(ids, par_row, rank, c0, c1, n_par, R, m, tokens);
}

__global__ void add_len_kernel(int* __restrict__ len, const int* __restrict__ m, int B) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b < B) len[b] += max(m[b], 0);
}
void launch_add_len(int* len, const int* m, int B, hipStream_t st) { add_len_kernel<<<(B + 63) / 64, 64, 0, st>>>(len, m, B); }

__global__ void add_scalar_kernel(int* __restrict__ p, int v) { *p += v; }
void launch_add_scalar(int* p, int v, hipStream_t st) { add_scalar_kernel<<<1, 1, 0, st>>>(p, v); }

__global__ void fill_i32_kernel(int* p, int v, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}
void launch_fill_i32(int* p, int v, int n, hipStream_t st) {
  if (n > 0) fill_i32_kernel<<<(n + 255) / 256, 256, 0, st>>>(p, v, n);
}

// ------------------------------------------------------------------------------------------
// greedy acceptance walk (one thread per sequence; the tree has at most 128 nodes)
// ------------------------------------------------------------------------------------------
__global__ void accept_walk_kernel(const int* __restrict__ argmax, const int* __restrict__ tokens,
                                   const int* __restrict__ first_child, const int* __restrict__ n_child, int n_nodes,
                                   int B, int R, const int* __restrict__ n_forced,
                                   const int* __restrict__ forced_next, int* __restrict__ m,
                                   int* __restrict__ acc_idx, int* __restrict__ new_tokens,
                                   int* __restrict__ next_tok, int child_stride) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= B) return;
  const size_t o = (size_t)b * R;
  first_child += (size_t)b * child_stride;
  n_child += (size_t)b * child_stride;
  int len, bonus;
  if (n_forced) {
    len = min(max(n_forced[b], 0), n_nodes);
    if (len == 0) { m[b] = 0; return; }
    for (int i = 0; i < len; ++i) acc_idx[o + i] = i;
    const int f = forced_next[b];
    bonus = f >= 0 ? f : argmax[(o + len - 1) * 16];
  } else {
    int u = 0;
    len = 1;
    acc_idx[o] = 0;
    for (;;) {
      const int t = argmax[(o + u) * 16];
      int found = -1;
      const int c0 = first_child[u], c1 = c0 + n_child[u];
      for (int c = c0; c < c1; ++c)
        if (tokens[o + c] == t) { found = c; break; }
      bonus = t;
      if (found < 0 || len >= R) break;
      u = found;
      acc_idx[o + len++] = u;
    }
  }
  for (int j = 1; j < len; ++j) {
    const int t = tokens[o + acc_idx[o + j]];
    new_tokens[o + j - 1] = t;
    next_tok[o + j - 1] = t;
  }
  new_tokens[o + len - 1] = bonus;
  next_tok[o + len - 1] = bonus;
  m[b] = len;
}
void launch_accept_walk(const int* argmax, const int* tokens, const int* first_child, const int* n_child, int n_nodes,
                        int B, int R, const int* n_forced, const int* forced_next, int* m, int* acc_idx,
                        int* new_tokens, int* next_tok, hipStream_t st, int child_stride) {
  accept_walk_kernel<<<(B + 63) / 64, 64, 0, st>>>(argmax, tokens, first_child, n_child, n_nodes, B, R, n_forced,
                                                   forced_next, m, acc_idx, new_tokens, next_tok, child_stride);
}

// ------------------------------------------------------------------------------------------
// KV compaction: slot L+i <- slot L+acc_idx[i], ascending i.  A thread owns one cache column for
// all rows, so the in-place moves of a column are ordered without any barrier.
// ------------------------------------------------------------------------------------------
template <typename KT>
__global__ void compact_kv_kernel(KT* __restrict__ kc, KT* __restrict__ vc, KVLayout kv, size_t k_layer_elems,
                                  size_t v_layer_elems, const int* __restrict__ len, const int* __restrict__ m,
                                  const int* __restrict__ acc_idx, int R) {
  const int col = blockIdx.x * blockDim.x + threadIdx.x, layer = blockIdx.y, b = blockIdx.z;
  const int width = kv.n_kv * kv.d;
  if (col >= width) return;
  const int mb = m[b], L = len[b];
  if (mb <= 0 || L + mb > kv.max_seq) return;
  KT* kbase = kc + (size_t)layer * k_layer_elems;
  KT* vbase = vc + (size_t)layer * v_layer_elems;
  const int head = col / kv.d, dim = col % kv.d;
  for (int i = 0; i < mb; ++i) {
    const int a = acc_idx[(size_t)b * R + i];
    if (a == i || a < 0 || L + a >= kv.max_seq) continue;
    mvkv(kbase, kv_k_at(kv, b, L + i, head) + dim, kv_k_at(kv, b, L + a, head) + dim, kv.plane);
    mvkv(vbase, kv_v_at(kv, b, head, dim, L + i), kv_v_at(kv, b, head, dim, L + a), kv.plane);
  }
}
void launch_compact_kv(void* k_cache, void* v_cache, int kvdtype, KVLayout kv, int n_layers, size_t k_layer_elems,
                       size_t v_layer_elems, const int* len, const int* m, const int* acc_idx, int B, int R,
                       hipStream_t st) {
  const int width = kv.n_kv * kv.d;
  dim3 grid((width + 255) / 256, n_layers, B);
  if (kvdtype == 0)
    compact_kv_kernel<float><<<grid, 256, 0, st>>>((float*)k_cache, (float*)v_cache, kv, k_layer_elems, v_layer_elems,
                                                   len, m, acc_idx, R);
  else
    compact_kv_kernel<bf16_t><<<grid, 256, 0, st>>>((bf16_t*)k_cache, (bf16_t*)v_cache, kv, k_layer_elems,
                                                    v_layer_elems, len, m, acc_idx, R);
}

__global__ void gather_hidden_kernel(const float* __restrict__ hidden, const int* __restrict__ acc_idx,
                                     const int* __restrict__ m, int R, int H, float* __restrict__ hid_acc) {
  const int i = blockIdx.x, b = blockIdx.y;
  if (i >= m[b]) return;
  const int a = acc_idx[(size_t)b * R + i];
  if (a < 0 || a >= R) return;
  for (int c = threadIdx.x; c < H; c += blockDim.x)
    hid_acc[((size_t)b * R + i) * H + c] = hidden[((size_t)b * R + a) * H + c];
}
void launch_gather_hidden(const float* hidden, const int* acc_idx, const int* m, int B, int R, int H, float* hid_acc,
                          hipStream_t st) {
  gather_hidden_kernel<<<dim3(R, B), 256, 0, st>>>(hidden, acc_idx, m, R, H, hid_acc);
}

template <typename KT>
__global__ void read_kv_kernel(const KT* __restrict__ kc, const KT* __restrict__ vc, KVLayout kv, int b, int slot0,
                               int n_slots, float* __restrict__ k_out, float* __restrict__ v_out) {
  const int width = kv.n_kv * kv.d;
  const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (size_t)n_slots * width) return;
  const int s = (int)(idx / width), col = (int)(idx % width);
  k_out[idx] = ldkv(kc, kv_k_at(kv, b, slot0 + s, col / kv.d) + col % kv.d, kv.plane);
  v_out[idx] = ldkv(vc, kv_v_at(kv, b, col / kv.d, col % kv.d, slot0 + s), kv.plane);
}
void launch_read_kv(const void* k_cache, const void* v_cache, int kvdtype, KVLayout kv, int b, int slot0, int n_slots,
                    float* k_out, float* v_out, hipStream_t st) {
  const size_t n = (size_t)n_slots * kv.n_kv * kv.d;
  if (n == 0) return;
  const unsigned blocks = (unsigned)((n + 255) / 256);
  if (kvdtype == 0)
    read_kv_kernel<float><<<blocks, 256, 0, st>>>((const float*)k_cache, (const float*)v_cache, kv, b, slot0, n_slots,
                                                  k_out, v_out);
  else
    read_kv_kernel<bf16_t><<<blocks, 256, 0, st>>>((const bf16_t*)k_cache, (const bf16_t*)v_cache, kv, b, slot0,
                                                   n_slots, k_out, v_out);
}

template <typename KT>
__global__ void write_kv_kernel(KT* __restrict__ kc, KT* __restrict__ vc, KVLayout kv, int b, int slot0, int n_slots,
                                const float* __restrict__ k_in, const float* __restrict__ v_in) {
  const int width = kv.n_kv * kv.d;
  const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (size_t)n_slots * width) return;
  const int s = (int)(idx / width), col = (int)(idx % width);
  stkv(kc, kv_k_at(kv, b, slot0 + s, col / kv.d) + col % kv.d, kv.plane, k_in[idx]);
  stkv(vc, kv_v_at(kv, b, col / kv.d, col % kv.d, slot0 + s), kv.plane, v_in[idx]);
}
void launch_write_kv(void* k_cache, void* v_cache, int kvdtype, KVLayout kv, int b, int slot0, int n_slots,
                     const float* k_in, const float* v_in, hipStream_t st) {
  const size_t n = (size_t)n_slots * kv.n_kv * kv.d;
  if (n == 0) return;
  const unsigned blocks = (unsigned)((n + 255) / 256);
  if (kvdtype == 0)
    write_kv_kernel<float><<<blocks, 256, 0, st>>>((float*)k_cache, (float*)v_cache, kv, b, slot0, n_slots, k_in, v_in);
  else
    write_kv_kernel<bf16_t><<<blocks, 256, 0, st>>>((bf16_t*)k_cache, (bf16_t*)v_cache, kv, b, slot0, n_slots, k_in,
                                                    v_in);
}

// ------------------------------------------------------------------------------------------
// split-bf16 planes and partial-sum consumers
// ------------------------------------------------------------------------------------------
__global__ void split_planes_kernel(const float* __restrict__ x, int ldx, bf16_t* __restrict__ hi,
                                    bf16_t* __restrict__ lo, int ldo, int K) {
  const size_t row = blockIdx.y;
  const int c = blockIdx.x * blockDim.x + threadIdx.x;
  if (c >= K) return;
  const float v = x[row * ldx + c];
  const bf16_t h = f32_to_bf16(v);
  hi[row * ldo + c] = h;
  lo[row * ldo + c] = f32_to_bf16(v - bf16_to_f32(h));
}
void launch_split_planes(const float* x, int ldx, bf16_t* hi, bf16_t* lo, int ldo, int rows, int K, hipStream_t st) {
  if (rows <= 0) return;
  split_planes_kernel<<<dim3((K + 255) / 256, rows), 256, 0, st>>>(x, ldx, hi, lo, ldo, K);
}

template <typename WT>
__global__ void reduce_kernel(const float* __restrict__ P, int splits, size_t sps, int ldp, const WT* __restrict__ bias,
                              float* __restrict__ Y, int ldy, int N, int mode) {
  const size_t row = blockIdx.y;
  const int c = blockIdx.x * blockDim.x + threadIdx.x;
  if (c >= N) return;
  float v = 0.f;
  for (int s = 0; s < splits; ++s) v += P[s * sps + row * ldp + c];
  if (bias) v += ldf(bias, c);
  float* y = Y + row * ldy + c;
  *y = mode == 1 ? *y + v : v;
}
void launch_reduce(const float* P, int splits, size_t split_stride, int ldp, const void* bias, int wdtype, float* Y,
                   int ldy, int M, int N, int mode, hipStream_t st) {
  if (M <= 0) return;
  dim3 grid((N + 255) / 256, M);
  if (wdtype == 0)
    reduce_kernel<float><<<grid, 256, 0, st>>>(P, splits, split_stride, ldp, (const float*)bias, Y, ldy, N, mode);
  else
    reduce_kernel<bf16_t><<<grid, 256, 0, st>>>(P, splits, split_stride, ldp, (const bf16_t*)bias, Y, ldy, N, mode);
}

// one 1024-thread block per row: residual add of the split-K partials (sixteen loads in flight per
// thread, summed in split order), then RMSNorm written as planes.  A thread keeps its (up to two)
// float4 of the new row in registers across the block-wide sum of squares; wider rows re-read them.
template <typename WT>
__global__ __launch_bounds__(1024) void reduce_add_norm_kernel(float* __restrict__ x, int ldx,
                                                               const float* __restrict__ P, int splits, size_t sps,
                                                               int ldp, const WT* __restrict__ gain, float eps,
                                                               bf16_t* __restrict__ hi, bf16_t* __restrict__ lo,
                                                               int ldo, int H, const WT* __restrict__ bias) {
  __shared__ float red[16];
  const size_t row = blockIdx.x;
  float* xr = x + row * ldx;
  const float* pr = P + row * ldp;
  float ss = 0.f;
  auto new_row = [&](int c) -> float4 {
    float4 v = bias ? make_float4(ldf(bias, c), ldf(bias, c + 1), ldf(bias, c + 2), ldf(bias, c + 3))
                    : *(const float4*)(xr + c);
    for (int s0 = 0; s0 < splits; s0 += 16) {
      float4 q[16];
#pragma unroll
      for (int j = 0; j < 16; ++j)
        q[j] = (s0 + j < splits) ? *(const float4*)(pr + (size_t)(s0 + j) * sps + c) : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
      for (int j = 0; j < 16; ++j) { v.x += q[j].x; v.y += q[j].y; v.z += q[j].z; v.w += q[j].w; }
    }
    if (splits > 0 || bias) *(float4*)(xr + c) = v;
    ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
    return v;
  };
  auto gain4 = [&](int c) { return make_float4(ldf(gain, c), ldf(gain, c + 1), ldf(gain, c + 2), ldf(gain, c + 3)); };
  const int c0 = threadIdx.x * 4;
  float4 keep[2], gn[2];
#pragma unroll
  for (int it = 0; it < 2; ++it) {  // (static indices: the two kept pieces live in registers)
    const int c = c0 + it * 4096;
    if (c < H) {
      if (gain) gn[it] = gain4(c);
      keep[it] = new_row(c);
    }
  }
  for (int c = c0 + 8192; c < H; c += 4096) new_row(c);
  if (!gain) return;
  ss = wave_sum(ss);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
  __syncthreads();
  float tot = 0.f;
#pragma unroll
  for (int w = 0; w < 16; ++w) tot += red[w];
  const float scale = 1.0f / sqrtf(tot / (float)H + eps);
  auto emit = [&](int c, float4 v, float4 g4) {
    const float o[4] = {v.x * scale * g4.x, v.y * scale * g4.y, v.z * scale * g4.z, v.w * scale * g4.w};
    bf16_t h[4], l[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      h[r] = f32_to_bf16(o[r]);
      l[r] = f32_to_bf16(o[r] - bf16_to_f32(h[r]));
    }
    *(uint2*)(hi + row * ldo + c) = make_uint2((unsigned)h[0] | ((unsigned)h[1] << 16), (unsigned)h[2] | ((unsigned)h[3] << 16));
    *(uint2*)(lo + row * ldo + c) = make_uint2((unsigned)l[0] | ((unsigned)l[1] << 16), (unsigned)l[2] | ((unsigned)l[3] << 16));
  };
#pragma unroll
  for (int it = 0; it < 2; ++it) {
    const int c = c0 + it * 4096;
    if (c < H) emit(c, keep[it], gn[it]);
  }
  for (int c = c0 + 8192; c < H; c += 4096) emit(c, *(const float4*)(xr + c), gain4(c));  // written by this same thread above
}
void launch_reduce_add_norm(float* x, int ldx, const float* P, int splits, size_t split_stride, int ldp,
                            const void* gain, int wdtype, float eps, bf16_t* hi, bf16_t* lo, int ldo, int rows, int H,
                            hipStream_t st, const void* bias) {
  if (rows <= 0) return;
  if (wdtype == 0)
    reduce_add_norm_kernel<float><<<rows, 1024, 0, st>>>(x, ldx, P, splits, split_stride, ldp, (const float*)gain, eps,
                                                        hi, lo, ldo, H, (const float*)bias);
  else
    reduce_add_norm_kernel<bf16_t><<<rows, 1024, 0, st>>>(x, ldx, P, splits, split_stride, ldp, (const bf16_t*)gain,
                                                         eps, hi, lo, ldo, H, (const bf16_t*)bias);
}

}  // namespace clv
