// Stand-alone probe (not part of libclover.so): do v_mfma_f32_16x16x32_bf16 instructions overlap ordinary vector-ALU
// instructions on one SIMD of gfx950 -- (a) of the same wavefront, interleaved in program order, (b) of a second
// wavefront on the same SIMD?  Also: the issue rate of dependent and independent accumulation chains.
//
//   hipcc -O3 --offload-arch=gfx950 -o /tmp/mfma_valu_overlap paper_2408_00264_amd/csrc/probes/mfma_valu_overlap.hip && /tmp/mfma_valu_overlap
//
// One workgroup of eight wavefronts; wavefronts w and w + 4 share a SIMD (two of them issuing only matrix
// instructions each take twice the time of one alone).  Only wavefront 0 (and 4, where stated) works; the others
// wait at the end.  Times are shader clocks per iteration of 24 matrix instructions.
#include <hip/hip_runtime.h>
#include <cstdio>
#define CK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("HIP error %s at line %d\n", hipGetErrorString(e), __LINE__); return 1; } } while (0)
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// NF: fma instructions after every matrix instruction (program order pinned); ROLE4: what wavefront 4 does
// (0 idle, 1 the same as wavefront 0, 2 only fma: 96 per iteration); NACC: independent accumulators of the chain
template <int NF, int ROLE4, int NACC>
__global__ __launch_bounds__(512) void k(long long* out, float* sink, int iters) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  bf16x8 a, b;
  for (int i = 0; i < 8; ++i) { a[i] = (__bf16)(0.001f * (lane + i)); b[i] = (__bf16)(0.002f * (lane - i)); }
  f32x4 acc[4];
  for (int j = 0; j < 4; ++j) acc[j] = (f32x4){0.f, 0.f, 0.f, 0.f};
  float v0 = 0.5f + lane, v1 = 0.6f + lane, v2 = 0.7f + lane, v3 = 0.8f + lane;
  const int role = wave == 0 ? 1 : wave == 4 ? ROLE4 : 0;
  __syncthreads();
  const long long t0 = clock64();
  if (role == 1) {
    for (int it = 0; it < iters; ++it)
#pragma unroll
      for (int r = 0; r < 24; ++r) {
        acc[r % NACC] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, acc[r % NACC], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        if (NF >= 1) v0 = __builtin_fmaf(v0, 0.999f, 0.001f);
        if (NF >= 2) v1 = __builtin_fmaf(v1, 0.999f, 0.001f);
        if (NF >= 3) v2 = __builtin_fmaf(v2, 0.999f, 0.001f);
        if (NF >= 4) v3 = __builtin_fmaf(v3, 0.999f, 0.001f);
        __builtin_amdgcn_sched_barrier(0);
      }
  } else if (role == 2) {
    for (int it = 0; it < iters; ++it)
#pragma unroll
      for (int r = 0; r < 24; ++r) {
        v0 = __builtin_fmaf(v0, 0.999f, 0.001f); v1 = __builtin_fmaf(v1, 0.999f, 0.001f);
        v2 = __builtin_fmaf(v2, 0.999f, 0.001f); v3 = __builtin_fmaf(v3, 0.999f, 0.001f);
      }
  }
  const long long t1 = clock64();
  const float s = acc[0][0] + acc[1][0] + acc[2][0] + acc[3][0] + v0 + v1 + v2 + v3;
  if (lane == 0) out[wave] = t1 - t0;
  if (s == 12345.678f) sink[threadIdx.x] = s;   // keeps the arithmetic alive
}

template <int NF, int ROLE4, int NACC>
static int run(long long* out, float* sink, const char* what) {
  const int iters = 1000;
  for (int rep = 0; rep < 2; ++rep) { k<NF, ROLE4, NACC><<<1, 512>>>(out, sink, iters); CK(hipDeviceSynchronize()); }
  long long h[8]; CK(hipMemcpy(h, out, sizeof(h), hipMemcpyDeviceToHost));
  printf("%-86s wavefront 0: %7.1f clk", what, (double)h[0] / iters);
  if (ROLE4) printf("   wavefront 4: %7.1f clk", (double)h[4] / iters);
  printf("\n"); fflush(stdout);
  return 0;
}

int main() {
  long long* out; float* sink; CK(hipMalloc(&out, 8 * 8)); CK(hipMalloc(&sink, 512 * 4));
  if (run<0, 0, 1>(out, sink, "24 MFMA, one dependent chain")) return 1;
  if (run<0, 0, 4>(out, sink, "24 MFMA, four independent chains")) return 1;
  if (run<1, 0, 4>(out, sink, "24 x (MFMA + 1 fma)")) return 1;
  if (run<2, 0, 4>(out, sink, "24 x (MFMA + 2 fma)")) return 1;
  if (run<4, 0, 4>(out, sink, "24 x (MFMA + 4 fma)")) return 1;
  if (run<0, 1, 4>(out, sink, "24 MFMA in wavefront 0 and in wavefront 4 (same SIMD)")) return 1;
  if (run<0, 2, 4>(out, sink, "24 MFMA in wavefront 0, 96 fma in wavefront 4 (alone: 96 fma = ~380 clk)")) return 1;
  if (run<4, 1, 4>(out, sink, "24 x (MFMA + 4 fma) in both")) return 1;
  return 0;
}
