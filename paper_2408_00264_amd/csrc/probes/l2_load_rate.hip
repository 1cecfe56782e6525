// Stand-alone probe (not part of libclover.so): how many bytes per clock can ONE compute unit pull from a buffer that
// stays in the L2 -- with 16-byte loads into registers, and with LDS-direct loads (global_load_lds_dwordx4)?  Four
// wavefronts (one per SIMD), eight loads of 1 KB in flight each; rate = bytes of all wavefronts / shader clocks of the
// slowest one.  The figure bounds what the activations cost a weight-streaming GEMM workgroup: they come through the
// same path as its weights.
//
//   hipcc -O3 --offload-arch=gfx950 -o /tmp/l2_load_rate paper_2408_00264_amd/csrc/probes/l2_load_rate.hip && /tmp/l2_load_rate
#include <hip/hip_runtime.h>
#include <cstdio>
#define CK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("HIP error %s at line %d\n", hipGetErrorString(e), __LINE__); return 1; } } while (0)
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
constexpr int SRC_BYTES = 256 * 1024;
template <int MODE>   // 0: LDS-direct, 2: loads to registers
__global__ __launch_bounds__(256) void k(const char* src, long long* out, int iters, unsigned* sink) {
  __shared__ __attribute__((aligned(16))) unsigned char lds[64 * 1024];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  unsigned char* my = lds + wave * 16 * 1024;
  u32x4 acc = {0, 0, 0, 0};
  __syncthreads();
  const long long t0 = clock64();
  for (int it = 0; it < iters; ++it) {
    const size_t off = ((size_t)(it * 8 * 1024 + wave * 64 * 1024)) % (SRC_BYTES - 8 * 1024);
    if (MODE == 0) {
#pragma unroll
      for (int j = 0; j < 8; ++j)
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src + off + j * 1024 + lane * 16),
                                         (__attribute__((address_space(3))) void*)(my + j * 1024), 16, 0, 0);
    } else {
      u32x4 v[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) v[j] = *(const u32x4*)(src + off + j * 1024 + lane * 16);
#pragma unroll
      for (int j = 0; j < 8; ++j) acc ^= v[j];
    }
  }
  __builtin_amdgcn_s_waitcnt(0);
  const long long t1 = clock64();
  if (lane == 0) out[wave] = t1 - t0;
  if (acc.x == 0x1234567u || lds[tid] == 0x7f) sink[tid] = acc.y;
}
int main() {
  char* src; long long* out; unsigned* sink;
  CK(hipMalloc(&src, SRC_BYTES)); CK(hipMemset(src, 1, SRC_BYTES)); CK(hipMalloc(&out, 64)); CK(hipMalloc(&sink, 1024));
  const int iters = 2000;
  const char* names[3] = {"LDS-direct loads", "", "loads to registers"};
  for (int mode = 0; mode < 3; mode += 2) {
    for (int rep = 0; rep < 2; ++rep) {
      if (mode == 0) k<0><<<1, 256>>>(src, out, iters, sink);
      if (mode == 2) k<2><<<1, 256>>>(src, out, iters, sink);
      CK(hipDeviceSynchronize());
    }
    long long h[8]; CK(hipMemcpy(h, out, sizeof(h), hipMemcpyDeviceToHost));
    long long mx = 0; for (int w = 0; w < 4; ++w) mx = h[w] > mx ? h[w] : mx;
    printf("%-40s %6.1f B/clk per CU (%5.1f clk per KB and wavefront)\n", names[mode], 4.0 * iters * 8 * 1024 / mx, (double)mx / (iters * 8)); fflush(stdout);
  }
  return 0;
}
