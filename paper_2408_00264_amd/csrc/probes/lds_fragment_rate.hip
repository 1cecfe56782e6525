// Stand-alone probe (not part of libclover.so): at which LDS row strides do the 16-byte fragment reads of the MFMA
// kernels (lane l reads row l % 16, 16-byte piece l / 16 -- one 16x32 bf16 operand) run at the full rate of a CU's LDS?
//
//   hipcc -O3 --offload-arch=gfx950 -o /tmp/lds_fragment_rate paper_2408_00264_amd/csrc/probes/lds_fragment_rate.hip && /tmp/lds_fragment_rate
//
// One workgroup of eight wavefronts (one CU) reads fragments from a 64 KB array for 2000 iterations of eight reads;
// the rate is bytes read by all wavefronts / shader clocks of the slowest one.  Nothing is written after set-up.
#include <hip/hip_runtime.h>
#include <cstdio>
#define CK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("HIP error %s at line %d\n", hipGetErrorString(e), __LINE__); return 1; } } while (0)
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
constexpr int LDS_BYTES = 64 * 1024;

// mode 0: address of lane = (lane % 16) * row_stride + (lane / 16) * 16;  mode 1: lane * 16 (a contiguous KB);
// mode 2: rows of 256 B without padding, piece index XOR row
__global__ __launch_bounds__(512) void read_kernel(long long* out, int iters, unsigned* sink, int row_stride, int mode) {
  __shared__ __attribute__((aligned(16))) unsigned char lds[LDS_BYTES];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, l16 = lane & 15, g4 = lane >> 4;
  for (int i = tid; i < LDS_BYTES / 4; i += blockDim.x) ((unsigned*)lds)[i] = i * 2654435761u;
  __syncthreads();
  int base = l16 * row_stride + g4 * 16;
  if (mode == 1) base = lane * 16;
  if (mode == 2) base = l16 * 256 + ((g4 ^ l16) & 15) * 16;
  u32x4 acc = {0, 0, 0, 0};
  const long long t0 = clock64();
  for (int it = 0; it < iters; ++it) {
    asm volatile("" : "+v"(base));   // opaque: the reads stay inside the loop
    u32x4 v[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) v[j] = *(const u32x4*)(lds + base + j * 4096);
#pragma unroll
    for (int j = 0; j < 8; ++j) acc ^= v[j];
  }
  const long long t1 = clock64();
  if (lane == 0) out[wave] = t1 - t0;
  if (acc.x == 0x12345u) sink[tid] = acc.y;   // keeps the reads alive
}

static int run(long long* out, unsigned* sink, int row_stride, int mode, const char* name) {
  const int iters = 2000;
  const int max_base = mode == 0 ? 15 * row_stride + 3 * 16 : mode == 1 ? 63 * 16 : 15 * 256 + 15 * 16;
  if (row_stride % 16 != 0 || max_base + 7 * 4096 + 16 > LDS_BYTES) { printf("%-34s skipped (out of range)\n", name); return 0; }
  for (int rep = 0; rep < 2; ++rep) { read_kernel<<<1, 512>>>(out, iters, sink, row_stride, mode); CK(hipDeviceSynchronize()); }
  long long h[8]; CK(hipMemcpy(h, out, sizeof(h), hipMemcpyDeviceToHost));
  long long mx = 0; for (int w = 0; w < 8; ++w) mx = h[w] > mx ? h[w] : mx;
  printf("%-34s %6.1f B/clk\n", name, 8.0 * iters * 8 * 1024 / mx); fflush(stdout);
  return 0;
}

int main() {
  long long* out; unsigned* sink; CK(hipMalloc(&out, 8 * 8)); CK(hipMalloc(&sink, 512 * 4));
  if (run(out, sink, 0, 1, "contiguous KB (lane * 16)")) return 1;
  if (run(out, sink, 0, 2, "256 B rows, piece XOR row")) return 1;
  char name[64];
  for (int stride = 16; stride <= 560; stride += 16) {
    snprintf(name, sizeof(name), "row stride %3d B (= %2d mod 64)", stride, stride % 64);
    if (run(out, sink, stride, 0, name)) return 1;
  }
  return 0;
}
