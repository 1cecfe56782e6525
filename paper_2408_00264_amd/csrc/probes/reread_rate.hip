// Stand-alone probe (not part of libclover.so): is a buffer that another kernel has just read faster to stream than a
// cold one -- is there a memory-side cache that the weights of the next GEMM could be prefetched into while the
// latency-bound kernels of a layer run?  256 workgroups stream S MB after (a) a 1 GB read of another buffer (cold),
// (b) the same and then a read of the S MB themselves, with ordinary or non-temporal loads.
//
//   hipcc -O3 --offload-arch=gfx950 -o /tmp/reread_rate paper_2408_00264_amd/csrc/probes/reread_rate.hip && /tmp/reread_rate
#include <hip/hip_runtime.h>
#include <cstdio>
#define CK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("HIP error %s at line %d\n", hipGetErrorString(e), __LINE__); return 1; } } while (0)
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
template <bool NT>
__global__ __launch_bounds__(512) void rd(const char* w, size_t wg_bytes, u32x4* sink) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const size_t per_wave = wg_bytes / 8;
  const char* base = w + (size_t)blockIdx.x * wg_bytes + (size_t)wave * per_wave;
  u32x4 acc = {0, 0, 0, 0};
  for (size_t off = 0; off < per_wave; off += 8 * 1024) {
    u32x4 v[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = NT ? __builtin_nontemporal_load((const u32x4*)(base + off + i * 1024 + lane * 16)) : *(const u32x4*)(base + off + i * 1024 + lane * 16);
#pragma unroll
    for (int i = 0; i < 8; ++i) acc ^= v[i];
  }
  if (acc.x == 0x12345678u) sink[blockIdx.x * 512 + threadIdx.x] = acc;
}
int main() {
  const int WGS = 256;
  const size_t BUF = (size_t)1 << 30;      // two 1 GB buffers: the one measured and one to push it out
  char *w, *flush; u32x4* sink;
  CK(hipMalloc(&w, BUF)); CK(hipMalloc(&flush, BUF)); CK(hipMalloc(&sink, (size_t)WGS * 512 * 16));
  CK(hipMemset(w, 1, BUF)); CK(hipMemset(flush, 2, BUF));
  hipStream_t st; CK(hipStreamCreate(&st));
  hipEvent_t a, b; CK(hipEventCreate(&a)); CK(hipEventCreate(&b));
  printf("%-8s %-10s %-12s %10s %10s\n", "MB", "first read", "state", "us", "TB/s");
  for (size_t mb : {32, 64, 128, 192, 256, 384, 512}) {
    const size_t wg_bytes = mb * 1024 * 1024 / WGS;                    // a multiple of 64 KB for every size above
    if (wg_bytes % (64 * 1024) != 0 || wg_bytes * WGS > BUF) { printf("bad size\n"); return 1; }
    for (int warm_nt = 0; warm_nt < 2; ++warm_nt)
      for (int state = 0; state < 2; ++state) {                        // 0: cold (flushed), 1: read just before
        float best = 1e9f;
        for (int rep = 0; rep < 3; ++rep) {
          rd<false><<<WGS, 512, 0, st>>>(flush, BUF / WGS, sink);      // push everything out
          if (state == 1) { if (warm_nt) rd<true><<<WGS, 512, 0, st>>>(w, wg_bytes, sink); else rd<false><<<WGS, 512, 0, st>>>(w, wg_bytes, sink); }
          CK(hipEventRecord(a, st));
          rd<true><<<WGS, 512, 0, st>>>(w, wg_bytes, sink);
          CK(hipEventRecord(b, st)); CK(hipStreamSynchronize(st));
          float ms; CK(hipEventElapsedTime(&ms, a, b)); if (ms < best) best = ms;
        }
        printf("%-8zu %-10s %-12s %10.1f %10.2f\n", mb, warm_nt ? "nt" : "plain", state ? "just read" : "cold", best * 1e3, mb * 1048576.0 / (best * 1e-3) / 1e12);
        fflush(stdout);
      }
  }
  return 0;
}
