// Stand-alone probe (not part of libclover.so): how fast can the wavefronts of one launch stream a buffer from HBM,
// as a function of the launch size, the wavefronts per compute unit and the loads each wavefront keeps in flight?
// The weight-streaming GEMMs are sized against these figures.
//
//   hipcc -O3 --offload-arch=gfx950 -o /tmp/stream_rate paper_2408_00264_amd/csrc/probes/stream_rate.hip && /tmp/stream_rate
//
// Every workgroup reads its own contiguous share of the buffer, every wavefront its own contiguous share of that,
// in bursts of U loads of 1 KB (16 bytes per lane, non-temporal), all issued before the first is consumed.
// "+X" rows: the same wavefronts also read as many bytes again from a 4 MB buffer that stays in the L2 (the
// activations of a GEMM).  Time = HIP events around the launch (they include ~2 us of dispatch).
#include <hip/hip_runtime.h>
#include <cstdio>
#define CK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("HIP error %s at line %d\n", hipGetErrorString(e), __LINE__); return 1; } } while (0)
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
constexpr size_t X_BYTES = 4u << 20;

template <int U, bool WITH_X>
__global__ __launch_bounds__(512) void stream_kernel(const char* w, const char* x, size_t wg_bytes, int waves, u32x4* sink) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  if (wave >= waves) return;
  const size_t per_wave = wg_bytes / waves;                  // a multiple of U KB (checked on the host)
  const char* base = w + (size_t)blockIdx.x * wg_bytes + (size_t)wave * per_wave;
  u32x4 acc = {0, 0, 0, 0};
  for (size_t off = 0; off < per_wave; off += (size_t)U * 1024) {
    u32x4 v[U], y[WITH_X ? U : 1];
#pragma unroll
    for (int i = 0; i < U; ++i) v[i] = __builtin_nontemporal_load((const u32x4*)(base + off + i * 1024 + lane * 16));
    if (WITH_X) {
      const size_t xo = (off + (size_t)wave * per_wave) % (X_BYTES - (size_t)U * 1024);   // stays inside the X buffer
#pragma unroll
      for (int i = 0; i < U; ++i) y[i] = *(const u32x4*)(x + (xo & ~(size_t)1023) + i * 1024 + lane * 16);
    }
#pragma unroll
    for (int i = 0; i < U; ++i) { acc ^= v[i]; if (WITH_X) acc ^= y[i]; }
  }
  if (acc.x == 0x12345678u) sink[blockIdx.x * 512 + threadIdx.x] = acc;   // keeps the loads alive
}

int main() {
  const int MAX_WG = 256;
  const size_t MAX_WG_BYTES = 8u << 20;
  char *w, *x; u32x4* sink;
  CK(hipMalloc(&w, (size_t)MAX_WG * MAX_WG_BYTES)); CK(hipMalloc(&x, X_BYTES)); CK(hipMalloc(&sink, (size_t)MAX_WG * 512 * 16));
  CK(hipMemset(w, 1, (size_t)MAX_WG * MAX_WG_BYTES)); CK(hipMemset(x, 2, X_BYTES));
  hipStream_t st; CK(hipStreamCreate(&st));
  hipEvent_t a, b; CK(hipEventCreate(&a)); CK(hipEventCreate(&b));
  printf("%-12s %-10s %-6s %-10s %-4s %10s %10s\n", "launch", "workgroups", "waves", "in flight", "+X", "us", "TB/s");
  for (size_t wg_bytes : {MAX_WG_BYTES, (size_t)1 << 20})
    for (int wgs : {256, 224})
      for (int cfg = 0; cfg < 6; ++cfg) {
        const int waves = (cfg == 2 || cfg == 3) ? 4 : 8, u = (cfg == 0 || cfg == 2 || cfg == 4) ? 8 : 16;
        const bool with_x = cfg >= 4;
        if ((wg_bytes / waves) % ((size_t)u * 1024) != 0 || (size_t)wgs * wg_bytes > (size_t)MAX_WG * MAX_WG_BYTES) { printf("bad sizes\n"); return 1; }
        float ms = 0.f;
        for (int rep = 0; rep < 3; ++rep) {
          CK(hipEventRecord(a, st));
          if (u == 8 && !with_x) stream_kernel<8, false><<<wgs, 512, 0, st>>>(w, x, wg_bytes, waves, sink);
          if (u == 16 && !with_x) stream_kernel<16, false><<<wgs, 512, 0, st>>>(w, x, wg_bytes, waves, sink);
          if (u == 8 && with_x) stream_kernel<8, true><<<wgs, 512, 0, st>>>(w, x, wg_bytes, waves, sink);
          if (u == 16 && with_x) stream_kernel<16, true><<<wgs, 512, 0, st>>>(w, x, wg_bytes, waves, sink);
          CK(hipEventRecord(b, st));
          CK(hipStreamSynchronize(st));
          CK(hipEventElapsedTime(&ms, a, b));
        }
        printf("%6.0f MB    %-10d %-6d %3d KB     %-4s %10.1f %10.2f\n", wgs * (double)wg_bytes / 1e6, wgs, waves, u, with_x ? "yes" : "no",
               ms * 1e3, wgs * (double)wg_bytes / (ms * 1e-3) / 1e12);
        fflush(stdout);
      }
  return 0;
}
