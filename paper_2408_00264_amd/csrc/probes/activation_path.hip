// Stand-alone probe (not part of libclover.so): a 224-workgroup launch streams 235 MB (the gate+up weights of the 8B
// shape) from HBM; beside it the same wavefronts read as many bytes again from a 4 MB buffer that stays in the L2 (what
// the activation planes are to a GEMM workgroup) -- with ordinary loads into registers, or with LDS-direct loads
// (global_load_lds_dwordx4).  Does the register path cost anything?  The last line checks the lane layout of the
// LDS-direct load (lane l's 16 bytes land at block + 16 l).
//
//   hipcc -O3 --offload-arch=gfx950 -o /tmp/activation_path paper_2408_00264_amd/csrc/probes/activation_path.hip && /tmp/activation_path
#include <hip/hip_runtime.h>
#include <cstdio>
#define CK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("HIP error %s at line %d\n", hipGetErrorString(e), __LINE__); return 1; } } while (0)
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
constexpr size_t X_BYTES = 4u << 20;
// mode 0: W only; 1: W + X plain loads; 2: W + X through global_load_lds (16 B per lane, 1 KB per instruction)
template <int MODE>
__global__ __launch_bounds__(512) void k(const char* w, const char* x, size_t wg_bytes, u32x4* sink, int* check) {
  __shared__ __attribute__((aligned(16))) char lds[8 * 8 * 1024];   // 8 wavefronts x 8 KB
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const size_t per_wave = wg_bytes / 8;
  const char* base = w + (size_t)blockIdx.x * wg_bytes + (size_t)wave * per_wave;
  char* my_lds = lds + wave * 8 * 1024;
  u32x4 acc = {0, 0, 0, 0};
  for (size_t off = 0; off < per_wave; off += 8 * 1024) {
    u32x4 v[8], y[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = __builtin_nontemporal_load((const u32x4*)(base + off + i * 1024 + lane * 16));
    const size_t xo = ((off + (size_t)wave * per_wave) % (X_BYTES - 8 * 1024)) & ~(size_t)1023;
    if (MODE == 1) {
#pragma unroll
      for (int i = 0; i < 8; ++i) y[i] = *(const u32x4*)(x + xo + i * 1024 + lane * 16);
    }
    if (MODE == 2) {
#pragma unroll
      for (int i = 0; i < 8; ++i)
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(x + xo + i * 1024 + lane * 16),
                                         (__attribute__((address_space(3))) void*)(my_lds + i * 1024), 16, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) { acc ^= v[i]; if (MODE == 1) acc ^= y[i]; }
    if (MODE == 2) {
      __builtin_amdgcn_s_waitcnt(0);   // everything landed (vmcnt 0)
      acc ^= *(const u32x4*)(my_lds + lane * 16);
    }
  }
  if (MODE == 2 && blockIdx.x == 0 && threadIdx.x < 64) {
    // lane layout check: after the last iteration LDS row i of this wavefront must equal x[xo_last + i*1024 + lane*16 ..]
    const size_t off = per_wave - 8 * 1024;
    const size_t xo = ((off + 0 * per_wave) % (X_BYTES - 8 * 1024)) & ~(size_t)1023;
    int ok = 1;
    for (int i = 0; i < 8; ++i) {
      const u32x4 a = *(const u32x4*)(lds + i * 1024 + lane * 16), b = *(const u32x4*)(x + xo + i * 1024 + lane * 16);
      ok &= (a.x == b.x && a.y == b.y && a.z == b.z && a.w == b.w);
    }
    if (!ok) atomicAdd(check, 1);
  }
  if (acc.x == 0x12345678u) sink[blockIdx.x * 512 + threadIdx.x] = acc;
}
int main() {
  const int WGS = 224; const size_t WG_BYTES = 1u << 20;
  char *w, *x; u32x4* sink; int* check;
  CK(hipMalloc(&w, (size_t)256 * WG_BYTES)); CK(hipMalloc(&x, X_BYTES)); CK(hipMalloc(&sink, (size_t)256 * 512 * 16)); CK(hipMalloc(&check, 4));
  CK(hipMemset(w, 1, (size_t)256 * WG_BYTES)); CK(hipMemset(check, 0, 4));
  // X holds its own word index so that the layout check means something
  { unsigned* hx = (unsigned*)malloc(X_BYTES); for (size_t i = 0; i < X_BYTES / 4; ++i) hx[i] = (unsigned)i * 2654435761u; CK(hipMemcpy(x, hx, X_BYTES, hipMemcpyHostToDevice)); free(hx); }
  hipStream_t st; CK(hipStreamCreate(&st));
  hipEvent_t a, b; CK(hipEventCreate(&a)); CK(hipEventCreate(&b));
  const char* names[3] = {"W only", "W + X plain loads", "W + X direct-to-LDS loads"};
  for (int mode = 0; mode < 3; ++mode) {
    float ms = 0;
    for (int rep = 0; rep < 4; ++rep) {
      CK(hipEventRecord(a, st));
      if (mode == 0) k<0><<<WGS, 512, 0, st>>>(w, x, WG_BYTES, sink, check);
      if (mode == 1) k<1><<<WGS, 512, 0, st>>>(w, x, WG_BYTES, sink, check);
      if (mode == 2) k<2><<<WGS, 512, 0, st>>>(w, x, WG_BYTES, sink, check);
      CK(hipEventRecord(b, st)); CK(hipStreamSynchronize(st)); CK(hipEventElapsedTime(&ms, a, b));
    }
    printf("%-28s %8.1f us\n", names[mode], ms * 1e3); fflush(stdout);
  }
  int h = -1; CK(hipMemcpy(&h, check, 4, hipMemcpyDeviceToHost));
  printf("layout check: %d lanes saw a mismatch (0 = LDS row i, lane l holds the 16 bytes lane l asked for)\n", h);
  return 0;
}
