// Persistent "phase program" kernel for the few-row decoder stack (M <= 64 rows, bf16 weights) on gfx950.
//
// One cooperative launch of one workgroup per compute unit walks a list of phases (embedding, GEMMs,
// RoPE + KV write, tree attention, split merge, residual add) with a grid-wide barrier after each.
// Why one kernel: a decoder layer at 64 rows is nine dependent kernels of 5..50 us, and every kernel
// boundary costs ~4.5 us of drain, cache write-back and dispatch during which no weight bytes move.
// Inside one kernel a barrier costs ~2.5 us and, more important, does not stop the memory pipeline.
//
// Coherence without cache flushes.  The eight XCDs have private L2 caches.
//   * Data another XCD reads later in the launch is stored write-through at agent scope
//     (buffer_store ... sc1); before reading it, after the grid barrier, one thread per workgroup executes
//     an agent-scope acquire (buffer_inv sc1), so plain loads miss in L1/L2 and may then be cached again --
//     which is what lets the 32 workgroups of an XCD share one activation slice.  No L2 write-back
//     (buffer_wbl2) is ever needed: nothing another XCD reads is left dirty.
//   * Data only workgroups of the SAME XCD read (sharded phases) is stored plainly into that XCD's L2; an
//     XCD-local barrier (one counter per XCD) and an L1 invalidate (buffer_inv sc0) are enough.  Such
//     buffers are private to one XCD for the whole launch, cache line by cache line, so no other L2 ever
//     holds a copy that could be written back over them.
//   * Barriers are relaxed agent-scope atomics; the workgroup-scope release in front waits for the
//     stores to be acknowledged.  Grid barrier: per-XCD counters plus one top counter (~4 us); XCD-local
//     barrier: the per-XCD counter alone (~1 us).
// Workgroups i and i + 8 share an XCD because the dispatcher hands consecutive workgroups to consecutive
// XCDs; every launch checks this against the hardware's XCC id register and raises the error flag if it
// does not hold (sharded results would then be invalid).
//
// The spin of every barrier is bounded (wall clock); on expiry a sticky abort flag makes every later
// barrier and launch return at once, and the error flag word reports it to the host.
#include "clover_internal.h"

#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <type_traits>

namespace clv {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

namespace {

union Frag {
  u32x4 u;
  bf16x8 v;
};

#define MG_AGENT __HIP_MEMORY_SCOPE_AGENT
constexpr int AUX_SC1 = 16;  // cache-policy bit of the buffer intrinsics: agent-scope write-through / coherent
constexpr int AUX_NT = 2;    // non-temporal (streamed weights)

constexpr int MG_NT = 512;
constexpr int MG_WAVES = 8;
constexpr int MG_KST = 256;          // K columns per activation stage
constexpr int MG_LDK = MG_KST + 8;   // LDS row stride (bf16): +16 B makes the fragment reads conflict-free
constexpr int MG_UW = 2;             // column-unit wavefront groups per workgroup
constexpr int MG_KW = 4;             // k-parts per stage
constexpr int MG_CH = 8 / MG_KW;     // 32-column k-tiles per wavefront and stage
constexpr int MG_NFW = 4;            // weight fragments (16 output columns each) per wavefront
constexpr int MG_PASS_BLOCKS = MG_UW * MG_NFW;  // 16-column blocks a workgroup finishes per pass over K

__device__ __forceinline__ __amdgpu_buffer_rsrc_t rsrc_of(const void* p, unsigned bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, bytes, 0x00020000);
}
__device__ __forceinline__ unsigned rn_bf16(float a) {
  unsigned u = __float_as_uint(a);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return u >> 16;
}
__device__ __forceinline__ float bf16_f32(unsigned h) { return __uint_as_float(h << 16); }
__device__ __forceinline__ void split2(float a, float b, unsigned& hi, unsigned& lo) {
  const unsigned ha = rn_bf16(a), hb = rn_bf16(b);
  hi = ha | (hb << 16);
  lo = rn_bf16(a - bf16_f32(ha)) | (rn_bf16(b - bf16_f32(hb)) << 16);
}
// Stores of a phase's results.  wt: write-through at agent scope (readers on other XCDs after a grid
// barrier); else plain stores into this XCD's L2 (readers on this XCD after an XCD-local barrier).  The
// buffer resource is built from a wavefront-uniform base pointer and the lane's position goes into the
// byte offset (< 4 GB): a resource that differed per lane would be issued one lane at a time.
struct WtBuf {
  __amdgpu_buffer_rsrc_t r;
  bool wt;
  __device__ __forceinline__ WtBuf(const void* base, int write_through) : r(rsrc_of(base, 0xFFFFFFFFu)), wt(write_through != 0) {}
  __device__ __forceinline__ void st128(size_t byte_off, f32x4 v) const {
    if (wt) __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, v), r, (unsigned)byte_off, 0, AUX_SC1);
    else __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, v), r, (unsigned)byte_off, 0, 0);
  }
  __device__ __forceinline__ void st64(size_t byte_off, u32x2 v) const {
    if (wt) __builtin_amdgcn_raw_buffer_store_b64(v, r, (unsigned)byte_off, 0, AUX_SC1);
    else __builtin_amdgcn_raw_buffer_store_b64(v, r, (unsigned)byte_off, 0, 0);
  }
  __device__ __forceinline__ void st32(size_t byte_off, unsigned v) const {
    if (wt) __builtin_amdgcn_raw_buffer_store_b32(v, r, (unsigned)byte_off, 0, AUX_SC1);
    else __builtin_amdgcn_raw_buffer_store_b32(v, r, (unsigned)byte_off, 0, 0);
  }
  __device__ __forceinline__ void st16(size_t byte_off, unsigned v) const {
    if (wt) __builtin_amdgcn_raw_buffer_store_b16((unsigned short)v, r, (unsigned)byte_off, 0, AUX_SC1);
    else __builtin_amdgcn_raw_buffer_store_b16((unsigned short)v, r, (unsigned)byte_off, 0, 0);
  }
};

// ------------------------------------------------------------------------------------------
// barriers
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ bool mg_aborted(MegaSync* s) {
  return __hip_atomic_load(&s->abort, __ATOMIC_RELAXED, MG_AGENT) != 0u;
}

// A barrier comes in two halves so that a phase can put independent memory requests between them.
// local: only the workgroups of this XCD group (blockIdx.x % 8) meet.  `seq`: number of this barrier among
// the barriers of its kind since the counters were zeroed (1-based, the same in every workgroup).
struct Barrier {
  MegaSync* s;
  long long limit_ticks;
  int* err_flag;
  bool no_inv;  // timing experiment only
};
__device__ __forceinline__ void barrier_arrive(const Barrier& b, bool local, unsigned seq) {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");  // this wave's stores are acknowledged (L2, or memory if write-through)
  __syncthreads();
  if (threadIdx.x == 0 && !mg_aborted(b.s)) {
    const unsigned n = gridDim.x, x = blockIdx.x & 7u;
    const unsigned per = (n + 7u - x) / 8u;  // workgroups with blockIdx.x % 8 == x
    if (local) {
      __hip_atomic_fetch_add(&b.s->lcount[x * 64], 1u, __ATOMIC_RELAXED, MG_AGENT);
    } else {
      const unsigned old = __hip_atomic_fetch_add(&b.s->xcount[x * 64], 1u, __ATOMIC_RELAXED, MG_AGENT);
      if (old + 1u == seq * per) __hip_atomic_fetch_add(&b.s->top, 1u, __ATOMIC_RELAXED, MG_AGENT);
    }
  }
}
__device__ __forceinline__ void barrier_wait(const Barrier& b, bool local, unsigned seq) {
  if (threadIdx.x == 0) {
    if (!mg_aborted(b.s)) {
      const unsigned n = gridDim.x, x = blockIdx.x & 7u;
      const unsigned* ctr = local ? &b.s->lcount[x * 64] : &b.s->top;
      const unsigned target = local ? seq * ((n + 7u - x) / 8u) : seq * (n < 8u ? n : 8u);
      const long long t0 = wall_clock64();
      while ((int)(__hip_atomic_load(ctr, __ATOMIC_RELAXED, MG_AGENT) - target) < 0) {
        __builtin_amdgcn_s_sleep(1);
        if (wall_clock64() - t0 > b.limit_ticks) {
          __hip_atomic_store(&b.s->abort, 1u, __ATOMIC_RELAXED, MG_AGENT);
          atomicOr(b.err_flag, 2);
          break;
        }
        if (mg_aborted(b.s)) break;
      }
    }
    if (!b.no_inv) {
      if (local) asm volatile("buffer_inv sc0" ::: "memory");   // this CU's L1 only: the data is in this XCD's L2
      else __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");    // L1 and the L2 lines other XCDs may have rewritten
    }
  }
  __syncthreads();
}

// ------------------------------------------------------------------------------------------
// GEMM phase:  out = X[M,K] * W[N,K]^T
//
// Three mappings of (K range, 16-column blocks) onto workgroups (x = workgroup % 8, the XCD group;
// j = workgroup / 8):
//   shard 0  K group kg = x % KG over the whole grid: the workgroups of an XCD share the activation
//            stages they read (L2 hits after the first); every column block has KG partial results.
//   shard 1  XCD x owns a set of column blocks (its heads, its FFN slice) over all of K, split again
//            into KG local K groups among its workgroups; partial results stay in this XCD.
//   shard 2  XCD x owns a K slice (the columns it produced itself in the previous phase) for ALL
//            column blocks; partial result x goes to the grid-wide residual sum.
// A workgroup finishes its column blocks in passes of MG_PASS_BLOCKS; in a pass wavefront (uw, kp)
// owns MG_NFW fragments and the k-tiles kp*MG_CH.. of every 256-column stage, streams its weights
// global -> registers two stages ahead and reads the activation fragments from the double-buffered
// LDS stage.  The k-parts are added through LDS after the last stage.
// ------------------------------------------------------------------------------------------
constexpr int MG_NBUF = 2;           // register buffers of weight fragments: loads run MG_NBUF - 1 stages ahead (more in
                                     // flight only lengthens the queue in front of the latency-critical activation loads)
constexpr int MG_NPRE = MG_NBUF - 1;  // stages whose weights are requested before the previous phase's barrier

typedef Frag WBuf[MG_NFW][MG_CH];

// where a workgroup stands in a GEMM phase
struct GemmPlan {
  int kg;                      // index of the partial result this workgroup contributes to
  int s_begin, s_end;          // its K stages
  int b_begin, b_end;          // its column blocks (shard 1: indices into the XCD's local block list)
  int n_blocks, KT, cb_per_pass, cb_per_wave;
  int rot;                     // rotation of the stage order
  bool idle;                   // nothing to do (whole workgroup)
};
__device__ __forceinline__ GemmPlan gemm_plan(const MegaPhase& ph) {
  GemmPlan g;
  const int nwg = gridDim.x, wg = blockIdx.x;
  const int x = wg & 7, j = wg >> 3, nw = nwg >> 3;  // XCD group, index and count of workgroups in it
  const int KG = ph.KG;
  g.KT = ph.K / 32;
  const int NS = ph.K / MG_KST;
  g.n_blocks = ph.N / 16;  // epi 1: blocks of F (each a gate and an up fragment)
  int part, parts, kgi, kgs, nb;
  if (ph.shard == 0) {
    kgi = x % KG; kgs = KG;
    parts = nwg / KG; part = x / KG + (8 / KG) * j;
    nb = g.n_blocks;
    g.s_begin = (int)((long long)kgi * NS / kgs);
    g.s_end = (int)((long long)(kgi + 1) * NS / kgs);
    g.kg = kgi;
  } else if (ph.shard == 1) {
    kgi = j % KG; kgs = KG;
    parts = nw / KG; part = j / KG;
    nb = 0;
#pragma unroll
    for (int sgm = 0; sgm < 3; ++sgm) nb += ph.seg_bnd[sgm][x + 1] - ph.seg_bnd[sgm][x];
    g.s_begin = (int)((long long)kgi * NS / kgs);
    g.s_end = (int)((long long)(kgi + 1) * NS / kgs);
    g.kg = kgi;
    if (part >= parts) nb = 0;  // workgroups beyond parts * KG have no share
  } else {
    parts = nw; part = j;
    nb = g.n_blocks;
    g.s_begin = ph.ks_bnd[x];
    g.s_end = ph.ks_bnd[x + 1];
    g.kg = x;
  }
  g.b_begin = (int)((long long)part * nb / parts);
  g.b_end = (int)((long long)(part + 1) * nb / parts);
  g.cb_per_pass = ph.epi == 1 ? MG_PASS_BLOCKS / 2 : MG_PASS_BLOCKS;  // column blocks per pass
  g.cb_per_wave = ph.epi == 1 ? MG_NFW / 2 : MG_NFW;
  g.idle = g.b_begin >= g.b_end || g.s_begin >= g.s_end;
  // Workgroups walk their stages in rotated order: every weight block has the same power-of-two size, and
  // walking them in lock-step would keep all workgroups on the same few HBM channels at any moment.
  g.rot = g.idle ? 0 : j % (g.s_end - g.s_begin);
  return g;
}
// column block index -> block row of W (shard 1: the XCD's local list -> global block)
__device__ __forceinline__ int gemm_global_block(const MegaPhase& ph, int lb) {
  if (ph.shard != 1) return lb;
  const int x = blockIdx.x & 7;
  int gb = 0, cum = 0;
#pragma unroll
  for (int sgm = 0; sgm < 3; ++sgm) {
    const int lo = ph.seg_bnd[sgm][x], len = ph.seg_bnd[sgm][x + 1] - lo;
    if (lb >= cum && lb < cum + len) gb = ph.seg_base[sgm] + lo + (lb - cum);
    cum += len;
  }
  return gb;
}
// fragments of wavefront (uw, kp) in the pass that starts at column block p0: byte offset of fragment f
// at stage 0 (k-tile kp*MG_CH), out of range for a missing fragment; cbk: its column block (the index
// of gemm_plan's range) or -1; gbk: the same block's row in W
__device__ __forceinline__ void gemm_frags(const MegaPhase& ph, const GemmPlan& g, int p0, int uw, int kp, int lane,
                                           unsigned (&wof)[MG_NFW], int (&cbk)[MG_NFW], int (&gbk)[MG_NFW]) {
#pragma unroll
  for (int f = 0; f < MG_NFW; ++f) {
    const int cb = p0 + uw * g.cb_per_wave + (ph.epi == 1 ? f / 2 : f);
    const bool live = !g.idle && cb < min(g.b_end, p0 + g.cb_per_pass);
    cbk[f] = live ? cb : -1;
    gbk[f] = live ? gemm_global_block(ph, cb) : 0;
    const int wrow = (ph.epi == 1 && (f & 1)) ? gbk[f] + g.n_blocks : gbk[f];  // up fragments follow the gate matrix
    wof[f] = live ? ((unsigned)wrow * (unsigned)g.KT + (unsigned)(kp * MG_CH)) * 1024u + (unsigned)lane * 16u : 0xFFFFFF00u;
  }
}
// weights of stage s into one register buffer; a stage past the end or a missing fragment is an
// out-of-range buffer load (returns zeros, moves no data), so every load is issued unconditionally and
// the memory-wait counters stay exact
__device__ __forceinline__ void gemm_load_w(const __amdgpu_buffer_rsrc_t rw, const unsigned (&wof)[MG_NFW],
                                            const int (&cbk)[MG_NFW], int s, bool live, WBuf& w) {
  const unsigned so = (unsigned)s * 8192u;
#pragma unroll
  for (int f = 0; f < MG_NFW; ++f) {
    const unsigned o = (cbk[f] >= 0 && live) ? wof[f] + so : 0xFFFFFF00u;
#pragma unroll
    for (int t = 0; t < MG_CH; ++t) w[f][t].u = __builtin_amdgcn_raw_buffer_load_b128(rw, o, t * 1024, AUX_NT);
  }
}

// The barrier that ends the previous phase is taken INSIDE this phase, after the weights of the first
// MG_NPRE stages have been requested: they do not depend on the previous phase, so the HBM stream keeps
// running while the workgroups wait for each other.
template <int MT>
__device__ __forceinline__ void gemm_phase(const MegaPhase& ph, const int tid, bf16_t* xs, const Barrier& bar,
                                           const unsigned barrier_seq /* 0: no barrier */, long long* stamp) {
  constexpr int ROWS = MT * 16;
  constexpr int PLANE = ROWS * MG_LDK;
  constexpr int BUF = 2 * PLANE;
  constexpr int XIT = 2 * ROWS * (MG_KST / 8) / MG_NT;  // 16-byte pieces per thread and stage (MT = 4: 8)
  static_assert(MT == 4, "the staging loops assume 64 rows");
  const int wave = tid >> 6, lane = tid & 63;
  const int l16 = lane & 15, g4 = lane >> 4;
  const int uw = wave / MG_KW, kp = wave % MG_KW;
  const bool local_bar = ph.sync != 0;
  const GemmPlan g = gemm_plan(ph);
  if (g.idle) {  // whole workgroup
    if (barrier_seq) { barrier_arrive(bar, local_bar, barrier_seq); barrier_wait(bar, local_bar, barrier_seq); }
    if (stamp && blockIdx.x == 0 && threadIdx.x == 0) *stamp = wall_clock64();
    return;
  }
  const int kg = g.kg, s_begin = g.s_begin, ns = g.s_end - g.s_begin, epi = ph.epi;
  const int rot = g.rot;
  auto stage_of = [&](int i) { const int r = i + rot; return s_begin + (r >= ns ? r - ns : r); };  // i < ns

  const __amdgpu_buffer_rsrc_t rw = rsrc_of(ph.W, ph.w_bytes);
  const unsigned ldx = (unsigned)ph.ldx;  // (a local copy: the descriptor is memory the compiler would re-read)
  const int dbg = ph.dbg;                 // timing experiments only: 1 no MFMA, 2 no activation staging, 4 no weight loads
  const unsigned x_bytes = (unsigned)ph.M * ldx * 2u;
  const __amdgpu_buffer_rsrc_t rxh = rsrc_of(ph.Xhi, x_bytes), rxl = rsrc_of(ph.Xlo, x_bytes);
  const unsigned x_row0 = ((unsigned)(tid >> 5) * ldx + (unsigned)(tid & 31) * 8u) * 2u;  // byte offset of this thread's piece of row tid/32

  for (int p0 = g.b_begin; p0 < g.b_end; p0 += g.cb_per_pass) {
    unsigned wof[MG_NFW];
    int cbk[MG_NFW], gbk[MG_NFW];
    gemm_frags(ph, g, p0, uw, kp, lane, wof, cbk, gbk);
    WBuf w[MG_NBUF];
    f32x4 acc[MG_NFW][MT];
#pragma unroll
    for (int f = 0; f < MG_NFW; ++f)
#pragma unroll
      for (int mb = 0; mb < MT; ++mb) acc[f][mb] = (f32x4){0.f, 0.f, 0.f, 0.f};

    u32x4 xv[XIT];
    auto x_load = [&](int i) {  // i-th stage of this workgroup; past the end: out of range (zeros, no traffic)
      const int s = stage_of(i);
#pragma unroll
      for (int it = 0; it < XIT; ++it) {
        constexpr int HALF = XIT / 2;  // iterations per plane, 16 rows each
        const unsigned o = (i < ns && !(dbg & 2)) ? x_row0 + (unsigned)((it % HALF) * 16) * ldx * 2u + (unsigned)s * (MG_KST * 2u) : 0xFFFFFF00u;
        xv[it] = __builtin_amdgcn_raw_buffer_load_b128(it < HALF ? rxh : rxl, o, 0, 0);  // rows >= M: out of range -> 0
      }
    };
    auto x_store = [&](int b) {
      if (dbg & 2) return;
#pragma unroll
      for (int it = 0; it < XIT; ++it) {
        constexpr int HALF = XIT / 2;
        const int r = (it % HALF) * 16 + (tid >> 5), sl = tid & 31;
        *(u32x4*)(xs + b * BUF + (it / HALF) * PLANE + r * MG_LDK + sl * 8) = xv[it];
      }
    };
    auto compute = [&](const WBuf& wb, int b) {
      if (dbg & 1) return;
      const bf16_t* hi = xs + b * BUF + l16 * MG_LDK + g4 * 8 + kp * MG_CH * 32;
      const bf16_t* lo = hi + PLANE;
#pragma unroll
      for (int t = 0; t < MG_CH; ++t) {
#pragma unroll
        for (int mb = 0; mb < MT; ++mb) {
          Frag bh, bl;
          bh.u = *(const u32x4*)(hi + mb * 16 * MG_LDK + t * 32);
          bl.u = *(const u32x4*)(lo + mb * 16 * MG_LDK + t * 32);
#pragma unroll
          for (int f = 0; f < MG_NFW; ++f)
            acc[f][mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wb[f][t].v, bl.v, acc[f][mb], 0, 0, 0);
#pragma unroll
          for (int f = 0; f < MG_NFW; ++f)
            acc[f][mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wb[f][t].v, bh.v, acc[f][mb], 0, 0, 0);
        }
      }
    };

    // ---- prologue: the first MG_NPRE stages of weights, the previous phase's barrier (first pass), the
    // first activation stage ----
    const bool first = p0 == g.b_begin;
    if (first && barrier_seq) barrier_arrive(bar, local_bar, barrier_seq);  // (its store wait must not see the loads below)
#pragma unroll
    for (int i = 0; i < MG_NPRE; ++i) gemm_load_w(rw, wof, cbk, stage_of(i), i < ns && !(dbg & 4), w[i]);
    if (first) {
      if (barrier_seq) barrier_wait(bar, local_bar, barrier_seq);
      if (stamp && blockIdx.x == 0 && threadIdx.x == 0) *stamp = wall_clock64();
    }
    x_load(0);
    x_store(0);
    __syncthreads();

    // ---- stage s: request the activations of s + 1 and the weights of s + MG_NPRE, multiply stage s ----
    auto stage = [&](auto ic, int i) {
      constexpr int I = decltype(ic)::value;
      const int lb = i & 1;
      x_load(i + 1);
      gemm_load_w(rw, wof, cbk, stage_of(i + MG_NPRE), i + MG_NPRE < ns && !(dbg & 4), w[(I + MG_NPRE) % MG_NBUF]);
      __builtin_amdgcn_sched_barrier(0);
      compute(w[I], lb);
      __builtin_amdgcn_sched_barrier(0);
      x_store(lb ^ 1);
      __syncthreads();
    };
    for (int i = 0; i < ns; i += MG_NBUF) {
      stage(std::integral_constant<int, 0>{}, i);
      if (i + 1 < ns) stage(std::integral_constant<int, 1 % MG_NBUF>{}, i + 1);
      if (MG_NBUF > 2 && i + 2 < ns) stage(std::integral_constant<int, 2 % MG_NBUF>{}, i + 2);
    }
    // (the last stage's barrier also frees the stage buffers)

    // ---- add the k-parts: parts 1.. hand their accumulators to part 0 through LDS ----
    {
      f32x4* red = (f32x4*)xs;
      if (kp != 0) {
        f32x4* dst = red + (size_t)(uw * (MG_KW - 1) + kp - 1) * MG_NFW * MT * 64 + lane;
#pragma unroll
        for (int f = 0; f < MG_NFW; ++f)
#pragma unroll
          for (int mb = 0; mb < MT; ++mb) dst[(f * MT + mb) * 64] = acc[f][mb];
      }
      __syncthreads();
      if (kp == 0) {
#pragma unroll
        for (int q = 0; q < MG_KW - 1; ++q) {
          const f32x4* src = red + (size_t)(uw * (MG_KW - 1) + q) * MG_NFW * MT * 64 + lane;
#pragma unroll
          for (int f = 0; f < MG_NFW; ++f)
#pragma unroll
            for (int mb = 0; mb < MT; ++mb) acc[f][mb] += src[(f * MT + mb) * 64];
        }
      }
    }

    // ---- epilogue: lane holds rows mb*16 + l16, columns 4*g4.. of each fragment ----
    if (kp == 0) {
      if (epi == 0) {
        // shard 1: this XCD's private partial buffer, indexed by the XCD's local columns
        const WtBuf wy(ph.shard == 1 ? ph.lbuf + (size_t)(blockIdx.x & 7) * ph.lbuf_stride : ph.Y, ph.wt);
        const size_t ybase = (size_t)kg * ph.split_stride;
#pragma unroll
        for (int f = 0; f < MG_NFW; ++f) {
          if (cbk[f] < 0) continue;
          const int col = cbk[f] * 16 + 4 * g4;
#pragma unroll
          for (int mb = 0; mb < MT; ++mb) {
            const int m = mb * 16 + l16;
            if (m < ph.M) wy.st128((ybase + (size_t)m * ph.ldy + col) * 4, acc[f][mb]);
          }
        }
      } else {
        const WtBuf wh(ph.Yhi, ph.wt), wl(ph.Ylo, ph.wt);
#pragma unroll
        for (int mb = 0; mb < MT; ++mb) {
          const int m = mb * 16 + l16;
          if (m >= ph.M) continue;
          const float4 q = *(const float4*)(ph.ss + (size_t)m * 4);
          const float sc = 1.0f / sqrtf((q.x + q.y + q.z + q.w) / (float)ph.H + ph.eps);
          if (epi == 1) {
#pragma unroll
            for (int f = 0; f < MG_NFW; f += 2) {
              if (cbk[f] < 0) continue;
              const int col = gbk[f] * 16 + 4 * g4;
              float o[4];
#pragma unroll
              for (int r = 0; r < 4; ++r) {
                const float gt = acc[f][mb][r] * sc, u = acc[f + 1][mb][r] * sc;
                o[r] = gt / (1.0f + expf(-gt)) * u;
              }
              unsigned h0, l0, h1, l1;
              split2(o[0], o[1], h0, l0);
              split2(o[2], o[3], h1, l1);
              const u32x2 h = {h0, h1}, l = {l0, l1};
              wh.st64(((size_t)m * ph.ldo + col) * 2, h);
              wl.st64(((size_t)m * ph.ldo + col) * 2, l);
            }
          } else {
#pragma unroll
            for (int f = 0; f < MG_NFW; ++f) {
              if (cbk[f] < 0) continue;
              const int col = gbk[f] * 16 + 4 * g4;
              const f32x4 v = acc[f][mb] * sc;
              *(float4*)(ph.Y + (size_t)m * ph.ldy + col) = make_float4(v[0], v[1], v[2], v[3]);
            }
          }
        }
      }
    }
    __syncthreads();  // the reduction buffer is free before the next pass stages into it
  }
}

// ------------------------------------------------------------------------------------------
// Residual phase: x[g, :] (+)= sum_kg P[kg][g][:]  (or x = embedding row), planes of x * gain for the next
// GEMM (the RMSNorm scale is applied by that GEMM's consumer) and per-quarter sums of squares.
// Item = (row g, quarter q of the columns).
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ void reduce_phase(const MegaPhase& ph, const int tid, float* redbuf) {
  const int lane = tid & 63, wave = tid >> 6;
  const int H = ph.H, Q = H / 4;
  const int n_items = ph.M * 4;
  const WtBuf wx(ph.x, 1), wh(ph.Yhi, 1), wl(ph.Ylo, 1), wss(ph.ss_out, 1);  // read by every XCD
  for (int item = blockIdx.x; item < n_items; item += gridDim.x) {
    const int g = item >> 2, q = item & 3;
    float ssq = 0.f;
    for (int c0 = 2 * tid; c0 < Q; c0 += 2 * MG_NT) {
      const int c = q * Q + c0;
      float2 v;
      if (ph.tok) {
        int t = ph.tok[g];
        t = t < 0 ? 0 : (t >= ph.vocab ? ph.vocab - 1 : t);
        const unsigned e = *(const unsigned*)(ph.table + (size_t)t * H + c);
        v = make_float2(bf16_f32(e & 0xFFFFu), bf16_f32(e >> 16));
      } else {
        v = *(const float2*)(ph.x + (size_t)g * H + c);
      }
      float2 pp[8];
#pragma unroll
      for (int k = 0; k < 8; ++k)
        pp[k] = k < ph.KG ? *(const float2*)(ph.Y + (size_t)k * ph.split_stride + (size_t)g * ph.ldy + c) : make_float2(0.f, 0.f);
#pragma unroll
      for (int k = 0; k < 8; ++k) { v.x += pp[k].x; v.y += pp[k].y; }
      wx.st64(((size_t)g * H + c) * 4, __builtin_bit_cast(u32x2, v));
      ssq += v.x * v.x + v.y * v.y;
      if (ph.gain) {
        const unsigned gg = *(const unsigned*)(ph.gain + c);
        unsigned h, l;
        split2(v.x * bf16_f32(gg & 0xFFFFu), v.y * bf16_f32(gg >> 16), h, l);
        wh.st32(((size_t)g * ph.ldo + c) * 2, h);
        wl.st32(((size_t)g * ph.ldo + c) * 2, l);
      }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) ssq += __shfl_xor(ssq, o, 64);
    __syncthreads();  // redbuf free (previous item)
    if (lane == 0) redbuf[wave] = ssq;
    __syncthreads();
    if (tid == 0) {
      float t = 0.f;
#pragma unroll
      for (int w = 0; w < MG_WAVES; ++w) t += redbuf[w];
      wss.st32(((size_t)g * 4 + q) * 4, __float_as_uint(t));
    }
  }
}

// ------------------------------------------------------------------------------------------
// RoPE + KV write phase (head_dim 128): sums the QKV partials, applies the deferred RMSNorm scale,
// rotates q and k (pairs i, i + 64), writes Q as pre-scaled planes, K rows and V^T columns as planes.
// Wavefront items: (row, q or k head) with one rotation pair per lane, then (sequence, 8 V^T lines)
// with one tree node per lane.
// ------------------------------------------------------------------------------------------
// the heads this workgroup's XCD group handles in the RoPE / attention / merge phases, where the workgroup
// stands among the workgroups that share them, and the buffers the three phases hand results over in
struct HeadShare {
  int q0, nq, kv0, nkv;   // first / number of query heads and of KV heads
  int widx, nwork;        // index / number of the workgroups sharing these heads
  const float* qkv;       // QKV partials [KG][M][ldy]: columns = (nq q heads, nkv k heads, nkv v heads) x 128
  float *o_part, *ml_part;  // [split][rows_total][nq][128] and [split][rows_total][nq][2]
};
__device__ __forceinline__ HeadShare head_share(const MegaPhase& ph) {
  HeadShare h;
  if (ph.shard) {
    const int x = blockIdx.x & 7;
    h.nq = ph.n_q / 8; h.nkv = ph.n_kv / 8;
    h.q0 = x * h.nq; h.kv0 = x * h.nkv;
    h.widx = blockIdx.x >> 3; h.nwork = gridDim.x >> 3;
    float* base = ph.lbuf + (size_t)x * ph.lbuf_stride;
    h.qkv = base; h.o_part = base + ph.lo_off; h.ml_part = base + ph.lml_off;
  } else {
    h.nq = ph.n_q; h.nkv = ph.n_kv; h.q0 = 0; h.kv0 = 0;
    h.widx = blockIdx.x; h.nwork = gridDim.x;
    h.qkv = ph.Y; h.o_part = ph.o_part; h.ml_part = ph.ml_part;
  }
  return h;
}

__device__ __forceinline__ float row_scale(const float* ss, int g, int H, float eps) {
  const float4 q = *(const float4*)(ss + (size_t)g * 4);
  return 1.0f / sqrtf((q.x + q.y + q.z + q.w) / (float)H + eps);
}

__device__ __forceinline__ void rope_phase(const MegaPhase& ph, const int tid) {
  const int lane = tid & 63;
  const HeadShare hs = head_share(ph);
  const int gw = hs.widx * MG_WAVES + (tid >> 6), n_gw = hs.nwork * MG_WAVES;
  const RowMap rm = ph.rm;
  const int d = 128, half = 64, n_kv = ph.n_kv;
  const int heads = hs.nq + hs.nkv;
  const int qk_items = rm.B * rm.n * heads;
  const int v_chunks = hs.nkv * d / 8;
  const int n_items = qk_items + rm.B * v_chunks;
  const int voff = heads * d;
  const WtBuf wqh(ph.q_hi, ph.wt), wql(ph.q_lo, ph.wt), wk(ph.k_hi, ph.wt), wv(ph.v_hi, ph.wt);
  for (int item = gw; item < n_items; item += n_gw) {
    if (item < qk_items) {
      const int li = item % heads, bi = item / heads, i = bi % rm.n, b = bi / rm.n;
      const int nv = rm.n_valid ? min(rm.n_valid[b], rm.n) : rm.n;
      const int L = ph.base_len[b];
      if (L + nv > ph.max_seq) {
        if (lane == 0 && i == 0 && li == 0) atomicOr(ph.err_flag, 1);
        continue;
      }
      if (i >= nv) continue;
      const int g = b * rm.R + i;
      const float sc = row_scale(ph.ss, g, ph.H, ph.eps);
      const float* src = hs.qkv + (size_t)g * ph.ldy + li * d + lane;
      float a1[8], a2[8];
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        a1[k] = k < ph.KG ? src[(size_t)k * ph.split_stride] : 0.f;
        a2[k] = k < ph.KG ? src[(size_t)k * ph.split_stride + half] : 0.f;
      }
      float x1 = 0.f, x2 = 0.f;
#pragma unroll
      for (int k = 0; k < 8; ++k) { x1 += a1[k]; x2 += a2[k]; }
      x1 *= sc; x2 *= sc;
      const float c = ph.cos_t[(size_t)g * half + lane], sn = ph.sin_t[(size_t)g * half + lane];
      const bool is_q = li < hs.nq;  // wavefront-uniform
      const float qs = is_q ? ph.q_scale : 1.0f;  // queries are stored pre-scaled by 1/sqrt(d)
      const float o1 = (x1 * c - x2 * sn) * qs, o2 = (x2 * c + x1 * sn) * qs;
      const unsigned h1 = rn_bf16(o1), h2 = rn_bf16(o2);
      const unsigned l1 = rn_bf16(o1 - bf16_f32(h1)), l2 = rn_bf16(o2 - bf16_f32(h2));
      if (is_q) {
        const size_t o = ((size_t)g * ph.ldq + (hs.q0 + li) * d + lane) * 2;
        wqh.st16(o, h1); wqh.st16(o + half * 2, h2);
        wql.st16(o, l1); wql.st16(o + half * 2, l2);
      } else {
        const size_t o = ((((size_t)b * ph.max_seq + (L + i)) * n_kv + (hs.kv0 + li - hs.nq)) * d + lane) * 2;
        wk.st16(o, h1); wk.st16(o + half * 2, h2);
        wk.st16(o + ph.k_plane * 2, l1); wk.st16(o + ph.k_plane * 2 + half * 2, l2);
      }
    } else {
      const int vi = item - qk_items, b = vi / v_chunks, e0 = (vi % v_chunks) * 8;  // e0: first of 8 V^T lines of this share
      const int nv = rm.n_valid ? min(rm.n_valid[b], rm.n) : rm.n;
      const int L = ph.base_len[b];
      if (L + nv > ph.max_seq) continue;
      for (int i = lane; i < nv; i += 64) {
        const int g = b * rm.R + i;
        const float sc = row_scale(ph.ss, g, ph.H, ph.eps);
        const float* src = hs.qkv + (size_t)g * ph.ldy + voff + e0;
        float4 va = {0.f, 0.f, 0.f, 0.f}, vb = {0.f, 0.f, 0.f, 0.f};
        float4 p0[8], p1[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) {  // all K-group partials in one batch of loads
          const bool in = k < ph.KG;
          p0[k] = in ? *(const float4*)(src + (size_t)k * ph.split_stride) : make_float4(0.f, 0.f, 0.f, 0.f);
          p1[k] = in ? *(const float4*)(src + (size_t)k * ph.split_stride + 4) : make_float4(0.f, 0.f, 0.f, 0.f);
        }
#pragma unroll
        for (int k = 0; k < 8; ++k) {
          va.x += p0[k].x; va.y += p0[k].y; va.z += p0[k].z; va.w += p0[k].w;
          vb.x += p1[k].x; vb.y += p1[k].y; vb.z += p1[k].z; vb.w += p1[k].w;
        }
        const float v[8] = {va.x * sc, va.y * sc, va.z * sc, va.w * sc, vb.x * sc, vb.y * sc, vb.z * sc, vb.w * sc};
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const size_t o = ((((size_t)b * n_kv + hs.kv0) * d + e0 + e) * ph.max_seq + L + i) * 2;
          const unsigned h = rn_bf16(v[e]);
          wv.st16(o, h);
          wv.st16(o + ph.v_plane * 2, rn_bf16(v[e] - bf16_f32(h)));
        }
      }
    }
  }
}

// ------------------------------------------------------------------------------------------
// Tree attention phase (head_dim 128, caches as bf16 planes); see kernels_attn.hip for the MFMA
// mapping.  Item = (sequence, KV head, chunk of 8/G groups of 32 nodes, key split): wavefront w is
// query head w % G of node group w / G; all eight wavefronts stage the K and V^T tiles.
// ------------------------------------------------------------------------------------------
constexpr int AT_D = 128, AT_TK = 32, AT_MB = 2;
constexpr int MG_MAX_SPLITS = 16;  // key splits of the attention phase (the merge holds one partial row per split in registers)
constexpr int AT_KLD = AT_D + 8, AT_VLD = AT_TK + 8;
constexpr int AT_KPLANE = AT_TK * AT_KLD, AT_VPLANE = AT_D * AT_VLD;
constexpr int AT_BUF = 2 * AT_KPLANE + 2 * AT_VPLANE;

// key tiles per split: the cached length is only known on the device; at least two tiles per split so
// that short contexts do not pay for partial results nobody needs
__device__ __forceinline__ int attn_tiles_per_split(int n_tiles, int n_splits) {
  return max(2, (n_tiles + n_splits - 1) / n_splits);
}

template <int G>
__device__ __forceinline__ void attn_phase(const MegaPhase& ph, const int tid, bf16_t* sm) {
  constexpr int NGW = MG_WAVES / G;  // node groups a workgroup serves at once
  const int wave = tid >> 6, lane = tid & 63;
  const int l16 = lane & 15, g4 = lane >> 4;
  const RowMap rm = ph.rm;
  const HeadShare hs = head_share(ph);
  const int n_kv = ph.n_kv;
  const int node_groups = (rm.n + 31) / 32;
  const int chunks = (node_groups + NGW - 1) / NGW;
  const int n_items = rm.B * hs.nkv * chunks * ph.n_splits;
  for (int item = hs.widx; item < n_items; item += hs.nwork) {
    const int split = item % ph.n_splits;
    int r = item / ph.n_splits;
    const int ck = r % chunks; r /= chunks;
    const int kvh = hs.kv0 + r % hs.nkv, b = r / hs.nkv;
    const int nv = rm.n_valid ? min(rm.n_valid[b], rm.n) : rm.n;
    const int L = ph.base_len[b];
    if (ck * NGW * 32 >= nv || L + nv > ph.max_seq) continue;  // whole workgroup
    const int total = L + nv;
    const int n_tiles = (total + AT_TK - 1) / AT_TK;
    const int tps = attn_tiles_per_split(n_tiles, ph.n_splits);
    const int t0 = split * tps, t1 = min(n_tiles, t0 + tps);
    if (t0 >= n_tiles) continue;  // the merge reads the first ceil(n_tiles / tps) splits only
    const int head = kvh * G + wave % G;
    const int ng = ck * NGW + wave / G;
    const bool active = ng * 32 < nv;  // wavefront-uniform

    Frag qh[AT_MB][4], ql[AT_MB][4];
    unsigned long long a0[AT_MB], a1[AT_MB];
#pragma unroll
    for (int mb = 0; mb < AT_MB; ++mb) {
      const int node = ng * 32 + mb * 16 + l16;
      const bool ok = active && node < nv;
      a0[mb] = ok ? ph.anc[2 * node] : 0ull;
      a1[mb] = ok ? ph.anc[2 * node + 1] : 0ull;
      const size_t qo = ((size_t)b * rm.R + (ok ? node : 0)) * ph.ldq + head * AT_D + g4 * 8;
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        qh[mb][ks].u = (u32x4){0u, 0u, 0u, 0u};
        ql[mb][ks].u = (u32x4){0u, 0u, 0u, 0u};
        if (ok) {
          qh[mb][ks].u = *(const u32x4*)(ph.q_hi + qo + ks * 32);
          ql[mb][ks].u = *(const u32x4*)(ph.q_lo + qo + ks * 32);
        }
      }
    }
    f32x4 O[8][AT_MB];
#pragma unroll
    for (int db = 0; db < 8; ++db)
#pragma unroll
      for (int mb = 0; mb < AT_MB; ++mb) O[db][mb] = (f32x4){0.f, 0.f, 0.f, 0.f};
    float m_run[AT_MB], l_run[AT_MB];
#pragma unroll
    for (int mb = 0; mb < AT_MB; ++mb) { m_run[mb] = -INFINITY; l_run[mb] = 0.f; }

    constexpr int KIT = 2 * AT_TK * 16 / MG_NT, VIT = 2 * AT_D * 4 / MG_NT;  // 2 and 2
    constexpr int AT_PT = 2;  // tiles requested at once: their memory latencies overlap
    u32x4 kra[AT_PT][KIT], vra[AT_PT][VIT];
    const bf16_t* kbase = ph.k_hi + (size_t)b * ph.max_seq * n_kv * AT_D + (size_t)kvh * AT_D;
    const bf16_t* vbase = ph.v_hi + ((size_t)b * n_kv + kvh) * AT_D * ph.max_seq;
    auto load_tile = [&](u32x4 (&kr)[KIT], u32x4 (&vr)[VIT], int t) {
#pragma unroll
      for (int it = 0; it < KIT; ++it) {
        const int idx = it * MG_NT + tid, plane = idx >> 9, rem = idx & 511, key = rem >> 4, sl = rem & 15;
        const int jk = min(t * AT_TK + key, ph.max_seq - 1);
        kr[it] = *(const u32x4*)(kbase + plane * ph.k_plane + (size_t)jk * n_kv * AT_D + sl * 8);
      }
#pragma unroll
      for (int it = 0; it < VIT; ++it) {
        const int idx = it * MG_NT + tid, plane = idx >> 9, rem = idx & 511, dr = rem >> 2, sl = rem & 3;
        const int jv = min(t * AT_TK + sl * 8, ph.max_seq - 8);
        vr[it] = *(const u32x4*)(vbase + plane * ph.v_plane + (size_t)dr * ph.max_seq + jv);
      }
    };
    auto store_tile = [&](const u32x4 (&kr)[KIT], const u32x4 (&vr)[VIT], int buf) {
      bf16_t* base = sm + buf * AT_BUF;
#pragma unroll
      for (int it = 0; it < KIT; ++it) {
        const int idx = it * MG_NT + tid, plane = idx >> 9, rem = idx & 511, key = rem >> 4, sl = rem & 15;
        // key k of the tile is row ((k/4)%2)*16 + (k/8)*4 + k%4: sub-tile tt holds keys 8g + 4tt + r at row 4g + r
        const int row = ((key >> 2) & 1) * 16 + (key >> 3) * 4 + (key & 3);
        *(u32x4*)(base + plane * AT_KPLANE + row * AT_KLD + sl * 8) = kr[it];
      }
#pragma unroll
      for (int it = 0; it < VIT; ++it) {
        const int idx = it * MG_NT + tid, plane = idx >> 9, rem = idx & 511, dr = rem >> 2, sl = rem & 3;
        *(u32x4*)(base + 2 * AT_KPLANE + plane * AT_VPLANE + dr * AT_VLD + sl * 8) = vr[it];
      }
    };
    auto compute = [&](int buf, int t) {
      const bf16_t* kb = sm + buf * AT_BUF + l16 * AT_KLD + g4 * 8;
      const bf16_t* vb = sm + buf * AT_BUF + 2 * AT_KPLANE + l16 * AT_VLD + g4 * 8;
      f32x4 s[2][AT_MB];
#pragma unroll
      for (int tt = 0; tt < 2; ++tt)
#pragma unroll
        for (int mb = 0; mb < AT_MB; ++mb) s[tt][mb] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int tt = 0; tt < 2; ++tt)
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
          Frag kh, kl;
          kh.u = *(const u32x4*)(kb + tt * 16 * AT_KLD + ks * 32);
          kl.u = *(const u32x4*)(kb + AT_KPLANE + tt * 16 * AT_KLD + ks * 32);
#pragma unroll
          for (int mb = 0; mb < AT_MB; ++mb) {
            s[tt][mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kl.v, qh[mb][ks].v, s[tt][mb], 0, 0, 0);
            s[tt][mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kh.v, ql[mb][ks].v, s[tt][mb], 0, 0, 0);
            s[tt][mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kh.v, qh[mb][ks].v, s[tt][mb], 0, 0, 0);
          }
        }
      Frag phh[AT_MB], pll[AT_MB];
#pragma unroll
      for (int mb = 0; mb < AT_MB; ++mb) {
        float sv[8];
        float tmax = -INFINITY;
#pragma unroll
        for (int e = 0; e < 8; ++e) {  // e-th key of this lane: slot t*32 + 8*g4 + e
          const int jk = t * AT_TK + 8 * g4 + e;
          bool vis = jk < L;
          if (!vis && jk < total) {
            const int wn = jk - L;
            vis = ((wn < 64 ? (a0[mb] >> wn) : (a1[mb] >> (wn - 64))) & 1ull) != 0ull;
          }
          if (a0[mb] == 0ull && a1[mb] == 0ull) vis = false;  // padding row
          sv[e] = vis ? s[e >> 2][mb][e & 3] : -INFINITY;
          tmax = fmaxf(tmax, sv[e]);
        }
        tmax = fmaxf(tmax, __shfl_xor(tmax, 16, 64));
        tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
        const float m_new = fmaxf(m_run[mb], tmax);
        const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
        const float corr = __expf(m_run[mb] - m_safe);  // exp(-inf) = 0 on the first visible tile
        float pe[8], psum = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) { pe[e] = __expf(sv[e] - m_safe); psum += pe[e]; }
        l_run[mb] = l_run[mb] * corr + psum;
        m_run[mb] = m_new;
#pragma unroll
        for (int db = 0; db < 8; ++db) O[db][mb] *= corr;
        unsigned h, l;
        split2(pe[0], pe[1], h, l); phh[mb].u.x = h; pll[mb].u.x = l;
        split2(pe[2], pe[3], h, l); phh[mb].u.y = h; pll[mb].u.y = l;
        split2(pe[4], pe[5], h, l); phh[mb].u.z = h; pll[mb].u.z = l;
        split2(pe[6], pe[7], h, l); phh[mb].u.w = h; pll[mb].u.w = l;
      }
#pragma unroll
      for (int db = 0; db < 8; ++db) {
        Frag vh, vl;
        vh.u = *(const u32x4*)(vb + db * 16 * AT_VLD);
        vl.u = *(const u32x4*)(vb + AT_VPLANE + db * 16 * AT_VLD);
#pragma unroll
        for (int mb = 0; mb < AT_MB; ++mb) {
          O[db][mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vl.v, phh[mb].v, O[db][mb], 0, 0, 0);
          O[db][mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vh.v, pll[mb].v, O[db][mb], 0, 0, 0);
          O[db][mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vh.v, phh[mb].v, O[db][mb], 0, 0, 0);
        }
      }
    };

    __syncthreads();  // the previous item (or phase) no longer reads the tile buffers
    for (int g0 = t0; g0 < t1; g0 += AT_PT) {  // uniform over the workgroup
#pragma unroll
      for (int j = 0; j < AT_PT; ++j)
        if (g0 + j < t1) load_tile(kra[j], vra[j], g0 + j);
#pragma unroll
      for (int j = 0; j < AT_PT; ++j) {
        if (g0 + j < t1) {
          // tile j goes to buffer j & 1: whoever stores tile j + 2 there has passed the barrier of tile
          // j + 1, which every wavefront reaches only after it has finished with tile j
          store_tile(kra[j], vra[j], j & 1);
          __syncthreads();
          if (active) compute(j & 1, g0 + j);
        }
      }
      __syncthreads();  // (AT_PT is even: the next group starts in buffer 0 again)
    }

    // ---- partial result of this split (write-through: the merge phase runs in other workgroups) ----
    const WtBuf wo(hs.o_part, ph.wt), wml(hs.ml_part, ph.wt);
    if (active) {
#pragma unroll
      for (int mb = 0; mb < AT_MB; ++mb) {
        const int node = ng * 32 + mb * 16 + l16;
        float lsum = l_run[mb];
        lsum += __shfl_xor(lsum, 16, 64);
        lsum += __shfl_xor(lsum, 32, 64);
        if (node >= nv) continue;
        const size_t prow = ((size_t)split * ph.rows_total + (size_t)b * rm.R + node) * hs.nq + (head - hs.q0);
#pragma unroll
        for (int db = 0; db < 8; ++db) wo.st128((prow * AT_D + db * 16 + 4 * g4) * 4, O[db][mb]);
        if (g4 == 0) {
          const u32x2 ml = {__float_as_uint(m_run[mb]), __float_as_uint(lsum)};
          wml.st64(prow * 2 * 4, ml);
        }
      }
    }
  }
}

// merge the key splits of one (row, head): out = sum_s e^{m_s - M} O_s / sum_s e^{m_s - M} l_s, as planes.
// Item = (row, group of 16 heads); 32 threads per head, four channels each.
__device__ __forceinline__ void merge_phase(const MegaPhase& ph, const int tid) {
  const RowMap rm = ph.rm;
  const HeadShare hs = head_share(ph);
  const int hgroups = (hs.nq + 15) / 16;
  const int n_items = rm.B * rm.n * hgroups;
  const WtBuf wh(ph.Yhi, ph.wt), wl(ph.Ylo, ph.wt);
  for (int item = hs.widx; item < n_items; item += hs.nwork) {
    const int hg = item % hgroups, bi = item / hgroups, i = bi % rm.n, b = bi / rm.n;
    const int nv = rm.n_valid ? min(rm.n_valid[b], rm.n) : rm.n;
    const int hl = hg * 16 + (tid >> 5), d4 = (tid & 31) * 4;  // head within the share
    if (i >= nv || hl >= hs.nq || ph.base_len[b] + nv > ph.max_seq) continue;
    const int head = hs.q0 + hl;
    const size_t row = (size_t)b * rm.R + i;
    const size_t sstride = (size_t)ph.rows_total * hs.nq;
    const size_t pr0 = row * hs.nq + hl;
    const int n_tiles = (ph.base_len[b] + nv + AT_TK - 1) / AT_TK;
    const int tps = attn_tiles_per_split(n_tiles, ph.n_splits);
    const int ns = (n_tiles + tps - 1) / tps;  // splits that hold a result
    // every load of the item is issued before the first wait: one memory round trip, not one per split
    float2 ml[MG_MAX_SPLITS];
    float4 o[MG_MAX_SPLITS];
#pragma unroll
    for (int k = 0; k < MG_MAX_SPLITS; ++k) {
      const bool in = k < ns;
      ml[k] = in ? *(const float2*)(hs.ml_part + (pr0 + k * sstride) * 2) : make_float2(-INFINITY, 0.f);
      o[k] = in ? *(const float4*)(hs.o_part + (pr0 + k * sstride) * AT_D + d4) : make_float4(0.f, 0.f, 0.f, 0.f);
    }
    float M = -INFINITY;
#pragma unroll
    for (int k = 0; k < MG_MAX_SPLITS; ++k) M = fmaxf(M, ml[k].x);
    float4 num = make_float4(0.f, 0.f, 0.f, 0.f);
    float den = 0.f;
#pragma unroll
    for (int k = 0; k < MG_MAX_SPLITS; ++k) {  // split order
      const float wgt = ml[k].x == -INFINITY ? 0.f : __expf(ml[k].x - M);
      den += wgt * ml[k].y;
      num.x += wgt * o[k].x; num.y += wgt * o[k].y; num.z += wgt * o[k].z; num.w += wgt * o[k].w;
    }
    unsigned h0, l0, h1, l1;
    split2(num.x / den, num.y / den, h0, l0);
    split2(num.z / den, num.w / den, h1, l1);
    const u32x2 h = {h0, h1}, l = {l0, l1};
    wh.st64((row * ph.ldo + head * AT_D + d4) * 2, h);
    wl.st64((row * ph.ldo + head * AT_D + d4) * 2, l);
  }
}

constexpr size_t MG_LDS_BYTES = (size_t)2 * 2 * 64 * MG_LDK * sizeof(bf16_t);  // two GEMM stages of 64 rows (135168 B)
static_assert((size_t)2 * AT_BUF * sizeof(bf16_t) <= MG_LDS_BYTES, "attention tiles fit the GEMM stage buffers");
static_assert((size_t)MG_UW * (MG_KW - 1) * MG_NFW * 4 * 64 * 16 <= MG_LDS_BYTES, "k-part reduction fits");

// stamps (optional): wall-clock ticks at which workgroup 0 started phase p (stamps[p]) and left the last one
__global__ __launch_bounds__(MG_NT) void mega_kernel(const MegaPhase* __restrict__ prog, int p_begin, int p_end,
                                                     MegaSync* sync, unsigned gseq_base, unsigned lseq_base,
                                                     long long limit_ticks, int* err_flag, long long* stamps,
                                                     int check_xcd /* the program has a grid barrier */) {
  extern __shared__ __attribute__((aligned(16))) bf16_t lds[];
  __shared__ float redbuf[MG_WAVES];
  if (mg_aborted(sync)) return;  // a previous launch timed out in a barrier: the counters are not trustworthy
  // Workgroups i and i + 8 must share an XCD: (XCC id - workgroup index) mod 8 is then one value for the
  // whole grid.  Workgroup 0 publishes its own, tagged with this launch's barrier count; at the end (behind
  // at least one grid barrier) every workgroup compares.
  const unsigned xcc_off = (__builtin_amdgcn_s_getreg(20 | (0 << 6) | (3 << 11)) - blockIdx.x) & 7u;  // HW_REG_XCC_ID, 4 bits
  const unsigned xcc_tag = (gseq_base << 3);
  if (blockIdx.x == 0 && threadIdx.x == 0) __hip_atomic_store(&sync->off_tag, xcc_tag | xcc_off, __ATOMIC_RELAXED, MG_AGENT);
  Barrier bar{sync, limit_ticks, err_flag, false};
  for (int p = p_begin; p < p_end; ++p) {
    const MegaPhase& ph = prog[p];
    // barrier between phase p - 1 and phase p (a GEMM phase takes it itself, behind its first weight loads)
    const bool local = ph.sync != 0;
    const unsigned bseq = p > p_begin ? (local ? lseq_base : gseq_base) + (unsigned)ph.bar_ord : 0u;
    bar.no_inv = (ph.dbg & 8) != 0;
    if (bseq && ph.op != MG_OP_GEMM) {
      barrier_arrive(bar, local, bseq);
      barrier_wait(bar, local, bseq);
    }
    if (stamps && blockIdx.x == 0 && threadIdx.x == 0 && ph.op != MG_OP_GEMM) stamps[p] = wall_clock64();
    // The thread index enters every phase through a value the compiler cannot see through: otherwise
    // it hoists each phase's index arithmetic out of this loop and keeps (spills) all of it across
    // all the other phases, with reloads and full memory waits inside the GEMM pipeline.
    int zero;
    asm volatile("v_mov_b32 %0, 0" : "=v"(zero));
    const int tid = (int)threadIdx.x + zero;
    switch (ph.op) {
      case MG_OP_GEMM: gemm_phase<4>(ph, tid, lds, bar, bseq, stamps ? stamps + p : nullptr); break;
      case MG_OP_REDUCE: reduce_phase(ph, tid, redbuf); break;
      case MG_OP_ROPE: rope_phase(ph, tid); break;
      case MG_OP_ATTN:
        switch (ph.n_q / ph.n_kv) {
          case 1: attn_phase<1>(ph, tid, lds); break;
          case 2: attn_phase<2>(ph, tid, lds); break;
          case 4: attn_phase<4>(ph, tid, lds); break;
          default: attn_phase<8>(ph, tid, lds); break;
        }
        break;
      case MG_OP_MERGE: merge_phase(ph, tid); break;
      default: break;
    }
  }
  if (stamps && blockIdx.x == 0 && threadIdx.x == 0) stamps[p_end] = wall_clock64();
  if (check_xcd && threadIdx.x == 0) {
    const unsigned v = __hip_atomic_load(&sync->off_tag, __ATOMIC_RELAXED, MG_AGENT);
    if ((v & ~7u) == xcc_tag && (v & 7u) != xcc_off) atomicOr(err_flag, 4);
  }
}

}  // namespace

// ------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------
size_t mega_lds_bytes() { return MG_LDS_BYTES; }

// number of workgroups one cooperative launch may use on the current device (0: not available)
int mega_grid_size() {
  static int cached = -1;
  if (cached >= 0) return cached;
  cached = 0;
  if (getenv("CLOVER_NO_MEGA")) return cached;
  int dev = 0, coop = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess) return cached;
  if (hipDeviceGetAttribute(&coop, hipDeviceAttributeCooperativeLaunch, dev) != hipSuccess || !coop) return cached;
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return cached;
  if (hipFuncSetAttribute((const void*)mega_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)MG_LDS_BYTES) != hipSuccess) {
    (void)hipGetLastError();
    return cached;
  }
  int per_cu = 0;
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, (const void*)mega_kernel, MG_NT, MG_LDS_BYTES) != hipSuccess || per_cu < 1) {
    (void)hipGetLastError();
    return cached;
  }
  cus -= cus % 8;  // the K-group mapping assumes workgroup i runs on XCD i % 8
  cached = cus >= 8 ? cus : 0;
  return cached;
}

int mega_barrier_timeout_ticks(long long* out) {
  int dev = 0, khz = 0;
  if (hipGetDevice(&dev) != hipSuccess) return -1;
  if (hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev) != hipSuccess || khz <= 0) khz = 100000;
  *out = (long long)khz * 2000;  // 2 s: far beyond any phase, short enough to end a broken launch
  return 0;
}

hipError_t launch_mega(const MegaPhase* prog_dev, int p_begin, int p_end, MegaSync* sync, unsigned gseq_base,
                       unsigned lseq_base, long long limit_ticks, int* err_flag, long long* stamps, int check_xcd,
                       int grid, hipStream_t st) {
  void* args[] = {(void*)&prog_dev, (void*)&p_begin, (void*)&p_end, (void*)&sync, (void*)&gseq_base, (void*)&lseq_base,
                  (void*)&limit_ticks, (void*)&err_flag, (void*)&stamps, (void*)&check_xcd};
  return hipLaunchCooperativeKernel((const void*)mega_kernel, dim3(grid), dim3(MG_NT), args, (unsigned)MG_LDS_BYTES, st);
}

// largest power-of-two K-group count (<= 8) that leaves every group a stage and every workgroup at
// most one pass of column blocks where the width allows it
int mega_pick_kg(int N, int K, int epi, int grid) {
  if (epi != 0) return 1;
  const int NS = K / MG_KST, n_blocks = N / 16;
  int kg = 8;
  while (kg > 1 && kg > NS) kg >>= 1;
  // fewer K groups when the columns alone give every workgroup a near-full pass (halves the partial-sum traffic)
  while (kg > 1 && (long long)n_blocks * kg / 2 >= (long long)grid * (MG_PASS_BLOCKS - 2) && (long long)n_blocks * kg / 2 <= (long long)grid * MG_PASS_BLOCKS)
    kg >>= 1;
  return kg;
}

bool mega_gemm_supported(int M, int N, int K) { return M >= 1 && M <= 64 && K % MG_KST == 0 && N % 16 == 0 && K / 32 * (N / 16) < (1 << 22); }

}  // namespace clv
