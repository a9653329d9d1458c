// What this machine attains on the two resources the roofline is drawn from, measured with
// kernels that do nothing else: a streaming read with the superkernel's own load map, and a
// loop of bf16 MFMAs on registers.  bench.py reports the superkernel's rates against these as
// well as against the datasheet peaks.  Not part of the library's ABI: a measuring aid in a
// shared object of its own.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
#define SK_GLOBAL __attribute__((address_space(1)))

// Every wave walks along groups of 32 rows, one 128-byte step at a time: four load instructions
// per step, each covering eight rows with their full 128-byte lines (the weight-streaming map of
// the skinny tile classes), a ring of NB steps in flight.  Groups are visited in a scattered
// order so that neighbouring workgroups do not walk neighbouring memory.
template <int NB>
__global__ void __launch_bounds__(256, 2) stream_read(const char *p, size_t row_bytes, size_t rows, f32x4 *sink) {
  const int lane = threadIdx.x & 63;
  const size_t wave = (size_t)blockIdx.x * 4 + (threadIdx.x >> 6), nwaves = (size_t)gridDim.x * 4;
  const size_t ngroups = rows / 32;
  const int nstep = (int)(row_bytes / 128);
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  for (size_t g0 = wave; g0 < ngroups; g0 += nwaves) {
    const size_t g = (g0 * 7919u + 104729u) % ngroups;  // 7919 is prime: a permutation when it does not divide ngroups
    size_t off[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) off[j] = (g * 32 + j * 8 + lane / 8) * row_bytes + (lane % 8) * 16;
    u32x4 w[NB][4];
#pragma unroll
    for (int u = 0; u < NB - 1; ++u)
#pragma unroll
      for (int j = 0; j < 4; ++j)
        w[u][j] = __builtin_nontemporal_load((const u32x4 SK_GLOBAL *)(uintptr_t)(p + off[j] + (size_t)(u < nstep ? u : 0) * 128));
    for (int i0 = 0; i0 < nstep; i0 += NB) {
#pragma unroll
      for (int u = 0; u < NB; ++u) {
        const int i = i0 + u;
        int ahead = i + NB - 1;
        if (ahead >= nstep) ahead = 0;  // loads past the end re-read the first step; never summed
#pragma unroll
        for (int j = 0; j < 4; ++j)
          w[(u + NB - 1) % NB][j] =
              __builtin_nontemporal_load((const u32x4 SK_GLOBAL *)(uintptr_t)(p + off[j] + (size_t)ahead * 128));
        if (i < nstep) {
#pragma unroll
          for (int j = 0; j < 4; ++j) acc += __builtin_bit_cast(f32x4, w[u][j]);
        }
      }
    }
  }
  if (acc.x == 12345.678f) sink[wave] = acc;  // keeps the loads alive; practically never taken
}

// Four independent 32x32x16 bf16 accumulations per wave, `iters` rounds.
__global__ void __launch_bounds__(256, 2) mfma_loop(int iters, float seed, f32x4 *sink) {
  bf16x8 a, b;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    a[i] = (__bf16)(seed + (float)threadIdx.x * 1e-3f);
    b[i] = (__bf16)(seed - (float)i * 1e-3f);
  }
  f32x16 c0, c1, c2, c3;
#pragma unroll
  for (int i = 0; i < 16; ++i) c0[i] = c1[i] = c2[i] = c3[i] = 0.f;
  for (int it = 0; it < iters; ++it) {
    c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c0, 0, 0, 0);
    c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c1, 0, 0, 0);
    c2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c2, 0, 0, 0);
    c3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c3, 0, 0, 0);
  }
  const float s = c0[0] + c1[1] + c2[2] + c3[3];
  if (s == 12345.678f) sink[blockIdx.x] = f32x4{s, s, s, s};
}

// What the LDS delivers to the fragment reads of the LDS-tile class: every wave of two workgroups per CU
// reads 16 bytes per lane from the padded 144-byte rows the tiles use (lane l: row l % 32, piece l / 32 + 2 kk),
// `iters` rounds of eight reads, nothing else.
__global__ void __launch_bounds__(256, 2) lds_read_loop(int iters, f32x4 *sink) {
  __shared__ __attribute__((aligned(16))) unsigned char lds[256 * 144];
  for (int i = threadIdx.x; i < 256 * 144 / 16; i += 256) ((f32x4 *)lds)[i] = f32x4{1.f, 2.f, 3.f, 4.f};
  __syncthreads();
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const unsigned char *base = lds + ((wave * 64) + (lane & 31)) * 144 + (lane >> 5) * 16;
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      acc += *(const f32x4 *)(base + kk * 32);
      acc += *(const f32x4 *)(base + 32 * 144 + kk * 32);
    }
    asm volatile("" : "+v"(acc));
  }
  if (acc[0] == 12345.678f) sink[blockIdx.x] = acc;
}

// The stage loop of the LDS-tile class by itself, without anything of the superkernel around it: sixteen
// 2048 x 2048 x 2048 bf16 products (C = A . B^T, both K-contiguous) in 128 x 128 tiles that are handed out
// statically (workgroup b takes tiles b, b + grid, ...), operands by direct global-to-LDS loads into two
// swizzled stage images, fragments one step ahead of the 32x32x16 MFMAs, one barrier per stage.
// MODE 0: the whole loop.  1: no operand loads (fragment reads, MFMAs and the barrier: what LDS and the
// matrix cores allow).  2: operand loads and barrier only (what the path from the L2s to LDS allows).
__device__ __forceinline__ void tile_dma16(const void *gptr, uint32_t lds_addr) {
  // lane i's 16 bytes land at lds_addr + 16 i
  // (one idle cycle between the write of M0 and the load that reads it: the compiler does not
  // add wait states in front of inline assembly)
  asm volatile("s_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(gptr), "{m0}"(lds_addr) : "memory");
}
template <int MODE>
__global__ void __launch_bounds__(256, 2) tile_loop(const uint16_t *A, const uint16_t *B, uint16_t *Cout, int M, int N, int K,
                                                    int nb, int rounds) {
  constexpr int SLOT = 256 * 128;
  __shared__ __attribute__((aligned(16))) unsigned char lds[2 * SLOT];
  const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)lds;
  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
  const int wm = wave & 1, wn = wave >> 1, l32 = lane & 31, half = lane >> 5;
  const int c_log = (lane & 7) ^ (((wave & 1) << 2) | (lane >> 4));
  const int frag_off = l32 * 128, frag_pos = half ^ ((l32 >> 1) & 7);
  const int TM = M / 128, TN = N / 128;
  for (int it = 0; it < rounds; ++it) {
    const int t = blockIdx.x + it * gridDim.x;
    if (t >= nb * TM * TN) break;
    const int b = t / (TM * TN), r = t - b * TM * TN, m0 = (r / TN) * 128, n0 = (r % TN) * 128;
    const char *pa[4], *pb[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      pa[i] = (const char *)(A + ((size_t)b * M + m0 + 8 * (wave + 4 * i) + (lane >> 3)) * K + c_log * 8);
      pb[i] = (const char *)(B + ((size_t)b * N + n0 + 8 * (wave + 4 * i) + (lane >> 3)) * K + c_log * 8);
    }
    f32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 16; ++j) acc[i >> 1][i & 1][j] = 0.f;
    const int nst = K / 64;
    auto issue = [&](int k, int slot) {
      if (MODE == 1) return;
      const uint32_t dst = lds_base + slot * SLOT + wave * 1024;
#pragma unroll
      for (int i = 0; i < 4; ++i) tile_dma16(pa[i] + (size_t)k * 128, dst + 4096 * i);
#pragma unroll
      for (int i = 0; i < 4; ++i) tile_dma16(pb[i] + (size_t)k * 128, dst + 128 * 128 + 4096 * i);
    };
    issue(0, 0);
    for (int h = 0; h < nst; ++h) {
      const int slot = h & 1;
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      __builtin_amdgcn_s_barrier();
      asm volatile("" ::: "memory");
      if (h + 1 < nst) issue(h + 1, slot ^ 1);
      __builtin_amdgcn_sched_barrier(0);
      if (MODE != 2) {
        const unsigned char *la = lds + slot * SLOT + wm * 2 * 4096 + frag_off;
        const unsigned char *lb = lds + slot * SLOT + 128 * 128 + wn * 2 * 4096 + frag_off;
        u32x4 fa[2][2], fb[2][2];
        auto frag = [&](int kk, u32x4(&xa)[2], u32x4(&xb)[2]) {
          const int pos = (frag_pos ^ (2 * kk)) << 4;
          xa[0] = *(const u32x4 *)(la + pos), xa[1] = *(const u32x4 *)(la + 4096 + pos);
          xb[0] = *(const u32x4 *)(lb + pos), xb[1] = *(const u32x4 *)(lb + 4096 + pos);
        };
        frag(0, fa[0], fb[0]);
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
          if (kk + 1 < 4) frag(kk + 1, fa[(kk + 1) & 1], fb[(kk + 1) & 1]);
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int fn = 0; fn < 2; ++fn)
#pragma unroll
            for (int fm = 0; fm < 2; ++fm)
              acc[fn][fm] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fb[kk & 1][fn]),
                                                                    __builtin_bit_cast(bf16x8, fa[kk & 1][fm]), acc[fn][fm], 0, 0, 0);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
    }
    // one output per lane and accumulator block keeps the products alive (a measuring aid: C is not a full result)
    uint16_t *C = Cout + (size_t)b * M * N;
#pragma unroll
    for (int fm = 0; fm < 2; ++fm)
#pragma unroll
      for (int fn = 0; fn < 2; ++fn)
        C[(size_t)(m0 + (wm * 2 + fm) * 32 + l32) * N + n0 + (wn * 2 + fn) * 32 + 4 * half] =
            (uint16_t)(__builtin_bit_cast(uint32_t, acc[fn][fm][0]) >> 16);
    __syncthreads();
  }
}

int cu_count() {
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess) return 0;
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
  return cus;
}

}  // namespace

extern "C" {

// Reads `bytes` of device memory at `buf` as rows of `row_bytes` (a multiple of 128; bytes a
// multiple of 32 rows) `launches` times after one warm-up; *gb_per_s = bytes / mean launch time.
// `sink` is device memory of at least 2 * CUs * 4 * 16 bytes.  Returns 0 or a hipError_t.
int sk_ceiling_stream_read(const void *buf, uint64_t bytes, uint64_t row_bytes, int launches, void *sink,
                           double *gb_per_s) {
  const int cus = cu_count();
  if (!buf || !sink || !gb_per_s || cus <= 0 || row_bytes == 0 || row_bytes % 128 || bytes % (32 * row_bytes) ||
      launches < 1)
    return (int)hipErrorInvalidValue;
  hipEvent_t e0, e1;
  hipError_t e = hipEventCreate(&e0);
  if (e != hipSuccess) return (int)e;
  e = hipEventCreate(&e1);
  if (e != hipSuccess) return (int)e;
  const dim3 grid(2 * cus), block(256);
  const size_t rows = bytes / row_bytes;
  hipLaunchKernelGGL(stream_read<2>, grid, block, 0, 0, (const char *)buf, (size_t)row_bytes, rows, (f32x4 *)sink);
  (void)hipEventRecord(e0, 0);
  for (int i = 0; i < launches; ++i)
    hipLaunchKernelGGL(stream_read<2>, grid, block, 0, 0, (const char *)buf, (size_t)row_bytes, rows, (f32x4 *)sink);
  (void)hipEventRecord(e1, 0);
  e = hipEventSynchronize(e1);
  float ms = 0.f;
  if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (e != hipSuccess) return (int)e;
  *gb_per_s = (double)bytes * launches / (ms * 1e-3) / 1e9;
  return 0;
}

// *tflops of `iters` rounds of four 32x32x16 bf16 MFMAs in every wave of 2 workgroups per CU.
int sk_ceiling_mfma_bf16(int iters, void *sink, double *tflops) {
  const int cus = cu_count();
  if (!sink || !tflops || cus <= 0 || iters < 1) return (int)hipErrorInvalidValue;
  hipEvent_t e0, e1;
  hipError_t e = hipEventCreate(&e0);
  if (e != hipSuccess) return (int)e;
  e = hipEventCreate(&e1);
  if (e != hipSuccess) return (int)e;
  const dim3 grid(2 * cus), block(256);
  hipLaunchKernelGGL(mfma_loop, grid, block, 0, 0, iters, 0.5f, (f32x4 *)sink);
  (void)hipEventRecord(e0, 0);
  hipLaunchKernelGGL(mfma_loop, grid, block, 0, 0, iters, 0.5f, (f32x4 *)sink);
  (void)hipEventRecord(e1, 0);
  e = hipEventSynchronize(e1);
  float ms = 0.f;
  if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (e != hipSuccess) return (int)e;
  const double flops = (double)grid.x * 4.0 * iters * 4.0 * (2.0 * 32 * 32 * 16);
  *tflops = flops / (ms * 1e-3) / 1e12;
  return 0;
}

// *bytes_per_clk_per_cu and *gb_per_s of `iters` rounds of eight 16-byte-per-lane LDS reads in every wave of 2 workgroups
// per CU (the clock is the device's current shader clock as HIP reports it, in kHz).
int sk_ceiling_lds_read(int iters, void *sink, double *gb_per_s, double *bytes_per_clk_per_cu) {
  const int cus = cu_count();
  if (!sink || !gb_per_s || !bytes_per_clk_per_cu || cus <= 0 || iters < 1) return (int)hipErrorInvalidValue;
  int dev = 0, khz = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e == hipSuccess) e = hipDeviceGetAttribute(&khz, hipDeviceAttributeClockRate, dev);
  if (e != hipSuccess) return (int)e;
  hipEvent_t e0, e1;
  e = hipEventCreate(&e0);
  if (e != hipSuccess) return (int)e;
  e = hipEventCreate(&e1);
  if (e != hipSuccess) return (int)e;
  const dim3 grid(2 * cus), block(256);
  hipLaunchKernelGGL(lds_read_loop, grid, block, 0, 0, iters, (f32x4 *)sink);
  (void)hipEventRecord(e0, 0);
  hipLaunchKernelGGL(lds_read_loop, grid, block, 0, 0, iters, (f32x4 *)sink);
  (void)hipEventRecord(e1, 0);
  e = hipEventSynchronize(e1);
  float ms = 0.f;
  if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (e != hipSuccess) return (int)e;
  const double bytes = (double)grid.x * 256.0 * iters * 8.0 * 16.0;
  *gb_per_s = bytes / (ms * 1e-3) / 1e9;
  *bytes_per_clk_per_cu = bytes / cus / (ms * 1e-3) / ((double)khz * 1e3);
  return 0;
}

// *tflops the stage loop of the LDS-tile class reaches by itself on sixteen 2048-cubed bf16 products (see
// tile_loop; mode 0, 1 or 2; counted as if every mode did the products).  a, b: 16 * 2048 * 2048 bf16 each,
// c: the same size, all device memory owned by the caller.
int sk_ceiling_tile_loop(int mode, const void *a, const void *b, void *c, double *tflops) {
  const int cus = cu_count();
  if (!a || !b || !c || !tflops || cus <= 0 || mode < 0 || mode > 2) return (int)hipErrorInvalidValue;
  const int M = 2048, N = 2048, K = 2048, nb = 16;
  const dim3 grid(2 * cus), block(256);
  const int rounds = (nb * (M / 128) * (N / 128) + (int)grid.x - 1) / (int)grid.x;
  hipEvent_t e0, e1;
  hipError_t e = hipEventCreate(&e0);
  if (e != hipSuccess) return (int)e;
  e = hipEventCreate(&e1);
  if (e != hipSuccess) return (int)e;
  auto launch = [&]() {
    const uint16_t *pa = (const uint16_t *)a, *pb = (const uint16_t *)b;
    uint16_t *pc = (uint16_t *)c;
    if (mode == 0)
      hipLaunchKernelGGL(tile_loop<0>, grid, block, 0, 0, pa, pb, pc, M, N, K, nb, rounds);
    else if (mode == 1)
      hipLaunchKernelGGL(tile_loop<1>, grid, block, 0, 0, pa, pb, pc, M, N, K, nb, rounds);
    else
      hipLaunchKernelGGL(tile_loop<2>, grid, block, 0, 0, pa, pb, pc, M, N, K, nb, rounds);
  };
  launch();
  (void)hipEventRecord(e0, 0);
  for (int i = 0; i < 5; ++i) launch();
  (void)hipEventRecord(e1, 0);
  e = hipEventSynchronize(e1);
  float ms = 0.f;
  if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (e != hipSuccess) return (int)e;
  *tflops = 2.0 * nb * M * N * (double)K * 5 / (ms * 1e-3) / 1e12;
  return 0;
}

}  // extern "C"
