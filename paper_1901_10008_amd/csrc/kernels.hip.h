// Device code of the superkernel (gfx950 / CDNA4 only).
//
// One persistent kernel walks the flat tile table (Section 5.3 of the paper:
// many small kernels repacked into one large execution block).  Every tile
// belongs to one operator in its canonical GEMM view
//     C[Mg,Ng] = A'[Mg,Kg] . Bs[Ng,Kg]^T          (fp32 accumulate)
// with both operands K-contiguous, so a 16-byte piece of a row is at the same
// time one 128-bit load and one MFMA operand (8 halves or 4 floats of K).
//
// Three families of tile code:
//   * skinny (Mg <= 64): weights go HBM -> registers -> MFMA directly; the
//     weight rows are the MFMA's row operand and the few activation rows its
//     column operand, so a lane ends up with four consecutive output columns.
//     Activations are staged through LDS.  The four waves of a workgroup take
//     different 32-row weight groups; long reductions are split over several
//     workgroups whose partial sums the last one to finish adds in fixed order.
//   * LDS tiles (128x128, or 128x64 for operators with at most 64 output
//     columns): staged GEMM with 32x32 MFMAs; the operands go global -> LDS
//     directly (buffer loads with the LDS modifier into a ring of swizzled
//     stage images), through a ring of registers only where an operator is
//     out of reach of 32-bit offsets; the activation operand may be gathered
//     on the fly from an NHWC image (implicit GEMM for convolutions, any stride).
//   * operands that cannot be read in aligned 16-byte pieces, and convolutions
//     on channel-major (NCHW) arrays, whose patch rows and output rows are not
//     contiguous: one output per thread for small rectangles, MFMA tiles
//     assembled element by element for larger ones; only in the kernel
//     instantiation for plans that need them.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "sk_internal.h"

namespace sk {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));

// Operand pointers reach the kernel through descriptors in memory, so the compiler cannot
// see that they are global addresses; say so explicitly (global_load instead of flat_load).
#define SK_GLOBAL __attribute__((address_space(1)))
template <class T>
__device__ __forceinline__ const T SK_GLOBAL *as_global(const void *p) {
  return (const T SK_GLOBAL *)(uintptr_t)p;
}
template <class T>
__device__ __forceinline__ T SK_GLOBAL *as_global_mut(void *p) {
  return (T SK_GLOBAL *)(uintptr_t)p;
}

// A record that every lane reads from the same address, returned in scalar registers.
template <class S>
__device__ __forceinline__ S load_uniform(const S *src) {
  static_assert(sizeof(S) % 4 == 0, "whole dwords");
  struct Words {
    uint32_t w[sizeof(S) / 4];
  } v;
  const uint32_t SK_GLOBAL *p = as_global<uint32_t>(src);
#pragma unroll
  for (unsigned i = 0; i < sizeof(S) / 4; ++i) v.w[i] = (uint32_t)__builtin_amdgcn_readfirstlane((int)p[i]);
  return __builtin_bit_cast(S, v);
}

// The same from a copy in LDS.
template <class S>
__device__ __forceinline__ S unpack_uniform(const uint32_t *src) {
  struct Words {
    uint32_t w[sizeof(S) / 4];
  } v;
#pragma unroll
  for (unsigned i = 0; i < sizeof(S) / 4; ++i) v.w[i] = (uint32_t)__builtin_amdgcn_readfirstlane((int)src[i]);
  return __builtin_bit_cast(S, v);
}

constexpr int WORK_DWORDS = (int)(sizeof(TileWork) / 4);
static_assert(WORK_DWORDS <= 64, "one dword of the record per lane");

constexpr int WG_THREADS = 256;
constexpr int LDS_ROW = 144;                  // 128 bytes of K + 16 bytes of padding (bank spread)
constexpr int LDS_TILE_BYTES = 512 * LDS_ROW;  // 72 KB per workgroup: two workgroups share a CU's 160 KB

// Queue counters of a table: [0] tiles handed out beyond the first grid-full, [1] finished workgroups,
// [16 * (1 + x)] entries handed out from die x's list of LDS tiles (a 64-byte line each).
constexpr int QUEUE_COUNTERS = 16 * 9 + 1;
__device__ __forceinline__ uint32_t *die_list_head(uint32_t *counters, uint32_t x) { return counters + 16u * (1u + x); }

struct KernelArgs {
  uint32_t *counters;   // see QUEUE_COUNTERS
  const TileWork *xwork;  // the LDS tiles' records, die by die (null: tiles are run where their ticket falls)
  const uint32_t *xoff;   // [9] where die x's list starts in xwork
  uint32_t *remaining;  // per operator: tiles not yet retired (null = no stamps)
  uint64_t *stamps;     // [n] completion ticks, [n] = start tick
  uint32_t n_problems;
  uint32_t tile_begin, tile_end;
  uint32_t dynamic;      // 1: tiles come from the atomic counter; 0: static stride over the range
  uint32_t write_start;  // 1: every workgroup lowers the start tick to its own first clock
  f32x4 *ws;             // split-K partial sums
  const uint32_t *ws_off;
  uint32_t *arrive;
};

#ifdef SK_DIAG_CLOCKS
// Diagnostic build (-DSK_DIAG_CLOCKS, a library of its own: see build_diag in build.py and tile_phases.py): thread 0
// of the first SK_DIAG_WGS workgroups stamps the 100 MHz device clock at the phase boundaries of its first
// SK_DIAG_TILES tiles.  Slots per tile: 0 tile taken up, 1 set-up done (before the first operand loads), 2 first
// main-loop step multiplied, 3 main loop done, 4 outputs stored (and split-reduction hand-over done), 5 next
// record handed to all waves, 6 = 1 + tile class + 100 * reduction slices, 7 = the ticket (low half) and the
// flags it was handed over with.
// (first 16 workgroups, 64 tiles each; -DSK_DIAG_WGS_N=512 -DSK_DIAG_TILES_N=24 stamps every workgroup of a launch)
#ifndef SK_DIAG_WGS_N
#define SK_DIAG_WGS_N 16
#endif
#ifndef SK_DIAG_TILES_N
#define SK_DIAG_TILES_N 64
#endif
constexpr int SK_DIAG_WGS = SK_DIAG_WGS_N, SK_DIAG_TILES = SK_DIAG_TILES_N;
__device__ uint64_t g_diag[SK_DIAG_WGS * SK_DIAG_TILES * 8];
#define SK_DIAG(slot_)                                                               \
  do {                                                                               \
    if (blockIdx.x < SK_DIAG_WGS && diag_tile < SK_DIAG_TILES && threadIdx.x == 0)   \
      g_diag[(blockIdx.x * SK_DIAG_TILES + diag_tile) * 8 + (slot_)] = wall_clock64(); \
  } while (0)
#else
#define SK_DIAG(slot_) \
  do {                 \
  } while (0)
#endif

// ---------------------------------------------------------------------------
// element helpers
// ---------------------------------------------------------------------------
template <int DT>
struct Elem;
template <>
struct Elem<SK_F32> {
  static constexpr int ES = 4;
};
template <>
struct Elem<SK_BF16> {
  static constexpr int ES = 2;
};
template <>
struct Elem<SK_F16> {
  static constexpr int ES = 2;
};

__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
  __bf16 h = (__bf16)f;  // v_cvt_pk_bf16_f32: nearest, ties to even; NaN stays NaN
  return (uint32_t)__builtin_bit_cast(uint16_t, h);
}
// Two outputs packed into one dword (lower column in the low half).
template <int DT>
__device__ __forceinline__ uint32_t cvt_pack(float lo, float hi) {
  typedef float f32x2 __attribute__((ext_vector_type(2)));
  const f32x2 v = {lo, hi};
  if constexpr (DT == SK_BF16) {
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
  } else {
    typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, f16x2));
  }
}
__device__ __forceinline__ uint32_t f32_to_f16_bits(float f) {
  _Float16 h = (_Float16)f;  // v_cvt_f16_f32: nearest, ties to even
  return (uint32_t)__builtin_bit_cast(uint16_t, h);
}

template <int DT>
__device__ __forceinline__ uint32_t cvt_bits(float f) {
  if constexpr (DT == SK_BF16) return f32_to_bf16_bits(f);
  if constexpr (DT == SK_F16) return f32_to_f16_bits(f);
  return __builtin_bit_cast(uint32_t, f);
}

// Store four consecutive outputs of one row (columns n .. n+3, clipped to n_end).
template <int DT>
__device__ __forceinline__ void store4(void *C, int64_t row_off, int n, int n_end, f32x4 v, bool vec_ok) {
  constexpr int ES = Elem<DT>::ES;
  char SK_GLOBAL *p = as_global_mut<char>(C) + (row_off + n) * ES;
  if (vec_ok && n + 3 < n_end) {
    if constexpr (ES == 4) {
      *(f32x4 SK_GLOBAL *)p = v;
    } else {
      u32x2 o;
      o.x = cvt_pack<DT>(v.x, v.y);
      o.y = cvt_pack<DT>(v.z, v.w);
      *(u32x2 SK_GLOBAL *)p = o;
    }
  } else {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      if (n + i < n_end) {
        if constexpr (ES == 4)
          ((float SK_GLOBAL *)p)[i] = v[i];
        else
          ((uint16_t SK_GLOBAL *)p)[i] = (uint16_t)cvt_bits<DT>(v[i]);
      }
    }
  }
}

template <int ES, bool NT>
__device__ __forceinline__ u32x4 load_piece_vec(const void *base, int64_t off) {
  const u32x4 SK_GLOBAL *p = (const u32x4 SK_GLOBAL *)(as_global<char>(base) + off * ES);
  if constexpr (NT)
    return __builtin_nontemporal_load(p);
  else
    return *p;
}

// The MFMA paths below require both operands to be readable in aligned 16-byte
// pieces (FLAG_VEC_A and FLAG_VEC_B: 16-byte aligned bases and row strides, Kg
// and, for a convolution, Cin multiples of a piece).  Everything else goes
// through run_generic.

// Loads in the MFMA paths are never placed under a branch (a conditional load makes the
// compiler wait for it at the end of the branch, which serialises the loads of a stage)
// and their values are not touched before they are consumed (a select right behind a
// load makes the wave wait for it at once).  So a piece that must read as zero (beyond K,
// in a convolution's padding, rows past Mg, idle slots of a ring) is not masked after the
// load: its address is replaced by that of a piece of zeros in device memory.

// Weight piece: row n of Bs[Ng,Kg], elements k .. k+CE-1; where !ok (beyond K, idle slots of the
// ring) a piece of zeros is read instead, so that a weight row that holds an infinity does
// not meet 0 * inf there.
__device__ __attribute__((aligned(16))) const uint32_t g_zero_piece[4] = {0u, 0u, 0u, 0u};
// Its address in vector registers.  (Given the symbol itself, the compiler selects between the two
// places with a branch and a load in either arm, and then waits for every load in flight.)
__device__ __forceinline__ uintptr_t zero_piece_address() {
  uintptr_t z = (uintptr_t)g_zero_piece;
  asm volatile("" : "+v"(z));
  return z;
}
template <int ES, bool NT>
__device__ __forceinline__ u32x4 fetch_B(const DevProblem &P, int64_t row_off, int k, bool ok, uintptr_t zeros) {
  const uintptr_t p = (uintptr_t)P.B + (uintptr_t)((row_off + k) * ES);
  const u32x4 SK_GLOBAL *q = (const u32x4 SK_GLOBAL *)(ok ? p : zeros);
  if constexpr (NT)
    return __builtin_nontemporal_load(q);
  else
    return *q;
}

// n / d with d given as multiplier and shift (FastDiv), 0 <= n < 2^31.
__device__ __forceinline__ int fast_div(int n, const uint32_t (&d)[2]) {
  return (int)(uint32_t)(((uint64_t)(uint32_t)n * d[0]) >> d[1]);
}

// Where row m of the activation operand starts.
struct RowA {
  int64_t base;  // plain: m*lda.  gather: offset of pixel (b, hb, wb), channel 0, the one under filter tap (0,0); may be negative
  int hb, wb;    // gather: ho*stride-pad_h, wo*stride-pad_w
};

__device__ __forceinline__ RowA row_of(const DevProblem &P, int m) {
  RowA r;
  if (!P.gather) {
    r.base = (int64_t)m * P.lda;
    r.hb = 0;
    r.wb = 0;
  } else {
    const int hw = P.Ho * P.Wo;
    const int b = fast_div(m, P.div_hw);
    const int rem = m - b * hw;
    const int ho = fast_div(rem, P.div_wo);
    const int wo = rem - ho * P.Wo;
    r.hb = ho * P.stride - P.pad_h;
    r.wb = wo * P.stride - P.pad_w;
    if (P.nchw)
      r.base = ((int64_t)b * P.Cin * P.H + r.hb) * P.W + r.wb;  // pixel (b, channel 0, hb, wb)
    else
      r.base = (((int64_t)b * P.H + r.hb) * P.W + r.wb) * P.Cin;
  }
  return r;
}

// Channel-major convolutions (element-wise paths only).  Element strides of the image along
// filter row, filter column and channel, and where output (m, n) lives in Y[Nb,Cout,Ho,Wo].
struct ImageStrides {
  int64_t sh, sw, sc;
};
__device__ __forceinline__ ImageStrides image_strides(const DevProblem &P) {
  if (P.nchw) return ImageStrides{(int64_t)P.W, 1, (int64_t)P.H * P.W};
  return ImageStrides{(int64_t)P.W * P.Cin, (int64_t)P.Cin, 1};
}
__device__ __forceinline__ int64_t nchw_out_base(const DevProblem &P, int m) {
  const int hw = P.Ho * P.Wo;
  const int b = fast_div(m, P.div_hw);
  return (int64_t)b * P.Ng * hw + (m - b * hw);  // + n * Ho*Wo
}
template <int DT>
__device__ __forceinline__ void store_elem(void *C, int64_t off, float v) {
  char SK_GLOBAL *c = as_global_mut<char>(C) + off * Elem<DT>::ES;
  if constexpr (DT == SK_F32)
    *(float SK_GLOBAL *)c = v;
  else
    *(uint16_t SK_GLOBAL *)c = (uint16_t)cvt_bits<DT>(v);
}

// Element k of the implicit patch row: k = (r*S + s)*Cin + c  ->  pixel (hb+r, wb+s), channel c.
__device__ __forceinline__ bool patch_offset(const DevProblem &P, const RowA &row, int k, int64_t &off) {
  const int tap = fast_div(k, P.div_cin);
  const int c = k - tap * P.Cin;
  const int r = fast_div(tap, P.div_s);
  const int s = tap - r * P.S;
  const int h = row.hb + r, w = row.wb + s;
  off = row.base + ((int64_t)r * P.W + s) * P.Cin + c;
  return (unsigned)h < (unsigned)P.H && (unsigned)w < (unsigned)P.W;
}

// Activation piece: elements k .. k+CE-1 of row `row` of A'.  Where the piece must read as
// zero (`ok` false on entry, or the tap falls into the padding) the piece of zeros is loaded.
template <int ES>
__device__ __forceinline__ u32x4 fetch_A(const DevProblem &P, const RowA &row, int k, bool ok, uintptr_t zeros) {
  int64_t off = row.base + k;
  if (P.gather) ok = patch_offset(P, row, k, off) && ok;
  const uintptr_t p = (uintptr_t)P.A + (uintptr_t)(off * ES);
  return *(const u32x4 SK_GLOBAL *)(ok ? p : zeros);
}

// Single elements as float, for run_generic.
template <int DT>
__device__ __forceinline__ float load_elem(const void *base, int64_t off) {
  if constexpr (DT == SK_F32) {
    return as_global<float>(base)[off];
  } else if constexpr (DT == SK_BF16) {
    return __builtin_bit_cast(float, (uint32_t)as_global<uint16_t>(base)[off] << 16);
  } else {
    return (float)as_global<_Float16>(base)[off];
  }
}

// ---------------------------------------------------------------------------
// MFMA wrappers: one 16-byte piece per lane and operand.
// 16x16: lane l gives row/column l%16 and K-slot l/16.  32x32: l%32 and l/32.
// The two operands use the same lane -> K-slot map, so which K elements a
// slot really holds does not matter as long as both operands agree.
// ---------------------------------------------------------------------------
template <int DT>
__device__ __forceinline__ void mma16(const u32x4 &a, const u32x4 &b, f32x4 &c) {
  if constexpr (DT == SK_BF16) {
    c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0,
                                                0);
  } else if constexpr (DT == SK_F16) {
    c = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
  } else {
    // (whole-vector casts: a bit cast applied to a single vector element reads element 0)
    const f32x4 af = __builtin_bit_cast(f32x4, a), bf = __builtin_bit_cast(f32x4, b);
#pragma unroll
    for (int j = 0; j < 4; ++j) c = __builtin_amdgcn_mfma_f32_16x16x4f32(af[j], bf[j], c, 0, 0, 0);
  }
}

template <int DT>
__device__ __forceinline__ void mma32(const u32x4 &a, const u32x4 &b, f32x16 &c) {
  if constexpr (DT == SK_BF16) {
    c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0,
                                                0);
  } else if constexpr (DT == SK_F16) {
    c = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
  } else {
    const f32x4 af = __builtin_bit_cast(f32x4, a), bf = __builtin_bit_cast(f32x4, b);
#pragma unroll
    for (int j = 0; j < 4; ++j) c = __builtin_amdgcn_mfma_f32_32x32x2f32(af[j], bf[j], c, 0, 0, 0);
  }
}

// ---------------------------------------------------------------------------
// skinny tiles
// ---------------------------------------------------------------------------
// A tile is all Mg (<= 16*RM) activation rows against n_len weight rows and a
// slice [k0, k0+k_len) of the reduction.  The four waves of the workgroup take
// different groups of 32 weight rows (two 16-row MFMA blocks per wave).
//
// Weights never touch LDS: each wave streams its rows HBM -> registers -> MFMA
// through a ring of NB reduction blocks (128 bytes per row each), so NB-1
// blocks of loads stay in flight while one is multiplied, and every wave walks
// along its rows in consecutive 128-byte steps.
//
// The activations (tiny, and gathered from an image for a convolution) are
// staged once per workgroup through LDS in chunks of SKINNY_CHUNK_BYTES,
// double-buffered, one barrier per chunk.
//
// Long reductions are cut into S slices that different workgroups take
// (records with S > 1).  Each slice leaves its fp32 partial sums in a
// workspace in register layout; the workgroup that arrives last adds the S
// partials in slice order (so the result does not depend on arrival order)
// and writes C.
// (8 KB = 4 / 2 / 1 blocks of K per chunk for 1 / 2 / 4 row blocks.  Measured against 16 and 32 KB
// the smaller chunk is faster for every class: fewer staging loads queued between the weight
// loads, less padding of short reductions to whole chunks.)
constexpr int SKINNY_CHUNK_BYTES = 8192;

constexpr int ilog2(int x) { return x <= 1 ? 0 : 1 + ilog2(x >> 1); }

// Two registers loaded with the full-line map hold, for a 16-row MFMA block,
//   first : lanes r16 < 8 -> (row r16, pieces 0..3)      lanes r16 >= 8 -> (row r16-8, pieces 4..7)
//   second: lanes r16 < 8 -> (row r16+8, pieces 0..3)    lanes r16 >= 8 -> (row r16,   pieces 4..7)
// fix_lo gives (row r16, pieces 0..3) in every lane, fix_hi (row r16, pieces 4..7): the halves
// that are in the wrong place come from the other register, rotated by 8 lanes within each row
// of 16 (DPP row_ror:8, written only to the upper resp. lower 8 lanes through the bank mask).
__device__ __forceinline__ u32x4 fix_lo(const u32x4 &first, const u32x4 &second) {
  u32x4 r;
#pragma unroll
  for (int i = 0; i < 4; ++i)
    r[i] = (uint32_t)__builtin_amdgcn_update_dpp((int)first[i], (int)second[i], 0x128, 0xF, 0xC, false);
  return r;
}
__device__ __forceinline__ u32x4 fix_hi(const u32x4 &first, const u32x4 &second) {
  u32x4 r;
#pragma unroll
  for (int i = 0; i < 4; ++i)
    r[i] = (uint32_t)__builtin_amdgcn_update_dpp((int)second[i], (int)first[i], 0x128, 0xF, 0x3, false);
  return r;
}

// One accumulator (16 bytes per lane, 1 KB per wave) written / read at device scope (through
// to memory, not left in or served from an XCD's L2) as two 64-bit relaxed atomics per lane.
// The 1 KB block holds the low halves of all 64 lanes first, then the high halves, so that
// each of the two instructions covers 512 contiguous bytes: a write-through of scattered
// 8-byte pieces would cost a partial-line memory write each.
__device__ __forceinline__ void store_device_scope(f32x4 *block, int lane, const f32x4 &v) {
  unsigned long long *q = (unsigned long long *)block;
  __hip_atomic_store(q + lane, __builtin_bit_cast(unsigned long long, __builtin_shufflevector(v, v, 0, 1)),
                     __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  __hip_atomic_store(q + 64 + lane, __builtin_bit_cast(unsigned long long, __builtin_shufflevector(v, v, 2, 3)),
                     __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ f32x4 load_device_scope(const f32x4 *block, int lane) {
  typedef float f32x2 __attribute__((ext_vector_type(2)));
  unsigned long long *q = (unsigned long long *)block;
  const f32x2 lo = __builtin_bit_cast(f32x2, __hip_atomic_load(q + lane, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
  const f32x2 hi =
      __builtin_bit_cast(f32x2, __hip_atomic_load(q + 64 + lane, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
  return f32x4{lo.x, lo.y, hi.x, hi.y};
}

// Memory order of the arrival count that hands split-reduction partials from one workgroup to another.
// The partials themselves are written and read with device-scope accesses that go through to memory
// (see store_device_scope), each wave waits for its own stores to complete (s_waitcnt) and the workgroup
// meets at a barrier before one thread counts it in, so on this hardware a relaxed count suffices.  The
// language memory model asks for release/acquire on the count as well; that variant is
// kept compilable (-DSK_SPLITK_ACQ_REL) and costs a write-back and an invalidate of the XCD's L2 per slice.
#ifdef SK_SPLITK_ACQ_REL
#define SK_ARRIVE_ORDER __ATOMIC_ACQ_REL
#else
#define SK_ARRIVE_ORDER __ATOMIC_RELAXED
#endif
#if defined(__HIP_DEVICE_COMPILE__) && !defined(__gfx950__)
#error "the split-reduction hand-over relies on gfx950's write-through device-scope stores"
#endif

struct SplitK {
  f32x4 *ws;                // partial sums of all split output rectangles
  const uint32_t *ws_off;   // per out_tile_id: offset of its partials in ws, in f32x4 units
  uint32_t *arrive;         // per out_tile_id: slices that have delivered (re-armed by the last one)
};

// The workgroup's next tile: claimed from the queue and its work record fetched while the
// current tile is still streaming, in two steps that each tile class places in its main loop.
//   claim(): thread 0 takes the next index from the queue (an atomic whose answer takes a
//     memory round trip).  Late in the tile, not at its start: a claimed tile cannot start
//     before its workgroup is free, so at the end of the launch tiles claimed early would
//     wait behind long tiles while other workgroups sit idle.
//   issue(): once the answer is there, lane i < WORK_DWORDS of every wave loads dword i of the
//     record (one register per lane).  Only wave 0 has the real index, and only its copy is
//     used.
// CLAIM_LEAD / ISSUE_GAP are counted in steps of the class's main loop (a step is one to two
// microseconds when the memory system is loaded).
struct Prefetch {
  const TileWork *work;
  uint32_t *counter;  // the queue (null: tiles are not handed out by the queue)
  uint32_t base;      // index of the first tile the queue hands out (0 when there is no queue)
  uint32_t next;      // next tile's index minus `base`; meaningful in lane 0 of wave 0 (in all lanes when there
                      // is no queue).  The queue's answer is left untouched until issue() needs it: anything
                      // computed from it at once would make the wave wait for the atomic, and with it for
                      // every load in flight.
  uint32_t last;      // last valid index of the launch
  int tid;            // this tile's copy of the thread index (see the tile loop)
  uint32_t word = 0;
  // An LDS tile is run by the die whose list holds it (see the tile loop).  While such a tile runs, the
  // workgroup also draws the next entry of its die's list (xhead not null), on the guess that its next
  // ticket falls on an LDS tile again: thread 1 draws beside thread 0 in the same atomic instruction, and
  // the one load of issue() brings the record of that entry (lanes below WORK_DWORDS) and, in lane 63, the
  // dword of the ticket's own record that holds its tile class.  (One atomic and one load as without
  // lists: with two of either in flight the compiler waits, in every step of the LDS-tile loops, until
  // one load at most is outstanding, which also counts the operand loads it does not see.)
  uint32_t *xhead = nullptr;
  const TileWork *xrec = nullptr;  // first record of the die's list
  uint32_t xlen = 0;               // its length (> 0 whenever xhead is set)
#ifdef SK_DIAG_CLOCKS
  int diag_tile = 0;
#endif
  __device__ __forceinline__ void claim() {
    // (lanes other than threads 0 and 1 keep whatever `next` held: it is never used, and any
    // instruction that touched the register here would have to wait for an earlier answer)
    if (counter && tid < (xhead ? 2 : 1)) next = atomicAdd(tid == 0 ? counter : xhead, 1u);
  }
  __device__ __forceinline__ void issue() {
    uint32_t idx = (uint32_t)__builtin_amdgcn_readfirstlane((int)next) + base;
    if (idx > last) idx = last;  // past the end of the table: the workgroup is about to leave
    const int lane = tid & 63;
    const uint32_t SK_GLOBAL *src = as_global<uint32_t>(work + idx) + (lane < WORK_DWORDS ? lane : 0);
    if (xhead) {
      uint32_t k = (uint32_t)__builtin_amdgcn_readlane((int)next, 1);
      if (k >= xlen) k = xlen - 1u;  // the list is used up
      src = lane == 63 ? as_global<uint32_t>(work + idx) + 1 : as_global<uint32_t>(xrec + k) + (lane < WORK_DWORDS ? lane : 0);
    }
    word = *src;
  }
  // step `i` of `total` main-loop steps
  __device__ __forceinline__ void at_step(int i, int total, int lead, int gap) {
    const int claim_at = total > lead ? total - lead : 0;
    const int issue_at = claim_at + gap < total ? claim_at + gap : total - 1;
    if (i == claim_at) claim();
    if (i == issue_at) issue();
  }
};
constexpr int CLAIM_LEAD = 8, ISSUE_GAP = 4;

template <int DT, int RM>
__device__ __forceinline__ void run_skinny(const DevProblem &P, const sk_tile &T, const SplitK &sp,
                                           unsigned char *lds, uint32_t *s_flag, Prefetch &pf) {
  constexpr int ES = Elem<DT>::ES;
  constexpr int CE = 16 / ES;
  constexpr int KB = 8 * CE;                        // reduction elements per block (128 bytes)
  constexpr int ROWS = 16 * RM;                     // activation rows held in LDS
  constexpr int CHUNK_BYTES = SKINNY_CHUNK_BYTES;
  constexpr int ROWB = CHUNK_BYTES / ROWS;          // bytes of K per row and chunk
  constexpr int LROW = ROWB + 16;                   // padded LDS row (bank spread)
  constexpr int BPC_LOG2 = ilog2(ROWB / 128);
  constexpr int BPC = 1 << BPC_LOG2;                // blocks per chunk: 4, 2, 1
  constexpr int PPR = ROWB / 16;                    // pieces per row and chunk
  constexpr int BUF = ROWS * LROW;                  // bytes per LDS buffer
  constexpr int NB = 2;                             // ring slots: one block in flight while one is multiplied.
  // (With every workgroup streaming, the memory system is saturated by far fewer bytes in flight
  // than the launch holds even at this depth; deeper rings only lengthen every load's wait.)
  static_assert(ROWB == BPC * 128, "chunk geometry");
  static_assert(2 * BUF <= LDS_TILE_BYTES, "activation chunks do not fit");

  const int tid = pf.tid;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform: keeps its branches scalar
  const int lane = tid & 63;
  const int r16 = lane & 15, q = lane >> 4;

  const int n_end = (int)T.n0 + (int)T.n_len;
  const int ngroups = ((int)T.n_len + 31) >> 5;
  const int iters = (ngroups + 3) >> 2;

  const int k0 = (int)T.k0, k_stop = (int)T.k0 + (int)T.k_len;
  const int nblocks = ((int)T.k_len + KB - 1) / KB;
  const int nchunks = (nblocks + BPC - 1) >> BPC_LOG2;
  const int nslots = nchunks << BPC_LOG2;  // block slots per wave (blocks past the end read as zero)

  const uintptr_t zeros = zero_piece_address();
  // staging map: thread -> SPT consecutive pieces of one activation row
  constexpr int SPT = CHUNK_BYTES / (WG_THREADS * 16);
  constexpr int TPR = PPR / SPT;  // threads per row
  const int s_row = tid / TPR;
  const int s_piece = (tid % TPR) * SPT;
  const bool s_ok = s_row < P.Mg;
  const RowA srow = row_of(P, s_ok ? s_row : 0);
  const int s_lds = s_row * LROW + s_piece * 16;
  u32x4 ar[SPT];
  // For a convolution: filter tap (g_r, g_s) and channel g_c of this thread's first piece in the
  // chunk that stage_load will fetch next, and g_off = ((g_r*W + g_s)*Cin + g_c), its distance in
  // elements from the pixel under tap (0,0).  Chunks are fetched in order (0, 1, ..., then 0 again
  // for the next pass), so the position moves on by additions; the divisions happen once per tile.
  int g_r = 0, g_s = 0, g_c = 0;
  int64_t g_off = 0;
  const int64_t next_filter_row = (int64_t)(P.W - P.S) * P.Cin;
  if (P.gather) {
    const int kk = k0 + s_piece * CE;
    const int tap = fast_div(kk, P.div_cin);
    g_c = kk - tap * P.Cin;
    g_r = fast_div(tap, P.div_s);
    g_s = tap - g_r * P.S;
    g_off = ((int64_t)g_r * P.W + g_s) * P.Cin + g_c;
  }
  const int g_r0 = g_r, g_s0 = g_s, g_c0 = g_c;
  const int64_t g_off0 = g_off;
  auto stage_load = [&](int c) {
    const int k = k0 + ((c << BPC_LOG2) * 8 + s_piece) * CE;
    if (!P.gather) {
#pragma unroll
      for (int i = 0; i < SPT; ++i) ar[i] = fetch_A<ES>(P, srow, k + i * CE, s_ok && k + i * CE < k_stop, zeros);
      return;
    }
    if (c == 0) {
      g_r = g_r0;
      g_s = g_s0;
      g_c = g_c0;
      g_off = g_off0;
    }
    // the thread's pieces follow one another in the patch row (a piece never straddles two taps:
    // Cin is a multiple of a piece); no branch between the loads
    int r = g_r, t = g_s, cc = g_c;
    int64_t off = g_off;
#pragma unroll
    for (int i = 0; i < SPT; ++i) {
      const bool ok = s_ok && k + i * CE < k_stop && (unsigned)(srow.hb + r) < (unsigned)P.H &&
                      (unsigned)(srow.wb + t) < (unsigned)P.W;
      const uintptr_t pa = (uintptr_t)P.A + (uintptr_t)((srow.base + off) * ES);
      ar[i] = *(const u32x4 SK_GLOBAL *)(ok ? pa : zeros);
      cc += CE;
      off += CE;
      const bool next_tap = cc >= P.Cin;
      cc -= next_tap ? P.Cin : 0;
      t += next_tap ? 1 : 0;
      const bool next_row = t == P.S;  // (only ever true right after a step to the next tap)
      t = next_row ? 0 : t;
      r += next_row ? 1 : 0;
      off += next_row ? next_filter_row : 0;
    }
    // on to the next chunk
    constexpr int KC = BPC * 8 * CE;
    g_c += KC;
    g_off += KC;
    while (g_c >= P.Cin) {
      g_c -= P.Cin;
      if (++g_s == P.S) {
        g_s = 0;
        ++g_r;
        g_off += next_filter_row;
      }
    }
  };
  auto stage_store = [&](int c) {
    unsigned char *base = lds + (c & 1) * BUF + s_lds;
#pragma unroll
    for (int i = 0; i < SPT; ++i) *(u32x4 *)(base + i * 16) = ar[i];
  };

  const bool vec_c = (P.flags & FLAG_VEC_C) != 0;
  const bool restage_each = nchunks > 1;

  // A wave's work is one stream of block slots: pass 0 (its first weight group) blocks
  // 0..nslots-1, then pass 1, ...  The weight loads run NB-1 slots ahead of the MFMAs and
  // keep running across pass boundaries, so the ring only drains at the end of the tile.
  // --- load stream (ahead) ---
  int p_it = 0, p_blk = 0;
  bool p_act = false;
  // Load map: instruction j of a block covers rows 8j..8j+7 of the 32-row group with their full
  // 128-byte lines: lane (r16, q) reads row 8j + r16%8, piece q + 4*(r16/8).  (Eight whole lines
  // per instruction stream measurably better than sixteen half lines.)  The MFMA wants row
  // r16 in lane r16 with pieces 0..3 resp. 4..7 in slot q; two DPP half-row swaps per pair of
  // registers put the data there when the block is consumed (see fix_lo / fix_hi).
  const int piece = q + 4 * (r16 >> 3);
  int64_t wrow[4] = {0, 0, 0, 0};
  auto set_load_rows = [&](int it) {
    const int g = it * 4 + wave;
    p_act = it < iters && g < ngroups;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int n = (int)T.n0 + g * 32 + j * 8 + (r16 & 7);
      if (n >= n_end) n = n_end - 1;  // rows past the edge repeat the last row; never stored
      wrow[j] = p_act ? (int64_t)n * P.ldb : 0;
    }
  };
  // The loads are unconditional (see fetch_B): slots past the end re-read the start of a row, and
  // slots that no pass will multiply (past the end of the tile, waves without a group) all read
  // the very first piece of the operand, so that the number of loads in flight at every point
  // of the loop is the same on every path and the waits stay exact.
  auto next_load = [&](u32x4(&w)[4]) {
    const int k = k0 + p_blk * KB + piece * CE;
    const bool in = p_act && k < k_stop;
#pragma unroll
    for (int j = 0; j < 4; ++j) w[j] = fetch_B<ES, true>(P, wrow[j], k, in, zeros);
    if (++p_blk == nslots) {
      p_blk = 0;
      ++p_it;
      set_load_rows(p_it);
    }
  };
  // --- compute stream ---
  int it = 0, blk = 0, buf = 1;
  f32x4 acc[2][RM];
#pragma unroll
  for (int rb = 0; rb < 2; ++rb)
#pragma unroll
    for (int mb = 0; mb < RM; ++mb) acc[rb][mb] = f32x4{0.f, 0.f, 0.f, 0.f};
  auto store_pass = [&]() {
    // lane holds, per (rb, mb): row m = mb*16 + lane%16, columns n_base + rb*16 + (lane/16)*4 + 0..3
    const int g = it * 4 + wave;
    const int n_base = (int)T.n0 + g * 32;
    if (g < ngroups) {
#pragma unroll
      for (int mb = 0; mb < RM; ++mb) {
        const int m = mb * 16 + r16;
        if (m < P.Mg) {
          const int64_t row_off = (int64_t)m * P.ldc;
#pragma unroll
          for (int rb = 0; rb < 2; ++rb) {
            const int n = n_base + rb * 16 + q * 4;
            if (n < n_end) store4<DT>(P.C, row_off, n, n_end, acc[rb][mb], vec_c);
          }
        }
      }
    }
  };

#ifdef SK_DIAG_CLOCKS
  const int diag_tile = pf.diag_tile;
#endif
  SK_DIAG(1);
  set_load_rows(0);
  stage_load(0);
  u32x4 w[NB][4];
#pragma unroll
  for (int u = 0; u < NB - 1; ++u) next_load(w[u]);
  if (!restage_each) {
    // the only activation chunk serves every pass
    stage_store(0);
    buf = 0;
    __syncthreads();
  }

  const int total = iters * nslots;
  for (int i0 = 0; i0 < total; i0 += NB) {
#pragma unroll
    for (int u = 0; u < NB; ++u) {
      const bool live = i0 + u < total;
      pf.at_step(i0 + u, total, CLAIM_LEAD, ISSUE_GAP);
      if (live && restage_each && (blk & (BPC - 1)) == 0) {
        // first block of a chunk: publish it, then start fetching the one after it
        // (chunk c+1 of this pass, or chunk 0 again for the next pass)
        buf ^= 1;
        stage_store(buf);
        __syncthreads();
        const int c_next = (blk >> BPC_LOG2) + 1;
        if (c_next < nchunks)
          stage_load(c_next);
        else if (it + 1 < iters)
          stage_load(0);
      }
      next_load(w[(u + NB - 1) % NB]);
      if (live) {
        if (it * 4 + wave < ngroups) {
          const unsigned char *abase = lds + buf * BUF + (blk & (BPC - 1)) * 128 + q * 16 + r16 * LROW;
          // All activation pieces of the block are requested from LDS first, each into registers
          // of its own (read one row block at a time into the same registers, every read would
          // wait for the MFMAs of the row block before it), and before the weights are touched:
          // the LDS round trip then overlaps the wait for the weight block.
          u32x4 a0[RM], a1[RM];
#pragma unroll
          for (int mb = 0; mb < RM; ++mb) {
            a0[mb] = *(const u32x4 *)(abase + mb * 16 * LROW);       // pieces 0..3
            a1[mb] = *(const u32x4 *)(abase + mb * 16 * LROW + 64);  // pieces 4..7
          }
          __builtin_amdgcn_sched_barrier(0);  // (the scheduler would sink the reads back to their uses)
          // rows 16rb..16rb+15: pieces 0..3 (x) and 4..7 (y) in MFMA lane order
          const u32x4 x0 = fix_lo(w[u][0], w[u][1]), y0 = fix_hi(w[u][0], w[u][1]);
          const u32x4 x1 = fix_lo(w[u][2], w[u][3]), y1 = fix_hi(w[u][2], w[u][3]);
#pragma unroll
          for (int mb = 0; mb < RM; ++mb) {
            mma16<DT>(x0, a0[mb], acc[0][mb]);
            mma16<DT>(x1, a0[mb], acc[1][mb]);
            mma16<DT>(y0, a1[mb], acc[0][mb]);
            mma16<DT>(y1, a1[mb], acc[1][mb]);
          }
        }
        if (i0 + u == 0) SK_DIAG(2);
        if (++blk == nslots && it + 1 < iters) {
          // this weight group is done; the next one's loads are already in flight
          store_pass();
#pragma unroll
          for (int rb = 0; rb < 2; ++rb)
#pragma unroll
            for (int mb = 0; mb < RM; ++mb) acc[rb][mb] = f32x4{0.f, 0.f, 0.f, 0.f};
          blk = 0;
          ++it;
        }
      }
    }
  }

  SK_DIAG(3);
  // last pass (the only one of a split rectangle, which has at most four weight groups)
  bool finish = true;
  if (T.S > 1) {
    // Deliver this slice's partial sums; the last slice to arrive adds all of them in slice
    // order.  The partials are written and read with device-scope accesses (they go through
    // to memory, past the per-XCD L2s), so no cache-wide release/acquire is needed: each wave
    // waits for its own stores, the workgroup meets at a barrier, one thread counts it in.
    f32x4 *mine = sp.ws + sp.ws_off[T.out_tile_id];
    const int slot = (wave * 2 * RM) * 64;  // this wave's 2*RM blocks of 64 x 16 bytes within a slice
#pragma unroll
    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
      for (int mb = 0; mb < RM; ++mb)
        store_device_scope(mine + (size_t)T.ks_idx * (4 * 2 * RM * 64) + slot + (rb * RM + mb) * 64, lane,
                           acc[rb][mb]);
    __builtin_amdgcn_s_waitcnt(0);  // all counters to zero: the stores above have completed
    __syncthreads();
    if (tid == 0)
      *s_flag = __hip_atomic_fetch_add(&sp.arrive[T.out_tile_id], 1u, SK_ARRIVE_ORDER, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    const uint32_t prev = *s_flag;
    finish = prev == (uint32_t)T.S - 1;
    if (finish) {
#pragma unroll
      for (int rb = 0; rb < 2; ++rb)
#pragma unroll
        for (int mb = 0; mb < RM; ++mb) acc[rb][mb] = f32x4{0.f, 0.f, 0.f, 0.f};
      // All partial sums of a slice are requested before the first is added, and those of the next AHEAD - 1
      // slices while this one's are added (left to the scheduler the loads went out two at a time, each pair
      // waited for: eight memory round trips per slice, which made an operator cut into dozens of slices
      // several times slower).  The sums are still taken in slice order.
      constexpr int AHEAD = 2;  // slices in flight (four or eight for the classes with fewer rows: measured, no gain)
      f32x4 part[AHEAD][2][RM];
      auto request = [&](int s2, f32x4(&dst)[2][RM]) {
#pragma unroll
        for (int rb = 0; rb < 2; ++rb)
#pragma unroll
          for (int mb = 0; mb < RM; ++mb)
            dst[rb][mb] = load_device_scope(mine + (size_t)s2 * (4 * 2 * RM * 64) + slot + (rb * RM + mb) * 64, lane);
      };
      const int S = (int)T.S;
#pragma unroll
      for (int u = 0; u < AHEAD - 1; ++u)
        if (u < S) request(u, part[u]);
      for (int s0 = 0; s0 < S; s0 += AHEAD) {
#pragma unroll
        for (int u = 0; u < AHEAD; ++u) {
          const int s2 = s0 + u;
          if (s2 + AHEAD - 1 < S) request(s2 + AHEAD - 1, part[(u + AHEAD - 1) % AHEAD]);
          __builtin_amdgcn_sched_barrier(0);
          if (s2 < S) {
#pragma unroll
            for (int rb = 0; rb < 2; ++rb)
#pragma unroll
              for (int mb = 0; mb < RM; ++mb) acc[rb][mb] += part[u][rb][mb];
          }
          __builtin_amdgcn_sched_barrier(0);
        }
      }
      if (tid == 0)  // re-arm for the next launch
        __hip_atomic_store(&sp.arrive[T.out_tile_id], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
  if (finish) store_pass();
  SK_DIAG(4);
}

// A slice of a split reduction hands its partial sums over; true in the workgroup that arrived last, with the
// sum of all slices (in slice order) in `acc`; false in the others, which have nothing left to do.
template <int FM, int FN>
__device__ __forceinline__ bool split_handover(const sk_tile &T, const SplitK &sp, uint32_t *s_flag, int tid,
                                               f32x16 (&acc)[FN][FM]) {
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lane = tid & 63;

    // A slice of a split reduction: same hand-over as in the skinny classes.  Partial sums go to
    // the workspace in register layout with device-scope stores (a slice is FN*FM*4 blocks of
    // 64 x 16 bytes per wave); the last slice to arrive adds all of them in slice order.
    constexpr int PER_WAVE = FN * FM * 4;          // 1 KB blocks per wave and slice
    constexpr int PER_SLICE = 4 * PER_WAVE * 64;   // f32x4 units per slice
    f32x4 *mine = sp.ws + sp.ws_off[T.out_tile_id] + wave * PER_WAVE * 64;
#pragma unroll
    for (int fn = 0; fn < FN; ++fn)
#pragma unroll
      for (int fm = 0; fm < FM; ++fm)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const f32x4 v = {acc[fn][fm][4 * j], acc[fn][fm][4 * j + 1], acc[fn][fm][4 * j + 2], acc[fn][fm][4 * j + 3]};
          store_device_scope(mine + (size_t)T.ks_idx * PER_SLICE + ((fn * FM + fm) * 4 + j) * 64, lane, v);
        }
    __builtin_amdgcn_s_waitcnt(0);  // all counters to zero: the stores above have completed
    __syncthreads();
    if (tid == 0)
      *s_flag = __hip_atomic_fetch_add(&sp.arrive[T.out_tile_id], 1u, SK_ARRIVE_ORDER, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    if (*s_flag != (uint32_t)T.S - 1) return false;
#pragma unroll
    for (int fn = 0; fn < FN; ++fn)
#pragma unroll
      for (int fm = 0; fm < FM; ++fm)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[fn][fm][i] = 0.f;
    // (all partial sums of a slice are requested before the first is added: see run_skinny)
    for (int s2 = 0; s2 < T.S; ++s2) {
      f32x4 part[FN][FM][4];
#pragma unroll
      for (int fn = 0; fn < FN; ++fn)
#pragma unroll
        for (int fm = 0; fm < FM; ++fm)
#pragma unroll
          for (int j = 0; j < 4; ++j)
            part[fn][fm][j] = load_device_scope(mine + (size_t)s2 * PER_SLICE + ((fn * FM + fm) * 4 + j) * 64, lane);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int fn = 0; fn < FN; ++fn)
#pragma unroll
        for (int fm = 0; fm < FM; ++fm)
#pragma unroll
          for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[fn][fm][4 * j + e] += part[fn][fm][j][e];
      __builtin_amdgcn_sched_barrier(0);
    }
    if (tid == 0)  // re-arm for the next launch
      __hip_atomic_store(&sp.arrive[T.out_tile_id], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return true;
}

// What follows the main loop of an LDS tile: the hand-over of a split reduction and the stores.
// lane holds, per (fn, fm): row l32 of the 32x32 block, columns 8*(i/4) + 4*half + (i%4).
template <int DT, int BM, int BN, int WAVES_M, int WAVES_N>
__device__ __forceinline__ void finish_tile(const DevProblem &P, const sk_tile &T, const SplitK &sp, unsigned char *lds,
                                            uint32_t *s_flag, int tid,
                                            f32x16 (&acc)[BN / (32 * WAVES_N)][BM / (32 * WAVES_M)]) {
  constexpr int ES = Elem<DT>::ES;
  constexpr int CE = 16 / ES;
  constexpr int FM = BM / (32 * WAVES_M);
  constexpr int FN = BN / (32 * WAVES_N);
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lane = tid & 63;
  const int wm = wave % WAVES_M, wn = wave / WAVES_M;
  const int l32 = lane & 31, half = lane >> 5;
  const int m0 = (int)T.m0, n0 = (int)T.n0;
  const int m_end = m0 + (int)T.m_len, n_end = n0 + (int)T.n_len;
  if (T.S > 1 && !split_handover<FM, FN>(T, sp, s_flag, tid, acc)) return;

  // lane holds, per (fn, fm): row m = l32, columns 8*(i/4) + 4*half + (i%4)
  //
  // Written from the accumulators a store instruction would cover 32 rows with 16 bytes each.
  // Where C allows 16-byte stores the tile goes through LDS instead (free by now: every wave has
  // passed the last stage's barrier) and leaves as whole rows: 16 lanes x 16 bytes side by side.
  constexpr int OROW = BN * ES + 16;  // padded row of the output tile in LDS
  static_assert(BM * OROW <= LDS_TILE_BYTES, "output tile does not fit the LDS buffer");
  const bool wide = ((uintptr_t)P.C % 16 == 0) && ((P.ldc * ES) % 16 == 0);
  if (wide) {
#pragma unroll
    for (int fm = 0; fm < FM; ++fm) {
      const int r = (wm * FM + fm) * 32 + l32;
#pragma unroll
      for (int fn = 0; fn < FN; ++fn) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int c = (wn * FN + fn) * 32 + 8 * j + 4 * half;
          unsigned char *q = lds + r * OROW + c * ES;
          if constexpr (ES == 4) {
            *(f32x4 *)q = f32x4{acc[fn][fm][4 * j], acc[fn][fm][4 * j + 1], acc[fn][fm][4 * j + 2], acc[fn][fm][4 * j + 3]};
          } else {
            u32x2 o;
            o.x = cvt_pack<DT>(acc[fn][fm][4 * j], acc[fn][fm][4 * j + 1]);
            o.y = cvt_pack<DT>(acc[fn][fm][4 * j + 2], acc[fn][fm][4 * j + 3]);
            *(u32x2 *)q = o;
          }
        }
      }
    }
    __syncthreads();
    constexpr int PIECES = BN * ES / 16;             // 16-byte pieces per output row
    constexpr int RPI = WG_THREADS / PIECES;         // rows per store instruction
    const int pc = tid % PIECES, pr = tid / PIECES;
    const int n = n0 + pc * CE;
#pragma unroll
    for (int i = 0; i < BM / RPI; ++i) {
      const int r = pr + i * RPI;
      const int m = m0 + r;
      if (m < m_end && n < n_end) {
        const u32x4 v = *(const u32x4 *)(lds + r * OROW + pc * 16);
        char SK_GLOBAL *dst = as_global_mut<char>(P.C) + ((int64_t)m * P.ldc + n) * ES;
        if (n + CE <= n_end) {
          *(u32x4 SK_GLOBAL *)dst = v;
        } else {
          // ragged right edge: element by element
#pragma unroll
          for (int e = 0; e < CE; ++e) {
            if (n + e < n_end) {
              if constexpr (ES == 4)
                ((uint32_t SK_GLOBAL *)dst)[e] = v[e];
              else
                ((uint16_t SK_GLOBAL *)dst)[e] = (uint16_t)(v[e / 2] >> (16 * (e & 1)));
            }
          }
        }
      }
    }
    // (the barrier at the end of every tile keeps the next tile's LDS writes behind these reads)
    return;
  }
  const bool vec_c = (P.flags & FLAG_VEC_C) != 0;
#pragma unroll
  for (int fm = 0; fm < FM; ++fm) {
    const int m = m0 + (wm * FM + fm) * 32 + l32;
    if (m < m_end) {
      const int64_t row_off = (int64_t)m * P.ldc;
#pragma unroll
      for (int fn = 0; fn < FN; ++fn) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int n = n0 + (wn * FN + fn) * 32 + 8 * j + 4 * half;
          if (n < n_end) {
            f32x4 v = {acc[fn][fm][4 * j], acc[fn][fm][4 * j + 1], acc[fn][fm][4 * j + 2], acc[fn][fm][4 * j + 3]};
            store4<DT>(P.C, row_off, n, n_end, v, vec_c);
          }
        }
      }
    }
  }
}

// ---------------------------------------------------------------------------
// LDS-staged tiles: BM x BN outputs per workgroup, 128 bytes of K per stage
// ---------------------------------------------------------------------------
// Operand pieces travel global memory -> registers -> LDS -> MFMA.  A ring of NS register
// stages keeps NS-1 stages of loads in flight.  LDS holds two stages: while the MFMAs of
// stage s read one buffer, the pieces of stage s+1 are written to the other, and one barrier
// per stage separates "everyone has written s+1 and finished reading s" from the next round.
//
// A stage costs a wave its whole instruction stream (address arithmetic, LDS traffic, MFMAs,
// barrier) back to back, so that stream is kept short: operand row pointers are formed once
// per tile, and the position in the implicit patch matrix (filter tap r,s and channel c of
// this thread's piece) advances by additions only -- no multiply or divide per stage.
template <int DT, int BM, int BN, int WAVES_M, int WAVES_N>
__device__ __forceinline__ void run_tile(const DevProblem &P, const sk_tile &T, const SplitK &sp, unsigned char *lds,
                                         uint32_t *s_flag, Prefetch &pf) {
  constexpr int ES = Elem<DT>::ES;
  constexpr int CE = 16 / ES;
  constexpr int KB = 8 * CE;                  // reduction elements per stage
  constexpr int FM = BM / (32 * WAVES_M);     // 32x32 blocks per wave along m
  constexpr int FN = BN / (32 * WAVES_N);     // ... along n
  constexpr int A_ITERS = BM / 32;            // 16-byte pieces per thread per stage, activations
  constexpr int B_ITERS = BN / 32;            // ... weights
  constexpr int STAGE = (BM + BN) * LDS_ROW;  // bytes of one stage in LDS
  constexpr int NS = 3;
  static_assert(WAVES_M * WAVES_N == 4, "four waves per workgroup");
  static_assert(2 * STAGE <= LDS_TILE_BYTES, "two stages do not fit the LDS buffer");

  const int tid = pf.tid;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lane = tid & 63;
  const int wm = wave % WAVES_M, wn = wave / WAVES_M;
  const int l32 = lane & 31, half = lane >> 5;

  const int m0 = (int)T.m0, n0 = (int)T.n0;
  const int m_end = m0 + (int)T.m_len, n_end = n0 + (int)T.n_len;
  const int k_begin = (int)T.k0, k_stop = (int)T.k0 + (int)T.k_len;

  // staging map: thread -> piece c8 of rows (tid/8) + 32*i
  const int c8 = tid & 7;
  const int srow = tid >> 3;
  const bool gvec = P.gather != 0;
  const char SK_GLOBAL *pa[A_ITERS];  // row start (for a convolution: the pixel under filter tap (0,0), may lie outside the image)
  int hb[A_ITERS], wb[A_ITERS];
#pragma unroll
  for (int i = 0; i < A_ITERS; ++i) {
    int m = m0 + srow + 32 * i;
    if (m >= m_end) m = m_end - 1;  // rows past the edge repeat the last row; never stored
    const RowA r = row_of(P, m);
    pa[i] = as_global<char>(P.A) + r.base * ES;
    hb[i] = r.hb;
    wb[i] = r.wb;
  }
  const char SK_GLOBAL *pb[B_ITERS];
#pragma unroll
  for (int i = 0; i < B_ITERS; ++i) {
    int n = n0 + srow + 32 * i;
    if (n >= n_end) n = n_end - 1;
    pb[i] = as_global<char>(P.B) + (int64_t)n * P.ldb * ES;
  }

  f32x16 acc[FN][FM];
#pragma unroll
  for (int fn = 0; fn < FN; ++fn)
#pragma unroll
    for (int fm = 0; fm < FM; ++fm)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[fn][fm][i] = 0.f;

  // position of this thread's piece in the patch row: tap (g_r, g_s), channel g_c;
  // tap_off = ((g_r*W + g_s)*Cin + g_c) elements from the pixel under tap (0,0)
  int g_r = 0, g_s = 0, g_c = 0;
  int64_t tap_off = 0;
  const int64_t next_filter_row = (int64_t)(P.W - P.S) * P.Cin;
  if (gvec) {
    const int k = k_begin + c8 * CE;
    const int tap = fast_div(k, P.div_cin);
    g_c = k - tap * P.Cin;
    g_r = fast_div(tap, P.div_s);
    g_s = tap - g_r * P.S;
    tap_off = ((int64_t)g_r * P.W + g_s) * P.Cin + g_c;
  }
  u32x4 ra[NS][A_ITERS], rb[NS][B_ITERS];
  const uintptr_t zeros = zero_piece_address();
  // Loads are unconditional (stages past the end of the reduction read clamped addresses and
  // are never multiplied), so the number of loads in flight is the same on every path.
  int k_load = k_begin + c8 * CE;  // reduction index of this thread's piece in the next stage to load
  auto gload = [&](u32x4(&xa)[A_ITERS], u32x4(&xb)[B_ITERS]) {
    const bool in = k_load < k_stop;
    if (gvec) {
#pragma unroll
      for (int i = 0; i < A_ITERS; ++i) {
        const bool ok = in && (unsigned)(hb[i] + g_r) < (unsigned)P.H && (unsigned)(wb[i] + g_s) < (unsigned)P.W;
        xa[i] = *(const u32x4 SK_GLOBAL *)(ok ? (uintptr_t)pa[i] + (uintptr_t)(tap_off * ES) : zeros);
      }
      g_c += KB;
      tap_off += KB;
      while (g_c >= P.Cin) {
        g_c -= P.Cin;
        if (++g_s == P.S) {
          g_s = 0;
          ++g_r;
          tap_off += next_filter_row;
        }
      }
    } else {
#pragma unroll
      for (int i = 0; i < A_ITERS; ++i)
        xa[i] = *(const u32x4 SK_GLOBAL *)(in ? (uintptr_t)pa[i] + (uintptr_t)((int64_t)k_load * ES) : zeros);
    }
#pragma unroll
    for (int i = 0; i < B_ITERS; ++i)
      xb[i] = *(const u32x4 SK_GLOBAL *)(in ? (uintptr_t)pb[i] + (uintptr_t)((int64_t)k_load * ES) : zeros);
    k_load += KB;
  };
  auto lstore = [&](int buf, const u32x4(&xa)[A_ITERS], const u32x4(&xb)[B_ITERS]) {
    unsigned char *a = lds + buf * STAGE + srow * LDS_ROW + c8 * 16;
    unsigned char *bb = a + BM * LDS_ROW;
#pragma unroll
    for (int i = 0; i < A_ITERS; ++i) *(u32x4 *)(a + 32 * i * LDS_ROW) = xa[i];
#pragma unroll
    for (int i = 0; i < B_ITERS; ++i) *(u32x4 *)(bb + 32 * i * LDS_ROW) = xb[i];
  };

  const int nstages = (k_stop - k_begin + KB - 1) / KB;
#pragma unroll
  for (int u = 0; u < NS - 1; ++u) gload(ra[u], rb[u]);
  lstore(0, ra[0], rb[0]);
  __syncthreads();
  int buf = 0;
  for (int s0 = 0; s0 < nstages; s0 += NS) {
#pragma unroll
    for (int u = 0; u < NS; ++u) {
      pf.at_step(s0 + u, nstages, CLAIM_LEAD, ISSUE_GAP);
      gload(ra[(u + NS - 1) % NS], rb[(u + NS - 1) % NS]);
      if (s0 + u < nstages) {
        // stage s0+u is in LDS buffer `buf`; put stage s0+u+1 (possibly past the end: zeros
        // times finite weights, never multiplied) into the other one while this one is used
        const unsigned char *la = lds + buf * STAGE;
        const unsigned char *lb = la + BM * LDS_ROW;
        // operand fragments of the first quarter of the stage are requested before the next
        // stage is written, those of quarter kk+1 before the MFMAs of quarter kk
        u32x4 fa[2][FM], fb[2][FN];
        auto frag = [&](int kk, u32x4(&xa)[FM], u32x4(&xb)[FN]) {
          const int piece = (2 * kk + half) * 16;
#pragma unroll
          for (int fm = 0; fm < FM; ++fm)
            xa[fm] = *(const u32x4 *)(la + ((wm * FM + fm) * 32 + l32) * LDS_ROW + piece);
#pragma unroll
          for (int fn = 0; fn < FN; ++fn)
            xb[fn] = *(const u32x4 *)(lb + ((wn * FN + fn) * 32 + l32) * LDS_ROW + piece);
        };
        frag(0, fa[0], fb[0]);
        lstore(buf ^ 1, ra[(u + 1) % NS], rb[(u + 1) % NS]);
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
          if (kk + 1 < 4) frag(kk + 1, fa[(kk + 1) & 1], fb[(kk + 1) & 1]);
#pragma unroll
          for (int fn = 0; fn < FN; ++fn)
#pragma unroll
            for (int fm = 0; fm < FM; ++fm) mma32<DT>(fb[kk & 1][fn], fa[kk & 1][fm], acc[fn][fm]);
        }
        __syncthreads();
        buf ^= 1;
      }
    }
  }

  finish_tile<DT, BM, BN, WAVES_M, WAVES_N>(P, T, sp, lds, s_flag, tid, acc);
}

// ---------------------------------------------------------------------------
// LDS tiles with lean operand addressing
// ---------------------------------------------------------------------------
// The stage of run_tile above spends more instructions on forming addresses than on anything
// else: per 16-byte piece a 64-bit add, two selects against the piece of zeros and, for a
// convolution, the bounds of the tap in both directions.  With two waves per SIMD those
// instructions, not the memory system, set the pace of a stage.  This variant keeps the same
// pipeline (ring of register stages, two LDS stages, the same LDS image, fragments and MFMAs)
// and reads its operands through buffer descriptors instead:
//   * one descriptor per operand and tile, based at the tile's first row, its size the extent of
//     the tile's rows: a piece's address is a 32-bit row offset kept in a register for the whole
//     tile plus a scalar offset that advances with the stage, and a piece that lies outside the
//     descriptor reads as zero, so a piece that must not be read gets the offset 2^31;
//   * for a convolution whose channel count is a multiple of a stage (64 elements of 2 bytes),
//     all pieces of a stage lie under one filter tap: the tap and its offset are scalar, and
//     whether a row's pixel under that tap lies in the image is one bit of a mask that is
//     worked out once per tile and row.
// It serves operators whose tile extents fit 31 bits of byte offset and, for convolutions,
// those with such channel counts and at most 31 filter taps; the others keep run_tile.
struct LeanOperands {
  uintptr_t baseA, baseB;  // first byte the descriptors cover
  uint32_t extA, extB;     // bytes they cover
  int64_t originA;         // element offset of baseA from P.A
};

// Whether the tile can take the lean path, and its descriptors.  All scalar (P and T are uniform).
template <int ES>
__device__ __forceinline__ bool lean_operands(const DevProblem &P, const sk_tile &T, LeanOperands &L) {
  constexpr int CE = 16 / ES;
  constexpr int KB = 8 * CE;
  constexpr int64_t LIMIT = (int64_t)1 << 31;
  const int64_t extB = ((int64_t)((int)T.n_len - 1) * P.ldb + P.Kg) * ES;
  L.baseB = (uintptr_t)P.B + (uintptr_t)((int64_t)T.n0 * P.ldb * ES);
  L.extB = (uint32_t)extB;
  int64_t extA;
  if (!P.gather) {
    extA = ((int64_t)((int)T.m_len - 1) * P.lda + P.Kg) * ES;
    L.originA = (int64_t)T.m0 * P.lda;
  } else {
    if (P.nchw || P.Cin % KB != 0 || P.R * P.S > 31) return false;
    // from the corner of the padded first image of the tile to the end of the array
    const int hw = P.Ho * P.Wo;
    const int b0 = fast_div((int)T.m0, P.div_hw);
    const int nb = fast_div(P.Mg + hw - 1, P.div_hw);
    L.originA = (((int64_t)b0 * P.H - P.pad_h) * P.W - P.pad_w) * P.Cin;
    const int b1 = fast_div((int)T.m0 + (int)T.m_len - 1, P.div_hw);
    // (the last image the tile touches must lie inside 2^31 bytes; the descriptor itself ends with the array)
    if ((((int64_t)(b1 + 1) * P.H * P.W) * P.Cin - L.originA) * ES >= LIMIT) return false;
    extA = (((int64_t)nb * P.H * P.W) * P.Cin - L.originA) * ES;
    if (extA >= LIMIT) extA = LIMIT - 1;
  }
  L.baseA = (uintptr_t)P.A + (uintptr_t)(L.originA * ES);
  L.extA = (uint32_t)extA;
  return extA < LIMIT && extB < LIMIT;
}

template <int DT, int BM, int BN, int WAVES_M, int WAVES_N, bool GATHER>
__device__ __forceinline__ void run_tile_lean(const DevProblem &P, const sk_tile &T, const SplitK &sp, unsigned char *lds,
                                              uint32_t *s_flag, Prefetch &pf, const LeanOperands &L) {
  constexpr int ES = Elem<DT>::ES;
  constexpr int CE = 16 / ES;
  constexpr int KB = 8 * CE;                  // reduction elements per stage
  constexpr int FM = BM / (32 * WAVES_M);     // 32x32 blocks per wave along m
  constexpr int FN = BN / (32 * WAVES_N);     // ... along n
  constexpr int A_ITERS = BM / 32;            // 16-byte pieces per thread per stage, activations
  constexpr int B_ITERS = BN / 32;            // ... weights
  constexpr int STAGE = (BM + BN) * LDS_ROW;  // bytes of one stage in LDS
  constexpr int NS = 3;
  constexpr uint32_t NOWHERE = 0x80000000u;   // an offset outside every descriptor: the piece reads as zero
  static_assert(WAVES_M * WAVES_N == 4, "four waves per workgroup");
  static_assert(2 * STAGE <= LDS_TILE_BYTES, "two stages do not fit the LDS buffer");

  const int tid = pf.tid;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lane = tid & 63;
  const int wm = wave % WAVES_M, wn = wave / WAVES_M;
  const int l32 = lane & 31, half = lane >> 5;

  const int m0 = (int)T.m0, n0 = (int)T.n0;
  const int m_end = m0 + (int)T.m_len, n_end = n0 + (int)T.n_len;
  const int k_begin = (int)T.k0, k_stop = (int)T.k0 + (int)T.k_len;

  const __amdgpu_buffer_rsrc_t descA = __builtin_amdgcn_make_buffer_rsrc((void *)L.baseA, 0, (int)L.extA, 0x00020000);
  const __amdgpu_buffer_rsrc_t descB = __builtin_amdgcn_make_buffer_rsrc((void *)L.baseB, 0, (int)L.extB, 0x00020000);

  // staging map: thread -> piece c8 of rows (tid/8) + 32*i
  const int c8 = tid & 7;
  const int srow = tid >> 3;
  uint32_t offA[A_ITERS];   // byte offset of this thread's piece of row i at reduction index 0 (tap (0,0), channel 0)
  uint32_t tapsA[A_ITERS];  // convolution: bit (r*S + s) set if the row's pixel under tap (r, s) lies in the image
#pragma unroll
  for (int i = 0; i < A_ITERS; ++i) {
    int m = m0 + srow + 32 * i;
    if (m >= m_end) m = m_end - 1;  // rows past the edge repeat the last row; never stored
    if constexpr (!GATHER) {
      offA[i] = (uint32_t)((m - m0) * (int)P.lda * ES) + (uint32_t)c8 * 16u;
      tapsA[i] = 0;
    } else {
      const RowA r = row_of(P, m);
      offA[i] = (uint32_t)((r.base - L.originA) * ES) + (uint32_t)c8 * 16u;
      // filter rows rr with 0 <= hb + rr < H form a range [lo, hi), and so do the filter columns
      const int hlo = max(0, -r.hb), hhi = min(P.R, P.H - r.hb);
      const int wlo = max(0, -r.wb), whi = min(P.S, P.W - r.wb);
      const uint32_t wmk = whi > wlo ? ((1u << whi) - 1u) & ~((1u << wlo) - 1u) : 0u;  // (at most 31 taps)
      uint32_t taps = 0;
      for (int rr = 0; rr < P.R; ++rr) taps |= (rr >= hlo && rr < hhi) ? wmk << (rr * P.S) : 0u;
      tapsA[i] = taps;
    }
  }
  uint32_t offB[B_ITERS];
#pragma unroll
  for (int i = 0; i < B_ITERS; ++i) {
    int n = n0 + srow + 32 * i;
    if (n >= n_end) n = n_end - 1;
    offB[i] = (uint32_t)((n - n0) * (int)P.ldb * ES) + (uint32_t)c8 * 16u;
  }

  f32x16 acc[FN][FM];
#pragma unroll
  for (int fn = 0; fn < FN; ++fn)
#pragma unroll
    for (int fm = 0; fm < FM; ++fm)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[fn][fm][i] = 0.f;

  // scalar position of the next stage to load: reduction index k_next; for a convolution the tap
  // (t_r, t_s) and the first channel t_c of the stage
  int k_next = k_begin;
  int t_r = 0, t_s = 0, t_c = 0;
  if constexpr (GATHER) {
    const int tap = fast_div(k_begin, P.div_cin);
    t_c = k_begin - tap * P.Cin;
    t_r = fast_div(tap, P.div_s);
    t_s = tap - t_r * P.S;
  }
  u32x4 ra[NS][A_ITERS], rb[NS][B_ITERS];
  // Loads are unconditional (stages past the end of the reduction read whatever lies there, or zeros
  // past the descriptor, and are never multiplied), so the number of loads in flight is the same on
  // every path.
  auto gload = [&](u32x4(&xa)[A_ITERS], u32x4(&xb)[B_ITERS]) {
    const uint32_t kbytes = (uint32_t)k_next * ES;
    if constexpr (GATHER) {
      // (no reduction tail: the reduction length is a multiple of the channel count, that of a stage)
      const uint32_t tapbit = 1u << ((t_r * P.S + t_s) & 31);
      const uint32_t tapoff = (uint32_t)(((t_r * P.W + t_s) * P.Cin + t_c) * ES);
#pragma unroll
      for (int i = 0; i < A_ITERS; ++i)
        xa[i] = __builtin_amdgcn_raw_buffer_load_b128(descA, (tapsA[i] & tapbit) ? offA[i] : NOWHERE, tapoff, 0);
#pragma unroll
      for (int i = 0; i < B_ITERS; ++i) xb[i] = __builtin_amdgcn_raw_buffer_load_b128(descB, offB[i], kbytes, 0);
      t_c += KB;
      if (t_c >= P.Cin) {
        t_c = 0;
        if (++t_s == P.S) {
          t_s = 0;
          ++t_r;
        }
      }
    } else {
      // this thread's piece lies beyond the end of the reduction (last stage of a length that is not a
      // multiple of a stage): nowhere
      const uint32_t tail = k_next + c8 * CE < k_stop ? 0u : NOWHERE;
#pragma unroll
      for (int i = 0; i < A_ITERS; ++i) xa[i] = __builtin_amdgcn_raw_buffer_load_b128(descA, offA[i] | tail, kbytes, 0);
#pragma unroll
      for (int i = 0; i < B_ITERS; ++i) xb[i] = __builtin_amdgcn_raw_buffer_load_b128(descB, offB[i] | tail, kbytes, 0);
    }
    k_next += KB;
  };
  auto lstore = [&](int buf, const u32x4(&xa)[A_ITERS], const u32x4(&xb)[B_ITERS]) {
    unsigned char *a = lds + buf * STAGE + srow * LDS_ROW + c8 * 16;
    unsigned char *bb = a + BM * LDS_ROW;
#pragma unroll
    for (int i = 0; i < A_ITERS; ++i) *(u32x4 *)(a + 32 * i * LDS_ROW) = xa[i];
#pragma unroll
    for (int i = 0; i < B_ITERS; ++i) *(u32x4 *)(bb + 32 * i * LDS_ROW) = xb[i];
  };

  const int nstages = (k_stop - k_begin + KB - 1) / KB;
#pragma unroll
  for (int u = 0; u < NS - 1; ++u) gload(ra[u], rb[u]);
  lstore(0, ra[0], rb[0]);
  __syncthreads();
  int buf = 0;
  for (int s0 = 0; s0 < nstages; s0 += NS) {
#pragma unroll
    for (int u = 0; u < NS; ++u) {
      pf.at_step(s0 + u, nstages, CLAIM_LEAD, ISSUE_GAP);
      gload(ra[(u + NS - 1) % NS], rb[(u + NS - 1) % NS]);
      if (s0 + u < nstages) {
        // stage s0+u is in LDS buffer `buf`; put stage s0+u+1 into the other one while this one is used
        const unsigned char *la = lds + buf * STAGE;
        const unsigned char *lb = la + BM * LDS_ROW;
        u32x4 fa[2][FM], fb[2][FN];
        auto frag = [&](int kk, u32x4(&xa)[FM], u32x4(&xb)[FN]) {
          const int piece = (2 * kk + half) * 16;
#pragma unroll
          for (int fm = 0; fm < FM; ++fm)
            xa[fm] = *(const u32x4 *)(la + ((wm * FM + fm) * 32 + l32) * LDS_ROW + piece);
#pragma unroll
          for (int fn = 0; fn < FN; ++fn)
            xb[fn] = *(const u32x4 *)(lb + ((wn * FN + fn) * 32 + l32) * LDS_ROW + piece);
        };
        frag(0, fa[0], fb[0]);
        lstore(buf ^ 1, ra[(u + 1) % NS], rb[(u + 1) % NS]);
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
          if (kk + 1 < 4) frag(kk + 1, fa[(kk + 1) & 1], fb[(kk + 1) & 1]);
#pragma unroll
          for (int fn = 0; fn < FN; ++fn)
#pragma unroll
            for (int fm = 0; fm < FM; ++fm) mma32<DT>(fb[kk & 1][fn], fa[kk & 1][fm], acc[fn][fm]);
        }
        __syncthreads();
        buf ^= 1;
      }
    }
  }
  finish_tile<DT, BM, BN, WAVES_M, WAVES_N>(P, T, sp, lds, s_flag, tid, acc);
}

// ---------------------------------------------------------------------------
// LDS tiles fed by direct global-to-LDS loads
// ---------------------------------------------------------------------------
// The same tile, fragments and MFMAs, but the operand pieces never pass through registers:
// a buffer load with the LDS modifier writes the 16 bytes of lane i at (M0 + 16 i) of the LDS,
// 1 KB per wave and instruction, and a piece whose offset lies outside the descriptor arrives
// as zeros.  What this removes from a stage: the register ring (96 registers), the LDS stores
// with their counted waits, and all but one or two instructions per piece.
//   * LDS image of a stage: (BM + BN) rows of 128 bytes, no padding (a load instruction fills
//     eight consecutive rows); position p of row r holds the row's piece p ^ ((r >> 1) & 7), so
//     the 16 lanes that a fragment read serves together (rows r .. r+15, one piece) fall into
//     16 different groups of four banks.  The swizzle is applied on the global side: lane i of
//     a load asks for piece (i & 7) ^ swizzle(row of the lane).
//   * a ring of NS such images (as many as fit LDS_TILE_BYTES): stages h+1 .. h+NS-2 are in
//     flight while stage h is multiplied; one barrier per stage says both "everyone's part of
//     stage h has landed" and "everyone is done with the image that stage h+NS-1 will overwrite".
//   * the compiler does not see these loads (inline assembly; told about them it would wait for
//     all of them before every LDS read), so the waits are written out: loads complete in order,
//     hence "at most n outstanding" with n the loads of the stages issued later.  Loads and
//     stores of the surrounding code that are also in flight only make these waits, and the
//     compiler's own, wait for more than they need.
//   * the compiler does not look into inline assembly for the wait states the hardware wants between
//     instructions either.  Two matter here: a scalar register written by a vector instruction (the
//     compiler keeps spilled scalars in lanes of a vector register and fetches them with v_readlane
//     wherever it needs them, also right in front of these loads) must not be read by a memory
//     instruction in the next five cycles, and M0 not by an LDS-writing load in the cycle after it
//     was written.  So all loads of a stage sit in ONE statement that opens with the five cycles
//     and moves M0 from piece to piece itself (the pieces of a wave lie 4 KB apart), and hands M0 back
//     as it got it.
template <int NA, int NBW>
__device__ __forceinline__ void dma_stage(__amdgpu_buffer_rsrc_t descA, __amdgpu_buffer_rsrc_t descB, const uint32_t (&va)[NA],
                                          const uint32_t (&vb)[NBW], uint32_t soffA, uint32_t soffB, uint32_t lds_addr) {
  static_assert(NA == 4 && (NBW == 4 || NBW == 2), "written out for 128 rows of activations and 128 or 64 of weights");
#define SK_DMA_NEXT "s_add_u32 m0, m0, 0x1000\n\ts_nop 0\n\t"
  if constexpr (NBW == 4) {
    asm volatile("s_nop 4\n\t"
                 "buffer_load_dwordx4 %0, %8, %10 offen lds\n\t" SK_DMA_NEXT
                 "buffer_load_dwordx4 %1, %8, %10 offen lds\n\t" SK_DMA_NEXT
                 "buffer_load_dwordx4 %2, %8, %10 offen lds\n\t" SK_DMA_NEXT
                 "buffer_load_dwordx4 %3, %8, %10 offen lds\n\t" SK_DMA_NEXT
                 "buffer_load_dwordx4 %4, %9, %11 offen lds\n\t" SK_DMA_NEXT
                 "buffer_load_dwordx4 %5, %9, %11 offen lds\n\t" SK_DMA_NEXT
                 "buffer_load_dwordx4 %6, %9, %11 offen lds\n\t" SK_DMA_NEXT
                 "buffer_load_dwordx4 %7, %9, %11 offen lds\n\t"
                 "s_sub_u32 m0, m0, 0x7000"
                 :
                 : "v"(va[0]), "v"(va[1]), "v"(va[2]), "v"(va[3]), "v"(vb[0]), "v"(vb[1]), "v"(vb[2]), "v"(vb[3]), "s"(descA),
                   "s"(descB), "s"(soffA), "s"(soffB), "{m0}"(lds_addr)
                 : "memory", "scc");
  } else {
    asm volatile("s_nop 4\n\t"
                 "buffer_load_dwordx4 %0, %6, %8 offen lds\n\t" SK_DMA_NEXT
                 "buffer_load_dwordx4 %1, %6, %8 offen lds\n\t" SK_DMA_NEXT
                 "buffer_load_dwordx4 %2, %6, %8 offen lds\n\t" SK_DMA_NEXT
                 "buffer_load_dwordx4 %3, %6, %8 offen lds\n\t" SK_DMA_NEXT
                 "buffer_load_dwordx4 %4, %7, %9 offen lds\n\t" SK_DMA_NEXT
                 "buffer_load_dwordx4 %5, %7, %9 offen lds\n\t"
                 "s_sub_u32 m0, m0, 0x5000"
                 :
                 : "v"(va[0]), "v"(va[1]), "v"(va[2]), "v"(va[3]), "v"(vb[0]), "v"(vb[1]), "s"(descA), "s"(descB), "s"(soffA),
                   "s"(soffB), "{m0}"(lds_addr)
                 : "memory", "scc");
  }
#undef SK_DMA_NEXT
}
template <int N>
__device__ __forceinline__ void wait_loads_but() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

template <int DT, int BM, int BN, bool GATHER>
__device__ __forceinline__ void run_tile_dma(const DevProblem &P, const sk_tile &T, const SplitK &sp, unsigned char *lds,
                                             uint32_t *s_flag, Prefetch &pf, const LeanOperands &L) {
  constexpr int ES = Elem<DT>::ES;
  constexpr int CE = 16 / ES;
  constexpr int KB = 8 * CE;                  // reduction elements per stage (128 bytes per row)
  constexpr int FM = BM / 64, FN = BN / 64;   // 32x32 blocks per wave along m and n (2 x 2 waves)
  constexpr int NA = BM / 32, NBW = BN / 32;  // load instructions per wave and stage: activations, weights
  constexpr int NPW = NA + NBW;
  constexpr int SLOT = (BM + BN) * 128;       // bytes of a stage in LDS
  constexpr int NS = LDS_TILE_BYTES / SLOT;   // ring slots
  constexpr uint32_t NOWHERE = 0x80000000u;   // an offset outside every descriptor: the piece arrives as zeros
  static_assert(NS == 2 || NS == 3, "waits below are written for two or three slots");
  static_assert(BM == 128, "a wave's pieces of a stage lie 4 KB apart, activations first (dma_stage)");
  static_assert(NPW < 32, "load counter");

  const int tid = pf.tid;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lane = tid & 63;
  const int wm = wave & 1, wn = wave >> 1;
  const int l32 = lane & 31, half = lane >> 5;

  const int m0 = (int)T.m0, n0 = (int)T.n0;
  const int m_end = m0 + (int)T.m_len, n_end = n0 + (int)T.n_len;
  const int k_begin = (int)T.k0, k_stop = (int)T.k0 + (int)T.k_len;

  const __amdgpu_buffer_rsrc_t descA = __builtin_amdgcn_make_buffer_rsrc((void *)L.baseA, 0, (int)L.extA, 0x00020000);
  const __amdgpu_buffer_rsrc_t descB = __builtin_amdgcn_make_buffer_rsrc((void *)L.baseB, 0, (int)L.extB, 0x00020000);

  // load map: instruction i of this wave fills rows 8 (wave + 4 i) .. + 7 of the operand's block; this lane
  // supplies position lane & 7 of row 8 (wave + 4 i) + lane / 8, which holds the logical piece c_log
  // (the swizzle of the lane's row is the same for every i)
  const int lrow = lane >> 3;
  const int c_log = (lane & 7) ^ (((wave & 1) << 2) | (lane >> 4));
  uint32_t offA[NA];   // byte offset of this lane's piece of row i at reduction index 0 (tap (0,0), channel 0)
  uint32_t tapsA[NA];  // convolution: bit (r*S + s) set if the row's pixel under tap (r, s) lies in the image
  // convolution, scalar: pixels per image, first image of the tile, bit rr*S for every filter row rr
  int g_hw = 0, g_b0 = 0;
  uint32_t g_rows = 0;
  if constexpr (GATHER) {
    g_hw = P.Ho * P.Wo;
    g_b0 = fast_div(m0, P.div_hw);
    for (int rr = 0; rr < P.R; ++rr) g_rows |= 1u << (rr * P.S);
  }
#pragma unroll
  for (int i = 0; i < NA; ++i) {
    const int m = m0 + 8 * (wave + 4 * i) + lrow;
    const bool in = m < m_end;  // rows past the edge arrive as zeros; never stored
    if constexpr (!GATHER) {
      offA[i] = in ? (uint32_t)((m - m0) * (int)P.lda * ES) + (uint32_t)c_log * 16u : NOWHERE;
      tapsA[i] = 0;
    } else {
      // Pixel (b, ho, wo) of the row; its offset from the descriptor's origin (the corner of the padded first
      // image of the tile) in 32 bits: lean_operands has checked that the tile's images lie within 2^31 bytes.
      const int mm = in ? m : m_end - 1;
      const int b = fast_div(mm, P.div_hw);
      const int rem = mm - b * g_hw;
      const int ho = fast_div(rem, P.div_wo);
      const int hs = ho * P.stride, ws = (rem - ho * P.Wo) * P.stride;  // row and column of tap (0,0) in the padded image
      offA[i] = (uint32_t)((((b - g_b0) * P.H + hs) * P.W + ws) * P.Cin * ES) + (uint32_t)c_log * 16u;
      // filter rows rr with 0 <= hb + rr < H form a range [lo, hi), and so do the filter columns; the
      // columns' bits times the bits rr*S of the rows in range is the mask of all taps in the image (no two
      // products overlap: the columns' bits lie below S; at most 31 taps)
      const int hb = hs - P.pad_h, wb = ws - P.pad_w;
      const int hlo = max(0, -hb), hhi = min(P.R, P.H - hb);
      const int wlo = max(0, -wb), whi = min(P.S, P.W - wb);
      const uint32_t wmk = whi > wlo ? ((1u << whi) - 1u) & ~((1u << wlo) - 1u) : 0u;
      const uint32_t rmk = hhi > hlo ? g_rows & ((1u << (hhi * P.S)) - 1u) & ~((1u << (hlo * P.S)) - 1u) : 0u;
      tapsA[i] = in ? wmk * rmk : 0u;
    }
  }
  uint32_t offB[NBW];
#pragma unroll
  for (int i = 0; i < NBW; ++i) {
    const int n = n0 + 8 * (wave + 4 * i) + lrow;
    offB[i] = n < n_end ? (uint32_t)((n - n0) * (int)P.ldb * ES) + (uint32_t)c_log * 16u : NOWHERE;
  }

  f32x16 acc[FN][FM];
#pragma unroll
  for (int fn = 0; fn < FN; ++fn)
#pragma unroll
    for (int fm = 0; fm < FM; ++fm)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[fn][fm][i] = 0.f;

  // scalar position of the next stage to load: reduction index k_next; for a convolution the tap
  // (t_r, t_s) and the first channel t_c of the stage
  int k_next = k_begin;
  int t_r = 0, t_s = 0, t_c = 0;
  if constexpr (GATHER) {
    const int tap = fast_div(k_begin, P.div_cin);
    t_c = k_begin - tap * P.Cin;
    t_r = fast_div(tap, P.div_s);
    t_s = tap - t_r * P.S;
  }
  const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)lds;
  const uint32_t my_blocks = lds_base + (uint32_t)wave * 1024u;  // + slot*SLOT + 4096 i (activations), + BM*128 + 4096 i (weights)
  auto issue = [&](int slot) {
    const uint32_t kbytes = (uint32_t)k_next * ES;
    const uint32_t dst = my_blocks + (uint32_t)slot * SLOT;
    uint32_t va[NA], vb[NBW];
    if constexpr (GATHER) {
      // (no reduction tail: the reduction length is a multiple of the channel count, that of a stage)
      const uint32_t tapbit = 1u << ((t_r * P.S + t_s) & 31);
      const uint32_t tapoff = (uint32_t)(((t_r * P.W + t_s) * P.Cin + t_c) * ES);
#pragma unroll
      for (int i = 0; i < NA; ++i) va[i] = (tapsA[i] & tapbit) ? offA[i] : NOWHERE;
#pragma unroll
      for (int i = 0; i < NBW; ++i) vb[i] = offB[i];
      dma_stage<NA, NBW>(descA, descB, va, vb, tapoff, kbytes, dst);
      t_c += KB;
      if (t_c >= P.Cin) {
        t_c = 0;
        if (++t_s == P.S) {
          t_s = 0;
          ++t_r;
        }
      }
    } else {
      // this lane's piece lies beyond the end of the reduction (last stage of a length that is not a
      // multiple of a stage): nowhere
      const uint32_t tail = k_next + c_log * CE < k_stop ? 0u : NOWHERE;
#pragma unroll
      for (int i = 0; i < NA; ++i) va[i] = offA[i] | tail;
#pragma unroll
      for (int i = 0; i < NBW; ++i) vb[i] = offB[i] | tail;
      dma_stage<NA, NBW>(descA, descB, va, vb, kbytes, kbytes, dst);
    }
    k_next += KB;
  };

  // fragment addresses inside a slot: row (w*F + f)*32 + l32, logical piece 2 kk + half at position
  // (2 kk + half) ^ swizzle(row), and swizzle(row) = (l32 >> 1) & 7 for every block of 32 rows
  const int frag_off = l32 * 128;
  const int frag_pos = half ^ ((l32 >> 1) & 7);  // position of piece `half`; piece 2 kk + half is at frag_pos ^ 2 kk
  const int a_base = wm * FM * 4096;
  const int b_base = BM * 128 + wn * FN * 4096;

#ifdef SK_DIAG_CLOCKS
  const int diag_tile = pf.diag_tile;
#endif
  SK_DIAG(1);
  const int nstages = (k_stop - k_begin + KB - 1) / KB;
  // (the previous tile's readers of this LDS buffer have passed the barrier at the end of their tile)
#pragma unroll
  for (int u = 0; u < NS - 1; ++u)
    if (u < nstages) issue(u);
  int slot = 0;
  for (int h = 0; h < nstages; ++h) {
    pf.at_step(h, nstages, CLAIM_LEAD, ISSUE_GAP);
    // this wave's loads of stage h have landed: the only loads issued after them are those of stage h+1
    if (NS == 3 && h + 1 < nstages)
      wait_loads_but<NPW>();
    else
      wait_loads_but<0>();
    __builtin_amdgcn_s_barrier();  // ... and everyone's; everyone is done with stage h-1
    asm volatile("" ::: "memory");
    if (h + NS - 1 < nstages) issue(slot == 0 ? NS - 1 : slot - 1);  // stage h+NS-1 into the slot stage h-1 used
    __builtin_amdgcn_sched_barrier(0);
    const unsigned char *la = lds + slot * SLOT + a_base + frag_off;
    const unsigned char *lb = lds + slot * SLOT + b_base + frag_off;
    // the fragments of step kk+1 are requested before the MFMAs of step kk (the scheduler is held to
    // that order: left alone it sinks every read to just above its first use).  Requesting all four
    // steps' fragments at the start of the stage was measured slower: the waves of a workgroup leave
    // the barrier together, and their reads then queue at the LDS.
    u32x4 fa[2][FM], fb[2][FN];
    auto frag = [&](int kk, u32x4(&xa)[FM], u32x4(&xb)[FN]) {
      const int pos = (frag_pos ^ (2 * kk)) << 4;
#pragma unroll
      for (int fm = 0; fm < FM; ++fm) xa[fm] = *(const u32x4 *)(la + fm * 4096 + pos);
#pragma unroll
      for (int fn = 0; fn < FN; ++fn) xb[fn] = *(const u32x4 *)(lb + fn * 4096 + pos);
    };
    frag(0, fa[0], fb[0]);
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      if (kk + 1 < 4) frag(kk + 1, fa[(kk + 1) & 1], fb[(kk + 1) & 1]);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int fn = 0; fn < FN; ++fn)
#pragma unroll
        for (int fm = 0; fm < FM; ++fm) mma32<DT>(fb[kk & 1][fn], fa[kk & 1][fm], acc[fn][fm]);
      __builtin_amdgcn_sched_barrier(0);
    }
    if (h == 0) SK_DIAG(2);
    slot = slot + 1 == NS ? 0 : slot + 1;
  }
  SK_DIAG(3);
  __syncthreads();  // everyone is done with the last stage before the output tile is staged in the same LDS
  finish_tile<DT, BM, BN, 2, 2>(P, T, sp, lds, s_flag, tid, acc);
  SK_DIAG(4);
}

// One LDS tile: the lean path where the operator allows it.
template <int DT, int BM, int BN>
__device__ __forceinline__ void run_lds_tile(const DevProblem &P, const sk_tile &T, const SplitK &sp, unsigned char *lds,
                                             uint32_t *s_flag, Prefetch &pf) {
#ifndef SK_NO_LEAN_TILES
  LeanOperands L;
  if (lean_operands<Elem<DT>::ES>(P, T, L)) {
#ifdef SK_REGISTER_RING_TILES
    if (P.gather)
      run_tile_lean<DT, BM, BN, 2, 2, true>(P, T, sp, lds, s_flag, pf, L);
    else
      run_tile_lean<DT, BM, BN, 2, 2, false>(P, T, sp, lds, s_flag, pf, L);
#else
    if (P.gather)
      run_tile_dma<DT, BM, BN, true>(P, T, sp, lds, s_flag, pf, L);
    else
      run_tile_dma<DT, BM, BN, false>(P, T, sp, lds, s_flag, pf, L);
#endif
    return;
  }
#endif
  run_tile<DT, BM, BN, 2, 2>(P, T, sp, lds, s_flag, pf);
}

// ---------------------------------------------------------------------------
// dispatch and the persistent shell
// ---------------------------------------------------------------------------
// ---------------------------------------------------------------------------
// generic tiles: operands that cannot be read in aligned 16-byte pieces
// (odd K, odd Cin, unaligned pointers or strides).  One output per thread and
// trip, plain fp32 multiply-adds in ascending k.  Correct for everything, fast
// for nothing; used for rectangles with next to no work.
// ---------------------------------------------------------------------------
// (Inlined, like every path of the kernel: as real calls the two slow paths gave the kernel a stack,
// and how well its fast paths then ran changed from build to build.  They exist only in the kernel
// instantiation for plans with such operands, which takes a few registers more.  They are given the
// records' addresses in memory rather than references to the caller's copies.)
template <int DT>
__device__ __forceinline__ void run_generic(const DevProblem *P_mem, const sk_tile *T_mem) {
  const DevProblem P = *P_mem;
  const sk_tile T = *T_mem;
  const int m_len = T.m_len, n_len = T.n_len;
  // a split reduction is done whole by the record of its first slice; the others have nothing to do
  if (T.ks_idx != 0) return;
  for (int idx = threadIdx.x; idx < m_len * n_len; idx += WG_THREADS) {
    const int m = (int)T.m0 + idx / n_len;
    const int n = (int)T.n0 + idx % n_len;
    const RowA row = row_of(P, m);
    const int64_t wrow = (int64_t)n * P.ldb;
    float acc = 0.f;
    if (!P.gather) {
      for (int k = 0; k < P.Kg; ++k)
        acc = __builtin_fmaf(load_elem<DT>(P.A, row.base + k), load_elem<DT>(P.B, wrow + k), acc);
    } else if (!P.nchw) {
      // taps in the order of the reduction index; those in the padding contribute nothing
      for (int r = 0; r < P.R; ++r) {
        if ((unsigned)(row.hb + r) >= (unsigned)P.H) continue;
        for (int t = 0; t < P.S; ++t) {
          if ((unsigned)(row.wb + t) >= (unsigned)P.W) continue;
          const int64_t xa = row.base + ((int64_t)r * P.W + t) * P.Cin;
          const int64_t wb = wrow + (int64_t)(r * P.S + t) * P.Cin;
          for (int c = 0; c < P.Cin; ++c)
            acc = __builtin_fmaf(load_elem<DT>(P.A, xa + c), load_elem<DT>(P.B, wb + c), acc);
        }
      }
    } else {
      // channel-major: reduction index (c*R + r)*S + t
      const int64_t plane = (int64_t)P.H * P.W;
      for (int c = 0; c < P.Cin; ++c)
        for (int r = 0; r < P.R; ++r) {
          if ((unsigned)(row.hb + r) >= (unsigned)P.H) continue;
          for (int t = 0; t < P.S; ++t) {
            if ((unsigned)(row.wb + t) >= (unsigned)P.W) continue;
            acc = __builtin_fmaf(load_elem<DT>(P.A, row.base + c * plane + (int64_t)r * P.W + t),
                                 load_elem<DT>(P.B, wrow + ((int64_t)c * P.R + r) * P.S + t), acc);
          }
        }
    }
    const int64_t c_off = P.nchw ? nchw_out_base(P, m) + (int64_t)n * P.Ho * P.Wo : (int64_t)m * P.ldc + n;
    store_elem<DT>(P.C, c_off, acc);
  }
}

// ---------------------------------------------------------------------------
// MFMA tiles for operands of any alignment (an image with 3 channels, an odd
// reduction length, unaligned bases): the staging map and the LDS layout of
// run_tile, but a 16-byte piece is put together from single elements, loaded one
// by one, and a stage is loaded, stored to LDS and multiplied before the next
// one is touched (the unpacked elements of one stage fill the registers that
// the packed pieces of a ring of stages would).  Any output rectangle is
// walked in blocks of 128 x 128; the slices of a split reduction (always a
// single block) meet in the workspace like those of the other tile classes.
// ---------------------------------------------------------------------------
template <int DT>
__device__ __forceinline__ void run_tile_any(const DevProblem *P_mem, const sk_tile *T_mem, const SplitK &sp,
                                             unsigned char *lds, uint32_t *s_flag) {
  constexpr int ES = Elem<DT>::ES;
  constexpr int CE = 16 / ES;
  constexpr int KB = 8 * CE;
  using elem_t = typename std::conditional<ES == 4, uint32_t, uint16_t>::type;
  const DevProblem P = *P_mem;
  const sk_tile T = *T_mem;
  const int tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63;
  const int wm = wave & 1, wn = wave >> 1;
  const int l32 = lane & 31, half = lane >> 5;
  const int c8 = tid & 7, srow = tid >> 3;
  const uintptr_t zeros = zero_piece_address();
  const int m_end = (int)T.m0 + (int)T.m_len, n_end = (int)T.n0 + (int)T.n_len;
  const bool vec_c = (P.flags & FLAG_VEC_C) != 0;
  const bool vec_b = (P.flags & FLAG_VEC_B) != 0;
  const ImageStrides im = image_strides(P);
  unsigned char *sa = lds + srow * LDS_ROW + c8 * 16;
  unsigned char *sb = sa + 128 * LDS_ROW;

  for (int mb = (int)T.m0; mb < m_end; mb += 128) {
    RowA rows[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      int m = mb + srow + 32 * i;
      if (m >= m_end) m = m_end - 1;  // rows past the edge repeat the last row; never stored
      rows[i] = row_of(P, m);
    }
    for (int nb = (int)T.n0; nb < n_end; nb += 128) {
      int64_t wrow[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        int n = nb + srow + 32 * i;
        if (n >= n_end) n = n_end - 1;
        wrow[i] = (int64_t)n * P.ldb;
      }
      f32x16 acc[2][2];
#pragma unroll
      for (int fn = 0; fn < 2; ++fn)
#pragma unroll
        for (int fm = 0; fm < 2; ++fm)
#pragma unroll
          for (int i = 0; i < 16; ++i) acc[fn][fm][i] = 0.f;

      // this record's slice of the reduction (all of it unless the rectangle is split)
      const int k_stop = (int)T.k0 + (int)T.k_len;
      for (int k0 = (int)T.k0; k0 < k_stop; k0 += KB) {
        const int k = k0 + c8 * CE;  // first reduction index of this thread's pieces
        // filter tap and channel of element k (convolutions); later elements by carrying
        int g_r = 0, g_s = 0, g_c = 0;
        if (P.gather && !P.nchw) {
          const int tap = fast_div(k, P.div_cin);
          g_c = k - tap * P.Cin;
          g_r = fast_div(tap, P.div_s);
          g_s = tap - g_r * P.S;
        } else if (P.gather) {  // channel-major: k = (c*R + r)*S + s
          const int cr = k / P.S;
          g_s = k - cr * P.S;
          g_c = cr / P.R;
          g_r = cr - g_c * P.R;
        }
        elem_t va[4][CE], vb[4][CE];
        // weight rows that can be read in 16-byte pieces (always so for channel-major convolutions with aligned
        // weights: a weight row is contiguous in either storage order) are: half the loads of the stage
        u32x4 wb16[4];
        if (vec_b) {
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const uintptr_t pb = (uintptr_t)P.B + (uintptr_t)((wrow[i] + k) * ES);
            wb16[i] = *(const u32x4 SK_GLOBAL *)(k < k_stop ? pb : zeros);
          }
        }
#pragma unroll
        for (int e = 0; e < CE; ++e) {
          const bool in = k + e < k_stop;
          const int64_t rel = P.gather ? g_r * im.sh + g_s * im.sw + g_c * im.sc : (int64_t)(k + e);
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const bool ok = in && (!P.gather || ((unsigned)(rows[i].hb + g_r) < (unsigned)P.H &&
                                                 (unsigned)(rows[i].wb + g_s) < (unsigned)P.W));
            const uintptr_t pa = (uintptr_t)P.A + (uintptr_t)((rows[i].base + rel) * ES);
            va[i][e] = *(const elem_t SK_GLOBAL *)(ok ? pa : zeros);
            if (!vec_b) {
              const uintptr_t pb = (uintptr_t)P.B + (uintptr_t)((wrow[i] + k + e) * ES);
              vb[i][e] = *(const elem_t SK_GLOBAL *)(in ? pb : zeros);
            } else {
              vb[i][e] = 0;
            }
          }
          if (!P.nchw) {
            if (++g_c == P.Cin) {
              g_c = 0;
              if (++g_s == P.S) {
                g_s = 0;
                ++g_r;
              }
            }
          } else if (++g_s == P.S) {
            g_s = 0;
            if (++g_r == P.R) {
              g_r = 0;
              ++g_c;
            }
          }
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          u32x4 qa, qb;
          if constexpr (ES == 4) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              qa[e] = va[i][e];
              qb[e] = vb[i][e];
            }
          } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              qa[e] = (uint32_t)va[i][2 * e] | ((uint32_t)va[i][2 * e + 1] << 16);
              qb[e] = (uint32_t)vb[i][2 * e] | ((uint32_t)vb[i][2 * e + 1] << 16);
            }
          }
          *(u32x4 *)(sa + 32 * i * LDS_ROW) = qa;
          *(u32x4 *)(sb + 32 * i * LDS_ROW) = vec_b ? wb16[i] : qb;
        }
        __syncthreads();
        const unsigned char *la = lds;
        const unsigned char *lb = lds + 128 * LDS_ROW;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
          const int piece = (2 * kk + half) * 16;
          u32x4 fa[2], fb[2];
#pragma unroll
          for (int f = 0; f < 2; ++f) {
            fa[f] = *(const u32x4 *)(la + ((wm * 2 + f) * 32 + l32) * LDS_ROW + piece);
            fb[f] = *(const u32x4 *)(lb + ((wn * 2 + f) * 32 + l32) * LDS_ROW + piece);
          }
#pragma unroll
          for (int fn = 0; fn < 2; ++fn)
#pragma unroll
            for (int fm = 0; fm < 2; ++fm) mma32<DT>(fb[fn], fa[fm], acc[fn][fm]);
        }
        __syncthreads();  // everyone has read the stage before the next one overwrites it
      }

      if (T.S > 1) {
        // A slice of a split reduction (such a rectangle is a single block here: at most 128 x 128, or
        // 16, 32 or 64 rows x 128 columns in the skinny classes).  Partial sums go to the rectangle's
        // workspace, which holds per slice `rows` x 128 (64 for the 64-column class) floats, as 16-byte
        // pieces indexed by (column group of 32, quad j, half, row); the last slice to arrive adds
        // all of them in slice order and stores the result.  Same hand-over as in run_tile.
        // The sixteen accumulator quads of a thread wait in LDS meanwhile (free by now: the last stage
        // ended with a barrier; a slot per thread and quad), so that the loops below can run rolled up:
        // unrolled over the accumulators they cost this kernel forty registers it does not have.
        typedef float f32x2 __attribute__((ext_vector_type(2)));
        static_assert(16 * WG_THREADS * 16 <= LDS_TILE_BYTES, "the accumulators do not fit the LDS buffer");
        f32x4 *slot = (f32x4 *)lds + tid;  // quad p of this thread: slot[p * WG_THREADS]
#pragma unroll
        for (int fn = 0; fn < 2; ++fn)
#pragma unroll
          for (int fm = 0; fm < 2; ++fm)
#pragma unroll
            for (int j = 0; j < 4; ++j)
              slot[((fn * 2 + fm) * 4 + j) * WG_THREADS] =
                  f32x4{acc[fn][fm][4 * j], acc[fn][fm][4 * j + 1], acc[fn][fm][4 * j + 2], acc[fn][fm][4 * j + 3]};
        const int rows = T.cls >= CLS_TILE_128x128 ? 128 : 16 << (T.cls / 3);
        const int groups = T.cls == CLS_TILE_128x64 ? 2 : 4;
        const size_t per_slice = (size_t)groups * 4 * 2 * rows;  // f32x4 units
        unsigned long long *mine = (unsigned long long *)(sp.ws + sp.ws_off[T.out_tile_id]);
        // where quad p = (fn*2 + fm)*4 + j of this thread lies in slice 0, or null if outside the rectangle's rows / columns
        auto piece = [&](int p) -> unsigned long long * {
          const int fn = p >> 3, fm = (p >> 2) & 1, j = p & 3;
          const int r = (wm * 2 + fm) * 32 + l32, cg = wn * 2 + fn;
          if (r >= rows || cg >= groups) return nullptr;
          return mine + 2 * ((size_t)((cg * 4 + j) * 2 + half) * rows + r);
        };
#pragma unroll 1
        for (int p = 0; p < 16; ++p) {
          unsigned long long *q = piece(p);
          if (q) {
            q += 2 * (size_t)T.ks_idx * per_slice;
            const f32x4 v = slot[p * WG_THREADS];
            __hip_atomic_store(q, __builtin_bit_cast(unsigned long long, f32x2{v.x, v.y}), __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(q + 1, __builtin_bit_cast(unsigned long long, f32x2{v.z, v.w}), __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
          }
        }
        __builtin_amdgcn_s_waitcnt(0);  // all counters to zero: the stores above have completed
        __syncthreads();
        if (tid == 0)
          *s_flag = __hip_atomic_fetch_add(&sp.arrive[T.out_tile_id], 1u, SK_ARRIVE_ORDER, __HIP_MEMORY_SCOPE_AGENT);
        __syncthreads();
        if (*s_flag != (uint32_t)T.S - 1) return;
#pragma unroll 1
        for (int p = 0; p < 16; ++p) {
          unsigned long long *q = piece(p);
          f32x4 sum = {0.f, 0.f, 0.f, 0.f};
          if (q) {
            for (int s2 = 0; s2 < T.S; ++s2, q += 2 * per_slice) {
              const f32x2 lo = __builtin_bit_cast(f32x2, __hip_atomic_load(q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
              const f32x2 hi = __builtin_bit_cast(f32x2, __hip_atomic_load(q + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
              sum += f32x4{lo.x, lo.y, hi.x, hi.y};
            }
          }
          slot[p * WG_THREADS] = sum;
        }
        if (tid == 0)  // re-arm for the next launch
          __hip_atomic_store(&sp.arrive[T.out_tile_id], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
        for (int fn = 0; fn < 2; ++fn)
#pragma unroll
          for (int fm = 0; fm < 2; ++fm)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
              const f32x4 v = slot[((fn * 2 + fm) * 4 + j) * WG_THREADS];
              acc[fn][fm][4 * j] = v.x;
              acc[fn][fm][4 * j + 1] = v.y;
              acc[fn][fm][4 * j + 2] = v.z;
              acc[fn][fm][4 * j + 3] = v.w;
            }
      }

      // lane holds, per (fn, fm): row l32, columns 8*(i/4) + 4*half + (i%4)
#pragma unroll
      for (int fm = 0; fm < 2; ++fm) {
        const int m = mb + (wm * 2 + fm) * 32 + l32;
        if (m < m_end) {
          const int64_t row_off = P.nchw ? nchw_out_base(P, m) : (int64_t)m * P.ldc;
          const int64_t plane = (int64_t)P.Ho * P.Wo;
#pragma unroll
          for (int fn = 0; fn < 2; ++fn) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
              const int n = nb + (wn * 2 + fn) * 32 + 8 * j + 4 * half;
              if (n < n_end) {
                f32x4 v = {acc[fn][fm][4 * j], acc[fn][fm][4 * j + 1], acc[fn][fm][4 * j + 2], acc[fn][fm][4 * j + 3]};
                if (!P.nchw) {
                  store4<DT>(P.C, row_off, n, n_end, v, vec_c);
                } else {
                  // consecutive output channels lie a plane apart
#pragma unroll
                  for (int q = 0; q < 4; ++q)
                    if (n + q < n_end) store_elem<DT>(P.C, row_off + (int64_t)(n + q) * plane, v[q]);
                }
              }
            }
          }
        }
      }
    }
  }
}

template <int DT, bool ANY_ALIGNMENT>
__device__ __forceinline__ void run_class(const DevProblem &P, const sk_tile &T, const DevProblem *P_mem,
                                          const sk_tile *T_mem, const SplitK &sp, unsigned char *lds,
                                          uint32_t *s_flag, Prefetch &pf) {
  const int cls = T.cls;
  if (ANY_ALIGNMENT && (P.flags & (FLAG_VEC_A | FLAG_VEC_B)) != (FLAG_VEC_A | FLAG_VEC_B)) {
    if constexpr (ANY_ALIGNMENT) {
      pf.claim();
      pf.issue();
      // One output per thread costs a thread (outputs / 256) * Kg dependent steps of about 0.1 us; a stage
      // of 64 (fp32: 32) reduction elements through the matrix cores costs a few us whatever the
      // rectangle.  So only rectangles that are done in a few dozen steps go the first way.
      const int per_thread = ((int)T.m_len * (int)T.n_len + WG_THREADS - 1) / WG_THREADS;
      if ((int64_t)per_thread * P.Kg <= 64)
        run_generic<DT>(P_mem, T_mem);
      else
        run_tile_any<DT>(P_mem, T_mem, sp, lds, s_flag);
    }
  } else if (cls == 0) {
    run_skinny<DT, 1>(P, T, sp, lds, s_flag, pf);
  } else if (cls == 3) {
    run_skinny<DT, 2>(P, T, sp, lds, s_flag, pf);
  } else if (cls == 6) {
    run_skinny<DT, 4>(P, T, sp, lds, s_flag, pf);
  } else if (cls == CLS_TILE_128x64) {
    run_lds_tile<DT, 128, 64>(P, T, sp, lds, s_flag, pf);
  } else {
    run_lds_tile<DT, 128, 128>(P, T, sp, lds, s_flag, pf);
  }
}

// Sets the start stamp to all ones ahead of a stamped launch (a kernel, not a memset: launches may be
// captured into graphs).
__global__ void sk_arm_start_stamp(uint64_t *slot) { *slot = ~0ull; }

// ONLY_DT >= 0: every operator of the plan has that element type (one third of the
// code, fewer registers); ONLY_DT < 0: operators of mixed types.
// ANY_ALIGNMENT false: every operator can be read in aligned 16-byte pieces, and the kernel
// does not carry the paths for the others (their calls cost the fast paths registers and a
// stack); true: operators of either kind.
template <int ONLY_DT, bool ANY_ALIGNMENT>
__global__ void __launch_bounds__(WG_THREADS, 2) sk_superkernel(const TileWork *__restrict__ work, KernelArgs a) {
  __shared__ __attribute__((aligned(16))) unsigned char lds[LDS_TILE_BYTES];
  // next record by parity; behind it [0] its ticket, [1] flags (MAIL_*), [2] its index in xwork, [3] the ticket
  // that waits while it runs
  __shared__ __attribute__((aligned(16))) uint32_t s_mail[2][WORK_DWORDS + 4];
  __shared__ uint32_t s_flag;
  const SplitK sp{a.ws, a.ws_off, a.arrive};
  enum : uint32_t { MAIL_RUN = 1, MAIL_FROM_LIST = 2, MAIL_PENDING = 4, MAIL_OWES = 8 };

  // Start of the launch = the earliest first clock of any workgroup (the host has set the slot to all ones).
  if (a.write_start && a.stamps && threadIdx.x == 0)
    __hip_atomic_fetch_min((unsigned long long *)&a.stamps[a.n_problems], (unsigned long long)wall_clock64(),
                           __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);

  // Tickets and lists.  The queue hands out positions of the table in order ("tickets"); the first ticket of
  // a workgroup is its block index.  A ticket that falls on a skinny tile is that tile.  A ticket that
  // falls on an LDS tile only says that one LDS tile is due: which one, the workgroup takes from the list
  // of its die (the host has sorted every LDS tile of the table into one of eight lists so that tiles
  // sharing operand panels meet behind one L2; workgroups go to the dies round robin by block index), and
  // from the other dies' lists once its own is used up.  While an LDS tile runs, the next entry of the
  // list is drawn together with the next ticket (Prefetch), on the guess that the ticket falls on an LDS
  // tile again; if it falls on a skinny tile instead, the entry runs first and the ticket's tile right after
  // it (its record is fetched while the entry runs, no new ticket is taken).  Work that is bound to a
  // workgroup is thus always its very next tile: an entry held back until the workgroup's next LDS ticket
  // left dozens of workgroups with a tile still to run when the tickets ran out, and cost mixed plans a
  // tenth of their time.  Such an entry ran without a ticket: the workgroup owes one, and the next ticket of
  // its own that falls on an LDS tile stands for nothing (it takes another ticket at once, and draws nothing
  // in advance while it owes).  Without that the LDS tiles as a whole ran ahead of their tickets by one tile
  // per wrong guess, and the launch ended on long skinny tiles with nothing short left to fill in.  What is
  // still owed when the tickets run out shows as tickets that find every list empty.  Every entry is drawn
  // exactly once and run by the workgroup that drew it, so every tile of the table runs exactly once.
  const uint32_t last = a.tile_end - 1u;
  const bool lists = a.xoff != nullptr;
  const uint32_t die = blockIdx.x & 7u;
  uint32_t xbeg = 0, xlen = 0;
  if (lists) {
    xbeg = a.xoff[die];
    xlen = a.xoff[die + 1] - xbeg;
  }
  uint32_t used_up = xlen == 0 ? 1u << die : 0u;  // lists seen empty (wave 0's copy is the one that counts)
  bool owes = false;                               // an entry of a list has run without a ticket

  const int wave0 = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6)) == 0;
  const int lane0 = (int)(threadIdx.x & 63u);
  const int wlane = lane0 < WORK_DWORDS ? lane0 : 0;
  // What the tile just run fetched for the next one (Prefetch): lane 0 of `got` holds the ticket (less
  // `got_base`), lane 1 the entry drawn from the die's list if `drew`; `got_word` the record of the ticket,
  // or, if `drew`, the record of that entry with the ticket's tile class in lane 63.
  uint32_t got = blockIdx.x, got_base = a.tile_begin;
  uint32_t got_word = 0;
  if (wave0) got_word = as_global<uint32_t>(work + (a.tile_begin + blockIdx.x <= last ? a.tile_begin + blockIdx.x : last))[wlane];
  bool drew = false;
  bool have_done = false;  // a tile has just been run: its operator and that operator's tile count
  uint32_t done_problem = 0, done_count = 0;
  int par = 0;
#ifdef SK_DIAG_CLOCKS
  int diag_tile = 0;
#endif
  for (;;) {
    if (wave0) {
      // wave 0 decides what runs next and hands the record to the other waves
      uint32_t idx = (uint32_t)__builtin_amdgcn_readfirstlane((int)got) + got_base;
      uint32_t word = got_word, flags = 0, xi = 0, waits = 0;
      if (!lists) {
        flags = idx <= last ? MAIL_RUN : 0u;
      } else {
        const uint32_t k = drew ? (uint32_t)__builtin_amdgcn_readlane((int)got, 1) : 0u;
        bool drawn = drew && k < xlen;  // `word` is the record of entry k of the die's list
        if (drew && !drawn) used_up |= 1u << die;
        bool have_record = !drew;       // `word` is the table's record at the ticket
        for (;;) {
          const bool ticket = idx <= last;
          // the ticket's tile class: sk_tile's dword 1, low half
          const uint32_t cls = (uint32_t)__builtin_amdgcn_readlane((int)word, have_record ? 1 : 63) & 0xffffu;
          if (ticket && cls >= CLS_TILE_128x128) {
            if (owes) {  // this ticket pays for the entry that ran without one
              owes = false;
              uint32_t n2 = 0;
              if (lane0 == 0) n2 = atomicAdd(&a.counters[0], 1u);
              idx = (uint32_t)__builtin_amdgcn_readfirstlane((int)n2) + a.tile_begin + gridDim.x;
              word = as_global<uint32_t>(work + (idx <= last ? idx : last))[wlane];
              have_record = true;
              continue;
            }
            if (drawn) {
              xi = xbeg + k;
              flags = MAIL_RUN | MAIL_FROM_LIST;
              break;
            }
            // nothing in hand: draw now, from the own list first
            bool found = false;
            for (uint32_t d = 0; d < 8u && !found; ++d) {
              const uint32_t x2 = (die + d) & 7u;
              if ((used_up >> x2) & 1u) continue;
              const uint32_t b2 = a.xoff[x2], l2 = a.xoff[x2 + 1] - b2;
              uint32_t k2 = l2;
              if (l2 != 0 && lane0 == 0) k2 = atomicAdd(die_list_head(a.counters, x2), 1u);
              k2 = (uint32_t)__builtin_amdgcn_readfirstlane((int)k2);
              if (k2 < l2) {
                xi = b2 + k2;
                found = true;
              } else {
                used_up |= 1u << x2;
              }
            }
            if (found) {
              word = as_global<uint32_t>(a.xwork + xi)[wlane];
              flags = MAIL_RUN | MAIL_FROM_LIST;
              break;
            }
            // every list is empty: the tile this ticket stood for has run already; take the next ticket
            uint32_t n2 = 0;
            if (lane0 == 0) n2 = atomicAdd(&a.counters[0], 1u);
            idx = (uint32_t)__builtin_amdgcn_readfirstlane((int)n2) + a.tile_begin + gridDim.x;
            word = as_global<uint32_t>(work + (idx <= last ? idx : last))[wlane];
            have_record = true;
            continue;
          }
          if (ticket) {  // a skinny tile: the ticket is the tile
            if (drawn) {  // the entry drawn in advance runs first; the ticket's tile follows it
              xi = xbeg + k;
              waits = idx;
              owes = true;
              flags = MAIL_RUN | MAIL_FROM_LIST | MAIL_PENDING;
            } else {
              flags = MAIL_RUN;
              // (a draw that found the list used up has left no record of the ticket)
              if (!have_record) word = as_global<uint32_t>(work + idx)[wlane];
            }
            break;
          }
          // the tickets are used up: run what is still in hand
          idx = last;
          if (drawn) {
            xi = xbeg + k;
            flags = MAIL_RUN | MAIL_FROM_LIST;
          }
          break;
        }
        if (owes) flags |= MAIL_OWES;
      }
      if (lane0 < WORK_DWORDS) s_mail[par][lane0] = word;
      if (lane0 == 0) {
        s_mail[par][WORK_DWORDS] = idx;
        s_mail[par][WORK_DWORDS + 1] = flags;
        s_mail[par][WORK_DWORDS + 2] = xi;
        s_mail[par][WORK_DWORDS + 3] = waits;
      }
    }
    __syncthreads();
    if (a.remaining && have_done && threadIdx.x == 0) {
      // the workgroup that retires an operator's last tile stamps it and re-arms the count
      const uint32_t left = atomicSub(&a.remaining[done_problem], 1u);
      if (left == 1u) {
        a.stamps[done_problem] = wall_clock64();
        a.remaining[done_problem] = done_count;
      }
    }
    const uint32_t flags = (uint32_t)__builtin_amdgcn_readfirstlane((int)s_mail[par][WORK_DWORDS + 1]);
#ifdef SK_DIAG_CLOCKS
    if (have_done) {
      SK_DIAG(5);
      ++diag_tile;
    }
#endif
    if (!(flags & MAIL_RUN)) break;
    const uint32_t t = (uint32_t)__builtin_amdgcn_readfirstlane((int)s_mail[par][WORK_DWORDS]);
    const TileWork W = unpack_uniform<TileWork>(s_mail[par]);
    const TileWork *cur =
        (flags & MAIL_FROM_LIST) ? a.xwork + (uint32_t)__builtin_amdgcn_readfirstlane((int)s_mail[par][WORK_DWORDS + 2]) : work + t;
    const bool pending = (flags & MAIL_PENDING) != 0;  // a ticket waits: this tile takes no new one
    owes = (flags & MAIL_OWES) != 0;
    const uint32_t waits = (uint32_t)__builtin_amdgcn_readfirstlane((int)s_mail[par][WORK_DWORDS + 3]);
    par ^= 1;

    // Everything a tile derives from the thread index is derived again for each tile, from a
    // copy the compiler cannot see through: hoisted out of this loop those values would stay
    // live across all tile classes, spill, and every reload of a spilled register waits for all
    // the loads and stores in flight.
    int tid = threadIdx.x;
    asm volatile("" : "+v"(tid));
    const bool queue = a.dynamic && !pending;
    Prefetch pf{work, queue ? &a.counters[0] : nullptr, queue ? a.tile_begin + gridDim.x : 0u,
                pending ? waits : t + gridDim.x, last, tid};
    const sk_tile &T = W.tile;
    drew = lists && T.cls >= CLS_TILE_128x128 && !pending && !owes && !((used_up >> die) & 1u);
    if (drew) {
      pf.xhead = die_list_head(a.counters, die);
      pf.xrec = a.xwork + xbeg;
      pf.xlen = xlen;
    }
#ifdef SK_DIAG_CLOCKS
    pf.diag_tile = diag_tile;
#endif
    SK_DIAG(0);
#ifdef SK_DIAG_CLOCKS
    if (blockIdx.x < SK_DIAG_WGS && diag_tile < SK_DIAG_TILES && threadIdx.x == 0)
      g_diag[(blockIdx.x * SK_DIAG_TILES + diag_tile) * 8 + 6] = 1 + T.cls + 100ull * T.S;
    if (blockIdx.x < SK_DIAG_WGS && diag_tile < SK_DIAG_TILES && threadIdx.x == 0)
      g_diag[(blockIdx.x * SK_DIAG_TILES + diag_tile) * 8 + 7] = ((uint64_t)flags << 32) | t;  // how it was handed over, and the ticket
#endif
    const DevProblem &P = W.prob;
    if constexpr (ONLY_DT >= 0) {
      run_class<ONLY_DT, ANY_ALIGNMENT>(P, T, &cur->prob, &cur->tile, sp, lds, &s_flag, pf);
    } else {
      switch (P.dtype) {
        case SK_BF16: run_class<SK_BF16, ANY_ALIGNMENT>(P, T, &cur->prob, &cur->tile, sp, lds, &s_flag, pf); break;
        case SK_F16: run_class<SK_F16, ANY_ALIGNMENT>(P, T, &cur->prob, &cur->tile, sp, lds, &s_flag, pf); break;
        default: run_class<SK_F32, ANY_ALIGNMENT>(P, T, &cur->prob, &cur->tile, sp, lds, &s_flag, pf); break;
      }
    }

    if (a.remaining) __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    got = pf.next;
    got_base = pf.base;
    got_word = pf.word;
    have_done = true;
    done_problem = T.problem;
    done_count = (uint32_t)P.tile_count;
  }

  // the last workgroup to leave re-arms the queue for the next launch
  if (a.dynamic && threadIdx.x == 0) {
    const uint32_t done = atomicAdd(&a.counters[1], 1u);
    if (done == gridDim.x - 1) {
      a.counters[0] = 0u;
      a.counters[1] = 0u;
      if (lists)
        for (uint32_t x = 0; x < 8u; ++x) *die_list_head(a.counters, x) = 0u;
      __threadfence();
    }
  }
}

}  // namespace sk
