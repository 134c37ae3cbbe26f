// Building blocks of the bf16 MFMA attention kernels (gfx950, wave64).
//
// Matrix-core instruction used throughout: v_mfma_f32_32x32x16_bf16, D[32x32] += A[32x16] B[16x32].
// Register layouts (lane l, g = l / 32, c = l % 32):
//   A: lane holds row i = c,    k = 8g + t (t = 0..7, one 16-byte fragment)
//   B: lane holds column j = c, k = 8g + t
//   D: lane holds column j = c, rows i = 8*(r/4) + 4g + r%4 for register r = 0..15
// All kernels keep the QUERY index on the D column, so a softmax row lives in one lane pair
// (l, l^32) and its statistics need a single cross-lane exchange.
//
// A D tile becomes the B operand of the next contraction without any shuffle: registers
// 8h..8h+7 of lane group g hold rows {16h + 8(t/4) + 4g + t%4}, which is read as "k slot
// (g, t) of k-step h".  The matching A operand presents the same rows in the same slots through
// transposed LDS reads (lds_frag_tr below), so no tile is stored permuted.
#pragma once

#include "bsa_common.h"

namespace bsa {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

__device__ inline f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

__device__ inline bf16x8 lds_frag(const uint16_t* p) { return *reinterpret_cast<const bf16x8*>(p); }
__device__ inline bf16x8 as_frag(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

__device__ inline uint32_t pack_bf16(float lo, float hi) {
  typedef __attribute__((ext_vector_type(2))) float f32x2;
  typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
  f32x2 v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

// registers 8h..8h+7 of a D tile -> one bf16 B-operand fragment
__device__ inline bf16x8 d_to_b(const f32x16& d, int h) {
  u32x4 v;
  v.x = pack_bf16(d[8 * h + 0], d[8 * h + 1]);
  v.y = pack_bf16(d[8 * h + 2], d[8 * h + 3]);
  v.z = pack_bf16(d[8 * h + 4], d[8 * h + 5]);
  v.w = pack_bf16(d[8 * h + 6], d[8 * h + 7]);
  return as_frag(v);
}

// Make the compiler treat x as consumed here, so that the wait for the (global) loads that
// produce it is placed at this point.  Used on loop-invariant operands before a pipelined
// loop: otherwise their first use inside the loop forces a wait for ALL outstanding loads,
// including the prefetch issued a moment earlier, which serialises the pipeline.
template <typename T>
__device__ inline void settle(T& x) {
  asm volatile("" : "+v"(x));
}

// ---- LDS tile format of the pipelined kernels -------------------------------------------
// A tile is 64 rows of D bf16, rows unpadded (D*2 bytes).  The 16-byte chunk c of row r is
// stored at chunk position c ^ swz<D>(r).  The LDS of gfx950 has 64 four-byte banks (256
// bytes per cycle); the swizzle makes both access patterns below conflict free:
//   * row fragments (A operand with the tile row on the MFMA row index): ds_read_b128, a
//     pass of 16 lanes reads the same chunk of 16 consecutive rows -> swz must be a bijection
//     on r mod 16 (d = 128: a row is one 256-byte line) or on (r / 2) mod 8 (d = 64: two rows
//     per line);
//   * transposed fragments (A operand with the CHANNEL on the MFMA row index and 8 tile
//     rows as contraction slots): two ds_read_b64_tr_b16, a pass of 32 lanes reads 4 aligned
//     chunks of 4 consecutive rows -> those rows must differ in bits [3:2] of swz.
// Tiles arrive by global->LDS DMA (global_load_lds_dwordx4: lane i's 16 bytes land at LDS
// base + 16*i), so the swizzle is applied on the global side: the lane that fills LDS slot
// (r, p) fetches chunk p ^ swz<D>(r) of row r.
template <int D>
__host__ __device__ constexpr int swz(int r) {
  return D == 128 ? (((r & 3) << 2) | ((r >> 2) & 3)) : ((((r >> 1) & 1) << 2) | ((r >> 2) & 3));
}

typedef __attribute__((address_space(3))) void* lds_ptr_t;
typedef __attribute__((address_space(1))) const void* gbl_ptr_t;
typedef short s16x4 __attribute__((ext_vector_type(4)));

// 16 bytes per lane, global -> LDS, no registers; completion is counted by vmcnt.
// Issued as inline assembly on purpose: when the compiler knows of a pending LDS DMA it
// waits for vmcnt(0) before every barrier and every LDS read it cannot disambiguate, which
// would drain the whole prefetch ring each step.  The kernels order DMA against LDS reads
// themselves: "s_waitcnt vmcnt(n)" for the tile about to be read, then a barrier.
__device__ inline void dma16(const void* gsrc, void* lds_wave_base) {
  // the LDS base travels in M0, a scalar register: make its wave-uniformity explicit
  const uint32_t lds_addr = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(lds_ptr_t)lds_wave_base);
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
               :
               : "v"(gsrc), "s"(lds_addr)
               : "memory", "m0");
}

// The same with every wave-uniform part already in scalar registers: a 64-bit scalar base,
// a 32-bit per-lane byte offset and the LDS address.  No vector arithmetic per instruction.
// (readfirstlane returns a signed int: each half is widened as unsigned, or a low half with
// bit 31 set would sign-extend over the high half.)
__device__ inline uint64_t uniform64(const void* p) {
  const uint64_t b = (uint64_t)(uintptr_t)p;
  return ((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)(b >> 32)) << 32) |
         (uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)b);
}
__device__ inline uint32_t uniform_lds(void* p) {
  return (uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(lds_ptr_t)p);
}
__device__ inline void dma16_raw(uint64_t sbase, uint32_t lane_offset, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
               :
               : "v"(lane_offset), "s"(sbase), "s"(lds_addr)
               : "memory", "m0");
}

// Barrier without the memory fence of __syncthreads() (see dma16): callers pair it with
// explicit waits.  The empty asm statements stop the compiler moving LDS accesses across it.
__device__ inline void raw_barrier() {
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

// A fragment from two transposed reads (contraction slots 0..3 and 4..7).
__device__ inline bf16x8 lds_frag_tr(const uint8_t* p0, const uint8_t* p1) {
  typedef __attribute__((address_space(3))) s16x4* lp;
  const s16x4 a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lp)p0);
  const s16x4 b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lp)p1);
  typedef short s16x8 __attribute__((ext_vector_type(8)));
  const s16x8 v = {a[0], a[1], a[2], a[3], b[0], b[1], b[2], b[3]};
  return __builtin_bit_cast(bf16x8, v);
}

// Reductions over a lane pair (l, l ^ 32): one v_permlane32_swap puts the two halves of the
// wavefront side by side (r[0] = the low half's values in both halves, r[1] = the high half's),
// so every lane combines its own value with its partner's without a trip through LDS.
__device__ inline float pair_max(float v) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ inline float pair_sum(float v) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

}  // namespace bsa
