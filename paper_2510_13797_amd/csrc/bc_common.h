// Shared device/host helpers for the gfx950 kernels (wave64 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/bc.h"

namespace bc {

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;

struct bf16_t { uint16_t bits; };   // storage tag for bf16 rows

constexpr float kNegBig = -1.0e30f;            // finite stand-in for -inf in running maxima
constexpr float kLog2e = 1.4426950408889634f;

template <typename T> struct Elem;
template <> struct Elem<float>  { static constexpr int size = 4; static constexpr int per16 = 4; };
template <> struct Elem<bf16_t> { static constexpr int size = 2; static constexpr int per16 = 8; };

// 2^x by the hardware instruction (inputs here are <= 0 or moderate; -1e30 gives 0)
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Swizzle of the 16-byte units of a 256-byte tile row in LDS (tiles of 32 rows): unit u of row
// `row` lives at position u ^ lds_swz(row).  Chosen so that both access patterns of the MFMA
// operands are conflict-free: the 128-bit reads of one unit from the 16 rows {a + 8b} get 16
// different positions, and the transposing 64-bit reads, which take two adjacent units from
// the 8 rows {a + 8*b0} per half wave, get 8 different unit pairs.
__device__ __forceinline__ int lds_swz(int row) {
  return ((row & 3) << 1) | (((row >> 3) & 1) << 3) | ((row >> 4) & 1);
}

// Swizzle of the 16-byte units of a tile row in LDS: unit u of row `row` lives at position
// u ^ tile_swz<D>(row).  D = 128 (16 units per row): lds_swz.  D = 64 (8 units per row, two rows
// per 256 bytes of banks): the 128-bit reads of one unit from the 8 rows {a, a+1, a+2, a+3, a+8,
// .., a+11} must hit 8 different 16-byte bank groups - the row parity gives two, bits 1 and 3 of
// the row the other four - and the transposing 64-bit reads of a half wave (rows {a..a+3} and
// {a+8..a+11}, two adjacent units each) the 32 different 8-byte slots, which the same bits give.
template <int D> __device__ __forceinline__ int tile_swz(int row);
template <> __device__ __forceinline__ int tile_swz<128>(int row) { return lds_swz(row); }
template <> __device__ __forceinline__ int tile_swz<64>(int row) {
  return (((row >> 1) & 1) << 1) | (((row >> 3) & 1) << 2);
}

// A wait for the wave's vector-memory counter with a count known at compile time (the
// instruction takes an immediate).
template <int N> __device__ __forceinline__ void wait_vmcnt() {
  static_assert(N >= 0 && N <= 40, "counts used by the kernels");
  if constexpr (N == 0) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  else if constexpr (N == 2) asm volatile("s_waitcnt vmcnt(2)" ::: "memory");
  else if constexpr (N == 3) asm volatile("s_waitcnt vmcnt(3)" ::: "memory");
  else if constexpr (N == 4) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
  else if constexpr (N == 5) asm volatile("s_waitcnt vmcnt(5)" ::: "memory");
  else if constexpr (N == 8) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
  else if constexpr (N == 12) asm volatile("s_waitcnt vmcnt(12)" ::: "memory");
  else if constexpr (N == 16) asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
  else if constexpr (N == 20) asm volatile("s_waitcnt vmcnt(20)" ::: "memory");
  else if constexpr (N == 24) asm volatile("s_waitcnt vmcnt(24)" ::: "memory");
  else static_assert(N < 0, "add the count");
}

// x minus one half of the bf16 pair hp, exactly, in one instruction: the bf16 dot product with a
// selector pair that holds -1 in that half and 0 in the other, accumulated onto x.  Used to split
// an fp32 value into two bf16 parts (hp holds the rounded high parts of two values).  The
// selectors must sit in registers: as an immediate the assembler encodes the pair as a 32-bit
// constant, which the instruction does not read as a pair.
struct HalfSelectors { uint32_t low, high; };
__device__ __forceinline__ HalfSelectors half_selectors() {
  uint32_t low = 0x0000bf80u, high = 0xbf800000u;          // (-1, 0) and (0, -1) as bf16 pairs
  asm volatile("" : "+s"(low), "+s"(high));                // opaque: stay in scalar registers
  return HalfSelectors{low, high};
}
// two floats -> one bf16 pair (round to nearest even, a in the low half)
__device__ __forceinline__ uint32_t pack2_bf16(float a, float b) {
  typedef __attribute__((ext_vector_type(2))) float f32x2_t_;
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2_t_{a, b}, bf16x2_t));
}
__device__ __forceinline__ float minus_half(float x, uint32_t hp, uint32_t selector) {
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, hp),
                                         __builtin_bit_cast(bf16x2_t, selector), x, false);
}

// One LDS-DMA instruction: every lane's 16 bytes at g go to LDS at lds_addr + 16 * lane (lds_addr
// the same for all lanes; the instruction takes it from M0).  Written out by hand so that the
// compiler does not know about it: it cannot tell which LDS reads such a load feeds and would
// put a wait for ALL outstanding loads (the next tiles' among them, and the fused decode step's
// ticket) in front of the tile reads in every pass of a tile loop.  The waits are the explicit ones in
// the kernel.  (M0 is not named as clobbered - the compiler reserves it and says so - and nothing
// else in these kernels uses it.)
template <bool STREAM>
__device__ __forceinline__ void lds_dma16(const char* g, const char* lds_dst) {
  const uint32_t a = __builtin_amdgcn_readfirstlane(
      (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const char*)lds_dst);
  if (STREAM)
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off nt"
                 : : "s"(a), "v"(g) : "memory");
  else
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
                 : : "s"(a), "v"(g) : "memory");
}

// The same with the address given as a base in scalar registers plus a 32-bit byte offset per lane
// and the LDS address as a number: no 64-bit vector arithmetic and no pointer conversion per
// instruction, which is what the issue rate of a tile's loads is bound by otherwise.
template <bool STREAM>
__device__ __forceinline__ void lds_dma16_s(uint32_t lane_offset, uint64_t base, uint32_t lds_addr) {
  if (STREAM)
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2 nt"
                 : : "s"(lds_addr), "v"(lane_offset), "s"(base) : "memory");
  else
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 : : "s"(lds_addr), "v"(lane_offset), "s"(base) : "memory");
}
// The number an LDS pointer stands for (uniform over the wave).
__device__ __forceinline__ uint32_t lds_address(const char* lds_ptr) {
  return __builtin_amdgcn_readfirstlane(
      (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const char*)lds_ptr);
}

// A 16-byte load into registers that the compiler does not count either (same reason).  The value
// is there only after an explicit wait: nothing may read the result before it.
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;
template <bool STREAM>
__device__ __forceinline__ void load16_uncounted(u32x4_t& dst, const char* g) {
  if (STREAM) asm volatile("global_load_dwordx4 %0, %1, off nt" : "=v"(dst) : "v"(g) : "memory");
  else asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(dst) : "v"(g) : "memory");
}
template <bool STREAM>
__device__ __forceinline__ void load16_uncounted_s(u32x4_t& dst, uint32_t lane_offset, uint64_t base) {
  if (STREAM) asm volatile("global_load_dwordx4 %0, %1, %2 nt" : "=v"(dst) : "v"(lane_offset), "s"(base) : "memory");
  else asm volatile("global_load_dwordx4 %0, %1, %2" : "=v"(dst) : "v"(lane_offset), "s"(base) : "memory");
}
// The point from which such a register may be used: right behind the explicit wait that covers its
// load.  Emits no instruction (the comment names the register for the check of the generated code:
// nothing may touch it between its load and this point).  The register is an input only: an
// in-out operand would make the mark a new definition, and the compiler joins the definitions of
// several marks of one variable by register copies - some of them in front of the wait.
template <typename R>
__device__ __forceinline__ void landed(const R& reg) {
  asm volatile("; landed %0" : : "v"(reg) : "memory");
}

// 16 bytes of a row -> floats
__device__ __forceinline__ void unpack16(const uint4& r, float (&f)[4], float) {
  f[0] = __uint_as_float(r.x); f[1] = __uint_as_float(r.y);
  f[2] = __uint_as_float(r.z); f[3] = __uint_as_float(r.w);
}
__device__ __forceinline__ void unpack16(const uint4& r, float (&f)[8], bf16_t) {
  f[0] = __uint_as_float(r.x << 16); f[1] = __uint_as_float(r.x & 0xffff0000u);
  f[2] = __uint_as_float(r.y << 16); f[3] = __uint_as_float(r.y & 0xffff0000u);
  f[4] = __uint_as_float(r.z << 16); f[5] = __uint_as_float(r.z & 0xffff0000u);
  f[6] = __uint_as_float(r.w << 16); f[7] = __uint_as_float(r.w & 0xffff0000u);
}

// x + (x of another lane), lane chosen by a DPP control word (row = 16 lanes)
template <int CTRL>
__device__ __forceinline__ float dpp_add(float x) {
  int y = __builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xf, 0xf, true);
  return x + __int_as_float(y);
}
constexpr int kDppXor1 = 0xB1;        // quad_perm [1,0,3,2]
constexpr int kDppXor2 = 0x4E;        // quad_perm [2,3,0,1]
constexpr int kDppHalfMirror = 0x141; // lane i <-> 7-i inside each 8
constexpr int kDppMirror = 0x140;     // lane i <-> 15-i inside each 16

// Sum over groups of LPR consecutive lanes; every lane of a group gets the sum.
// After the two quad steps all lanes of a quad agree, so the mirrors act as xor 4 / xor 8.
template <int LPR>
__device__ __forceinline__ float group_allreduce_sum(float x) {
  static_assert(LPR == 8 || LPR == 16 || LPR == 32, "lanes per row");
  x = dpp_add<kDppXor1>(x);
  x = dpp_add<kDppXor2>(x);
  x = dpp_add<kDppHalfMirror>(x);
  if (LPR >= 16) x = dpp_add<kDppMirror>(x);
  if (LPR >= 32) x += __shfl_xor(x, 16, 64);
  return x;
}

// All-reduce over the four 16-lane rows of a wave (lane l with l ^ 16 and l ^ 32) by the two
// row-swap instructions of gfx950 instead of two LDS-routed shuffles.  permlane16_swap(x, x)
// returns {rows 0,0,2,2 ; rows 1,1,3,3} of x, permlane32_swap(y, y) {lower half twice ; upper
// half twice}, so combining the two results of each gives every lane the value over all rows.
__device__ __forceinline__ float rows_allreduce_max(float x) {
  const uint32_t u = __float_as_uint(x);
  const auto a = __builtin_amdgcn_permlane16_swap(u, u, false, false);
  const uint32_t v = __float_as_uint(fmaxf(__uint_as_float(a[0]), __uint_as_float(a[1])));
  const auto b = __builtin_amdgcn_permlane32_swap(v, v, false, false);
  return fmaxf(__uint_as_float(b[0]), __uint_as_float(b[1]));
}
__device__ __forceinline__ float rows_allreduce_sum(float x) {
  const uint32_t u = __float_as_uint(x);
  const auto a = __builtin_amdgcn_permlane16_swap(u, u, false, false);
  const uint32_t v = __float_as_uint(__uint_as_float(a[0]) + __uint_as_float(a[1]));
  const auto b = __builtin_amdgcn_permlane32_swap(v, v, false, false);
  return __uint_as_float(b[0]) + __uint_as_float(b[1]);
}

inline hipStream_t as_stream(void* s) { return reinterpret_cast<hipStream_t>(s); }

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// x > 0 and finite, decided on the bit pattern: a floating-point comparison would let a NaN
// through in files built with the assumption that NaNs do not occur.
inline bool positive_finite(float x) {
  uint32_t u;
  __builtin_memcpy(&u, &x, sizeof(u));
  return u > 0u && u < 0x7f800000u;
}
inline bool nonnegative_finite(float x) {      // either zero included
  uint32_t u;
  __builtin_memcpy(&u, &x, sizeof(u));
  return u < 0x7f800000u || u == 0x80000000u;
}

inline int32_t check_shape(const bc_shape* sh) {
  if (!sh) return BC_ERR_ARG;
  if (sh->B < 1 || sh->Hq < 1 || sh->Hkv < 1) return BC_ERR_SHAPE;
  if (sh->Hq % sh->Hkv != 0 || sh->Hq / sh->Hkv > 8) return BC_ERR_SHAPE;
  if (sh->d != 64 && sh->d != 128) return BC_ERR_SHAPE;
  if (sh->kv_dtype != BC_F32 && sh->kv_dtype != BC_BF16) return BC_ERR_SHAPE;
  return BC_OK;
}

inline int32_t check_cache(const bc_cache* c) {
  if (!c || !c->k_slab || !c->v_slab || !c->base || !c->cap || !c->P || !c->c || !c->nb ||
      !c->w || !c->err)
    return BC_ERR_ARG;
  if (!aligned16(c->k_slab) || !aligned16(c->v_slab)) return BC_ERR_ARG;
  if (c->max_cap < 1) return BC_ERR_ARG;
  if (c->uniform_P < 0 || c->uniform_cap < 0) return BC_ERR_ARG;
  if (c->uniform_P > 0 && (c->uniform_cap != c->max_cap || c->uniform_P > c->uniform_cap)) return BC_ERR_ARG;
  return BC_OK;
}

inline int elem_size(int32_t dtype) { return dtype == BC_BF16 ? 2 : 4; }

inline int32_t launch_status() {
  return hipGetLastError() == hipSuccess ? BC_OK : BC_ERR_HIP;
}

// Row offsets divided by the window stride c + 1 (Fig. 2: c tokens and their beacon), for
// offsets below 2^26.  The multiplier is floor(2^32 / stride) + 1, so the product's high word
// overestimates offset / stride by less than offset / 2^32 < 1/64: it is the quotient, or one
// more - and never more while rows * stride fits in 32 bits, which `exact` records (uniform, so
// the correction is skipped by a scalar branch at the paper's ratios).  Ratios beyond any row
// count behave like 2^26: no window ever closes.
struct WindowStride {
  int c, stride;
  uint32_t magic;
  bool exact;
};
__device__ __forceinline__ WindowStride window_stride(int c_table, int rows) {
  WindowStride ws;
  ws.c = min(c_table, 1 << 26);
  ws.stride = ws.c + 1;
  ws.magic = ws.c > 0 ? (uint32_t)(0x100000000ull / (uint32_t)ws.stride) + 1u : 0u;
  ws.exact = (uint64_t)(uint32_t)max(rows, 0) * (uint32_t)max(ws.stride, 1) < 0x100000000ull;
  return ws;
}
__device__ __forceinline__ uint32_t window_of(const WindowStride& ws, uint32_t offset) {
  uint32_t q = __umulhi(offset, ws.magic);
  if (!ws.exact) q -= (q * (uint32_t)ws.stride > offset) ? 1u : 0u;
  return q;
}

}  // namespace bc
