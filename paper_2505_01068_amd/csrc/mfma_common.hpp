// Device helpers for the bf16 MFMA kernels (gfx950, 64-wide wavefronts).
//
// Lane layout of v_mfma_f32_32x32x16_bf16 (checked on hardware), lane l,
// lo = l % 32, hi = l / 32:
//   A (32 x 16): lane holds row  m = lo, k = 8*hi .. 8*hi+7   (8 bf16, 16 bytes)
//   B (16 x 32): lane holds col  n = lo, k = 8*hi .. 8*hi+7
//   C (32 x 32): lane holds col  n = lo; register r = 4*i + j holds row 8*i + 4*hi + j
//
// "Row permutation": when the A rows of a 32-row block are fed in the order
// perm32(m) below, register r of the result on lane half `hi` belongs to the
// ACTUAL row 16*(r/8) + 8*hi + (r%8): registers 0..7 and 8..15 are then two runs
// of 8 consecutive rows, exactly the k-slots (8*hi .. 8*hi+7) a lane must supply
// as the B operand of the next MFMA.  This lets softmax probabilities go from
// the accumulator of one product into the operand of the next without leaving
// registers.
#pragma once
#include "common.hpp"

namespace imattn {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

constexpr int LDS_LD = 72;  // bf16 per row of a padded LDS tile (128 x 128 GEMM): 64 + 8 pad, 144 B keeps 16-byte reads conflict-free

__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// m (0..31) -> actual row fed as MFMA row m (see header comment)
__device__ __forceinline__ int perm32(int m) {
  const int i = m >> 3, h = (m >> 2) & 1, j = m & 3;
  return ((i >> 1) << 4) + (h << 3) + ((i & 1) << 2) + j;
}

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) {
  union { u32x4 u; bf16x8 b; } x;
  x.u = v;
  return x.b;
}

// pack two floats to two bf16 (round to nearest even) in one dword: low half = a
__device__ __forceinline__ unsigned pack_bf16(float a, float b) {
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  typedef float f32x2 __attribute__((ext_vector_type(2)));
  union { bf16x2 h; unsigned u; } x;
  f32x2 f = {a, b};
  x.h = __builtin_convertvector(f, bf16x2);
  return x.u;
}

__device__ __forceinline__ bf16x8 pack8(const float* v) {
  u32x4 u;
  u[0] = pack_bf16(v[0], v[1]);
  u[1] = pack_bf16(v[2], v[3]);
  u[2] = pack_bf16(v[4], v[5]);
  u[3] = pack_bf16(v[6], v[7]);
  return as_bf16x8(u);
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// acc + the sum of the eight bf16 values of v: four two-element dot products against (1, 1)
// (v_dot2c_f32_bf16), half the instructions of eight fp32 additions.
__device__ __forceinline__ float sum_bf16x8(bf16x8 v, float acc) {
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  union { bf16x8 v; bf16x2 h[4]; } x;
  x.v = v;
  const bf16x2 ones = __builtin_bit_cast(bf16x2, 0x3f803f80u);
#pragma unroll
  for (int i = 0; i < 4; ++i) acc = __builtin_amdgcn_fdot2_f32_bf16(x.h[i], ones, acc, false);
  return acc;
}

// Transposed fragment from a K-MAJOR tile (row = contraction index k, columns = m) using the
// gfx950 LDS transpose read.  ds_read_b64_tr_b16 exchanges data inside each group of 16 lanes:
// result[lane i][e] = data[lane 4e + i/4][i % 4] (checked on hardware), where data[lane j] are the
// four 16-bit elements lane j's address points at.  With lane j pointing at (row k0 + j/4,
// columns m0 + 4*(j%4) ..+3) a group reads a 4 x 16 block and lane i receives column m0 + i, rows
// k0..k0+3.  Two reads give the 8 consecutive k a 32x32x16 operand needs: lane l gets
// m = m_base + (l % 32), k = k_base + 8*(l / 32) + 0..7.
typedef short v4i16 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ bf16x8 lds_frag_tr(const bf16_t* lds, int ld, int k_base, int m_base, int lane) {
  const int j = lane & 15, g = lane >> 4;
  const bf16_t* p = lds + (k_base + 8 * (g >> 1) + (j >> 2)) * ld + m_base + 16 * (g & 1) + 4 * (j & 3);
  typedef v4i16 __attribute__((address_space(3))) * lds_v4_ptr;
  const v4i16 a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4_ptr)(p));
  const v4i16 b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4_ptr)(p + 4 * ld));
  union { v4i16 h[2]; bf16x8 v; } x;
  x.h[0] = a;
  x.h[1] = b;
  return x.v;
}

// The same fragment with the 32 columns in the order perm32 (lane lo receives column m_base + perm32(lo)): the
// columns of each group of 16 lanes are exchanged in blocks of four, which the transpose read does when the
// lanes' addresses point at the exchanged blocks.
__device__ __forceinline__ bf16x8 lds_frag_tr_perm(const bf16_t* lds, int ld, int k_base, int m_base, int lane) {
  const int j = lane & 15, g = lane >> 4, q = j & 3;
  const bf16_t* p = lds + (k_base + 8 * (g >> 1) + (j >> 2)) * ld + m_base + 16 * (g & 1) + 4 * (((q & 1) << 1) | (q >> 1));
  typedef v4i16 __attribute__((address_space(3))) * lds_v4_ptr;
  const v4i16 a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4_ptr)(p));
  const v4i16 b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4_ptr)(p + 4 * ld));
  union { v4i16 h[2]; bf16x8 v; } x;
  x.h[0] = a;
  x.h[1] = b;
  return x.v;
}

// ---- asynchronous global -> LDS copy ----
// One instruction moves 16 (or 4) bytes per lane from the lane's global address to LDS address
// (wave-uniform base) + 16 (or 4) * lane, with no staging register.  It counts in vmcnt like any
// load and completes in issue order.
// Written as inline assembly on purpose: when the compiler sees the corresponding builtin it
// treats every later LDS read as dependent on the copy and drains vmcnt to zero in front of it,
// which serialises a prefetch ring.  The kernels order the copies against their LDS reads
// themselves (s_waitcnt vmcnt(n) + workgroup barrier).  The compiler's own vmcnt bookkeeping for
// ordinary loads stays safe: the counter counts these copies too and returns are in order, so its
// waits can only be longer than it thinks, never shorter.  M0 is a reserved register: the compiler
// never keeps a value live in it across statements (it writes it immediately before each of its own
// uses) and warns that a clobber entry for a reserved register has no defined meaning, so none is listed.
__device__ __forceinline__ unsigned lds_offset(const void* lds_ptr) {  // wave-uniform by contract -> SGPR
  return (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)(uintptr_t)lds_ptr);
}
__device__ __forceinline__ void dma16(const void* gptr, const void* lds_wave_base) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
               :: "s"(lds_offset(lds_wave_base)), "v"(gptr) : "memory");
}
// same, global address = wave-uniform base + per-lane unsigned 32-bit byte offset
__device__ __forceinline__ void dma16_off(const void* gbase, unsigned byte_off, const void* lds_wave_base) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
               :: "s"(lds_offset(lds_wave_base)), "v"(byte_off), "s"(gbase) : "memory");
}
__device__ __forceinline__ void dma4_off(const void* gbase, unsigned byte_off, const void* lds_wave_base) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, %2"
               :: "s"(lds_offset(lds_wave_base)), "v"(byte_off), "s"(gbase) : "memory");
}
__device__ __forceinline__ void dma4(const void* gptr, const void* lds_wave_base) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, off"
               :: "s"(lds_offset(lds_wave_base)), "v"(gptr) : "memory");
}

// ---- swizzled, unpadded 64-column tiles (attention kernels) ----
// A tile row is 128 bytes = 8 chunks of 16 bytes; chunk c of row r is stored at chunk position
// c ^ sw_f(r).  sw_f depends on r % 16 only.  With it both access patterns below are free of bank
// conflicts (measured: 16-byte row reads ~250 B/clk/CU, transpose reads ~225 B/clk/CU, against 136
// B/clk/CU for transpose reads of rows padded to 144 bytes):
//  - 16-byte reads of one chunk column over 16 consecutive rows: (r & 1) picks the bank half and
//    the three bits of sw_f are a bijection of (r >> 1) & 7;
//  - transpose reads touch, per 32 lanes, rows r0..r0+3 (r0 % 4 == 0) x one aligned 64-byte span:
//    r and r+1 sit in opposite bank halves, r+2 moves the span by 64 bytes (bit 2 of sw_f).
constexpr int SW_LD = 64;
__device__ __forceinline__ int sw_f(int r) { return (((r >> 1) & 1) << 2) | ((r >> 2) & 3); }

// 16-byte fragment: row row16 + lrow (row16 % 16 == 0, 0 <= lrow < 32), chunk column `chunk`
__device__ __forceinline__ bf16x8 lds_frag_sw(const bf16_t* lds, int row16, int lrow, int chunk) {
  return as_bf16x8(*(const u32x4*)(lds + (row16 + lrow) * SW_LD + ((chunk ^ sw_f(lrow)) << 3)));
}

// transposed fragment as lds_frag_tr, from a swizzled tile; k_base % 16 == 0, m_base % 32 == 0
__device__ __forceinline__ bf16x8 lds_frag_tr_sw(const bf16_t* lds, int k_base, int m_base, int lane) {
  const int j = lane & 15, g = lane >> 4;
  const int lrow = 8 * (g >> 1) + (j >> 2);                  // second read: lrow + 4, i.e. sw_f ^ 1
  const int lchunk = 2 * (g & 1) + ((j & 3) >> 1), within = 4 * (j & 1);
  const int f = sw_f(lrow);
  const int mb = m_base >> 3;
  typedef v4i16 __attribute__((address_space(3))) * lds_v4_ptr;
  const bf16_t* p0 = lds + (k_base + lrow) * SW_LD + (((mb | lchunk) ^ f) << 3) + within;
  const bf16_t* p1 = lds + (k_base + lrow + 4) * SW_LD + (((mb | lchunk) ^ f ^ 1) << 3) + within;
  const v4i16 a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4_ptr)(p0));
  const v4i16 b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4_ptr)(p1));
  union { v4i16 h[2]; bf16x8 v; } x;
  x.h[0] = a;
  x.h[1] = b;
  return x.v;
}

__device__ __forceinline__ bf16x8 lds_frag(const bf16_t* lds, int row, int col) {
  return as_bf16x8(*(const u32x4*)(lds + row * LDS_LD + col));
}

}  // namespace imattn
