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

constexpr int LDS_LD = 72;  // bf16 elements per LDS tile row: 64 + 8 pad (144 B keeps 16-byte reads conflict-free)

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

// Padded-transposed token axis: segment s starts at tp_off[s] (multiple of 8);
// Tp = sum of round_up_8(seg_len).  Pad columns of a transposed buffer hold 0.
struct GeoT {
  int tp_off[IM_MAX_SEG + 1];
  int Tp;
};

// Stage a 64-row x 64-column bf16 tile from global memory into LDS (row stride
// LDS_LD) with 256 threads: two 16-byte loads per thread.
//   row r of the tile lives at  base + rowidx(r) * gstride  (rowidx clamps tails)
struct TileRegs {
  u32x4 v[2];
};

// rows = tokens: tile row r is token row min(r0 + r, rmax) of a [.., ld] activation matrix
__device__ __forceinline__ void load_rows_tile(TileRegs& t, const bf16_t* base, long ld, int r0, int rmax, int tid) {
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    const int r = (tid >> 3) + u * 32, c = (tid & 7) * 8;
    const int rr = min(r0 + r, rmax);
    t.v[u] = *(const u32x4*)(base + (long)rr * ld + c);
  }
}

// rows = channels, columns = tokens c0 .. c0+63 of a transposed [C, Tp] matrix;
// columns >= cmax are zero-filled (cmax relative to the same origin as c0).
__device__ __forceinline__ void load_cols_tile(TileRegs& t, const bf16_t* base, long tp, int c0, int cmax, int tid) {
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    const int r = (tid >> 3) + u * 32, c = c0 + (tid & 7) * 8;
    u32x4 v = {0u, 0u, 0u, 0u};
    if (c < cmax) {
      v = *(const u32x4*)(base + (long)r * tp + c);
      if (c + 8 > cmax) {
        const int keep = cmax - c;  // 1..7 valid elements
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const unsigned lo_ok = (2 * e < keep) ? 0xffffu : 0u, hi_ok = (2 * e + 1 < keep) ? 0xffff0000u : 0u;
          v[e] &= (lo_ok | hi_ok);
        }
      }
    }
    t.v[u] = v;
  }
}

__device__ __forceinline__ void store_tile(const TileRegs& t, bf16_t* lds, int tid) {
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    const int r = (tid >> 3) + u * 32, c = (tid & 7) * 8;
    *(u32x4*)(lds + r * LDS_LD + c) = t.v[u];
  }
}

__device__ __forceinline__ bf16x8 lds_frag(const bf16_t* lds, int row, int col) {
  return as_bf16x8(*(const u32x4*)(lds + row * LDS_LD + col));
}

}  // namespace imattn
