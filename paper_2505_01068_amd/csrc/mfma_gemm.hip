// bf16 MFMA GEMM  C[M,N] = sum_k A(m,k) B(n,k), fp32 accumulation, for the
// projections around IM attention at model widths that fill the matrix cores.
//
// Workgroup tile 128 x 128 x 64, four waves in a 2 x 2 grid, each wave 64 x 64 as
// 2 x 2 v_mfma_f32_32x32x16_bf16 blocks.  The MFMA "A" operand is fed from the
// B tile and the "B" operand from the A tile, i.e. the wave computes C^T: each
// lane then owns one output ROW m and four consecutive columns per register
// quad (8-byte row-major stores).
//
// Either operand may be stored m-major (rows = m, K contiguous: activations as
// the left operand, weights used transposed) or k-major (rows = k: weights
// [d_in, d_out] in the forward, and BOTH operands of the weight gradients
// x^T dQ whose contraction runs over token rows).  k-major tiles are staged
// row-major and read with the LDS transpose read, so no operand is ever
// transposed in HBM.  Further variants by descriptor: three B matrices
// partitioning N (k-major) or K (m-major), deterministic split-K with a
// fixed-order reduction, bias / residual / GELU epilogues.
#include "mfma_common.hpp"
#include "mfma_path.hpp"

namespace imattn {

constexpr int GM = 128, GN = 128, GK = 64;
constexpr int KM_LD = 160;  // row stride (bf16) of a k-major LDS tile: 128 + 32 pad -> conflict-free transpose reads

__device__ __forceinline__ float gelu_exact_f(float x) { return 0.5f * x * (1.f + erff(x * 0.70710678118654752440f)); }

struct Tile128 {
  u32x4 v[4];
};

// m-major operand: tile rows r0..r0+127 (clamped to rmax), K columns c0..c0+63 (zero beyond cmax)
__device__ __forceinline__ void load_mm(Tile128& t, const bf16_t* base, long ld, int r0, int rmax, int c0, int cmax,
                                        int tid) {
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int r = (tid >> 3) + u * 32, c = c0 + (tid & 7) * 8;
    const int rr = min(r0 + r, rmax);
    u32x4 v = {0u, 0u, 0u, 0u};
    if (c < cmax) v = *(const u32x4*)(base + (long)rr * ld + c);  // K is a multiple of 8 for every caller
    t.v[u] = v;
  }
}
__device__ __forceinline__ void store_mm(const Tile128& t, bf16_t* lds, int tid) {
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int r = (tid >> 3) + u * 32, c = (tid & 7) * 8;
    *(u32x4*)(lds + r * LDS_LD + c) = t.v[u];
  }
}
// k-major operand: tile rows k0..k0+63 (zero beyond kmax), columns c0..c0+127 (zero beyond cmax);
// the columns may be spread over up to three matrices of n_per columns each
__device__ __forceinline__ void load_km(Tile128& t, const bf16_t* const* mats, int n_per, long ld, int k0, int kmax,
                                        int c0, int cmax, int tid) {
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int r = (tid >> 4) + u * 16, c = c0 + (tid & 15) * 8;
    u32x4 v = {0u, 0u, 0u, 0u};
    if (k0 + r < kmax && c < cmax) {
      const bf16_t* m = mats[0];
      int cc = c;
      if (n_per > 0) { m = mats[c / n_per]; cc = c % n_per; }
      v = *(const u32x4*)(m + (long)(k0 + r) * ld + cc);
    }
    t.v[u] = v;
  }
}
__device__ __forceinline__ void store_km(const Tile128& t, bf16_t* lds, int tid) {
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int r = (tid >> 4) + u * 16, c = (tid & 15) * 8;
    *(u32x4*)(lds + r * KM_LD + c) = t.v[u];
  }
}

template <bool AKM, bool BKM>
__global__ __launch_bounds__(256) void mfma_gemm_kernel(MGemm p) {
  __shared__ __attribute__((aligned(16))) bf16_t sA[AKM ? GK * KM_LD : GM * LDS_LD];
  __shared__ __attribute__((aligned(16))) bf16_t sB[BKM ? GK * KM_LD : GN * LDS_LD];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, lo = lane & 31, hi = lane >> 5;
  const int wm = wave >> 1, wn = wave & 1;
  int bx, by, bz;
  xcd_block_index(bx, by, bz);
  const int m0 = by * GM, n0 = bx * GN;

  const int ktiles = (p.K + GK - 1) / GK;
  const int per_split = (ktiles + p.split_k - 1) / p.split_k;
  const int it_begin = bz * per_split, it_end = min(ktiles, it_begin + per_split);

  f32x16 acc[2][2];  // [n block][m block]: rows of the accumulator = n, cols = m
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;

  const bf16_t* amat[3] = {p.A, p.A, p.A};
  const bf16_t* bmat[3] = {p.B[0], p.B[1], p.B[2]};
  Tile128 ta, tb;
  auto prefetch = [&](int it) {
    const int k0 = it * GK;
    if (AKM) load_km(ta, amat, 0, p.lda, k0, p.K, m0, p.M, tid);
    else load_mm(ta, p.A, p.lda, m0, p.M - 1, k0, p.K, tid);
    if (BKM) {
      load_km(tb, bmat, p.b_nper, p.ldb, k0, p.K, n0, p.N, tid);
    } else {
      const bf16_t* Bp = p.B[0];
      int kk = k0, kmax = p.K;
      if (p.b_kper > 0) { Bp = p.B[k0 / p.b_kper]; kk = k0 % p.b_kper; kmax = p.b_kper; }
      load_mm(tb, Bp, p.ldb, n0, p.N - 1, kk, kmax, tid);
    }
  };
  if (it_begin < it_end) prefetch(it_begin);
  for (int it = it_begin; it < it_end; ++it) {
    __syncthreads();
    if (AKM) store_km(ta, sA, tid); else store_mm(ta, sA, tid);
    if (BKM) store_km(tb, sB, tid); else store_mm(tb, sB, tid);
    __syncthreads();
    if (it + 1 < it_end) prefetch(it + 1);
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      bf16x8 fa[2], fb[2];
#pragma unroll
      for (int x = 0; x < 2; ++x) {
        fa[x] = AKM ? lds_frag_tr(sA, KM_LD, s * 16, wm * 64 + x * 32, lane)
                    : lds_frag(sA, wm * 64 + x * 32 + lo, s * 16 + hi * 8);
        fb[x] = BKM ? lds_frag_tr(sB, KM_LD, s * 16, wn * 64 + x * 32, lane)
                    : lds_frag(sB, wn * 64 + x * 32 + lo, s * 16 + hi * 8);
      }
#pragma unroll
      for (int nb = 0; nb < 2; ++nb)
#pragma unroll
        for (int mb = 0; mb < 2; ++mb) acc[nb][mb] = mfma32(fb[nb], fa[mb], acc[nb][mb]);
    }
  }

  // ---- epilogue: lane owns row m; registers 4i..4i+3 are columns n = 8i + 4hi + 0..3 of the block ----
#pragma unroll
  for (int mb = 0; mb < 2; ++mb) {
    const int m = m0 + wm * 64 + mb * 32 + lo;
    if (m >= p.M) continue;
#pragma unroll
    for (int nb = 0; nb < 2; ++nb)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int n = n0 + wn * 64 + nb * 32 + 8 * i + 4 * hi;
        if (n >= p.N) continue;  // N is a multiple of 4 for every caller
        float v[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) v[j] = acc[nb][mb][4 * i + j];
        if (p.partial) {
          *(float4*)(p.partial + ((long)bz * p.M + m) * p.N + n) = make_float4(v[0], v[1], v[2], v[3]);
          continue;
        }
        if (p.n_per > 0) {
          const int sel = n / p.n_per, nn = n % p.n_per;
          if (p.bias[sel]) {
#pragma unroll
            for (int j = 0; j < 4; ++j) v[j] += bf2f(p.bias[sel][nn + j]);
          }
        }
        if (p.gelu) {
#pragma unroll
          for (int j = 0; j < 4; ++j) v[j] = gelu_exact_f(v[j]);
        }
        if (p.res) {
          const u32x2 rv = *(const u32x2*)(p.res + (long)m * p.ldc + n);
          v[0] += __uint_as_float(rv[0] << 16); v[1] += __uint_as_float(rv[0] & 0xffff0000u);
          v[2] += __uint_as_float(rv[1] << 16); v[3] += __uint_as_float(rv[1] & 0xffff0000u);
        }
        const u32x2 pk = {pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3])};
        *(u32x2*)(p.C + (long)m * p.ldc + n) = pk;
      }
  }
}

// partial[z][M][N] -> out (fp32), z summed in fixed order; output column blocks may go to 3 matrices
__global__ void mfma_splitk_reduce_kernel(const float* partial, int split_k, int M, int N, float* o0, float* o1,
                                          float* o2, int n_per) {
  const long n_out = (long)M * N;
  for (long i = blockIdx.x * (long)blockDim.x + threadIdx.x; i < n_out; i += (long)gridDim.x * blockDim.x) {
    float s = 0.f;
    for (int z = 0; z < split_k; ++z) s += partial[z * n_out + i];
    const int m = i / N, n = i % N;
    if (n_per > 0) {
      float* o = (n / n_per == 0) ? o0 : (n / n_per == 1) ? o1 : o2;
      if (o) o[(long)m * n_per + n % n_per] = s;
    } else {
      o0[i] = s;
    }
  }
}

int mfma_gemm_split(int M, int N, int K) {
  const long tiles = (long)((M + GM - 1) / GM) * ((N + GN - 1) / GN);
  const int ktiles = (K + GK - 1) / GK;
  if (tiles >= 256 || ktiles < 16) return 1;
  int s = (int)((512 + tiles - 1) / tiles);
  if (s > ktiles / 4) s = ktiles / 4;
  return s < 1 ? 1 : s;
}

void launch_mfma_gemm(const MGemm& p, hipStream_t st) {
  dim3 grid((p.N + GN - 1) / GN, (p.M + GM - 1) / GM, p.split_k);
  if (p.a_kmajor && p.b_kmajor) hipLaunchKernelGGL((mfma_gemm_kernel<true, true>), grid, dim3(256), 0, st, p);
  else if (p.b_kmajor) hipLaunchKernelGGL((mfma_gemm_kernel<false, true>), grid, dim3(256), 0, st, p);
  else if (p.a_kmajor) hipLaunchKernelGGL((mfma_gemm_kernel<true, false>), grid, dim3(256), 0, st, p);
  else hipLaunchKernelGGL((mfma_gemm_kernel<false, false>), grid, dim3(256), 0, st, p);
}
void launch_splitk_reduce(const float* partial, int split_k, int M, int N, float* o0, float* o1, float* o2, int n_per,
                          hipStream_t st) {
  hipLaunchKernelGGL(mfma_splitk_reduce_kernel, dim3(256), dim3(256), 0, st, partial, split_k, M, N, o0, o1, o2, n_per);
}

}  // namespace imattn
