// bf16 MFMA GEMM  C[M,N] = A[M,K] * B[N,K]^T  (both operands K-contiguous), fp32
// accumulation, for the projections around IM attention at model widths that
// fill the matrix cores (d a multiple of 64).
//
// Workgroup tile 128 x 128 x 64, four waves in a 2 x 2 grid, each wave 64 x 64 as
// 2 x 2 v_mfma_f32_32x32x16_bf16 blocks.  The MFMA "A" operand is fed from the
// B tile and the "B" operand from the A tile, i.e. the wave computes C^T: each
// lane then owns one output ROW m and four consecutive columns per register
// quad, so row-major stores are 8 bytes per lane and stores into the
// token-transposed copy ([B, C, Tp]) run along consecutive tokens.
//
// Variants selected by the descriptor: up to three B matrices partitioning K
// (dx = [dQ|dK|dV] [Wq|Wk|Wv]^T), K running over `kb` batches of `kt` columns
// (weight gradients over the padded token axis), deterministic split-K with a
// fixed-order reduction, bias / residual / GELU epilogues, and an optional second
// output transposed per batch element.
#include "mfma_common.hpp"
#include "mfma_path.hpp"

namespace imattn {

constexpr int GM = 128, GN = 128, GK = 64;

__device__ __forceinline__ float gelu_exact_f(float x) { return 0.5f * x * (1.f + erff(x * 0.70710678118654752440f)); }

// 128 rows x 64 cols: 4 x 16-byte loads per thread; rows >= rmax clamp, cols >= cmax zero
struct Tile128 {
  u32x4 v[4];
};
__device__ __forceinline__ void load128(Tile128& t, const bf16_t* base, long ld, int r0, int rmax, int c0, int cmax,
                                        int tid) {
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int r = (tid >> 3) + u * 32, c = c0 + (tid & 7) * 8;
    const int rr = min(r0 + r, rmax);
    u32x4 v = {0u, 0u, 0u, 0u};
    if (c < cmax) {
      v = *(const u32x4*)(base + (long)rr * ld + c);
      if (c + 8 > cmax) {
        const int keep = cmax - c;
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
__device__ __forceinline__ void store128(const Tile128& t, bf16_t* lds, int tid) {
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int r = (tid >> 3) + u * 32, c = (tid & 7) * 8;
    *(u32x4*)(lds + r * LDS_LD + c) = t.v[u];
  }
}

__global__ __launch_bounds__(256) void mfma_gemm_kernel(MGemm p) {
  __shared__ __attribute__((aligned(16))) bf16_t sA[GM * LDS_LD];
  __shared__ __attribute__((aligned(16))) bf16_t sB[GN * LDS_LD];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, lo = lane & 31, hi = lane >> 5;
  const int wm = wave >> 1, wn = wave & 1;
  const int m0 = blockIdx.y * GM, n0 = blockIdx.x * GN;

  // the K loop runs over (batch, k-tile) pairs; this split takes a contiguous range of them
  const int tiles_per_batch = (p.kt + GK - 1) / GK;
  const int total = p.kb * tiles_per_batch;
  const int per_split = (total + p.split_k - 1) / p.split_k;
  const int it_begin = blockIdx.z * per_split, it_end = min(total, it_begin + per_split);

  f32x16 acc[2][2];  // [n block][m block]: rows of the accumulator = n, cols = m
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;

  Tile128 ta, tb;
  auto prefetch = [&](int it) {
    const int bb = it / tiles_per_batch, k0 = (it % tiles_per_batch) * GK;
    load128(ta, p.A + (long)bb * p.a_bs, p.lda, m0, p.M - 1, k0, p.kt, tid);
    const bf16_t* Bp = p.B[0];
    int kk = k0;
    if (p.b_kper > 0) { Bp = p.B[k0 / p.b_kper]; kk = k0 % p.b_kper; }
    load128(tb, Bp + (long)bb * p.b_bs, p.ldb, n0, p.N - 1, kk, p.b_kper > 0 ? p.b_kper : p.kt, tid);
  };
  if (it_begin < it_end) prefetch(it_begin);
  for (int it = it_begin; it < it_end; ++it) {
    __syncthreads();
    store128(ta, sA, tid);
    store128(tb, sB, tid);
    __syncthreads();
    if (it + 1 < it_end) prefetch(it + 1);
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      bf16x8 fa[2], fb[2];
#pragma unroll
      for (int x = 0; x < 2; ++x) {
        fa[x] = lds_frag(sA, wm * 64 + x * 32 + lo, s * 16 + hi * 8);
        fb[x] = lds_frag(sB, wn * 64 + x * 32 + lo, s * 16 + hi * 8);
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
    // row -> (batch element, padded token) for the transposed output
    long ct_row = 0;
    int ct_pad = 0;
    if (p.Ct) {
      const int bb = m / p.T, t = m % p.T;
      int sg = 0;
      while (sg + 1 < p.n_seg && t >= p.seg_off[sg + 1]) ++sg;
      ct_row = (long)bb * p.ct_bs + p.tp_off[sg] + (t - p.seg_off[sg]);
      if (t == p.seg_off[sg + 1] - 1) ct_pad = p.tp_off[sg + 1] - (p.tp_off[sg] + (t - p.seg_off[sg])) - 1;
    }
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
          *(float4*)(p.partial + ((long)blockIdx.z * p.M + m) * p.N + n) = make_float4(v[0], v[1], v[2], v[3]);
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
        if (p.C) *(u32x2*)(p.C + (long)m * p.ldc + n) = pk;
        if (p.Ct) {
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            bf16_t* col = p.Ct + (long)(n + j) * p.Tp + ct_row;
            col[0] = (bf16_t)((j & 1) ? (pk[j >> 1] >> 16) : (pk[j >> 1] & 0xffffu));
            for (int z = 1; z <= ct_pad; ++z) col[z] = 0;
          }
        }
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

// x [B, T, C] rows -> xT [B, C, Tp] with zero pad columns (one 64 x 64 tile per workgroup via LDS)
__global__ __launch_bounds__(256) void transpose_pad_kernel(const bf16_t* __restrict__ x, long ld, int C, int T,
                                                            int n_seg, GeoT gt, Geo g, bf16_t* __restrict__ xt) {
  __shared__ bf16_t tile[64][66];
  const int b = blockIdx.z, c0 = blockIdx.y * 64;
  // blockIdx.x enumerates 64-column tiles of the padded axis
  const int tp0 = blockIdx.x * 64;
  const int tid = threadIdx.x;
  for (int i = tid; i < 64 * 64; i += 256) {
    const int tt = i / 64, cc = i % 64;  // padded token tp0+tt, channel c0+cc
    const int tp = tp0 + tt;
    bf16_t v = 0;
    if (tp < gt.Tp && c0 + cc < C) {
      int sg = 0;
      while (sg + 1 < n_seg && tp >= gt.tp_off[sg + 1]) ++sg;
      const int pos = tp - gt.tp_off[sg];
      if (pos < g.seg_len[sg]) v = x[((long)b * T + g.seg_off[sg] + pos) * ld + c0 + cc];
    }
    tile[tt][cc] = v;
  }
  __syncthreads();
  for (int i = tid; i < 64 * 64; i += 256) {
    const int cc = i / 64, tt = i % 64;
    if (tp0 + tt < gt.Tp && c0 + cc < C) xt[((long)b * C + c0 + cc) * gt.Tp + tp0 + tt] = tile[tt][cc];
  }
}

// W [K, N] row-major -> Wt [N, K]
__global__ __launch_bounds__(256) void transpose_w_kernel(const bf16_t* __restrict__ w, int K, int N,
                                                          bf16_t* __restrict__ wt) {
  __shared__ bf16_t tile[64][66];
  const int k0 = blockIdx.y * 64, n0 = blockIdx.x * 64, tid = threadIdx.x;
  for (int i = tid; i < 64 * 64; i += 256) {
    const int kk = i / 64, nn = i % 64;
    tile[kk][nn] = (k0 + kk < K && n0 + nn < N) ? w[(long)(k0 + kk) * N + n0 + nn] : (bf16_t)0;
  }
  __syncthreads();
  for (int i = tid; i < 64 * 64; i += 256) {
    const int nn = i / 64, kk = i % 64;
    if (k0 + kk < K && n0 + nn < N) wt[(long)(n0 + nn) * K + k0 + kk] = tile[kk][nn];
  }
}

int mfma_gemm_split(int M, int N, int total_ktiles) {
  const long tiles = (long)((M + GM - 1) / GM) * ((N + GN - 1) / GN);
  if (tiles >= 256 || total_ktiles < 16) return 1;
  int s = (int)((512 + tiles - 1) / tiles);
  if (s > total_ktiles / 4) s = total_ktiles / 4;
  return s < 1 ? 1 : s;
}

void launch_mfma_gemm(const MGemm& p, hipStream_t st) {
  dim3 grid((p.N + GN - 1) / GN, (p.M + GM - 1) / GM, p.split_k);
  hipLaunchKernelGGL(mfma_gemm_kernel, grid, dim3(256), 0, st, p);
}
void launch_splitk_reduce(const float* partial, int split_k, int M, int N, float* o0, float* o1, float* o2, int n_per,
                          hipStream_t st) {
  hipLaunchKernelGGL(mfma_splitk_reduce_kernel, dim3(256), dim3(256), 0, st, partial, split_k, M, N, o0, o1, o2, n_per);
}
void launch_transpose_pad(const bf16_t* x, long ld, int C, const Geo& g, const GeoT& gt, bf16_t* xt, hipStream_t st) {
  dim3 grid((gt.Tp + 63) / 64, (C + 63) / 64, g.B);
  hipLaunchKernelGGL(transpose_pad_kernel, grid, dim3(256), 0, st, x, ld, C, g.T, g.n_seg, gt, g, xt);
}
void launch_transpose_w(const bf16_t* w, int K, int N, bf16_t* wt, hipStream_t st) {
  dim3 grid((N + 63) / 64, (K + 63) / 64);
  hipLaunchKernelGGL(transpose_w_kernel, grid, dim3(256), 0, st, w, K, N, wt);
}

}  // namespace imattn
