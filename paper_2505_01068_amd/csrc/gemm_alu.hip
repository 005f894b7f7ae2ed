// fp32-ALU GEMM with strided operands, used for the projections of the small
// multimodal-sentiment shapes (d = 32..64: the whole weight fits in a few LDS
// tiles and the work is bandwidth / launch bound, not MFMA bound) and as the
// fp32 path of the library.  Also: deterministic column sums and LayerNorm.
#include "common.hpp"

namespace imattn {

constexpr int GA_BM = 64, GA_BN = 64, GA_BK = 16, GA_THREADS = 256;

struct GemmDev {
  const void* A;
  long sam, sak;
  const void* B[3];
  long sbk, sbn;
  int b_split, n_per, k_per;
  const void* bias[3];
  void* C[3];
  int c_split, bias_split;
  long ldc;
  const void* res;
  int M, N, K, gelu, split_k;
  float* partial;
  int kb, kt;
  long sab, sbb;
};

__device__ __forceinline__ float gelu_exact(float x) { return 0.5f * x * (1.f + erff(x * 0.70710678118654752440f)); }

template <typename TA, typename TB, typename TC>
__global__ __launch_bounds__(GA_THREADS) void gemm_alu_kernel(GemmDev g) {
  __shared__ __attribute__((aligned(16))) float As[GA_BK][GA_BM + 4];
  __shared__ __attribute__((aligned(16))) float Bs[GA_BK][GA_BN + 4];
  const int tid = threadIdx.x;
  const int m0 = blockIdx.y * GA_BM, n0 = blockIdx.x * GA_BN;
  const int tx = tid % 16, ty = tid / 16;
  const TA* A = (const TA*)g.A;

  // K range of this split
  const int ktiles = (g.K + GA_BK - 1) / GA_BK;
  const int per_split = (ktiles + g.split_k - 1) / g.split_k;
  const int kt_begin = blockIdx.z * per_split;
  const int kt_end = min(ktiles, kt_begin + per_split);

  float acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;

  const bool a_kfast = (g.sak == 1);
  const bool b_nfast = (g.sbn == 1);
  // The next k-tile is fetched into registers while the current one is multiplied (the global round
  // trip would otherwise be exposed once per 16-deep tile).
  float ra[4], rb[4];
  auto fetch = [&](int kt) {
    const int kbase = kt * GA_BK;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int idx = tid + u * GA_THREADS;
      int m, k;
      if (a_kfast) { k = idx % GA_BK; m = idx / GA_BK; } else { m = idx % GA_BM; k = idx / GA_BM; }
      const int gm = m0 + m, gk = kbase + k;
      float v = 0.f;
      if (gm < g.M && gk < g.K) {
        long off;
        if (g.kb > 1) { const int bb = gk / g.kt, kk = gk % g.kt; off = bb * g.sab + (long)kk * g.sak; }
        else off = (long)gk * g.sak;
        v = ldf(A + (long)gm * g.sam + off);
      }
      ra[u] = v;
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int idx = tid + u * GA_THREADS;
      int n, k;
      if (b_nfast) { n = idx % GA_BN; k = idx / GA_BN; } else { k = idx % GA_BK; n = idx / GA_BK; }
      const int gn = n0 + n, gk = kbase + k;
      float v = 0.f;
      if (gn < g.N && gk < g.K) {
        int sel = 0, kk = gk, nn = gn;
        long boff = 0;
        if (g.b_split == 1) { sel = gn / g.n_per; nn = gn % g.n_per; }
        else if (g.b_split == 2) { sel = gk / g.k_per; kk = gk % g.k_per; }
        if (g.kb > 1) { const int bb = gk / g.kt; kk = gk % g.kt; boff = bb * g.sbb; }
        v = ldf((const TB*)g.B[sel] + boff + (long)kk * g.sbk + (long)nn * g.sbn);
      }
      rb[u] = v;
    }
  };
  if (kt_begin < kt_end) fetch(kt_begin);
  for (int kt = kt_begin; kt < kt_end; ++kt) {
    __syncthreads();
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int idx = tid + u * GA_THREADS;
      if (a_kfast) As[idx % GA_BK][idx / GA_BK] = ra[u]; else As[idx / GA_BM][idx % GA_BM] = ra[u];
      if (b_nfast) Bs[idx / GA_BN][idx % GA_BN] = rb[u]; else Bs[idx % GA_BK][idx / GA_BK] = rb[u];
    }
    __syncthreads();
    if (kt + 1 < kt_end) fetch(kt + 1);
#pragma unroll
    for (int k = 0; k < GA_BK; ++k) {
      const float4 a = *(const float4*)&As[k][ty * 4];
      const float4 b = *(const float4*)&Bs[k][tx * 4];
      const float av[4] = {a.x, a.y, a.z, a.w}, bv[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(av[i], bv[j], acc[i][j]);
    }
  }

#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int gm = m0 + ty * 4 + i;
    if (gm >= g.M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int gn = n0 + tx * 4 + j;
      if (gn >= g.N) continue;
      float v = acc[i][j];
      if (g.split_k > 1) {
        g.partial[((long)blockIdx.z * g.M + gm) * g.N + gn] = v;
        continue;
      }
      int sel = 0, nn = gn;
      if (g.n_per > 0) { sel = gn / g.n_per; nn = gn % g.n_per; }
      const int bsel = g.bias_split ? sel : 0;
      if (g.bias[bsel]) v += ldf((const TC*)g.bias[bsel] + (g.bias_split ? nn : gn));
      if (g.gelu) v = gelu_exact(v);
      if (g.c_split) {
        stf((TC*)g.C[sel] + (long)gm * g.ldc + nn, v);
      } else {
        if (g.res) v += ldf((const TC*)g.res + (long)gm * g.ldc + gn);
        stf((TC*)g.C[0] + (long)gm * g.ldc + gn, v);
      }
    }
  }
}

// Sum split-K partials in a fixed order and write fp32 outputs (weight gradients).  A block of 256
// threads owns 64 consecutive outputs; thread (zz, o) sums partials z = zz, zz+4, ... and the four
// sub-sums are added in a fixed order, so the result does not depend on scheduling.
__global__ __launch_bounds__(256) void gemm_splitk_reduce_kernel(GemmDev g) {
  __shared__ float part[4][64];
  const long n_out = (long)g.M * g.N;
  const int o = threadIdx.x & 63, zz = threadIdx.x >> 6;
  const long i = (long)blockIdx.x * 64 + o;
  float s = 0.f;
  if (i < n_out)
    for (int z = zz; z < g.split_k; z += 4) s += g.partial[z * n_out + i];
  part[zz][o] = s;
  __syncthreads();
  if (zz == 0 && i < n_out) {
    s = (part[0][o] + part[1][o]) + (part[2][o] + part[3][o]);
    const int gm = i / g.N, gn = i % g.N;
    int sel = 0, nn = gn;
    if (g.n_per > 0) { sel = gn / g.n_per; nn = gn % g.n_per; }
    if (g.c_split) ((float*)g.C[sel])[(long)gm * g.ldc + nn] = s;
    else ((float*)g.C[0])[(long)gm * g.ldc + gn] = s;
  }
}

size_t gemm_alu_partial_bytes(int M, int N, int K, int* split_k) {
  // Split only reductions that are much longer than the output is wide (weight gradients).
  int s = 1;
  const long tiles = (long)((M + GA_BM - 1) / GA_BM) * ((N + GA_BN - 1) / GA_BN);
  if (K >= 2048 && tiles < 256) {
    s = (int)((512 + tiles - 1) / tiles);
    const int ktiles = (K + GA_BK - 1) / GA_BK;
    if (s > ktiles / 8) s = ktiles / 8;
    if (s > 128) s = 128;
    if (s < 1) s = 1;
  }
  if (split_k) *split_k = s;
  return s > 1 ? (size_t)s * M * N * sizeof(float) : 0;
}

int launch_gemm_alu(const GemmDesc& d, int a_bf16, int b_bf16, int c_bf16, hipStream_t st) {
  GemmDev g;
  g.A = d.A; g.sam = d.sam; g.sak = d.sak;
  for (int i = 0; i < 3; ++i) { g.B[i] = d.B[i]; g.bias[i] = d.bias[i]; g.C[i] = d.C[i]; }
  g.sbk = d.sbk; g.sbn = d.sbn; g.b_split = d.b_split; g.n_per = d.n_per; g.k_per = d.k_per; g.c_split = d.c_split;
  g.bias_split = d.bias_split; g.ldc = d.ldc;
  g.res = d.res; g.M = d.M; g.N = d.N; g.K = d.K; g.gelu = d.gelu;
  g.split_k = d.split_k > 1 ? d.split_k : 1; g.partial = d.partial;
  g.kb = d.kb > 1 ? d.kb : 1; g.kt = d.kb > 1 ? d.kt : d.K; g.sab = d.sab; g.sbb = d.sbb;
  if (g.M <= 0 || g.N <= 0) return IM_OK;
  dim3 grid((g.N + GA_BN - 1) / GA_BN, (g.M + GA_BM - 1) / GA_BM, g.split_k), block(GA_THREADS);
  const int key = (a_bf16 ? 4 : 0) | (b_bf16 ? 2 : 0) | (c_bf16 ? 1 : 0);
  switch (key) {
    case 0: hipLaunchKernelGGL((gemm_alu_kernel<float, float, float>), grid, block, 0, st, g); break;
    case 7: hipLaunchKernelGGL((gemm_alu_kernel<bf16_t, bf16_t, bf16_t>), grid, block, 0, st, g); break;
    case 6: hipLaunchKernelGGL((gemm_alu_kernel<bf16_t, bf16_t, float>), grid, block, 0, st, g); break;
    default: set_error("gemm_alu: unsupported operand type combination %d", key); return IM_ERR_UNSUPPORTED;
  }
  if (g.split_k > 1)
    hipLaunchKernelGGL(gemm_splitk_reduce_kernel, dim3((unsigned)(((long)g.M * g.N + 63) / 64)), dim3(256), 0, st, g);
  return IM_OK;
}

// ---- column sums (bias gradients): stage 1 sums blocks of rows, stage 2 sums the blocks in order ----
// ---- weight gradient of a narrow layer: C[M, N] = A[R, M]^T G[R, N], M <= 64, N <= 256, R long ----
// The general GEMM above spends its time in a latency-bound loop of R / split 16-deep k-tiles.  Here a
// block stages WS_RB rows of A and G in LDS with all loads in flight at once and every thread keeps a
// TM x TN patch of the output in registers (thread (ty, tx): rows ty + 8 i, columns tx + 32 j, so the
// LDS reads are broadcasts / consecutive words).  Each block writes one partial [M, N]; the caller
// reduces the partials in a fixed order.
constexpr int WS_RB = 32;
constexpr int WS_MAX_BLOCKS = 1024;
template <typename T, int TM, int TN>
__global__ __launch_bounds__(256) void wgrad_small_kernel(const T* __restrict__ A, long lda, const T* __restrict__ G,
                                                          long ldg, int R, int M, int N, float* __restrict__ partial) {
  __shared__ float sm[WS_RB * (64 + 256)];
  float* sA = sm;
  float* sG = sm + WS_RB * M;
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
  float acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) acc[i][j] = 0.f;
  int mi[TM], nj[TN];
#pragma unroll
  for (int i = 0; i < TM; ++i) mi[i] = min(ty + 8 * i, M - 1);
#pragma unroll
  for (int j = 0; j < TN; ++j) nj[j] = min(tx + 32 * j, N - 1);
  const int nchunks = (R + WS_RB - 1) / WS_RB;
  for (int ch = blockIdx.x; ch < nchunks; ch += gridDim.x) {
    const long row0 = (long)ch * WS_RB;
    __syncthreads();
    for (int e = threadIdx.x; e < WS_RB * M; e += 256) {
      const int r = e / M, m = e - r * M;
      sA[e] = row0 + r < R ? ldf(A + (row0 + r) * lda + m) : 0.f;
    }
    for (int e = threadIdx.x; e < WS_RB * N; e += 256) {
      const int r = e / N, n = e - r * N;
      sG[e] = row0 + r < R ? ldf(G + (row0 + r) * ldg + n) : 0.f;
    }
    __syncthreads();
#pragma unroll 4
    for (int r = 0; r < WS_RB; ++r) {
      float a[TM], g[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i) a[i] = sA[r * M + mi[i]];
#pragma unroll
      for (int j = 0; j < TN; ++j) g[j] = sG[r * N + nj[j]];
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = fmaf(a[i], g[j], acc[i][j]);
    }
  }
  float* out = partial + (long)blockIdx.x * M * N;
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    const int m = ty + 8 * i;
    if (m >= M) continue;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int n = tx + 32 * j;
      if (n < N) out[(long)m * N + n] = acc[i][j];
    }
  }
}

// out[m, n] = sum_z partial[z][m][n], z in a fixed order; column block s of n_per columns goes to the [M, n_per]
// matrix o<s> (NULL = dropped) when n_per > 0, else everything to o0.  A block of 256 threads owns 16
// consecutive outputs: thread (g, o) sums z = g, g + 16, ... with four running sums (independent loads in
// flight), then the 16 groups are added in a fixed order.
__global__ __launch_bounds__(256) void wgrad_small_reduce_kernel(const float* __restrict__ partial, int nz, int M, int N,
                                                                 float* o0, float* o1, float* o2, int n_per) {
  __shared__ float red[16][16];
  const int o = threadIdx.x & 15, g = threadIdx.x >> 4;
  const long n_out = (long)M * N;
  const long i = (long)blockIdx.x * 16 + o;
  float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
  if (i < n_out) {
    int z = g;
    for (; z + 48 < nz; z += 64) {
      s0 += partial[(long)z * n_out + i];
      s1 += partial[(long)(z + 16) * n_out + i];
      s2 += partial[(long)(z + 32) * n_out + i];
      s3 += partial[(long)(z + 48) * n_out + i];
    }
    for (; z < nz; z += 16) s0 += partial[(long)z * n_out + i];
  }
  red[g][o] = (s0 + s1) + (s2 + s3);
  __syncthreads();
  if (g == 0 && i < n_out) {
    float v = 0.f;
#pragma unroll
    for (int k = 0; k < 16; ++k) v += red[k][o];
    const int m = (int)(i / N), n = (int)(i - (long)m * N);
    if (n_per > 0) {
      float* dst = (n / n_per == 0) ? o0 : (n / n_per == 1) ? o1 : o2;
      if (dst) dst[(long)m * n_per + n % n_per] = v;
    } else {
      o0[i] = v;
    }
  }
}
void launch_wgrad_small_reduce(const float* partial, int nz, int M, int N, float* o0, float* o1, float* o2, int n_per,
                               hipStream_t st) {
  const long n_out = (long)M * N;
  hipLaunchKernelGGL(wgrad_small_reduce_kernel, dim3((unsigned)((n_out + 15) / 16)), dim3(256), 0, st, partial, nz, M, N, o0,
                     o1, o2, n_per);
}

bool wgrad_small_ok(int M, int N, int n_per) {
  (void)n_per;
  return M >= 1 && M <= 64 && N >= 1 && N <= 256;
}
int wgrad_small_blocks(int R) {
  const int nchunks = (R + WS_RB - 1) / WS_RB;
  return nchunks < WS_MAX_BLOCKS ? nchunks : WS_MAX_BLOCKS;
}
size_t wgrad_small_partial_bytes(int M, int N, int R) { return (size_t)wgrad_small_blocks(R) * M * N * sizeof(float); }

template <typename T, int TM>
static void launch_wgrad_small_tn(const T* A, long lda, const T* G, long ldg, int R, int M, int N, float* partial, int blocks,
                                  hipStream_t st) {
  const int tn = (N + 31) / 32;
  if (tn <= 2) hipLaunchKernelGGL((wgrad_small_kernel<T, TM, 2>), dim3(blocks), dim3(256), 0, st, A, lda, G, ldg, R, M, N, partial);
  else if (tn <= 4) hipLaunchKernelGGL((wgrad_small_kernel<T, TM, 4>), dim3(blocks), dim3(256), 0, st, A, lda, G, ldg, R, M, N, partial);
  else if (tn <= 6) hipLaunchKernelGGL((wgrad_small_kernel<T, TM, 6>), dim3(blocks), dim3(256), 0, st, A, lda, G, ldg, R, M, N, partial);
  else hipLaunchKernelGGL((wgrad_small_kernel<T, TM, 8>), dim3(blocks), dim3(256), 0, st, A, lda, G, ldg, R, M, N, partial);
}
template <typename T>
static void launch_wgrad_small_t(const T* A, long lda, const T* G, long ldg, int R, int M, int N, float* partial, int blocks,
                                 hipStream_t st) {
  const int tm = (M + 7) / 8;
  if (tm <= 4) launch_wgrad_small_tn<T, 4>(A, lda, G, ldg, R, M, N, partial, blocks, st);
  else if (tm <= 5) launch_wgrad_small_tn<T, 5>(A, lda, G, ldg, R, M, N, partial, blocks, st);
  else launch_wgrad_small_tn<T, 8>(A, lda, G, ldg, R, M, N, partial, blocks, st);
}
// Writes wgrad_small_blocks(R) partial [M, N] matrices; returns that count (the number of partials to reduce).
int launch_wgrad_small(const void* A, long lda, const void* G, long ldg, int R, int M, int N, int in_bf16, float* partial,
                       hipStream_t st) {
  const int blocks = wgrad_small_blocks(R);
  if (in_bf16) launch_wgrad_small_t<bf16_t>((const bf16_t*)A, lda, (const bf16_t*)G, ldg, R, M, N, partial, blocks, st);
  else launch_wgrad_small_t<float>((const float*)A, lda, (const float*)G, ldg, R, M, N, partial, blocks, st);
  return blocks;
}

// Column sums of up to four [R, n] matrices in two deterministic stages (one launch each for all of
// them: blockIdx.z selects the matrix).  Stage 1: a block of 256 threads = 4 row groups x 64 columns
// sums CS_ROWS rows (thread (g, c): rows r0 + g, r0 + g + 4, ..., with four independent running sums so
// loads overlap), then the 4 groups are added in a fixed order through LDS.  Stage 2 adds the
// per-block partials ([matrix][row block][n]) the same way with 16 groups x 16 columns.
constexpr int CS_ROWS = 256;
struct ColsumArgs {
  const void* a[4];
  long lda[4];
  float* out[4];   // nullptr: this matrix is skipped
};

template <typename T>
__global__ __launch_bounds__(256) void colsum_stage1(ColsumArgs q, int R, int n, float* __restrict__ partial) {
  __shared__ float red[4][64];
  const int z = blockIdx.z;
  if (!q.out[z]) return;
  const T* __restrict__ a = (const T*)q.a[z];
  const long lda = q.lda[z];
  const int tx = threadIdx.x & 63, g = threadIdx.x >> 6;
  const int c = blockIdx.x * 64 + tx;
  const int r0 = blockIdx.y * CS_ROWS, r1 = min(R, r0 + CS_ROWS);
  float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
  if (c < n) {
    int r = r0 + g;
    for (; r + 12 < r1; r += 16) {
      s0 += ldf(a + (long)r * lda + c);
      s1 += ldf(a + (long)(r + 4) * lda + c);
      s2 += ldf(a + (long)(r + 8) * lda + c);
      s3 += ldf(a + (long)(r + 12) * lda + c);
    }
    for (; r < r1; r += 4) s0 += ldf(a + (long)r * lda + c);
  }
  red[g][tx] = (s0 + s1) + (s2 + s3);
  __syncthreads();
  if (g == 0 && c < n)
    partial[((long)z * gridDim.y + blockIdx.y) * n + c] = (red[0][tx] + red[1][tx]) + (red[2][tx] + red[3][tx]);
}
__global__ __launch_bounds__(256) void colsum_stage2(const float* __restrict__ partial, int nblk, int n, ColsumArgs q) {
  // 16 groups x 16 columns: group g adds row blocks g, g + 16, ... in ascending order, then the 16 group sums are
  // added in a fixed order (a block of 4 groups x 64 columns left one workgroup walking through all the partials)
  __shared__ float red[16][16];
  const int z = blockIdx.z;
  if (!q.out[z]) return;
  const int tx = threadIdx.x & 15, g = threadIdx.x >> 4;
  const int c = blockIdx.x * 16 + tx;
  float s = 0.f;
  if (c < n)
    for (int b = g; b < nblk; b += 16) s += partial[((long)z * nblk + b) * n + c];
  red[g][tx] = s;
  __syncthreads();
  if (g != 0 || c >= n) return;
  for (int k = 1; k < 16; ++k) s += red[k][tx];
  q.out[z][c] = s;
}
// bytes of `partial` for ONE matrix; launch_colsum_multi needs count times as much
size_t colsum_partial_bytes(int R, int n) { return (size_t)((R + CS_ROWS - 1) / CS_ROWS) * n * sizeof(float); }

int launch_colsum_multi(const void* const* a, const long* lda, float* const* out, int count, int R, int n, int a_bf16,
                        float* partial, hipStream_t st) {
  ColsumArgs q;
  bool any = false;
  for (int i = 0; i < 4; ++i) {   // count <= 4
    q.a[i] = i < count ? a[i] : nullptr;
    q.lda[i] = i < count ? lda[i] : 0;
    q.out[i] = i < count ? out[i] : nullptr;
    any = any || q.out[i];
  }
  if (!any) return IM_OK;
  const int nblk = (R + CS_ROWS - 1) / CS_ROWS;
  dim3 grid((n + 63) / 64, nblk, count), block(256);
  if (a_bf16) hipLaunchKernelGGL((colsum_stage1<bf16_t>), grid, block, 0, st, q, R, n, partial);
  else hipLaunchKernelGGL((colsum_stage1<float>), grid, block, 0, st, q, R, n, partial);
  hipLaunchKernelGGL(colsum_stage2, dim3((n + 15) / 16, 1, count), dim3(256), 0, st, partial, nblk, n, q);
  return IM_OK;
}
int launch_colsum(const void* a, long lda, int R, int n, int a_bf16, float* out, float* partial, hipStream_t st) {
  return launch_colsum_multi(&a, &lda, &out, 1, R, n, a_bf16, partial, st);
}

// ---- LayerNorm over the feature axis: one wavefront per row, two-pass (mean, then variance) in fp32 ----
template <typename T>
__global__ __launch_bounds__(256) void layernorm_kernel(const T* __restrict__ x, const T* __restrict__ gamma,
                                                        const T* __restrict__ beta, T* __restrict__ y, int R, int d,
                                                        float eps) {
  const int wave = threadIdx.x / 64, lane = threadIdx.x % 64;
  const long r = (long)blockIdx.x * 4 + wave;
  if (r >= R) return;
  const T* xr = x + r * d;
  float s = 0.f;
  for (int e = lane; e < d; e += 64) s += ldf(xr + e);
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
  const float mu = s / d;
  float v = 0.f;
  for (int e = lane; e < d; e += 64) { const float t = ldf(xr + e) - mu; v = fmaf(t, t, v); }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  const float rstd = rsqrtf(v / d + eps);
  for (int e = lane; e < d; e += 64) stf(y + r * d + e, (ldf(xr + e) - mu) * rstd * ldf(gamma + e) + ldf(beta + e));
}

// bf16 rows of d = 8 LPR elements (LPR a power of two <= 32): LPR lanes share a row, each holds 8
// consecutive elements (one 16-byte load), and a wave normalises 64 / LPR rows at once.  At d = 64 that is
// 8 rows per wave and full-width loads and stores instead of one row and 2 bytes per lane.
template <int LPR>
__global__ __launch_bounds__(256) void layernorm_rows_kernel(const bf16_t* __restrict__ x,
                                                             const bf16_t* __restrict__ gamma,
                                                             const bf16_t* __restrict__ beta,
                                                             bf16_t* __restrict__ y, int R, float eps) {
  typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
  constexpr int RPW = 64 / LPR, d = 8 * LPR;
  const int wave = threadIdx.x / 64, lane = threadIdx.x % 64;
  const long r = ((long)blockIdx.x * 4 + wave) * RPW + lane / LPR;
  const int c = (lane % LPR) * 8;
  const bool live = r < R;
  float v[8], gm[8], bt[8];
  {
    u32x4 raw = {0u, 0u, 0u, 0u};
    if (live) raw = *(const u32x4*)(x + r * d + c);
    const u32x4 gr = *(const u32x4*)(gamma + c), br = *(const u32x4*)(beta + c);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      v[2 * j] = __uint_as_float(raw[j] << 16); v[2 * j + 1] = __uint_as_float(raw[j] & 0xffff0000u);
      gm[2 * j] = __uint_as_float(gr[j] << 16); gm[2 * j + 1] = __uint_as_float(gr[j] & 0xffff0000u);
      bt[2 * j] = __uint_as_float(br[j] << 16); bt[2 * j + 1] = __uint_as_float(br[j] & 0xffff0000u);
    }
  }
  float s = 0.f;
#pragma unroll
  for (int j = 0; j < 8; ++j) s += v[j];
#pragma unroll
  for (int o = LPR / 2; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
  const float mu = s * (1.f / d);
  float q = 0.f;
#pragma unroll
  for (int j = 0; j < 8; ++j) { const float t = v[j] - mu; q = fmaf(t, t, q); }
#pragma unroll
  for (int o = LPR / 2; o > 0; o >>= 1) q += __shfl_xor(q, o, 64);
  const float rstd = rsqrtf(q * (1.f / d) + eps);
  if (!live) return;
  u32x4 out;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const float a = (v[2 * j] - mu) * rstd * gm[2 * j] + bt[2 * j], b = (v[2 * j + 1] - mu) * rstd * gm[2 * j + 1] + bt[2 * j + 1];
    out[j] = (unsigned)f2bf(a) | ((unsigned)f2bf(b) << 16);
  }
  *(u32x4*)(y + r * d + c) = out;
}

// ---- pieces of the encoder-layer backward ----
__device__ __forceinline__ float gelu_f(float z) { return 0.5f * z * (1.f + erff(z * 0.70710678118654752440f)); }
// d/dz [z Phi(z)] = Phi(z) + z phi(z)
__device__ __forceinline__ float gelu_grad_f(float z) {
  return 0.5f * (1.f + erff(z * 0.70710678118654752440f)) + z * __expf(-0.5f * z * z) * 0.39894228040143267794f;
}
template <typename T>
__global__ void gelu_fwd_kernel(const T* __restrict__ z, T* __restrict__ a, long n) {
  for (long i = blockIdx.x * (long)blockDim.x + threadIdx.x; i < n; i += (long)gridDim.x * blockDim.x) stf(a + i, gelu_f(ldf(z + i)));
}
template <typename T>
__global__ void gelu_bwd_kernel(const T* __restrict__ z, T* __restrict__ g, long n) {  // g: da in, dz out
  for (long i = blockIdx.x * (long)blockDim.x + threadIdx.x; i < n; i += (long)gridDim.x * blockDim.x)
    stf(g + i, ldf(g + i) * gelu_grad_f(ldf(z + i)));
}
// bf16, 8 elements (16 bytes) per thread and step
__device__ __forceinline__ void unpack8(const uint4& r, float (&v)[8]) {
  const unsigned w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
  for (int j = 0; j < 4; ++j) { v[2 * j] = __uint_as_float(w[j] << 16); v[2 * j + 1] = __uint_as_float(w[j] & 0xffff0000u); }
}
__device__ __forceinline__ uint4 pack8_rne(const float (&v)[8]) {
  unsigned w[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) w[j] = (unsigned)f2bf(v[2 * j]) | ((unsigned)f2bf(v[2 * j + 1]) << 16);
  return make_uint4(w[0], w[1], w[2], w[3]);
}
// Phi(x), the standard normal CDF, with erf from Abramowitz & Stegun 7.1.26 (|error| <= 1.5e-7, far below the
// bf16 rounding of the results): a reciprocal, an exp2 and six multiply-adds instead of the library erff.
__device__ __forceinline__ float phi_as_f(float x) {
  const float u = fabsf(x) * 0.70710678118654752440f;
  const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f, u, 1.f));
  float pl = fmaf(1.061405429f, t, -1.453152027f);
  pl = fmaf(pl, t, 1.421413741f);
  pl = fmaf(pl, t, -0.284496736f);
  pl = fmaf(pl, t, 0.254829592f);
  const float e = pl * t * __builtin_amdgcn_exp2f(-1.44269504088896340736f * u * u);  // 1 - erf(u)
  return x >= 0.f ? 1.f - 0.5f * e : 0.5f * e;
}
__global__ void gelu_fwd8_kernel(const bf16_t* __restrict__ z, bf16_t* __restrict__ a, long n8) {
  for (long i = blockIdx.x * (long)blockDim.x + threadIdx.x; i < n8; i += (long)gridDim.x * blockDim.x) {
    float v[8];
    unpack8(*(const uint4*)(z + 8 * i), v);
#pragma unroll
    for (int j = 0; j < 8; ++j) v[j] *= phi_as_f(v[j]);
    *(uint4*)(a + 8 * i) = pack8_rne(v);
  }
}
__global__ void gelu_bwd8_kernel(const bf16_t* __restrict__ z, bf16_t* __restrict__ g, long n8) {
  for (long i = blockIdx.x * (long)blockDim.x + threadIdx.x; i < n8; i += (long)gridDim.x * blockDim.x) {
    float v[8], w[8];
    unpack8(*(const uint4*)(z + 8 * i), v);
    unpack8(*(const uint4*)(g + 8 * i), w);
#pragma unroll
    for (int j = 0; j < 8; ++j)   // d/dz [z Phi(z)] = Phi(z) + z phi(z)
      w[j] *= phi_as_f(v[j]) + v[j] * __expf(-0.5f * v[j] * v[j]) * 0.39894228040143267794f;
    *(uint4*)(g + 8 * i) = pack8_rne(w);
  }
}
static bool vec8_ok(const void* a, const void* b, long n) { return n % 8 == 0 && (((uintptr_t)a | (uintptr_t)b) & 15) == 0; }
int launch_gelu_fwd(const void* z, void* a, long n, int bf16, hipStream_t st) {
  if (bf16 && vec8_ok(z, a, n)) {
    const long n8 = n / 8;
    const int blocks8 = (int)((n8 + 255) / 256 < 8192 ? (n8 + 255) / 256 : 8192);
    hipLaunchKernelGGL(gelu_fwd8_kernel, dim3(blocks8), dim3(256), 0, st, (const bf16_t*)z, (bf16_t*)a, n8);
    return IM_OK;
  }
  const int blocks = (int)((n + 255) / 256 < 8192 ? (n + 255) / 256 : 8192);
  if (bf16) hipLaunchKernelGGL((gelu_fwd_kernel<bf16_t>), dim3(blocks), dim3(256), 0, st, (const bf16_t*)z, (bf16_t*)a, n);
  else hipLaunchKernelGGL((gelu_fwd_kernel<float>), dim3(blocks), dim3(256), 0, st, (const float*)z, (float*)a, n);
  return IM_OK;
}
int launch_gelu_bwd(const void* z, void* g, long n, int bf16, hipStream_t st) {
  if (bf16 && vec8_ok(z, g, n)) {
    const long n8 = n / 8;
    const int blocks8 = (int)((n8 + 255) / 256 < 8192 ? (n8 + 255) / 256 : 8192);
    hipLaunchKernelGGL(gelu_bwd8_kernel, dim3(blocks8), dim3(256), 0, st, (const bf16_t*)z, (bf16_t*)g, n8);
    return IM_OK;
  }
  const int blocks = (int)((n + 255) / 256 < 8192 ? (n + 255) / 256 : 8192);
  if (bf16) hipLaunchKernelGGL((gelu_bwd_kernel<bf16_t>), dim3(blocks), dim3(256), 0, st, (const bf16_t*)z, (bf16_t*)g, n);
  else hipLaunchKernelGGL((gelu_bwd_kernel<float>), dim3(blocks), dim3(256), 0, st, (const float*)z, (float*)g, n);
  return IM_OK;
}

// LayerNorm backward of one row per wave: with xhat = (x - mean) * rstd and a = gamma * dy,
//   dx = rstd * (a - mean(a) - xhat * mean(a * xhat)) + res,      t = dy * xhat
// (the column sums of t and dy over all rows are the gradients of gamma and beta).
template <typename T>
__global__ __launch_bounds__(256) void layernorm_bwd_kernel(const T* __restrict__ x, const T* __restrict__ gamma,
                                                            const T* __restrict__ dy, const T* __restrict__ res,
                                                            T* __restrict__ dx, T* __restrict__ t, int R, int d,
                                                            float eps) {
  const int wave = threadIdx.x / 64, lane = threadIdx.x % 64;
  const long r = (long)blockIdx.x * 4 + wave;
  if (r >= R) return;
  const T* xr = x + r * d;
  const T* gr = dy + r * d;
  float s = 0.f;
  for (int e = lane; e < d; e += 64) s += ldf(xr + e);
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
  const float mu = s / d;
  float v = 0.f;
  for (int e = lane; e < d; e += 64) { const float c = ldf(xr + e) - mu; v = fmaf(c, c, v); }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  const float rstd = rsqrtf(v / d + eps);
  float m1 = 0.f, m2 = 0.f;
  for (int e = lane; e < d; e += 64) {
    const float a = ldf(gamma + e) * ldf(gr + e), xh = (ldf(xr + e) - mu) * rstd;
    m1 += a;
    m2 = fmaf(a, xh, m2);
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) { m1 += __shfl_xor(m1, o, 64); m2 += __shfl_xor(m2, o, 64); }
  m1 /= d;
  m2 /= d;
  for (int e = lane; e < d; e += 64) {
    const float g = ldf(gr + e), a = ldf(gamma + e) * g, xh = (ldf(xr + e) - mu) * rstd;
    stf(dx + r * d + e, rstd * (a - m1 - xh * m2) + (res ? ldf(res + r * d + e) : 0.f));
    stf(t + r * d + e, g * xh);
  }
}
// The same for bf16 rows of d = 8 LPR elements, LPR lanes per row and 64 / LPR rows per wave (see layernorm_rows_kernel).
template <int LPR>
__global__ __launch_bounds__(256) void layernorm_bwd_rows_kernel(const bf16_t* __restrict__ x, const bf16_t* __restrict__ gamma,
                                                                 const bf16_t* __restrict__ dy, const bf16_t* __restrict__ res,
                                                                 bf16_t* __restrict__ dx, bf16_t* __restrict__ t, int R,
                                                                 float eps) {
  constexpr int RPW = 64 / LPR, d = 8 * LPR;
  const int wave = threadIdx.x / 64, lane = threadIdx.x % 64;
  const long r = ((long)blockIdx.x * 4 + wave) * RPW + lane / LPR;
  const int c = (lane % LPR) * 8;
  const bool live = r < R;
  const long at = (live ? r : 0) * d + c;
  float xv[8], gv[8], gm[8], rs[8];
  unpack8(*(const uint4*)(x + at), xv);
  unpack8(*(const uint4*)(dy + at), gv);
  unpack8(*(const uint4*)(gamma + c), gm);
  if (res) unpack8(*(const uint4*)(res + at), rs);
  auto rowsum = [&](float v) {
#pragma unroll
    for (int o = LPR / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
  };
  float s = 0.f;
#pragma unroll
  for (int j = 0; j < 8; ++j) s += xv[j];
  const float mu = rowsum(s) * (1.f / d);
  float q = 0.f;
#pragma unroll
  for (int j = 0; j < 8; ++j) { const float w = xv[j] - mu; q = fmaf(w, w, q); }
  const float rstd = rsqrtf(rowsum(q) * (1.f / d) + eps);
  float m1 = 0.f, m2 = 0.f, xh[8], a[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    a[j] = gm[j] * gv[j];
    xh[j] = (xv[j] - mu) * rstd;
    m1 += a[j];
    m2 = fmaf(a[j], xh[j], m2);
  }
  m1 = rowsum(m1) * (1.f / d);
  m2 = rowsum(m2) * (1.f / d);
  if (!live) return;
  float o1[8], o2[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    o1[j] = rstd * (a[j] - m1 - xh[j] * m2) + (res ? rs[j] : 0.f);
    o2[j] = gv[j] * xh[j];
  }
  *(uint4*)(dx + at) = pack8_rne(o1);
  *(uint4*)(t + at) = pack8_rne(o2);
}
int launch_layernorm_bwd(const void* x, const void* gamma, const void* dy, const void* res, void* dx, void* t, int R,
                         int d, float eps, int bf16, hipStream_t st) {
  dim3 grid((R + 3) / 4), block(256);
  const uintptr_t al = (uintptr_t)x | (uintptr_t)gamma | (uintptr_t)dy | (uintptr_t)res | (uintptr_t)dx | (uintptr_t)t;
  if (bf16 && (al & 15) == 0 && (d == 64 || d == 128 || d == 256)) {
    const int lpr = d / 8, rows_per_block = 4 * (64 / lpr);
    const dim3 g2((R + rows_per_block - 1) / rows_per_block);
#define LNB_ROWS(L) hipLaunchKernelGGL((layernorm_bwd_rows_kernel<L>), g2, block, 0, st, (const bf16_t*)x, (const bf16_t*)gamma, \
                                       (const bf16_t*)dy, (const bf16_t*)res, (bf16_t*)dx, (bf16_t*)t, R, eps)
    if (lpr == 8) LNB_ROWS(8); else if (lpr == 16) LNB_ROWS(16); else LNB_ROWS(32);
#undef LNB_ROWS
    return IM_OK;
  }
  if (bf16)
    hipLaunchKernelGGL((layernorm_bwd_kernel<bf16_t>), grid, block, 0, st, (const bf16_t*)x, (const bf16_t*)gamma,
                       (const bf16_t*)dy, (const bf16_t*)res, (bf16_t*)dx, (bf16_t*)t, R, d, eps);
  else
    hipLaunchKernelGGL((layernorm_bwd_kernel<float>), grid, block, 0, st, (const float*)x, (const float*)gamma,
                       (const float*)dy, (const float*)res, (float*)dx, (float*)t, R, d, eps);
  return IM_OK;
}

int launch_layernorm(const void* x, const void* gamma, const void* beta, void* y, int R, int d, float eps, int bf16,
                     hipStream_t st) {
  dim3 grid((R + 3) / 4), block(256);
  const bool aligned = (((uintptr_t)x | (uintptr_t)y | (uintptr_t)gamma | (uintptr_t)beta) & 15) == 0;
  if (bf16 && aligned && (d == 64 || d == 128 || d == 256)) {
    const int lpr = d / 8, rows_per_block = 4 * (64 / lpr);
    const dim3 g2((R + rows_per_block - 1) / rows_per_block);
#define LN_ROWS(L) hipLaunchKernelGGL((layernorm_rows_kernel<L>), g2, block, 0, st, (const bf16_t*)x, (const bf16_t*)gamma, \
                                      (const bf16_t*)beta, (bf16_t*)y, R, eps)
    if (lpr == 8) LN_ROWS(8); else if (lpr == 16) LN_ROWS(16); else LN_ROWS(32);
#undef LN_ROWS
    return IM_OK;
  }
  if (bf16)
    hipLaunchKernelGGL((layernorm_kernel<bf16_t>), grid, block, 0, st, (const bf16_t*)x, (const bf16_t*)gamma,
                       (const bf16_t*)beta, (bf16_t*)y, R, d, eps);
  else
    hipLaunchKernelGGL((layernorm_kernel<float>), grid, block, 0, st, (const float*)x, (const float*)gamma,
                       (const float*)beta, (float*)y, R, d, eps);
  return IM_OK;
}

}  // namespace imattn
