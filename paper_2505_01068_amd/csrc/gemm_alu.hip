// fp32-ALU GEMM with strided operands, used for the projections of the small
// multimodal-sentiment shapes (d = 32..64: the whole weight fits in a few LDS
// tiles and the work is bandwidth / launch bound, not MFMA bound) and as the
// fp32 path of the library.  Also: deterministic column sums and LayerNorm.
#include <type_traits>
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

// ---------------------------------------------------------------------------------------------
// fp32 GEMM of a tall matrix with a small weight on the fp32 matrix instruction
// (v_mfma_f32_32x32x2_f32: products and sums in fp32, twice the vector FMA rate): the projections of the
// narrow models (d = 32..64: [rows, d] x [d, 3d], [rows, 3d] x [3d, d], ...).  One pass over A, no tiles of A
// in LDS: the product is computed transposed, C^T = B^T A^T, so that a lane owns one output row --
//   matrix-instruction "A" operand = the weight: lane (n = lane % 32, h = lane / 32) holds B(k = h Kh + j, n)
//     for step j; the whole weight sits in LDS in exactly that order (Kh x NB x 64 floats, one conflict-free
//     4-byte read per instruction), filled once per workgroup with 16-byte loads;
//   "B" operand = a 32-row block of A: lane (m, h) holds A(m, h Kh + j), i.e. the lane reads Kh CONSECUTIVE
//     elements of its row (16-byte loads, all requested at once) -- the contraction index is simply visited in
//     the order (0, Kh), (1, Kh + 1), ..., which both operands agree on;
//   accumulator register r of block nb = column nb 32 + 8 (r / 4) + 4 h + r % 4 of row m: four consecutive
//     columns per register quad; the accumulators start at the bias and are stored with 16-byte stores.
// A wave owns a 32-row block and at most two 32-column blocks (wider outputs are shared by two waves that read
// the same rows): at these sizes the kernel is not bound by the matrix pipe but by the instructions around it,
// executed by waves that have a SIMD to themselves, so the work per wave is kept short and the index arithmetic
// out of the loops.  K is padded to a multiple of 8 with zeros (LDS is cleared first; A elements past K are not
// loaded).
typedef float f32x16s __attribute__((ext_vector_type(16)));
constexpr int SK_MAX_LDS_FLOATS = 12288;   // 48 KB: Kh * NB * 64 floats
constexpr int SK_MAX_CH = 16;              // 4-element chunks of a lane's half row held in registers: K <= 128
constexpr int SK_NBW = 2;                  // 32-column blocks per wave (the kernel is written for 2)

// fill: 0 = element by element (any strides), 1 = B(k, n .. n+3) contiguous, 2 = B(k .. k+3, n) contiguous
template <bool AVEC, int NCH>   // NCH = Kh / 4: 4-element chunks of a lane's half row (straight-line code per size)
__global__ __launch_bounds__(256) void gemm_skinny_kernel(GemmDev g, int NB, int nparts, int fill) {
  constexpr int Kh = 4 * NCH;
  extern __shared__ __attribute__((aligned(16))) float wl[];   // [Kh][NB][64]
  const int tid = threadIdx.x, lane = tid & 63, h = lane >> 5, ml = lane & 31;
  const float* A = (const float*)g.A;
  const int nblk = (g.M + 31) >> 5;
  const int units = nblk * nparts, stride = gridDim.x * 4;   // stride is a multiple of nparts (1 or 2)
  const int k0 = h * Kh;
  float x[NCH][4];
  auto load_rows = [&](int rb) {
    const int m = rb * 32 + ml;
    const int mr = m < g.M ? m : g.M - 1;   // rows past the end read the last row; they are not stored
    const float* arow = A + (long)mr * g.sam;
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
      if (AVEC) {
        const float4 v = *(const float4*)(arow + k0 + 4 * c);
        x[c][0] = v.x; x[c][1] = v.y; x[c][2] = v.z; x[c][3] = v.w;
      } else {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int k = k0 + 4 * c + u;
          x[c][u] = k < g.K ? arow[(long)k * g.sak] : 0.f;
        }
      }
    }
  };
  int unit = blockIdx.x * 4 + (tid >> 6);
  const int nb0 = (unit % nparts) * SK_NBW;   // the same for every unit of this wave
  if (unit < units) load_rows(unit / nparts);

  // accumulators start at the bias
  f32x16s binit[SK_NBW];
#pragma unroll
  for (int nb = 0; nb < SK_NBW; ++nb)
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int n0 = (nb0 + nb) * 32 + 8 * q + 4 * h;
      float4 bv = make_float4(0.f, 0.f, 0.f, 0.f);
      if (n0 < g.N) {
        int sel = 0, nn = n0;
        if (g.bias_split) { sel = (n0 >= g.n_per) + (n0 >= 2 * g.n_per); nn = n0 - sel * g.n_per; }
        const float* bp = sel == 0 ? (const float*)g.bias[0] : sel == 1 ? (const float*)g.bias[1] : (const float*)g.bias[2];
        if (bp) bv = *(const float4*)(bp + nn);
      }
      binit[nb][4 * q] = bv.x; binit[nb][4 * q + 1] = bv.y; binit[nb][4 * q + 2] = bv.z; binit[nb][4 * q + 3] = bv.w;
    }

  // the weight into LDS
  const int nw = Kh * NB * 64;
  for (int i = tid * 4; i < nw; i += 1024) *(float4*)(wl + i) = make_float4(0.f, 0.f, 0.f, 0.f);
  __syncthreads();
  if (fill == 1) {
    const int Q = g.N >> 2, G = g.K * Q;
    for (int base = tid; base < G; base += 4 * 256) {
      float4 wv[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int gi = base + u * 256;
        wv[u] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (gi < G) {
          const int k = gi / Q, n0 = (gi - k * Q) * 4;
          int sel = 0, kk = k, nn = n0;
          if (g.b_split == 1) { sel = (n0 >= g.n_per) + (n0 >= 2 * g.n_per); nn = n0 - sel * g.n_per; }
          else if (g.b_split == 2) { sel = (k >= g.k_per) + (k >= 2 * g.k_per); kk = k - sel * g.k_per; }
          const float* bp = sel == 0 ? (const float*)g.B[0] : sel == 1 ? (const float*)g.B[1] : (const float*)g.B[2];
          wv[u] = *(const float4*)(bp + (long)kk * g.sbk + nn);
        }
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int gi = base + u * 256;
        if (gi < G) {
          const int k = gi / Q, n0 = (gi - k * Q) * 4;
          const int hh = k >= Kh, j = k - hh * Kh;
          *(float4*)(wl + (j * NB + (n0 >> 5)) * 64 + hh * 32 + (n0 & 31)) = wv[u];
        }
      }
    }
  } else if (fill == 2) {
    const int Q = g.K >> 2, G = g.N * Q;
    for (int base = tid; base < G; base += 4 * 256) {
      float4 wv[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int gi = base + u * 256;
        wv[u] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (gi < G) {
          const int n = gi / Q, kb = (gi - n * Q) * 4;
          int sel = 0, kk = kb, nn = n;
          if (g.b_split == 1) { sel = (n >= g.n_per) + (n >= 2 * g.n_per); nn = n - sel * g.n_per; }
          else if (g.b_split == 2) { sel = (kb >= g.k_per) + (kb >= 2 * g.k_per); kk = kb - sel * g.k_per; }
          const float* bp = sel == 0 ? (const float*)g.B[0] : sel == 1 ? (const float*)g.B[1] : (const float*)g.B[2];
          wv[u] = *(const float4*)(bp + (long)nn * g.sbn + kk);
        }
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int gi = base + u * 256;
        if (gi < G) {
          const int n = gi / Q, kb = (gi - n * Q) * 4;
          const int hh = kb >= Kh, j = kb - hh * Kh;   // Kh and kb are multiples of 4: the four k share a half
          float* dst = wl + (j * NB + (n >> 5)) * 64 + hh * 32 + (n & 31);
          dst[0] = wv[u].x; dst[NB * 64] = wv[u].y; dst[2 * NB * 64] = wv[u].z; dst[3 * NB * 64] = wv[u].w;
        }
      }
    }
  } else {
    for (int idx = tid; idx < nw; idx += 256) {
      const int l = idx & 63, nb = (idx >> 6) % NB, j = idx / (64 * NB);
      const int n = nb * 32 + (l & 31), k = (l >> 5) * Kh + j;
      if (n < g.N && k < g.K) {
        int sel = 0, kk = k, nn = n;
        if (g.b_split == 1) { sel = (n >= g.n_per) + (n >= 2 * g.n_per); nn = n - sel * g.n_per; }
        else if (g.b_split == 2) { sel = (k >= g.k_per) + (k >= 2 * g.k_per); kk = k - sel * g.k_per; }
        const float* bp = sel == 0 ? (const float*)g.B[0] : sel == 1 ? (const float*)g.B[1] : (const float*)g.B[2];
        wl[idx] = bp[(long)kk * g.sbk + (long)nn * g.sbn];
      }
    }
  }
  __syncthreads();

  for (; unit < units; unit += stride) {
    const int rb = unit / nparts;
    const int m = rb * 32 + ml;
    f32x16s acc[SK_NBW];
#pragma unroll
    for (int nb = 0; nb < SK_NBW; ++nb) acc[nb] = binit[nb];
    // a wave whose second column block does not exist (odd NB) multiplies its first block twice; nothing of the
    // copy is stored.  No branch around a matrix instruction: the accumulators stay where they are.
    const float* wbase = wl + nb0 * 64 + lane;
    const int second = nb0 + 1 < NB ? 64 : 0;
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const float* wrow = wbase + (c * 4 + u) * NB * 64;
        acc[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(wrow[0], x[c][u], acc[0], 0, 0, 0);
        acc[1] = __builtin_amdgcn_mfma_f32_32x32x2f32(wrow[second], x[c][u], acc[1], 0, 0, 0);
      }
      __builtin_amdgcn_sched_barrier(0);   // one chunk's weight reads at a time (hoisted together they take 2 * Kh registers)
    }
    if (unit + stride < units) load_rows((unit + stride) / nparts);
    if (m >= g.M) continue;
#pragma unroll
    for (int nb = 0; nb < SK_NBW; ++nb)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int n0 = (nb0 + nb) * 32 + 8 * q + 4 * h;
        if (n0 >= g.N) continue;
        float4 v = make_float4(acc[nb][4 * q], acc[nb][4 * q + 1], acc[nb][4 * q + 2], acc[nb][4 * q + 3]);
        float* dst;
        if (g.c_split) {
          const int sel = (n0 >= g.n_per) + (n0 >= 2 * g.n_per);
          float* cp = sel == 0 ? (float*)g.C[0] : sel == 1 ? (float*)g.C[1] : (float*)g.C[2];
          dst = cp + (long)m * g.ldc + (n0 - sel * g.n_per);
        } else {
          dst = (float*)g.C[0] + (long)m * g.ldc + n0;
          if (g.res) {
            const float4 r = *(const float4*)((const float*)g.res + (long)m * g.ldc + n0);
            v.x += r.x; v.y += r.y; v.z += r.z; v.w += r.w;
          }
        }
        *(float4*)dst = v;
      }
  }
}

static bool aligned16(const void* p) { return (((uintptr_t)p) & 15) == 0; }

// true if the launch was done by the matrix-instruction kernel above
static bool launch_gemm_skinny(const GemmDev& g, hipStream_t st) {
  // (a GELU epilogue stays with the ALU kernel: erf inlined once per accumulator register is too much code)
  if (g.gelu || g.split_k > 1 || g.kb > 1 || g.M < 1024 || g.N > 128 || g.K > 8 * SK_MAX_CH) return false;
  const int NB = (g.N + 31) / 32;
  const int Kh = ((g.K + 7) / 8) * 4;
  if ((long)Kh * NB * 64 > SK_MAX_LDS_FLOATS) return false;
  if ((g.b_split == 1 || g.c_split || g.bias_split) && g.n_per <= 0) return false;
  if (g.b_split == 2 && (g.k_per <= 0 || g.K > 3 * g.k_per)) return false;
  if (g.n_per > 0 && g.N > 3 * g.n_per) return false;
  const bool avec = g.sak == 1 && g.K % 8 == 0 && g.sam % 4 == 0 && aligned16(g.A);
  // outputs, residual and biases are accessed four columns at a time
  const bool split_n = g.c_split || g.bias_split;
  bool cvec = g.N % 4 == 0 && g.ldc % 4 == 0 && (!split_n || g.n_per % 4 == 0) && (!g.res || aligned16(g.res));
  const int nbuf = split_n ? (g.N + g.n_per - 1) / g.n_per : 1;
  for (int i = 0; i < (g.c_split ? nbuf : 1); ++i) cvec = cvec && g.C[i] && aligned16(g.C[i]);
  for (int i = 0; i < (g.bias_split ? nbuf : 1); ++i) cvec = cvec && (!g.bias[i] || aligned16(g.bias[i]));
  if (!cvec) return false;   // the ALU kernel takes those
  // how the weight can be read
  const int nB = g.b_split ? (g.b_split == 1 ? (g.N + g.n_per - 1) / g.n_per : (g.K + g.k_per - 1) / g.k_per) : 1;
  bool b_al = true;
  for (int i = 0; i < nB; ++i) b_al = b_al && aligned16(g.B[i]);
  int fill = 0;
  if (b_al && g.sbn == 1 && g.sbk % 4 == 0 && g.N % 4 == 0 && (g.b_split != 1 || g.n_per % 4 == 0)) fill = 1;
  else if (b_al && g.sbk == 1 && g.sbn % 4 == 0 && g.K % 4 == 0 && (g.b_split != 2 || g.k_per % 4 == 0)) fill = 2;
  const int nblk = (g.M + 31) / 32;
  const int nparts = (NB + SK_NBW - 1) / SK_NBW;   // 1 or 2
  const dim3 grid(std::min((nblk * nparts + 3) / 4, 2048)), block(256);
  const size_t lds = (size_t)Kh * NB * 64 * sizeof(float);
#define SK_CASE(N_)                                                                                               \
  case N_:                                                                                                        \
    if (avec) hipLaunchKernelGGL((gemm_skinny_kernel<true, N_>), grid, block, lds, st, g, NB, nparts, fill);       \
    else hipLaunchKernelGGL((gemm_skinny_kernel<false, N_>), grid, block, lds, st, g, NB, nparts, fill);           \
    break
  switch (Kh / 4) {
    SK_CASE(1); SK_CASE(2); SK_CASE(3); SK_CASE(4); SK_CASE(5); SK_CASE(6); SK_CASE(7); SK_CASE(8);
    SK_CASE(9); SK_CASE(10); SK_CASE(11); SK_CASE(12); SK_CASE(13); SK_CASE(14); SK_CASE(15); SK_CASE(16);
    default: return false;
  }
#undef SK_CASE
  return true;
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
  if (!a_bf16 && !b_bf16 && !c_bf16 && launch_gemm_skinny(g, st)) return IM_OK;
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

// The same weight gradient on the fp32 matrix instruction: C = A^T G is a product whose contraction runs over the
// rows, and both operands are read exactly as they lie in memory -- lane (c = lane % 32, h = lane / 32) takes
// column c of row r + h, a coalesced 128-byte piece per half wave; no LDS in the loop.  A workgroup of 4 waves owns
// `rows_per_wg` consecutive rows, a quarter each; the four accumulator sets are added through LDS as
// (w0 + w2) + (w1 + w3), a fixed order, and the workgroup writes one partial result IN ACCUMULATOR ORDER
// ([block][register quad][lane][4]: 16-byte stores, no index arithmetic); wgrad_mfma_reduce_kernel adds the
// partials in a fixed order and undoes the layout.  Columns past M resp. N read the last valid column: they only
// reach accumulator rows / columns that nobody reads.
struct WgradProblem {
  const float* A;
  long lda;
  const float* G;
  long ldg;
  int M, N;
  float* partial;
  float *o0, *o1, *o2;   // outputs of the reduction (see wgrad_mfma_reduce_kernel)
  int n_per;
  int n_off;             // column of the whole gradient that column 0 of this problem is (a gradient split by columns)
};
template <int MB, int NB>
__device__ __forceinline__ void wgrad_mfma_body(const float* __restrict__ A, long lda, const float* __restrict__ G, long ldg,
                                                int R, int M, int N, int rows_per_wg, float* __restrict__ partial,
                                                float* red_base) {
  constexpr int NBLK = MB * NB;
  float(*red)[NBLK * 16 * 64] = (float(*)[NBLK * 16 * 64])red_base;
  const int lane = threadIdx.x & 63, c = lane & 31, h = lane >> 5;
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // scalar: the row range of the wave is wave-uniform
  const int rpw = rows_per_wg >> 2;   // a multiple of 16
  const long row0 = (long)blockIdx.x * rows_per_wg + (long)w * rpw;
  f32x16s acc[MB][NB];
#pragma unroll
  for (int i = 0; i < MB; ++i)
#pragma unroll
    for (int j = 0; j < NB; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
  int ca[MB], cg[NB];
#pragma unroll
  for (int i = 0; i < MB; ++i) ca[i] = min(i * 32 + c, M - 1);
#pragma unroll
  for (int j = 0; j < NB; ++j) cg[j] = min(j * 32 + c, N - 1);
  const bool full = row0 + rpw <= R;   // wave-uniform: only the last rows of the matrix need the row test
  // Eight rows (four contraction steps) per group; the next group's 4 (MB + NB) loads are in flight while the
  // current group is multiplied.  rpw is a multiple of 16: two groups per trip, in two fixed register sets.
  float a0[4][MB], g0[4][NB], a1[4][MB], g1[4][NB];
  // A pair of rows per contraction step: the pair's address is wave-uniform (scalar registers), the lane adds its
  // row of the pair and its column as one 32-bit offset that never changes.
  int la[MB], lg[NB];
#pragma unroll
  for (int i = 0; i < MB; ++i) la[i] = h * (int)lda + ca[i];
#pragma unroll
  for (int j = 0; j < NB; ++j) lg[j] = h * (int)ldg + cg[j];
  auto load = [&](int r, float (&a)[4][MB], float (&g)[4][NB]) {
    if (full) {
      const float* pa = A + (row0 + r) * lda;
      const float* pg = G + (row0 + r) * ldg;
#pragma unroll
      for (int u = 0; u < 4; ++u) {
#pragma unroll
        for (int i = 0; i < MB; ++i) a[u][i] = pa[2 * u * lda + la[i]];
#pragma unroll
        for (int j = 0; j < NB; ++j) g[u][j] = pg[2 * u * ldg + lg[j]];
      }
    } else {
      // the last rows of the matrix: every load is issued, at an address inside the matrix, and rows past the end
      // are replaced by zeros afterwards
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const long row = row0 + r + 2 * u;
        const long rc = row < R ? row : (long)R - 1;
        const bool pair = row + 1 < R;   // wave-uniform: the second row of the pair exists
        const bool ok = row + h < R;
        const float* pa = A + rc * lda;
        const float* pg = G + rc * ldg;
#pragma unroll
        for (int i = 0; i < MB; ++i) {
          const float v = pa[pair ? la[i] : ca[i]];
          a[u][i] = ok ? v : 0.f;
        }
#pragma unroll
        for (int j = 0; j < NB; ++j) {
          const float v = pg[pair ? lg[j] : cg[j]];
          g[u][j] = ok ? v : 0.f;
        }
      }
    }
  };
  auto multiply = [&](const float (&a)[4][MB], const float (&g)[4][NB]) {
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[u][i], g[u][j], acc[i][j], 0, 0, 0);
  };
  load(0, a0, g0);
  for (int r = 0; r < rpw; r += 16) {
    load(r + 8, a1, g1);
    multiply(a0, g0);
    if (r + 16 < rpw) load(r + 16, a0, g0);
    multiply(a1, g1);
  }
  // (w0 + w2) + (w1 + w3) through LDS, 16 bytes per lane and access
  auto put = [&](float* dst) {
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
      for (int j = 0; j < NB; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q)
          *(float4*)(dst + (((i * NB + j) * 4 + q) * 64 + lane) * 4) =
              make_float4(acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]);
  };
  auto add = [&](const float* src) {
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
      for (int j = 0; j < NB; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const float4 v = *(const float4*)(src + (((i * NB + j) * 4 + q) * 64 + lane) * 4);
          acc[i][j][4 * q] += v.x; acc[i][j][4 * q + 1] += v.y; acc[i][j][4 * q + 2] += v.z; acc[i][j][4 * q + 3] += v.w;
        }
  };
  if (w >= 2) put(red[w - 2]);
  __syncthreads();
  if (w < 2) add(red[w]);
  __syncthreads();
  if (w == 1) put(red[0]);
  __syncthreads();
  if (w != 0) return;
  add(red[0]);
  put(partial + (long)blockIdx.x * (NBLK * 16 * 64));
}
template <int MB, int NB>
__global__ __launch_bounds__(256) void wgrad_mfma_f32_kernel(WgradProblem p, int R, int rows_per_wg) {
  __shared__ __attribute__((aligned(16))) float red[2 * MB * NB * 16 * 64];
  wgrad_mfma_body<MB, NB>(p.A, p.lda, p.G, p.ldg, R, p.M, p.N, rows_per_wg, p.partial, red);
}
// two weight gradients over the same rows in one launch (blockIdx.y picks the problem)
template <int MB0, int NB0, int MB1, int NB1>
__global__ __launch_bounds__(256) void wgrad_mfma_f32_pair_kernel(WgradProblem p0, WgradProblem p1, int R, int rows_per_wg) {
  constexpr int NBLK = MB0 * NB0 > MB1 * NB1 ? MB0 * NB0 : MB1 * NB1;
  __shared__ __attribute__((aligned(16))) float red[2 * NBLK * 16 * 64];
  if (blockIdx.y == 0) wgrad_mfma_body<MB0, NB0>(p0.A, p0.lda, p0.G, p0.ldg, R, p0.M, p0.N, rows_per_wg, p0.partial, red);
  else wgrad_mfma_body<MB1, NB1>(p1.A, p1.lda, p1.G, p1.ldg, R, p1.M, p1.N, rows_per_wg, p1.partial, red);
}

// Three problems of 2 x 2 blocks over the same rows (blockIdx.y picks the problem).  For 32 < d <= 42 the wide
// gradient [dWq | dWk | dWv] is split at column 64 into two such problems beside dWo.  Here a wave owns one BLOCK
// and all rows of the workgroup instead of all blocks and a quarter of the rows: 16 accumulator registers, no sum
// across the waves at the end, and room for the loads of three groups of eight rows in flight behind the group being
// multiplied at several workgroups per CU.  The partial result has the layout of wgrad_mfma_body.
__global__ __launch_bounds__(256) void wgrad_mfma_f32_tri_kernel(WgradProblem p0, WgradProblem p1, WgradProblem p2, int R,
                                                                 int rows_per_wg) {
  const WgradProblem& p = blockIdx.y == 0 ? p0 : blockIdx.y == 1 ? p1 : p2;
  const float* __restrict__ A = p.A;
  const float* __restrict__ G = p.G;
  const long lda = p.lda, ldg = p.ldg;
  const int lane = threadIdx.x & 63, c = lane & 31, h = lane >> 5;
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int bi = w >> 1, bj = w & 1;
  const long row0 = (long)blockIdx.x * rows_per_wg;   // rows_per_wg is a multiple of 32
  const int ca = min(bi * 32 + c, p.M - 1), cg = min(bj * 32 + c, p.N - 1);
  const int la = h * (int)lda + ca, lg = h * (int)ldg + cg;
  const bool full = row0 + rows_per_wg <= R;   // uniform: only the last rows of the matrix need the row test
  f32x16s acc;
#pragma unroll
  for (int r = 0; r < 16; ++r) acc[r] = 0.f;
  float a[4][4], g[4][4];   // [register set][contraction step of the group]
  auto multiply = [&](const float (&av)[4], const float (&gv)[4]) {
#pragma unroll
    for (int u = 0; u < 4; ++u) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(av[u], gv[u], acc, 0, 0, 0);
  };
  // The whole loop exists twice, with and without the row test, and its last trip is peeled: no branch between a
  // group's loads and its use, so the waits count exactly the loads requested after it.
  auto run = [&](auto full_tag) {
    constexpr bool FULL = decltype(full_tag)::value;
    auto load = [&](int r, float (&av)[4], float (&gv)[4]) {
      if constexpr (FULL) {
        const float* pa = A + (row0 + r) * lda;
        const float* pg = G + (row0 + r) * ldg;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          av[u] = pa[2 * u * lda + la];
          gv[u] = pg[2 * u * ldg + lg];
        }
      } else {
#pragma unroll
        for (int u = 0; u < 4; ++u) {   // every load is issued, inside the matrix; rows past the end become zeros
          const long row = row0 + r + 2 * u;
          const long rc = row < R ? row : (long)R - 1;
          const bool pair = row + 1 < R, ok = row + h < R;
          const float va = A[rc * lda + (pair ? la : ca)];
          const float vg = G[rc * ldg + (pair ? lg : cg)];
          av[u] = ok ? va : 0.f;
          gv[u] = ok ? vg : 0.f;
        }
      }
    };
    load(0, a[0], g[0]);
    load(8, a[1], g[1]);
    load(16, a[2], g[2]);
    int r = 0;
    for (; r + 32 < rows_per_wg; r += 32) {
      load(r + 24, a[3], g[3]);
      multiply(a[0], g[0]);
      load(r + 32, a[0], g[0]);
      multiply(a[1], g[1]);
      load(r + 40, a[1], g[1]);
      multiply(a[2], g[2]);
      load(r + 48, a[2], g[2]);
      multiply(a[3], g[3]);
    }
    load(r + 24, a[3], g[3]);
    multiply(a[0], g[0]);
    multiply(a[1], g[1]);
    multiply(a[2], g[2]);
    multiply(a[3], g[3]);
  };
  if (full) run(std::true_type{});
  else run(std::false_type{});
  float* dst = p.partial + (long)blockIdx.x * (4 * 16 * 64);
#pragma unroll
  for (int q = 0; q < 4; ++q)
    *(float4*)(dst + (((bi * 2 + bj) * 4 + q) * 64 + lane) * 4) =
        make_float4(acc[4 * q], acc[4 * q + 1], acc[4 * q + 2], acc[4 * q + 3]);
}

// out[m, n] = sum_z partial[z] (accumulator order, see above), z ascending in 16 interleaved groups that are then
// added in a fixed order; column block s of n_per columns goes to o<s> (NULL = dropped) when n_per > 0.
// A thread sums one accumulator QUAD (16 bytes: four rows of one column) of its share of the partial results, so
// the 16 threads of a group read 256 contiguous bytes of every partial result; grid.x covers the quads of the
// largest problem, 16 per workgroup.
__global__ __launch_bounds__(256) void wgrad_mfma_reduce_kernel(WgradProblem p0, WgradProblem p1, WgradProblem p2, int nz) {
  __shared__ float4 red[16][16];
  const WgradProblem& p = blockIdx.y == 0 ? p0 : blockIdx.y == 1 ? p1 : p2;
  const float4* __restrict__ partial = (const float4*)p.partial;
  const int M = p.M, N = p.N, NB = (N + 31) / 32, nblk = ((M + 31) / 32) * NB, n_per = p.n_per;
  const int o = threadIdx.x & 15, g = threadIdx.x >> 4;
  const int nquad = nblk * 4 * 64;          // quads of one partial result: [block][register quad][lane]
  const int i = blockIdx.x * 16 + o;
  float4 s[4];
#pragma unroll
  for (int k = 0; k < 4; ++k) s[k] = make_float4(0.f, 0.f, 0.f, 0.f);
  if (i < nquad) {
    // eight partial results per trip, all requested (at an index inside the array) before the first is added
    for (int z = g; z < nz; z += 128) {
      float4 v[8];
#pragma unroll
      for (int k = 0; k < 8; ++k) v[k] = partial[(long)min(z + 16 * k, nz - 1) * nquad + i];
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        if (z + 16 * k < nz) {
          float4& t = s[k & 3];
          t.x += v[k].x; t.y += v[k].y; t.z += v[k].z; t.w += v[k].w;
        }
      }
    }
  }
  red[g][o] = make_float4((s[0].x + s[1].x) + (s[2].x + s[3].x), (s[0].y + s[1].y) + (s[2].y + s[3].y),
                          (s[0].z + s[1].z) + (s[2].z + s[3].z), (s[0].w + s[1].w) + (s[2].w + s[3].w));
  __syncthreads();
  if (g == 0 && i < nquad) {
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
    for (int k = 0; k < 16; ++k) { v.x += red[k][o].x; v.y += red[k][o].y; v.z += red[k][o].z; v.w += red[k][o].w; }
    // quad q of lane (c, h) in block (bi, bj): rows 32 bi + 8 q + 4 h + 0..3, column 32 bj + c
    const int lane = i & 63, q = (i >> 6) & 3, blk = i >> 8, bi = blk / NB, bj = blk - bi * NB;
    const int n = bj * 32 + (lane & 31), m0 = bi * 32 + 8 * q + 4 * (lane >> 5);
    if (n < N) {
      const float vv[4] = {v.x, v.y, v.z, v.w};
      float* dst = p.o0;
      long ld = N, col = n;
      if (n_per > 0) {
        const int gn = n + p.n_off;
        dst = (gn / n_per == 0) ? p.o0 : (gn / n_per == 1) ? p.o1 : p.o2;
        ld = n_per; col = gn % n_per;
      }
      if (dst) {
#pragma unroll
        for (int j = 0; j < 4; ++j)
          if (m0 + j < M) dst[(long)(m0 + j) * ld + col] = vv[j];
      }
    }
  }
}

static int wgrad_mfma_rows_per_wg(int R) {
  // at most 1024 workgroups = partial results, and at least 128 rows each (measured at 29 600 rows, 40 x 120:
  // 64 rows 22 us, 128 rows 17 us, 256 rows 25 us including the reduction); a multiple of 64: every wave then has
  // a multiple of 16 rows = two groups of four steps per trip
  const int rows = std::max((R + 1023) / 1024, 128);
  return ((rows + 63) / 64) * 64;
}
bool wgrad_mfma_ok(int M, int N, int R, int in_bf16) { return !in_bf16 && M <= 64 && N <= 128 && R >= 1024; }
size_t wgrad_mfma_partial_bytes(int M, int N, int R) {
  const int rows = wgrad_mfma_rows_per_wg(R);
  return (size_t)((R + rows - 1) / rows) * ((M + 31) / 32) * ((N + 31) / 32) * 16 * 64 * sizeof(float);
}
// Up to two gradients with 33..64 rows through wgrad_mfma_f32_tri_kernel: `a` (at most 128 columns; more than 64
// only with column-block outputs) becomes one or two problems of at most 64 columns, `b` (optional, at most 64
// columns) one more.  The partial results lie one problem after the other from `partial` on.  A gradient's bits do
// not depend on what else the launch computes.
static void launch_wgrad_mfma_f32_tri(const WgradProblem* a, const WgradProblem* b, int R, float* partial, hipStream_t st) {
  // rows per workgroup: a multiple of 32, those of the layout that the workspace is sized for
  const int rows3 = (wgrad_mfma_rows_per_wg(R) + 31) / 32 * 32;
  const int blocks3 = (R + rows3 - 1) / rows3;
  const long pstride = (long)blocks3 * 4 * 16 * 64;
  WgradProblem ps[3];
  int n = 0;
  auto push = [&](const WgradProblem& src, int col0, int ncols) {
    ps[n] = src;
    ps[n].G = src.G + col0;
    ps[n].N = ncols;
    ps[n].n_off = col0;
    ps[n].partial = partial + n * pstride;
    ++n;
  };
  if (a->N > 64) { push(*a, 0, 64); push(*a, 64, a->N - 64); }
  else push(*a, 0, a->N);
  if (b) push(*b, 0, b->N);
  for (int k = n; k < 3; ++k) ps[k] = ps[0];
  hipLaunchKernelGGL(wgrad_mfma_f32_tri_kernel, dim3(blocks3, n), dim3(256), 0, st, ps[0], ps[1], ps[2], R, rows3);
  hipLaunchKernelGGL(wgrad_mfma_reduce_kernel, dim3(4 * 16, n), dim3(256), 0, st, ps[0],
                     ps[1], ps[2], blocks3);
}
// C[M, N] = A[R, M]^T G[R, N] into o0 (n_per == 0) or column blocks of n_per columns into o0 | o1 | o2
void launch_wgrad_mfma_f32(const float* A, long lda, const float* G, long ldg, int R, int M, int N, float* partial,
                           float* o0, float* o1, float* o2, int n_per, hipStream_t st) {
  const int rows = wgrad_mfma_rows_per_wg(R);
  const int blocks = (R + rows - 1) / rows;
  const int MB = (M + 31) / 32, NB = (N + 31) / 32;
  const WgradProblem p{A, lda, G, ldg, M, N, partial, o0, o1, o2, n_per};
  if (MB == 2 && (N <= 64 || n_per > 0)) {
    launch_wgrad_mfma_f32_tri(&p, nullptr, R, partial, st);
    return;
  }
#define WM_LAUNCH(MBV, NBV) hipLaunchKernelGGL((wgrad_mfma_f32_kernel<MBV, NBV>), dim3(blocks), dim3(256), 0, st, p, R, rows)
  if (MB == 1) {
    if (NB == 1) WM_LAUNCH(1, 1); else if (NB == 2) WM_LAUNCH(1, 2); else if (NB == 3) WM_LAUNCH(1, 3); else WM_LAUNCH(1, 4);
  } else {
    if (NB == 1) WM_LAUNCH(2, 1); else if (NB == 2) WM_LAUNCH(2, 2); else if (NB == 3) WM_LAUNCH(2, 3); else WM_LAUNCH(2, 4);
  }
#undef WM_LAUNCH
  hipLaunchKernelGGL(wgrad_mfma_reduce_kernel, dim3(MB * NB * 16, 1), dim3(256), 0, st, p, p, p, blocks);
}
// The two weight gradients of an attention block in one pair of launches:
//   [dWq | dWk | dWv] = X^T [dQ | dK | dV]  (d x 3d, column blocks of d columns into q0 | q1 | q2, NULL = dropped)
//   dWo               = O^T dY              (d x d)
// partial: wgrad_mfma_partial_bytes(d, 3 d, R) + wgrad_mfma_partial_bytes(d, d, R) bytes.
void launch_wgrad_mfma_f32_attn(const float* X, const float* dQKV, const float* O, const float* dY, int R, int d,
                                float* partial, float* q0, float* q1, float* q2, float* dwo, hipStream_t st) {
  const int MB = (d + 31) / 32, NB0 = (3 * d + 31) / 32;
  if (MB == 2) {
    const WgradProblem wide{X, d, dQKV, 3L * d, d, 3 * d, partial, q0, q1, q2, d, 0};
    const WgradProblem wo{O, d, dY, d, d, d, nullptr, dwo, nullptr, nullptr, 0, 0};
    launch_wgrad_mfma_f32_tri(&wide, &wo, R, partial, st);
    return;
  }
  const int rows = wgrad_mfma_rows_per_wg(R);
  const int blocks = (R + rows - 1) / rows;
  float* partial1 = partial + wgrad_mfma_partial_bytes(d, 3 * d, R) / sizeof(float);
  const WgradProblem p0{X, d, dQKV, 3L * d, d, 3 * d, partial, q0, q1, q2, d};
  const WgradProblem p1{O, d, dY, d, d, d, partial1, dwo, nullptr, nullptr, 0};
  const dim3 grid(blocks, 2), block(256);
  if (NB0 == 3) hipLaunchKernelGGL((wgrad_mfma_f32_pair_kernel<1, 3, 1, 1>), grid, block, 0, st, p0, p1, R, rows);
  else if (NB0 == 2) hipLaunchKernelGGL((wgrad_mfma_f32_pair_kernel<1, 2, 1, 1>), grid, block, 0, st, p0, p1, R, rows);
  else hipLaunchKernelGGL((wgrad_mfma_f32_pair_kernel<1, 1, 1, 1>), grid, block, 0, st, p0, p1, R, rows);
  hipLaunchKernelGGL(wgrad_mfma_reduce_kernel, dim3(MB * NB0 * 16, 2), dim3(256), 0, st, p0, p1, p1, blocks);
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
// Stage 1 with 16-byte loads, for matrices whose rows allow them (n and lda multiples of the vector width, base
// aligned, n <= 256 vectors): a block covers all n columns of its CS_ROWS rows as (n / VW column groups) x (row
// groups); a thread requests eight rows at a time.  The element-per-thread kernel above walks 64 rows per thread
// with four loads in flight, which at 30 000 rows is sixteen exposed round trips per launch.
template <typename T>
__global__ __launch_bounds__(256) void colsum_stage1_vec(ColsumArgs q, int R, int n, float* __restrict__ partial) {
  constexpr int VW = 16 / sizeof(T);
  __shared__ float red[256 * VW];
  const int z = blockIdx.z;
  if (!q.out[z]) return;
  const T* __restrict__ a = (const T*)q.a[z];
  const long lda = q.lda[z];
  const int CG = n / VW, RG = 256 / CG;
  const int cg = threadIdx.x % CG, rg = threadIdx.x / CG;
  const int r0 = blockIdx.y * CS_ROWS, r1 = min(R, r0 + CS_ROWS);
  float s[VW];
#pragma unroll
  for (int e = 0; e < VW; ++e) s[e] = 0.f;
  if (rg < RG) {
    for (int r = r0 + rg; r < r1; r += 8 * RG) {
      uint4 v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int rr = min(r + u * RG, r1 - 1);   // every load is issued (no branch, no wait per row); rows past the
        v[u] = *(const uint4*)(a + (long)rr * lda + cg * VW);   // block are read again and dropped below
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        if (r + u * RG >= r1) v[u] = make_uint4(0u, 0u, 0u, 0u);
        const unsigned w[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          if (sizeof(T) == 2) { s[2 * e] += __uint_as_float(w[e] << 16); s[2 * e + 1] += __uint_as_float(w[e] & 0xffff0000u); }
          else s[e] += __uint_as_float(w[e]);
        }
      }
    }
#pragma unroll
    for (int e = 0; e < VW; ++e) red[rg * n + cg * VW + e] = s[e];
  }
  __syncthreads();
  for (int c = threadIdx.x; c < n; c += 256) {
    float t = red[c];
    for (int g = 1; g < RG; ++g) t += red[g * n + c];
    partial[((long)z * gridDim.y + blockIdx.y) * n + c] = t;
  }
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

// One launch for a list of second-stage sums (blockIdx.y = job).  A block is 16 output quads x 16 lanes over the
// partials: lane zl adds partials zl, zl + 16, ... in ascending order, then the 16 lane sums are added in a fixed
// order through LDS -- the same order as colsum_stage2 and the parallel split-K reduction use on their own.
__global__ __launch_bounds__(256) void reduce_list_kernel(ReduceList l) {
  __shared__ float4 red[16][16];
  const ReduceJob& j = l.job[blockIdx.y];
  const long n_out = (long)j.M * j.N;
  const int ql = threadIdx.x & 15, zl = threadIdx.x >> 4;
  if ((long)blockIdx.x * 64 >= n_out) return;   // block-uniform
  const long i = ((long)blockIdx.x * 16 + ql) * 4;
  float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
  if (i < n_out) {
    int z = zl;
    for (; z + 48 < j.nparts; z += 64) {   // four requests in flight; added in the same ascending order
      float4 v[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) v[u] = *(const float4*)(j.partial + (z + 16 * u) * n_out + i);
#pragma unroll
      for (int u = 0; u < 4; ++u) { s.x += v[u].x; s.y += v[u].y; s.z += v[u].z; s.w += v[u].w; }
    }
    for (; z < j.nparts; z += 16) {
      const float4 v = *(const float4*)(j.partial + z * n_out + i);
      s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
    }
  }
  red[zl][ql] = s;
  __syncthreads();
  if (zl != 0 || i >= n_out) return;
  for (int k = 1; k < 16; ++k) {
    const float4 v = red[k][ql];
    s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
  }
  const int m = (int)(i / j.N), n = (int)(i % j.N);
  float* o = j.o[0];
  long at = i;
  if (j.n_per > 0) {
    const int sel = n / j.n_per;
    o = sel == 0 ? j.o[0] : sel == 1 ? j.o[1] : j.o[2];
    at = (long)m * j.n_per + n % j.n_per;
  }
  if (!o) return;
  o[at] = s.x; o[at + 1] = s.y; o[at + 2] = s.z; o[at + 3] = s.w;   // caller pointers: no alignment assumed
}
bool reduce_deferrable(int M, int N, int nparts) {
  return N % 4 == 0 && (long)M * N <= 4L * 65536 && (long)M * N * nparts * 4 <= (8L << 20);
}
void reduce_push(ReduceList* l, const float* partial, int nparts, int M, int N, float* o0, float* o1, float* o2, int n_per) {
  ReduceJob& j = l->job[l->n++];
  j.partial = partial; j.nparts = nparts; j.M = M; j.N = N; j.n_per = n_per;
  j.o[0] = o0; j.o[1] = o1; j.o[2] = o2;
}
void launch_reduce_list(const ReduceList& l, hipStream_t st) {
  if (l.n == 0) return;
  long mx = 0;
  for (int i = 0; i < l.n; ++i) mx = std::max(mx, (long)l.job[i].M * l.job[i].N);
  hipLaunchKernelGGL(reduce_list_kernel, dim3((unsigned)((mx + 63) / 64), l.n), dim3(256), 0, st, l);
}

int launch_colsum_multi(const void* const* a, const long* lda, float* const* out, int count, int R, int n, int a_bf16,
                        float* partial, hipStream_t st, ReduceList* defer) {
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
  const int vw = a_bf16 ? 8 : 4;
  bool vec = n % vw == 0 && n / vw <= 256;
  for (int i = 0; i < count; ++i)
    if (q.out[i]) vec = vec && q.lda[i] % vw == 0 && (reinterpret_cast<uintptr_t>(q.a[i]) & 15) == 0;
  if (vec && a_bf16) hipLaunchKernelGGL((colsum_stage1_vec<bf16_t>), dim3(1, nblk, count), block, 0, st, q, R, n, partial);
  else if (vec) hipLaunchKernelGGL((colsum_stage1_vec<float>), dim3(1, nblk, count), block, 0, st, q, R, n, partial);
  else if (a_bf16) hipLaunchKernelGGL((colsum_stage1<bf16_t>), grid, block, 0, st, q, R, n, partial);
  else hipLaunchKernelGGL((colsum_stage1<float>), grid, block, 0, st, q, R, n, partial);
  if (defer && reduce_deferrable(1, n, nblk) && defer->n + count <= 16) {
    for (int i = 0; i < count; ++i)
      if (q.out[i]) reduce_push(defer, partial + (long)i * nblk * n, nblk, 1, n, q.out[i], nullptr, nullptr, 0);
    return IM_OK;
  }
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
