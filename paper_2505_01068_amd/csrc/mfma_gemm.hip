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

// GELU(x) = x Phi(x) = max(x, 0) - |x| erfc(|x| / sqrt 2) / 2, with erfc(u) = 2^(-u p(u)) for a quartic p fitted on
// [0, 6.5] (|error| of erfc <= 6e-7, of GELU <= 1.2e-6 in fp32 -- three orders below the bf16 rounding of the
// result; the coefficients below are those of p with the 1 / sqrt 2 folded in).  Four multiply-adds for p, one
// for the exponent, one exp2, a multiply, a maximum and a subtraction: the epilogue of the first MLP GEMM
// evaluates this for every hidden element, and the library erff takes several dozen instructions.
__device__ __forceinline__ float gelu_erf_f(float x) {
  const float a = fabsf(x);
  float p = fmaf(0.0005204590852372348f, a, -0.007397513370960951f);
  p = fmaf(p, a, 0.05256124213337898f);
  p = fmaf(p, a, 0.4592546820640564f);
  p = fmaf(p, a, 1.1510913372039795f);
  const float e = __builtin_amdgcn_exp2f(fmaf(-p, a, -1.f));   // erfc(|x| / sqrt 2) / 2
  return fmaxf(x, 0.f) - e * a;
}

// d/dx [x Phi(x)] = Phi(x) + x phi(x), Phi from the same erfc form, phi(x) = exp(-x^2 / 2) / sqrt(2 pi)
__device__ __forceinline__ float gelu_grad_f(float x) {
  const float a = fabsf(x);
  float p = fmaf(0.0005204590852372348f, a, -0.007397513370960951f);
  p = fmaf(p, a, 0.05256124213337898f);
  p = fmaf(p, a, 0.4592546820640564f);
  p = fmaf(p, a, 1.1510913372039795f);
  const float e = __builtin_amdgcn_exp2f(fmaf(-p, a, -1.f));   // erfc(|x| / sqrt 2) / 2
  const float Phi = x >= 0.f ? 1.f - e : e;
  const float pdf = 0.39894228040143267794f * __builtin_amdgcn_exp2f(-0.72134752044448170368f * x * x);
  return fmaf(x, pdf, Phi);
}

template <int U>
struct TileRegs {
  u32x4 v[U];
};
typedef TileRegs<4> Tile128;

// m-major operand: tile rows r0..r0+32U-1 (clamped to rmax), K columns c0..c0+63 (zero beyond cmax)
template <int U>
__device__ __forceinline__ void load_mm(TileRegs<U>& t, const bf16_t* base, long ld, int r0, int rmax, int c0, int cmax,
                                        int tid) {
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int r = (tid >> 3) + u * 32, c = c0 + (tid & 7) * 8;
    const int rr = min(r0 + r, rmax);
    u32x4 v = {0u, 0u, 0u, 0u};
    if (c < cmax) v = *(const u32x4*)(base + (long)rr * ld + c);  // K is a multiple of 8 for every caller
    t.v[u] = v;
  }
}
template <int U>
__device__ __forceinline__ void store_mm(const TileRegs<U>& t, bf16_t* lds, int tid) {
#pragma unroll
  for (int u = 0; u < U; ++u) {
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
      if (n_per > 0) {   // select chain, not a dynamic index: the three pointers stay in scalar registers
        const int bi = c / n_per;
        m = bi == 0 ? mats[0] : bi == 1 ? mats[1] : mats[2];
        cc = c - bi * n_per;
      }
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

// LayerNorm of the staged rows of a row-major A tile whose 64 columns are the whole feature row
// (K == 64): the 8 lanes that hold a row (8 elements each) share its mean and variance through three
// shuffles; two-pass in fp32 and rounded to bf16 exactly as the stand-alone kernel does.
template <int U>
__device__ __forceinline__ void ln_tile_rows(TileRegs<U>& t, const bf16_t* gamma, const bf16_t* beta, float eps, int tid) {
  const int c = (tid & 7) * 8;
  const u32x4 gr = *(const u32x4*)(gamma + c), br = *(const u32x4*)(beta + c);
#pragma unroll
  for (int u = 0; u < U; ++u) {
    float v[8];
#pragma unroll
    for (int j = 0; j < 4; ++j) { v[2 * j] = __uint_as_float(t.v[u][j] << 16); v[2 * j + 1] = __uint_as_float(t.v[u][j] & 0xffff0000u); }
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < 8; ++j) s += v[j];
#pragma unroll
    for (int o = 4; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
    const float mu = s * (1.f / 64.f);
    float q = 0.f;
#pragma unroll
    for (int j = 0; j < 8; ++j) { const float w = v[j] - mu; q = fmaf(w, w, q); }
#pragma unroll
    for (int o = 4; o > 0; o >>= 1) q += __shfl_xor(q, o, 64);
    const float rstd = rsqrtf(q * (1.f / 64.f) + eps);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const float a = (v[2 * j] - mu) * rstd * __uint_as_float(gr[j] << 16) + __uint_as_float(br[j] << 16);
      const float b = (v[2 * j + 1] - mu) * rstd * __uint_as_float(gr[j] & 0xffff0000u) + __uint_as_float(br[j] & 0xffff0000u);
      t.v[u][j] = pack_bf16(a, b);
    }
  }
}

// EPI: the epilogue may apply GELU and add a residual (separate instantiation, so that the plain
// bias epilogue of the attention projections stays a few hundred instructions long).
// Bias of the 4 consecutive output columns n .. n+3 (n % 4 == 0) as fp32; 0 without a bias or past
// N.  The columns lie in one of at most three blocks of width n_per (one bias vector each), so the
// block index needs no integer division.
__device__ __forceinline__ void bias4(const MGemm& p, const bf16_t* const (&bias)[3], int n, float (&out)[4]) {
  out[0] = out[1] = out[2] = out[3] = 0.f;
  if (p.n_per <= 0 || n >= p.N) return;
  const int sel = (n >= p.n_per) + (n >= 2 * p.n_per);
  const bf16_t* bp = sel == 0 ? bias[0] : sel == 1 ? bias[1] : bias[2];
  if (!bp) return;
  const bf16_t* q = bp + (n - sel * p.n_per);
  if ((reinterpret_cast<uintptr_t>(bp) & 7) == 0) {
    const u32x2 v = *(const u32x2*)q;
    out[0] = __uint_as_float(v[0] << 16); out[1] = __uint_as_float(v[0] & 0xffff0000u);
    out[2] = __uint_as_float(v[1] << 16); out[3] = __uint_as_float(v[1] & 0xffff0000u);
  } else {
#pragma unroll
    for (int j = 0; j < 4; ++j) out[j] = bf2f(q[j]);
  }
}

// The same for NQ column groups at once: every load is issued before the first value is used (one call of bias4
// per group is a conditional load and a wait per group, eight memory round trips in front of a tile's main loop).
template <int NQ>
__device__ __forceinline__ void bias4_many(const MGemm& p, const bf16_t* const (&bias)[3], const int (&n)[NQ],
                                           float (&out)[NQ][4]) {
  const bf16_t* any = bias[0] ? bias[0] : bias[1] ? bias[1] : bias[2];
  if (p.n_per <= 0 || !any) {
#pragma unroll
    for (int q = 0; q < NQ; ++q) out[q][0] = out[q][1] = out[q][2] = out[q][3] = 0.f;
    return;
  }
  const bool al = ((reinterpret_cast<uintptr_t>(bias[0]) | reinterpret_cast<uintptr_t>(bias[1]) |
                    reinterpret_cast<uintptr_t>(bias[2])) & 7) == 0;
  const bf16_t* src[NQ];
  bool have[NQ];
#pragma unroll
  for (int q = 0; q < NQ; ++q) {
    const int nn = n[q] < p.N ? n[q] : 0;
    const int sel = (nn >= p.n_per) + (nn >= 2 * p.n_per);
    const bf16_t* bp = sel == 0 ? bias[0] : sel == 1 ? bias[1] : bias[2];
    have[q] = bp != nullptr && n[q] < p.N;
    src[q] = (bp ? bp : any) + (nn - sel * p.n_per);   // every bias vector has n_per elements: a valid address either way
  }
  u32x2 raw[NQ];
  if (al) {
#pragma unroll
    for (int q = 0; q < NQ; ++q) raw[q] = *(const u32x2*)src[q];
  } else {
    unsigned short h[NQ][4];
#pragma unroll
    for (int q = 0; q < NQ; ++q)
#pragma unroll
      for (int j = 0; j < 4; ++j) h[q][j] = src[q][j];
#pragma unroll
    for (int q = 0; q < NQ; ++q) raw[q] = u32x2{(unsigned)h[q][0] | ((unsigned)h[q][1] << 16), (unsigned)h[q][2] | ((unsigned)h[q][3] << 16)};
  }
#pragma unroll
  for (int q = 0; q < NQ; ++q) {
    out[q][0] = have[q] ? __uint_as_float(raw[q][0] << 16) : 0.f; out[q][1] = have[q] ? __uint_as_float(raw[q][0] & 0xffff0000u) : 0.f;
    out[q][2] = have[q] ? __uint_as_float(raw[q][1] << 16) : 0.f; out[q][3] = have[q] ? __uint_as_float(raw[q][1] & 0xffff0000u) : 0.f;
  }
}

// TM = rows of the tile: 128, or 64 (m-major A only; each wave then owns 32 x 64) for shapes whose 128-row
// tiles would not fill the chip -- with about one workgroup per CU nothing overlaps the chain load ->
// LDS -> MFMA -> epilogue loads -> store of a workgroup, and twice as many half-size workgroups finish sooner.
template <bool AKM, bool BKM, bool EPI, int TM>
__device__ __forceinline__ void mfma_gemm_tile(const MGemm& p, int bx, int by, int bz, int pz) {
  static_assert(TM == GM || (TM == 64 && !AKM), "the 64-row tile exists for m-major A only");
  constexpr int MB = TM / 64;  // 32-row blocks per wave
  __shared__ __attribute__((aligned(16))) bf16_t sA[AKM ? GK * KM_LD : TM * LDS_LD];
  __shared__ __attribute__((aligned(16))) bf16_t sB[BKM ? GK * KM_LD : GN * LDS_LD];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, lo = lane & 31, hi = lane >> 5;
  const int wm = wave >> 1, wn = wave & 1;
  const int m0 = by * TM, n0 = bx * GN;
  // pz = 1: the second problem of a paired launch, whose tensors lie at the byte offsets p.z_* from the first one's
  auto zoff = [&](const bf16_t* q, long off) { return q && pz ? (const bf16_t*)((const char*)q + off) : q; };
  const bf16_t* const pA = zoff(p.A, p.z_a);
  const bf16_t* const pln_g = zoff(p.ln_g, p.z_ln_g);
  const bf16_t* const pln_b = zoff(p.ln_b, p.z_ln_b);
  const bf16_t* const pres = zoff(p.res, p.z_res);
  bf16_t* const pC = (bf16_t*)zoff(p.C, p.z_c);
  const bf16_t* pbias[3] = {zoff(p.bias[0], p.z_bias[0]), zoff(p.bias[1], p.z_bias[1]), zoff(p.bias[2], p.z_bias[2])};

  const int ktiles = (p.K + GK - 1) / GK;
  const int per_split = (ktiles + p.split_k - 1) / p.split_k;
  const int it_begin = bz * per_split, it_end = min(ktiles, it_begin + per_split);

  // [n block][m block]: rows of the accumulator = n, cols = m; registers 4i..4i+3 are columns
  // n = 8i + 4hi + 0..3 of the block.  The accumulators start at the bias of their column (split-K launches
  // carry no bias), so the epilogue has nothing to add.
  f32x16 acc[2][MB];

  const bf16_t* amat[3] = {pA, pA, pA};
  const bf16_t* bmat[3] = {zoff(p.B[0], p.z_b[0]), zoff(p.B[1], p.z_b[1]), zoff(p.B[2], p.z_b[2])};
  TileRegs<TM / 32> ta;
  Tile128 tb;
  auto prefetch = [&](int it) {
    const int k0 = it * GK;
    if constexpr (AKM) load_km(ta, amat, 0, p.lda, k0, p.K, m0, p.M, tid);
    else {
      load_mm(ta, pA, p.lda, m0, p.M - 1, k0, p.K, tid);
      if (pln_g) ln_tile_rows(ta, pln_g, pln_b, p.ln_eps, tid);  // K == 64: this is the only k-tile
    }
    if (BKM) {
      load_km(tb, bmat, p.b_nper, p.ldb, k0, p.K, n0, p.N, tid);
    } else {
      const bf16_t* Bp = bmat[0];
      int kk = k0, kmax = p.K;
      if (p.b_kper > 0) {
        const int bi = k0 / p.b_kper;
        Bp = bi == 0 ? bmat[0] : bi == 1 ? bmat[1] : bmat[2];
        kk = k0 - bi * p.b_kper; kmax = p.b_kper;
      }
      load_mm(tb, Bp, p.ldb, n0, p.N - 1, kk, kmax, tid);
    }
  };
  if (it_begin < it_end) prefetch(it_begin);
  {   // the bias values are requested behind the first tile, all eight groups at once
    int nq[8];
    float bq[8][4];
#pragma unroll
    for (int nb = 0; nb < 2; ++nb)
#pragma unroll
      for (int i = 0; i < 4; ++i) nq[nb * 4 + i] = p.partial ? p.N : n0 + wn * 64 + nb * 32 + 8 * i + 4 * hi;
    bias4_many<8>(p, pbias, nq, bq);
#pragma unroll
    for (int nb = 0; nb < 2; ++nb)
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
          for (int jj = 0; jj < 4; ++jj) acc[nb][mb][4 * i + jj] = bq[nb * 4 + i][jj];
  }
  for (int it = it_begin; it < it_end; ++it) {
    __syncthreads();
    if constexpr (AKM) store_km(ta, sA, tid); else store_mm(ta, sA, tid);
    if (BKM) store_km(tb, sB, tid); else store_mm(tb, sB, tid);
    __syncthreads();
    if (it + 1 < it_end) prefetch(it + 1);
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      bf16x8 fa[MB], fb[2];
#pragma unroll
      for (int x = 0; x < MB; ++x)
        fa[x] = AKM ? lds_frag_tr(sA, KM_LD, s * 16, wm * 32 * MB + x * 32, lane)
                    : lds_frag(sA, wm * 32 * MB + x * 32 + lo, s * 16 + hi * 8);
#pragma unroll
      for (int x = 0; x < 2; ++x)
        fb[x] = BKM ? lds_frag_tr(sB, KM_LD, s * 16, wn * 64 + x * 32, lane)
                    : lds_frag(sB, wn * 64 + x * 32 + lo, s * 16 + hi * 8);
#pragma unroll
      for (int nb = 0; nb < 2; ++nb)
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) acc[nb][mb] = mfma32(fb[nb], fa[mb], acc[nb][mb]);
    }
  }

  // ---- epilogue: lane owns row m; registers 4i..4i+3 are columns n = 8i + 4hi + 0..3 of the block ----
  if (p.partial) {  // split-K: fp32 partial sums, 16 bytes per lane
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
      const int m = m0 + wm * 32 * MB + mb * 32 + lo;
      if (m >= p.M) continue;
#pragma unroll
      for (int nb = 0; nb < 2; ++nb)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int n = n0 + wn * 64 + nb * 32 + 8 * i + 4 * hi;
          if (n >= p.N) continue;  // N is a multiple of 4 for every caller
          *(float4*)(p.partial + ((long)bz * p.M + m) * p.N + n) =
              make_float4(acc[nb][mb][4 * i], acc[nb][mb][4 * i + 1], acc[nb][mb][4 * i + 2], acc[nb][mb][4 * i + 3]);
        }
    }
    return;
  }
  // Direct 8-byte stores (a lane owns a row of the accumulator tile).  Staging the tile through LDS
  // for 16-byte row-contiguous stores was measured slower here: with three workgroups per CU the
  // stores of one overlap the loads of the others, and the extra barrier costs more than it saves.
#pragma unroll
  for (int mb = 0; mb < MB; ++mb) {
    const int m = m0 + wm * 32 * MB + mb * 32 + lo;
    if (m >= p.M) continue;
    // the residual (or saved pre-activation) values of the lane's row: all eight requests before the first use --
    // loaded where they are added, each was a memory round trip of its own
    u32x2 rvs[2][4];
    if constexpr (EPI) {
      if (pres) {
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const int n = n0 + wn * 64 + nb * 32 + 8 * i + 4 * hi;
            rvs[nb][i] = *(const u32x2*)(pres + (long)m * p.ldc + (n < p.N ? n : 0));
          }
      }
    }
#pragma unroll
    for (int nb = 0; nb < 2; ++nb)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int n = n0 + wn * 64 + nb * 32 + 8 * i + 4 * hi;
        if (n >= p.N) continue;  // N is a multiple of 4 for every caller
        float v[4];
        const float cs = (p.scale0_on && n < p.n_per) ? p.scale0 : 1.f;
#pragma unroll
        for (int j = 0; j < 4; ++j) v[j] = acc[nb][mb][4 * i + j] * cs;
        if constexpr (EPI) {
          if (p.gelu == MGEMM_GELU_BOTH) {
            // the pre-activation goes to C as it is; C2 gets GELU of the ROUNDED pre-activation, the value a
            // backward pass will read back
            const u32x2 pre = {pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3])};
            *(u32x2*)(pC + (long)m * p.ldc + n) = pre;
            const u32x2 act = {pack_bf16(gelu_erf_f(__uint_as_float(pre[0] << 16)), gelu_erf_f(__uint_as_float(pre[0] & 0xffff0000u))),
                               pack_bf16(gelu_erf_f(__uint_as_float(pre[1] << 16)), gelu_erf_f(__uint_as_float(pre[1] & 0xffff0000u)))};
            *(u32x2*)(p.C2 + (long)m * p.ldc + n) = act;
            continue;
          }
          if (p.gelu == MGEMM_GELU_GRAD) {   // C = (A B) * GELU'(res)
            const u32x2 rv = rvs[nb][i];
            v[0] *= gelu_grad_f(__uint_as_float(rv[0] << 16)); v[1] *= gelu_grad_f(__uint_as_float(rv[0] & 0xffff0000u));
            v[2] *= gelu_grad_f(__uint_as_float(rv[1] << 16)); v[3] *= gelu_grad_f(__uint_as_float(rv[1] & 0xffff0000u));
          } else {
            if (p.gelu) {
#pragma unroll
              for (int j = 0; j < 4; ++j) v[j] = gelu_erf_f(v[j]);
            }
            if (pres) {
              const u32x2 rv = rvs[nb][i];
              v[0] += __uint_as_float(rv[0] << 16); v[1] += __uint_as_float(rv[0] & 0xffff0000u);
              v[2] += __uint_as_float(rv[1] << 16); v[3] += __uint_as_float(rv[1] & 0xffff0000u);
            }
          }
        }
        const u32x2 pk = {pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3])};
        *(u32x2*)(pC + (long)m * p.ldc + n) = pk;
      }
  }
}

template <bool AKM, bool BKM, bool EPI, int TM = GM>
__global__ __launch_bounds__(256, 3) void mfma_gemm_kernel(MGemm p) {  // three workgroups per CU: at most 168 registers
  int bx, by, bz;
  xcd_block_index(bx, by, bz);
  mfma_gemm_tile<AKM, BKM, EPI, TM>(p, bx, by, bz, 0);
}
// Two independent GEMMs of the same shape in one launch (grid z = 2, no split-K): the layers of two encoders
// that run side by side.  Each fills about half a launch on its own; together the tail of one is filled by the other.
template <bool AKM, bool BKM, bool EPI, int TM = GM>
__global__ __launch_bounds__(256, 3) void mfma_gemm_pair_kernel(MGemm p) {
  int bx, by, bz;
  xcd_block_index(bx, by, bz);
  mfma_gemm_tile<AKM, BKM, EPI, TM>(p, bx, by, 0, bz);
}

// ------------------------------------------------------------------------------------------
// Q|K|V projection of narrow models (d = 64 or 128), optionally with the LayerNorm of the input rows inside.
//
// At these widths the whole problem is a few hundred rows per CU and the 128 x 128 tile kernel spends its time
// in one load -> LDS -> multiply -> store chain per workgroup.  Here a WAVE owns 32 rows: it loads them straight
// into the operand layout of the matrix instruction (lane = row, 8 consecutive features per 16-byte load),
// normalises them in registers once (a row lies in two lanes: one exchange per statistic) and multiplies them by
// Wq, Wk and Wv in turn.  The workgroup holds all three d x d weights in LDS, k-major as stored, read with the
// transpose read; biases, pre-multiplied by the score scale for Q, sit there as fp32 and enter in the one
// multiply-add per element of the epilogue.  Vector instructions per row are what bounds this kernel (the first
// version gave every projection its own wave and normalised every row three times: 14 instead of 9 us per launch).
// Up to two problems (two encoders) per launch.
struct QkvRows {
  const bf16_t* x[2]; const bf16_t* w[2][3]; const bf16_t* bias[2][3];
  const bf16_t* ln_g[2]; const bf16_t* ln_b[2];
  bf16_t* qkv[2];
  int R, groups; float ln_eps, qscale;   // groups = ceil(R / 128)
};
template <int D> constexpr int qkv_rows_lds_bytes() { return 3 * D * (D + 32) * 2 + 5 * D * 4; }
template <int D>
__global__ __launch_bounds__(256) void qkv_rows_kernel(QkvRows p) {
  constexpr int KS = D / 16, NBK = D / 32, LD = D + 32;   // row stride = 64 bytes mod 256: conflict-free transpose reads
  constexpr int WCH = D * D / 8 / 256;                    // 16-byte requests per thread and weight
  extern __shared__ __attribute__((aligned(16))) unsigned char qkv_smem[];
  bf16_t* const sW = (bf16_t*)qkv_smem;                   // [3][D][LD]
  float* const sG = (float*)(qkv_smem + 3 * D * LD * 2);  // gamma, beta, then the three biases
  float* const sBt = sG + D;
  float* const sBias = sG + 2 * D;
  int rg, z;
  {
    int lin, u0, u1;
    xcd_block_index(lin, u0, u1);
    rg = lin % p.groups; z = lin / p.groups;
  }
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, lo = lane & 31, hi = lane >> 5;
  const bf16_t* const x = z ? p.x[1] : p.x[0];
  const bf16_t* const ln_g = z ? p.ln_g[1] : p.ln_g[0];
  const bf16_t* const ln_b = z ? p.ln_b[1] : p.ln_b[0];
  bf16_t* const out = z ? p.qkv[1] : p.qkv[0];

  const int m = (rg * 4 + wave) * 32 + lo;
  const long mc = min(m, p.R - 1);
  u32x4 xr[KS];
#pragma unroll
  for (int s = 0; s < KS; ++s) xr[s] = *(const u32x4*)(x + mc * D + s * 16 + hi * 8);
  {   // the weights as stored: every request of the three is in flight before the first is written to LDS
    u32x4 wr[3][WCH];
#pragma unroll
    for (int part = 0; part < 3; ++part) {
      const bf16_t* const w = z ? p.w[1][part] : p.w[0][part];
#pragma unroll
      for (int i = 0; i < WCH; ++i) {
        const int idx = tid + i * 256, k = idx / (D / 8), c = (idx % (D / 8)) * 8;
        wr[part][i] = *(const u32x4*)(w + (long)k * D + c);
      }
    }
#pragma unroll
    for (int part = 0; part < 3; ++part)
#pragma unroll
      for (int i = 0; i < WCH; ++i) {
        const int idx = tid + i * 256, k = idx / (D / 8), c = (idx % (D / 8)) * 8;
        *(u32x4*)(sW + (part * D + k) * LD + c) = wr[part][i];
      }
  }
  if (tid < D) {
    // the five per-column vectors: every load issued (a NULL vector reads the first weight instead, which has more
    // than D elements, and counts as zero) before the first value goes to LDS
    const bf16_t* const safe = z ? p.w[1][0] : p.w[0][0];
    const bf16_t* src[5];
    src[0] = ln_g; src[1] = ln_b;
#pragma unroll
    for (int part = 0; part < 3; ++part) src[2 + part] = z ? p.bias[1][part] : p.bias[0][part];
    float v[5];
#pragma unroll
    for (int u = 0; u < 5; ++u) v[u] = __uint_as_float((unsigned)(src[u] ? src[u] : safe)[tid] << 16);
#pragma unroll
    for (int u = 0; u < 5; ++u) v[u] = src[u] ? v[u] : 0.f;
    sG[tid] = v[0];
    sBt[tid] = v[1];
    sBias[tid] = v[2] * p.qscale;
    sBias[D + tid] = v[3];
    sBias[2 * D + tid] = v[4];
  }
  __syncthreads();

  bf16x8 xa[KS];
  if (ln_g) {   // two-pass in fp32, rounded to bf16 as the stand-alone LayerNorm kernel does
    float sum = 0.f;
#pragma unroll
    for (int s = 0; s < KS; ++s) sum = sum_bf16x8(as_bf16x8(xr[s]), sum);
    sum += __shfl_xor(sum, 32, 64);
    const float mu = sum * (1.f / D);
    float t[KS][8];
    float q = 0.f;
#pragma unroll
    for (int s = 0; s < KS; ++s)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        t[s][2 * j] = __uint_as_float(xr[s][j] << 16) - mu;
        t[s][2 * j + 1] = __uint_as_float(xr[s][j] & 0xffff0000u) - mu;
        q = fmaf(t[s][2 * j], t[s][2 * j], q);
        q = fmaf(t[s][2 * j + 1], t[s][2 * j + 1], q);
      }
    q += __shfl_xor(q, 32, 64);
    const float rstd = rsqrtf(q * (1.f / D) + p.ln_eps);
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      const float4 g0 = *(const float4*)(sG + s * 16 + hi * 8), g1 = *(const float4*)(sG + s * 16 + hi * 8 + 4);
      const float4 b0 = *(const float4*)(sBt + s * 16 + hi * 8), b1 = *(const float4*)(sBt + s * 16 + hi * 8 + 4);
      const float gg[8] = {g0.x, g0.y, g0.z, g0.w, g1.x, g1.y, g1.z, g1.w};
      const float bb[8] = {b0.x, b0.y, b0.z, b0.w, b1.x, b1.y, b1.z, b1.w};
      float y[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) y[j] = fmaf(t[s][j], rstd * gg[j], bb[j]);
      xa[s] = pack8(y);
    }
  } else {
#pragma unroll
    for (int s = 0; s < KS; ++s) xa[s] = as_bf16x8(xr[s]);
  }

  bf16_t* const orow = out + (long)m * (3 * D) + 8 * hi;
#pragma unroll
  for (int part = 0; part < 3; ++part) {
    // register 4i + j of block nb is column 32 nb + 8i + 4hi + j
    f32x16 acc[NBK];
#pragma unroll
    for (int nb = 0; nb < NBK; ++nb)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[nb][r] = 0.f;
#pragma unroll
    for (int s = 0; s < KS; ++s)
#pragma unroll
      for (int nb = 0; nb < NBK; ++nb)
        acc[nb] = mfma32(lds_frag_tr(sW + part * D * LD, LD, s * 16, nb * 32, lane), xa[s], acc[nb]);

    // Two neighbouring register quads hold columns 8i + 4hi + 0..3 and 8(i+1) + 4hi + 0..3; swapping the upper
    // half-wave of the first with the lower half-wave of the second leaves every lane 8 consecutive columns.
    const float cs = part == 0 ? p.qscale : 1.f;
    u32x4 o[NBK][2];
#pragma unroll
    for (int nb = 0; nb < NBK; ++nb)
#pragma unroll
      for (int ip = 0; ip < 2; ++ip) {
        const float4 ba = *(const float4*)(sBias + part * D + nb * 32 + 16 * ip + 4 * hi);
        const float4 bb = *(const float4*)(sBias + part * D + nb * 32 + 16 * ip + 8 + 4 * hi);
        const unsigned a0 = pack_bf16(fmaf(acc[nb][8 * ip], cs, ba.x), fmaf(acc[nb][8 * ip + 1], cs, ba.y));
        const unsigned a1 = pack_bf16(fmaf(acc[nb][8 * ip + 2], cs, ba.z), fmaf(acc[nb][8 * ip + 3], cs, ba.w));
        const unsigned b0 = pack_bf16(fmaf(acc[nb][8 * ip + 4], cs, bb.x), fmaf(acc[nb][8 * ip + 5], cs, bb.y));
        const unsigned b1 = pack_bf16(fmaf(acc[nb][8 * ip + 6], cs, bb.z), fmaf(acc[nb][8 * ip + 7], cs, bb.w));
        const u32x2 s0 = __builtin_amdgcn_permlane32_swap(a0, b0, false, false);
        const u32x2 s1 = __builtin_amdgcn_permlane32_swap(a1, b1, false, false);
        o[nb][ip][0] = s0[0]; o[nb][ip][1] = s1[0]; o[nb][ip][2] = s0[1]; o[nb][ip][3] = s1[1];
      }
    if (m < p.R) {
#pragma unroll
      for (int nb = 0; nb < NBK; ++nb)
#pragma unroll
        for (int ip = 0; ip < 2; ++ip) *(u32x4*)(orow + part * D + nb * 32 + 16 * ip) = o[nb][ip];
    }
  }
}

// ------------------------------------------------------------------------------------------
// Large-tile kernel with asynchronous global->LDS staging.
//
// The 128 x 128 kernel above is bound by bytes in flight, not by the matrix cores: one
// register-staged k-tile per workgroup covers well under the L2/HBM round trip.  Here the
// tile is 256 x 256, a quarter of the operand traffic per flop, and operands go straight from
// global memory into a ring of four 32-deep LDS stages with global_load_lds_dwordx4 (no staging
// registers), three stages in flight while one is multiplied, one barrier per stage.
// 8 waves, each 128 x 64 = 4 x 2 MFMA blocks (128 accumulator registers, two waves per SIMD).  The
// first version had 4 waves of 128 x 128 (256 accumulator registers, ONE wave per SIMD): a wave alone
// on a SIMD issues vector instructions at half rate and nothing overlaps its LDS waits, its prologue
// or its epilogue -- with 8 waves the QKV + output projections take 0.129 instead of 0.157 ms and the
// weight gradients 0.122 instead of 0.129 ms, although every MFMA now needs 1.5x the LDS fragment reads.
//
// A direct load writes lane i's 16 bytes at (wave-uniform LDS base) + 16 i, so rows cannot be
// padded; bank conflicts are avoided by XOR-swizzling the 16-byte chunk index instead:
//   m-major tile [256 rows][4 chunks]  : chunk kc of row r sits at r*4 + (kc ^ ((r >> 2) & 3))
//   k-major tile [32 rows][32 chunks]  : chunk c of row k sits at k*32 + (c ^ ((k & 3) << 2))
// (16 consecutive rows read at one kc, resp. the 4 x 4 chunk footprint of a transpose read, then
// cover all 64 banks exactly once).  Each lane fetches the global chunk that belongs in its slot.
constexpr int DM = 256, DN = 256, DK = 32, DSTAGES = 4;
constexpr int DMA_STAGE_BYTES = (DM + DN) * DK * 2;           // 32 KB
constexpr int DMA_LDS_BYTES = DSTAGES * DMA_STAGE_BYTES;      // 128 KB

typedef __attribute__((address_space(3))) void* lds_void_ptr;
typedef const __attribute__((address_space(1))) void* glb_void_ptr;

// NWV waves per workgroup: 8 (each wave 128 x 64, two waves per SIMD) or 4 (each wave 128 x 128, one wave per SIMD).
template <bool AKM, bool BKM, bool EPI, int NWV>
__global__ __launch_bounds__(NWV * 64) void mfma_gemm_dma_kernel(MGemm p) {
  extern __shared__ __attribute__((aligned(1024))) bf16_t smem[];
  constexpr int NWN = NWV / 2;          // wave grid: 2 (rows) x NWN (columns)
  constexpr int WCOLS = DN / NWN;       // columns of a wave's sub-tile: 128 or 64
  constexpr int NBN = WCOLS / 32;       // 32-column blocks per wave: 4 or 2
  constexpr int CH = 1024 / (NWV * 64); // 16-byte chunks per thread, operand and stage: 4 or 2
  const int tid = threadIdx.x, lane = tid & 63, lo = lane & 31, hi = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / NWN, wn = wave % NWN;
  int bx, by, bz;
  xcd_block_index(bx, by, bz);
  const int m0 = by * DM, n0 = bx * DN;

  const int ktiles = p.K / DK;  // K % 32 == 0 is required by the launcher
  const int per_split = (ktiles + p.split_k - 1) / p.split_k;
  const int it_begin = bz * per_split, it_end = min(ktiles, it_begin + per_split);
  const int n_it = max(0, it_end - it_begin);

  // ---- per-thread source pointers of the CH + CH chunks it fetches per stage (advanced by DK per stage) ----
  const bf16_t* ga[CH];
  const bf16_t* gb[CH];   // k-major B: source pointer; m-major B: only the offset inside one matrix is used
  long gboff[CH];
  long a_step, b_step;
#pragma unroll
  for (int j = 0; j < CH; ++j) {
    const int slot = (wave * CH + j) * 64 + lane;  // chunk slot inside the 1024-chunk tile
    if (AKM) {
      const int k = slot >> 5, pos = slot & 31, c = pos ^ ((k & 3) << 2);
      const int col = min(m0 + c * 8, p.M - 8);
      ga[j] = p.A + (long)(it_begin * DK + k) * p.lda + col;
    } else {
      const int r = slot >> 2, pos = slot & 3, kc = pos ^ ((r >> 2) & 3);
      ga[j] = p.A + (long)min(m0 + r, p.M - 1) * p.lda + it_begin * DK + kc * 8;
    }
    if (BKM) {
      const int k = slot >> 5, pos = slot & 31, c = pos ^ ((k & 3) << 2);
      const int col = min(n0 + c * 8, p.N - 8);
      const bf16_t* mat = p.B[0];
      int cc = col;
      if (p.b_nper > 0) { mat = p.B[col / p.b_nper]; cc = col % p.b_nper; }
      gb[j] = mat + (long)(it_begin * DK + k) * p.ldb + cc;
    } else {
      const int r = slot >> 2, pos = slot & 3, kc = pos ^ ((r >> 2) & 3);
      gb[j] = p.B[0];
      gboff[j] = (long)min(n0 + r, p.N - 1) * p.ldb + kc * 8;  // k offset added per stage (K may be split over B[])
    }
    if (BKM) gboff[j] = 0;
  }
  a_step = AKM ? (long)DK * p.lda : DK;
  b_step = BKM ? (long)DK * p.ldb : DK;

  auto issue = [&](int it_rel) {  // fetch stage it_rel (relative to it_begin) into ring slot it_rel % DSTAGES
    char* base = (char*)smem + (it_rel % DSTAGES) * DMA_STAGE_BYTES;
#pragma unroll
    for (int j = 0; j < CH; ++j) {
      const bf16_t* src = ga[j] + (long)it_rel * a_step;
      dma16(src, base + (wave * CH + j) * 1024);
    }
#pragma unroll
    for (int j = 0; j < CH; ++j) {
      const bf16_t* src;
      if (BKM) {
        src = gb[j] + (long)it_rel * b_step;
      } else {
        const int k0 = (it_begin + it_rel) * DK;
        const bf16_t* mat = p.B[0];
        int kk = k0;
        if (p.b_kper > 0) { mat = p.B[k0 / p.b_kper]; kk = k0 % p.b_kper; }
        src = mat + gboff[j] + kk;
      }
      dma16(src, base + DM * DK * 2 + (wave * CH + j) * 1024);
    }
  };

  // [n block][m block]; registers 4i..4i+3 are columns n = 8i + 4hi + 0..3 of the block.  The
  // accumulators start at the bias of their column (split-K launches carry no bias).
  f32x16 acc[NBN][4];
#pragma unroll
  for (int nb = 0; nb < NBN; ++nb)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      float bv[4] = {0.f, 0.f, 0.f, 0.f};
      if (!p.partial) bias4(p, p.bias, n0 + wn * WCOLS + nb * 32 + 8 * i + 4 * hi, bv);
#pragma unroll
      for (int mb = 0; mb < 4; ++mb)
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) acc[nb][mb][4 * i + jj] = bv[jj];
    }

  // ---- LDS byte offsets of this lane's fragments inside a stage ----
  int offA[2][4], offB[2][NBN];   // [k-step][block]; for k-major operands the second transpose read is +4 rows
  int offA2[2][4], offB2[2][NBN];
#pragma unroll
  for (int ks = 0; ks < 2; ++ks)
#pragma unroll
    for (int x = 0; x < 4; ++x) {
      if (AKM) {
        const int j = lane & 15, gq = lane >> 4;
        const int kr = ks * 16 + 8 * (gq >> 1) + (j >> 2), col = wm * 128 + x * 32 + 16 * (gq & 1) + 4 * (j & 3);
        offA[ks][x] = (kr * 32 + ((col >> 3) ^ ((kr & 3) << 2))) * 16 + (col & 7) * 2;
        offA2[ks][x] = ((kr + 4) * 32 + ((col >> 3) ^ (((kr + 4) & 3) << 2))) * 16 + (col & 7) * 2;
      } else {
        const int row = wm * 128 + x * 32 + lo, kc = ks * 2 + hi;
        offA[ks][x] = (row * 4 + (kc ^ ((row >> 2) & 3))) * 16;
        offA2[ks][x] = 0;
      }
      if (x < NBN) {
        if (BKM) {
          const int j = lane & 15, gq = lane >> 4;
          const int kr = ks * 16 + 8 * (gq >> 1) + (j >> 2), col = wn * WCOLS + x * 32 + 16 * (gq & 1) + 4 * (j & 3);
          offB[ks][x] = DM * DK * 2 + (kr * 32 + ((col >> 3) ^ ((kr & 3) << 2))) * 16 + (col & 7) * 2;
          offB2[ks][x] = DM * DK * 2 + ((kr + 4) * 32 + ((col >> 3) ^ (((kr + 4) & 3) << 2))) * 16 + (col & 7) * 2;
        } else {
          const int row = wn * WCOLS + x * 32 + lo, kc = ks * 2 + hi;
          offB[ks][x] = DM * DK * 2 + (row * 4 + (kc ^ ((row >> 2) & 3))) * 16;
          offB2[ks][x] = 0;
        }
      }
    }
  auto frag = [&](const char* st, int o1, int o2, bool km) -> bf16x8 {
    if (!km) return as_bf16x8(*(const u32x4*)(st + o1));
    typedef v4i16 __attribute__((address_space(3))) * lds_v4_ptr;
    union { v4i16 h[2]; bf16x8 v; } x;
    x.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4_ptr)(st + o1));
    x.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4_ptr)(st + o2));
    return x.v;
  };

  // ---- pipeline: stages it+1 .. it+3 in flight while stage it is multiplied ----
#pragma unroll
  for (int s = 0; s < DSTAGES - 1; ++s)
    if (s < n_it) issue(s);
  for (int it = 0; it < n_it; ++it) {
    // this lane's loads of stage `it` have landed when at most the loads of the later stages remain
    const int later = min(DSTAGES - 2, n_it - 1 - it);
    // (2 CH loads per thread and stage).  A bare s_barrier is used: __syncthreads() would also drain vmcnt.
    if (NWV == 4) {
      if (later >= 2) asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
      else if (later == 1) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
      else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    } else {
      if (later >= 2) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
      else if (later == 1) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
      else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    }
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    if (it + DSTAGES - 1 < n_it) issue(it + DSTAGES - 1);
    const char* st = (const char*)smem + (it % DSTAGES) * DMA_STAGE_BYTES;
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
      bf16x8 fa[4], fb[NBN];
#pragma unroll
      for (int x = 0; x < 4; ++x) fa[x] = frag(st, offA[ks][x], offA2[ks][x], AKM);
#pragma unroll
      for (int x = 0; x < NBN; ++x) fb[x] = frag(st, offB[ks][x], offB2[ks][x], BKM);
#pragma unroll
      for (int nb = 0; nb < NBN; ++nb)
#pragma unroll
        for (int mb = 0; mb < 4; ++mb) acc[nb][mb] = mfma32(fb[nb], fa[mb], acc[nb][mb]);
    }
  }

  // ---- epilogue ----
  if (p.partial) {  // split-K: fp32 partial sums, 16 bytes per lane
#pragma unroll
    for (int mb = 0; mb < 4; ++mb) {
      const int m = m0 + wm * 128 + mb * 32 + lo;
      if (m >= p.M) continue;
#pragma unroll
      for (int nb = 0; nb < NBN; ++nb)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int n = n0 + wn * WCOLS + nb * 32 + 8 * i + 4 * hi;
          if (n >= p.N) continue;
          *(float4*)(p.partial + ((long)bz * p.M + m) * p.N + n) =
              make_float4(acc[nb][mb][4 * i], acc[nb][mb][4 * i + 1], acc[nb][mb][4 * i + 2], acc[nb][mb][4 * i + 3]);
        }
    }
    return;
  }
  // bf16 output: a lane owns a ROW of the accumulator tile (8 bytes per register quad), which would
  // make every store touch 64 different cache lines.  The wave's 128 x WCOLS tile therefore goes through
  // its own share of the (now idle) stage ring, 64 rows at a time, and leaves as 16-byte stores in
  // which WCOLS / 8 consecutive lanes cover one row segment of 2 WCOLS bytes.
  __builtin_amdgcn_s_barrier();  // every wave has finished reading the last stage
  asm volatile("" ::: "memory");
  constexpr int EP_LD = WCOLS + 8;   // bf16 per staged row
  static_assert(64 * EP_LD * 2 <= DMA_LDS_BYTES / NWV, "a wave's staging area must fit in its share of the ring");
  bf16_t* stg = smem + wave * (DMA_LDS_BYTES / 2 / NWV);
  // a tile inside the matrix stores without bounds checks
  const bool interior = m0 + DM <= p.M && n0 + DN <= p.N;
#pragma unroll
  for (int half = 0; half < 2; ++half) {
#pragma unroll
    for (int mq = 0; mq < 2; ++mq) {
      const int mb = half * 2 + mq;
      const int m = m0 + wm * 128 + mb * 32 + lo;
      u32x2 rvs[NBN][4];   // the row's residual values, all requested before the first is added
      if constexpr (EPI) {
        if (p.res) {
#pragma unroll
          for (int nb = 0; nb < NBN; ++nb)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              const int n = n0 + wn * WCOLS + nb * 32 + 8 * i + 4 * hi;
              rvs[nb][i] = *(const u32x2*)(p.res + (long)min(m, p.M - 1) * p.ldc + (n < p.N ? n : 0));
            }
        }
      }
#pragma unroll
      for (int nb = 0; nb < NBN; ++nb)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int nl = nb * 32 + 8 * i + 4 * hi;
          const int n = n0 + wn * WCOLS + nl;
          float v[4];
          const float cs = (p.scale0_on && n < p.n_per) ? p.scale0 : 1.f;
#pragma unroll
          for (int j = 0; j < 4; ++j) v[j] = acc[nb][mb][4 * i + j] * cs;
          if constexpr (EPI) {
            if (p.gelu) {
#pragma unroll
              for (int j = 0; j < 4; ++j) v[j] = gelu_erf_f(v[j]);
            }
            if (p.res && (interior || (m < p.M && n < p.N))) {
              const u32x2 rv = rvs[nb][i];
              v[0] += __uint_as_float(rv[0] << 16); v[1] += __uint_as_float(rv[0] & 0xffff0000u);
              v[2] += __uint_as_float(rv[1] << 16); v[3] += __uint_as_float(rv[1] & 0xffff0000u);
            }
          }
          const u32x2 pk = {pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3])};
          *(u32x2*)(stg + (mq * 32 + lo) * EP_LD + nl) = pk;
        }
    }
    // 64 rows x CPR chunks of 16 bytes; lane -> (row = RPP t + lane / CPR, chunk = lane % CPR)
    constexpr int CPR = WCOLS / 8, RPP = 64 / CPR, NT = 64 / RPP;
    const int row0 = lane / CPR, ch = lane % CPR;
    const int mrow = m0 + wm * 128 + half * 64 + row0, n = n0 + wn * WCOLS + ch * 8;
    bf16_t* cp = p.C + (long)mrow * p.ldc + n;
    const bf16_t* sp = stg + row0 * EP_LD + ch * 8;
    if (interior) {
#pragma unroll
      for (int t = 0; t < NT; ++t) *(u32x4*)(cp + (long)(RPP * t) * p.ldc) = *(const u32x4*)(sp + RPP * t * EP_LD);
    } else {
#pragma unroll
      for (int t = 0; t < NT; ++t)   // N is a multiple of 8 on this path
        if (mrow + RPP * t < p.M && n < p.N)
          *(u32x4*)(cp + (long)(RPP * t) * p.ldc) = *(const u32x4*)(sp + RPP * t * EP_LD);
    }
  }
}

// ------------------------------------------------------------------------------------------
// The same kernel for row-major A and k-major B with a 288 x 256 tile and twelve waves (3 x 4, each 96 x 64:
// three waves per SIMD).  The tile height is chosen for the launch, not for the CU: 36 864 rows are 128 tiles of
// 288, so N = 1536 gives 768 workgroups = exactly three rounds of the 256 CUs (256-row tiles: 864 = three rounds
// and a fourth with 96), and N = 512 gives 256 = one round (256-row tiles: 288 = one round and a second with 32).
// Per stage 288 x 4 + 32 x 32 = 2176 16-byte chunks for 768 threads: thread t copies A chunks t and t + 768 (< 1152)
// and B chunks t and t + 768 (< 1024), i.e. waves 0-3 issue 4 copies per stage, waves 4-5 three, waves 6-11 two --
// each wave waits for its own count.
constexpr int TM = 288, TWAVES = 12;
constexpr int T_A_BYTES = TM * DK * 2;                         // 18 KB
constexpr int T_STAGE_BYTES = T_A_BYTES + DN * DK * 2;         // 34 KB
constexpr int T_LDS_BYTES = DSTAGES * T_STAGE_BYTES;           // 136 KB
constexpr int T_STG_BYTES = 10240;                             // epilogue staging per wave: 64 rows x 72 bf16 (9216) rounded up

template <bool EPI>
__global__ __launch_bounds__(TWAVES * 64) void mfma_gemm_dma12_kernel(MGemm p) {
  extern __shared__ __attribute__((aligned(1024))) bf16_t smem[];
  constexpr int NBN = 2, MBW = 3, WCOLS = 64, NT_THREADS = TWAVES * 64;
  const int tid = threadIdx.x, lane = tid & 63, lo = lane & 31, hi = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 2, wn = wave & 3;
  int bx, by, bz;
  xcd_block_index(bx, by, bz);
  const int m0 = by * TM, n0 = bx * DN;
  const int n_it = p.K / DK;   // K % 32 == 0 is required by the launcher; no split-K on this path

  // ---- source pointers of this thread's chunks (advanced by DK per stage) ----
  const bool a2 = tid + NT_THREADS < TM * 4, b2 = tid + NT_THREADS < DN * 4;   // wave-uniform
  const bf16_t* ga[2];
  const bf16_t* gb[2];
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int slot = j * NT_THREADS + tid;
    {
      const int sa = min(slot, TM * 4 - 1);
      const int r = sa >> 2, pos = sa & 3, kc = pos ^ ((r >> 2) & 3);
      ga[j] = p.A + (long)min(m0 + r, p.M - 1) * p.lda + kc * 8;
    }
    {
      const int sb = min(slot, DN * 4 - 1);
      const int k = sb >> 5, pos = sb & 31, c = pos ^ ((k & 3) << 2);
      const int col = min(n0 + c * 8, p.N - 8);
      const bf16_t* mat = p.B[0];
      int cc = col;
      if (p.b_nper > 0) {
        const int sel = col / p.b_nper;
        mat = sel == 0 ? p.B[0] : sel == 1 ? p.B[1] : p.B[2];
        cc = col - sel * p.b_nper;
      }
      gb[j] = mat + (long)k * p.ldb + cc;
    }
  }
  const long b_step = (long)DK * p.ldb;
  auto issue = [&](int it) {   // stage `it` into ring slot it % DSTAGES
    char* base = (char*)smem + (it % DSTAGES) * T_STAGE_BYTES;
    dma16(ga[0] + (long)it * DK, base + wave * 1024);
    if (a2) dma16(ga[1] + (long)it * DK, base + (TWAVES + wave) * 1024);
    dma16(gb[0] + (long)it * b_step, base + T_A_BYTES + wave * 1024);
    if (b2) dma16(gb[1] + (long)it * b_step, base + T_A_BYTES + (TWAVES + wave) * 1024);
  };

  // [n block][m block]; registers 4i..4i+3 are columns n = 8i + 4hi + 0..3 of the block; they start at the bias
  f32x16 acc[NBN][MBW];
#pragma unroll
  for (int nb = 0; nb < NBN; ++nb) {   // one column block at a time (register budget of three waves per SIMD)
    int nq[4];
    float bq[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i) nq[i] = n0 + wn * WCOLS + nb * 32 + 8 * i + 4 * hi;
    bias4_many<4>(p, p.bias, nq, bq);
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int mb = 0; mb < MBW; ++mb)
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) acc[nb][mb][4 * i + jj] = bq[i][jj];
  }

  // ---- LDS byte offsets of this lane's fragments inside a stage ----
  int offA[2][MBW], offB[2][NBN], offB2[2][NBN];
#pragma unroll
  for (int ks = 0; ks < 2; ++ks) {
#pragma unroll
    for (int x = 0; x < MBW; ++x) {
      const int row = wm * 96 + x * 32 + lo, kc = ks * 2 + hi;
      offA[ks][x] = (row * 4 + (kc ^ ((row >> 2) & 3))) * 16;
    }
#pragma unroll
    for (int x = 0; x < NBN; ++x) {
      const int j = lane & 15, gq = lane >> 4;
      const int kr = ks * 16 + 8 * (gq >> 1) + (j >> 2), col = wn * WCOLS + x * 32 + 16 * (gq & 1) + 4 * (j & 3);
      offB[ks][x] = T_A_BYTES + (kr * 32 + ((col >> 3) ^ ((kr & 3) << 2))) * 16 + (col & 7) * 2;
      offB2[ks][x] = T_A_BYTES + ((kr + 4) * 32 + ((col >> 3) ^ (((kr + 4) & 3) << 2))) * 16 + (col & 7) * 2;
    }
  }
  auto frag_t = [&](const char* st, int o1, int o2) -> bf16x8 {
    typedef v4i16 __attribute__((address_space(3))) * lds_v4_ptr;
    union { v4i16 h[2]; bf16x8 v; } x;
    x.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4_ptr)(st + o1));
    x.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4_ptr)(st + o2));
    return x.v;
  };

  // ---- pipeline: stages it+1 .. it+3 in flight while stage it is multiplied ----
  const int ncopy = 2 + (a2 ? 1 : 0) + (b2 ? 1 : 0);   // this wave's copies per stage: 4, 3 or 2
#pragma unroll
  for (int s = 0; s < DSTAGES - 1; ++s)
    if (s < n_it) issue(s);
  for (int it = 0; it < n_it; ++it) {
    // this wave's copies of stage `it` have landed when at most the copies of the later stages remain
    const int later = min(DSTAGES - 2, n_it - 1 - it);
    if (later == 0) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    else if (ncopy == 4) { if (later >= 2) asm volatile("s_waitcnt vmcnt(8)" ::: "memory"); else asm volatile("s_waitcnt vmcnt(4)" ::: "memory"); }
    else if (ncopy == 3) { if (later >= 2) asm volatile("s_waitcnt vmcnt(6)" ::: "memory"); else asm volatile("s_waitcnt vmcnt(3)" ::: "memory"); }
    else { if (later >= 2) asm volatile("s_waitcnt vmcnt(4)" ::: "memory"); else asm volatile("s_waitcnt vmcnt(2)" ::: "memory"); }
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    if (it + DSTAGES - 1 < n_it) issue(it + DSTAGES - 1);
    const char* st = (const char*)smem + (it % DSTAGES) * T_STAGE_BYTES;
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
      bf16x8 fa[MBW], fb[NBN];
#pragma unroll
      for (int x = 0; x < MBW; ++x) fa[x] = as_bf16x8(*(const u32x4*)(st + offA[ks][x]));
#pragma unroll
      for (int x = 0; x < NBN; ++x) fb[x] = frag_t(st, offB[ks][x], offB2[ks][x]);
#pragma unroll
      for (int nb = 0; nb < NBN; ++nb)
#pragma unroll
        for (int mb = 0; mb < MBW; ++mb) acc[nb][mb] = mfma32(fb[nb], fa[mb], acc[nb][mb]);
    }
  }

  // ---- epilogue: the wave's 96 x 64 tile through its own staging area, 32 rows at a time, 16-byte stores ----
  __builtin_amdgcn_s_barrier();  // every wave has finished reading the last stage
  asm volatile("" ::: "memory");
  constexpr int EP_LD = WCOLS + 8;   // bf16 per staged row
  static_assert(32 * EP_LD * 2 <= T_STG_BYTES && TWAVES * T_STG_BYTES <= T_LDS_BYTES, "staging areas must fit in the ring");
  bf16_t* stg = smem + wave * (T_STG_BYTES / 2);
  const bool interior = m0 + TM <= p.M && n0 + DN <= p.N;
#pragma unroll
  for (int mb = 0; mb < MBW; ++mb) {
    const int m = m0 + wm * 96 + mb * 32 + lo;
#pragma unroll
    for (int nb = 0; nb < NBN; ++nb) {
      u32x2 rvs[4];   // the row's residual values of this column block, requested together (168 registers: not all eight)
      if constexpr (EPI) {
        if (p.res) {
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const int n = n0 + wn * WCOLS + nb * 32 + 8 * i + 4 * hi;
            rvs[i] = *(const u32x2*)(p.res + (long)min(m, p.M - 1) * p.ldc + (n < p.N ? n : 0));
          }
        }
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int nl = nb * 32 + 8 * i + 4 * hi;
        const int n = n0 + wn * WCOLS + nl;
        float v[4];
        const float cs = (p.scale0_on && n < p.n_per) ? p.scale0 : 1.f;
#pragma unroll
        for (int j = 0; j < 4; ++j) v[j] = acc[nb][mb][4 * i + j] * cs;
        if constexpr (EPI) {
          if (p.gelu) {
#pragma unroll
            for (int j = 0; j < 4; ++j) v[j] = gelu_erf_f(v[j]);
          }
          if (p.res && (interior || (m < p.M && n < p.N))) {
            const u32x2 rv = rvs[i];
            v[0] += __uint_as_float(rv[0] << 16); v[1] += __uint_as_float(rv[0] & 0xffff0000u);
            v[2] += __uint_as_float(rv[1] << 16); v[3] += __uint_as_float(rv[1] & 0xffff0000u);
          }
        }
        const u32x2 pk = {pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3])};
        *(u32x2*)(stg + lo * EP_LD + nl) = pk;
      }
    }
    // 32 rows x 8 chunks of 16 bytes; lane -> (row = 8 t + lane / 8, chunk = lane % 8).  The staging area is
    // private to the wave and its LDS instructions complete in order: no barrier between the passes.
    const int row0 = lane >> 3, ch = lane & 7;
    const int mrow = m0 + wm * 96 + mb * 32 + row0, n = n0 + wn * WCOLS + ch * 8;
    bf16_t* cp = p.C + (long)mrow * p.ldc + n;
    const bf16_t* sp = stg + row0 * EP_LD + ch * 8;
    u32x4 out[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) out[t] = *(const u32x4*)(sp + 8 * t * EP_LD);
    if (interior) {
#pragma unroll
      for (int t = 0; t < 4; ++t) *(u32x4*)(cp + (long)(8 * t) * p.ldc) = out[t];
    } else {
#pragma unroll
      for (int t = 0; t < 4; ++t)   // N is a multiple of 8 on this path
        if (mrow + 8 * t < p.M && n < p.N) *(u32x4*)(cp + (long)(8 * t) * p.ldc) = out[t];
    }
  }
}

// ------------------------------------------------------------------------------------------
// Whole MLP sub-block of an encoder layer at model width D = 64 or 128 in one kernel:
//   y = h + GELU(LN(h) W1 + b1) W2 + b2        (h [R, D], W1 [D, d_ff], W2 [d_ff, D], d_ff % 64 == 0)
// and, with PROJ, also the attention's output projection and residual in front of it:
//   h = x + O Wo + bo                          (O, x [R, D]; h is rounded to bf16 and kept in LDS only)
// A workgroup owns 64 rows.  The hidden layer is walked in chunks of 64 columns: the chunk
// z_j = GELU(LN(h) W1[:, j] + b1[j]) (64 x 64) goes to LDS as bf16 and is at once multiplied into the
// 64 x D output accumulator with W2[j, :], so the [R, d_ff] activation never exists in memory and the
// launches output projection, LayerNorm, first GEMM, second GEMM become one.  Four waves in a 2 x 2 grid: each
// owns 32 x 32 of a z chunk and 32 x D/2 of the output; the same transposed-product tiles as
// mfma_gemm_kernel (a lane owns an output row; registers 4i..4i+3 are columns 8i + 4hi + 0..3 of a 32-column block).
// NQ groups of four consecutive bf16 of a bias vector (element offsets off[q], multiples of 4) as fp32; zeros
// for a NULL vector.  All loads are issued together: written as `b ? bf2f(b[k]) : 0.f` per element, every element
// became a conditional 2-byte load with a wait of its own (96 of them in front of the layer tail at width 128).
template <int NQ>
__device__ __forceinline__ void bias_quads(const bf16_t* b, const int (&off)[NQ], float (&out)[NQ][4]) {
  if (!b) {
#pragma unroll
    for (int q = 0; q < NQ; ++q) out[q][0] = out[q][1] = out[q][2] = out[q][3] = 0.f;
    return;
  }
  u32x2 raw[NQ];
  if ((reinterpret_cast<uintptr_t>(b) & 7) == 0) {
#pragma unroll
    for (int q = 0; q < NQ; ++q) raw[q] = *(const u32x2*)(b + off[q]);
  } else {
    unsigned short h[NQ][4];
#pragma unroll
    for (int q = 0; q < NQ; ++q)
#pragma unroll
      for (int j = 0; j < 4; ++j) h[q][j] = b[off[q] + j];
#pragma unroll
    for (int q = 0; q < NQ; ++q) raw[q] = u32x2{(unsigned)h[q][0] | ((unsigned)h[q][1] << 16), (unsigned)h[q][2] | ((unsigned)h[q][3] << 16)};
  }
#pragma unroll
  for (int q = 0; q < NQ; ++q) {
    out[q][0] = __uint_as_float(raw[q][0] << 16); out[q][1] = __uint_as_float(raw[q][0] & 0xffff0000u);
    out[q][2] = __uint_as_float(raw[q][1] << 16); out[q][3] = __uint_as_float(raw[q][1] & 0xffff0000u);
  }
}
struct MlpTailArgs {
  const bf16_t* h; const bf16_t* ln_g; const bf16_t* ln_b; float ln_eps;
  const bf16_t* w1; const bf16_t* b1; const bf16_t* w2; const bf16_t* b2;
  bf16_t* y; int R, d_ff;
  const bf16_t* o; const bf16_t* wo; const bf16_t* bo;   // PROJ: h above is x, the residual of the projection
  long ldy;                                              // row stride of y (d, or wider: y is a column block)
};
// ROWS x COLS bf16 tile as 16-byte chunks, chunk (tid + 256 u): row = chunk / (COLS / 8), so the COLS / 8 lanes that
// hold a row are consecutive.  Rows are clamped to rmax.
template <int ROWS, int COLS>
struct ChunkTile {
  static constexpr int CPR = COLS / 8, N = ROWS * CPR / 256;
  u32x4 v[N];
  __device__ __forceinline__ void load(const bf16_t* base, long ld, int r0, int rmax, int tid) {
#pragma unroll
    for (int u = 0; u < N; ++u) {
      const int idx = tid + u * 256, r = idx / CPR, c = (idx % CPR) * 8;
      v[u] = *(const u32x4*)(base + (long)min(r0 + r, rmax) * ld + c);
    }
  }
  __device__ __forceinline__ void store(bf16_t* lds, int ld, int tid) const {
#pragma unroll
    for (int u = 0; u < N; ++u) {
      const int idx = tid + u * 256, r = idx / CPR, c = (idx % CPR) * 8;
      *(u32x4*)(lds + r * ld + c) = v[u];
    }
  }
  __device__ __forceinline__ void load_lds(const bf16_t* lds, int ld, int tid) {
#pragma unroll
    for (int u = 0; u < N; ++u) {
      const int idx = tid + u * 256, r = idx / CPR, c = (idx % CPR) * 8;
      v[u] = *(const u32x4*)(lds + r * ld + c);
    }
  }
  // LayerNorm of every row (COLS = the whole feature row): two-pass in fp32, as the stand-alone kernel
  __device__ __forceinline__ void layernorm(const bf16_t* gamma, const bf16_t* beta, float eps, int tid) {
    const int c = (tid % CPR) * 8;
    const u32x4 gr = *(const u32x4*)(gamma + c), br = *(const u32x4*)(beta + c);
#pragma unroll
    for (int u = 0; u < N; ++u) {
      float x[8];
#pragma unroll
      for (int j = 0; j < 4; ++j) { x[2 * j] = __uint_as_float(v[u][j] << 16); x[2 * j + 1] = __uint_as_float(v[u][j] & 0xffff0000u); }
      float s = 0.f;
#pragma unroll
      for (int j = 0; j < 8; ++j) s += x[j];
#pragma unroll
      for (int o = CPR / 2; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
      const float mu = s * (1.f / COLS);
      float q = 0.f;
#pragma unroll
      for (int j = 0; j < 8; ++j) { const float w = x[j] - mu; q = fmaf(w, w, q); }
#pragma unroll
      for (int o = CPR / 2; o > 0; o >>= 1) q += __shfl_xor(q, o, 64);
      const float rstd = rsqrtf(q * (1.f / COLS) + eps);
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const float a = (x[2 * j] - mu) * rstd * __uint_as_float(gr[j] << 16) + __uint_as_float(br[j] << 16);
        const float b = (x[2 * j + 1] - mu) * rstd * __uint_as_float(gr[j] & 0xffff0000u) + __uint_as_float(br[j] & 0xffff0000u);
        v[u][j] = pack_bf16(a, b);
      }
    }
  }
};
__device__ __forceinline__ bf16x8 frag_rows(const bf16_t* lds, int ld, int row, int col) {  // m-major operand fragment
  return as_bf16x8(*(const u32x4*)(lds + row * ld + col));
}
template <int D, bool PROJ>
__device__ __forceinline__ void mlp_tail_tile(const MlpTailArgs& p) {
  constexpr int LDD = D + 8, LDC = 64 + 8;   // row strides (bf16) of tiles with D resp. 64 columns
  constexpr int NB = D / 64;                 // 32-column output blocks per wave
  // LDS: LN(h) rows | W1 chunk (rows k < D, 64 hidden columns) | W2 chunk (rows k < 64, D columns; PROJ: a Wo
  // chunk) | PROJ only: a 64-column chunk of O, then the h rows.  The two weight tiles are also the buffer
  // through which the waves exchange their partial outputs at the end.
  constexpr int N_A = 64 * LDD, N_W1 = D * LDC, N_W2 = 64 * LDD, N_Z = PROJ ? 64 * LDC : 0, N_H = PROJ ? 64 * LDD : 0;
  __shared__ __attribute__((aligned(16))) bf16_t smem[N_A + N_W1 + N_W2 + N_Z + N_H];
  bf16_t* const sA = smem;
  bf16_t* const sW1 = sA + N_A;
  bf16_t* const sW2 = sW1 + N_W1;
  bf16_t* const sZ = sW2 + N_W2;
  bf16_t* const sH = sZ + N_Z;
  static_assert((N_W1 + N_W2) * 2 >= 4 * NB * 16 * 64 * 4, "the exchange buffer must fit in the weight tiles");
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, lo = lane & 31, hi = lane >> 5;
  const int wm = wave >> 1, wn = wave & 1;
  const int m0 = blockIdx.x * 64;
  const int row = wm * 32 + lo;              // the output row of this lane inside the tile
  ChunkTile<64, D> ta;
  ChunkTile<D, 64> t1;
  ChunkTile<64, D> t2;
  if constexpr (PROJ) {
    // h = x + O Wo + bo, the contraction in chunks of 64: O chunk -> sZ, Wo chunk -> sW2, h (bf16) -> sH
    f32x16 acc[NB];
    {
      int off[NB * 4];
      float bq[NB * 4][4];
#pragma unroll
      for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int i = 0; i < 4; ++i) off[nb * 4 + i] = wn * (D / 2) + nb * 32 + 8 * i + 4 * hi;
      bias_quads<NB * 4>(p.bo, off, bq);
#pragma unroll
      for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int j = 0; j < 4; ++j) acc[nb][4 * i + j] = bq[nb * 4 + i][j];
    }
    // every chunk of O and Wo (one or two) and the residual rows are requested at once, before the first is used
    constexpr int NKC = D / 64;
    ChunkTile<64, 64> to[NKC];
    ChunkTile<64, D> tw[NKC];
#pragma unroll
    for (int kc = 0; kc < NKC; ++kc) {
      to[kc].load(p.o + kc * 64, D, m0, p.R - 1, tid);
      tw[kc].load(p.wo + (long)kc * 64 * D, D, 0, 63, tid);
    }
    const int mr = min(m0 + row, p.R - 1);
    u32x2 resv[NB][4];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
      for (int i = 0; i < 4; ++i) resv[nb][i] = *(const u32x2*)(p.h + (long)mr * D + wn * (D / 2) + nb * 32 + 8 * i + 4 * hi);
#pragma unroll
    for (int kc = 0; kc < NKC; ++kc) {
      if (kc) __syncthreads();
      to[kc].store(sZ, LDC, tid);
      tw[kc].store(sW2, LDD, tid);
      __syncthreads();
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        const bf16x8 fa = frag_rows(sZ, LDC, row, s * 16 + hi * 8);
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) acc[nb] = mfma32(lds_frag_tr(sW2, LDD, s * 16, wn * (D / 2) + nb * 32, lane), fa, acc[nb]);
      }
    }
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int n = wn * (D / 2) + nb * 32 + 8 * i + 4 * hi;
        const u32x2 rv = resv[nb][i];
        const u32x2 pk = {pack_bf16(acc[nb][4 * i] + __uint_as_float(rv[0] << 16), acc[nb][4 * i + 1] + __uint_as_float(rv[0] & 0xffff0000u)),
                          pack_bf16(acc[nb][4 * i + 2] + __uint_as_float(rv[1] << 16), acc[nb][4 * i + 3] + __uint_as_float(rv[1] & 0xffff0000u))};
        *(u32x2*)(sH + row * LDD + n) = pk;
      }
    __syncthreads();  // sH complete; every wave is done with sZ and sW2
    ta.load_lds(sH, LDD, tid);
  } else {
    ta.load(p.h, D, m0, p.R - 1, tid);
  }
  ta.layernorm(p.ln_g, p.ln_b, p.ln_eps, tid);
  ta.store(sA, LDD, tid);
  const int nchunk = p.d_ff / 64;
  // W1[:, 64 j .. 64 j + 63] (rows = k < D) and W2[64 j .. 64 j + 63, :] (rows = k < 64), requested TWO chunks ahead
  // into two alternating register sets: with one chunk of arithmetic (16 matrix instructions per wave) between
  // request and use, the trip to L2 was exposed in every chunk
  ChunkTile<D, 64> t1b;
  ChunkTile<64, D> t2b;
  // ... and with them the 16 bias values the lane's z accumulator starts from.  The z block of a wave is 32 rows x
  // 32 hidden columns wn * 32 ..; W1's columns are fed in the order perm32, so register 8 u + e of the block
  // is hidden column 16 u + 8 hi + e: two runs of 8 consecutive columns, the k-slots of the lane in the second product.
  u32x4 bia[2], bib[2];
  const bool b1_vec = (reinterpret_cast<uintptr_t>(p.b1) & 15) == 0;
  auto fetch = [&](int j, ChunkTile<D, 64>& a, ChunkTile<64, D>& b, u32x4 (&bi)[2]) {
    a.load(p.w1 + j * 64, p.d_ff, 0, D - 1, tid);
    b.load(p.w2 + (long)j * 64 * D, D, 0, 63, tid);
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const bf16_t* q = p.b1 + j * 64 + wn * 32 + 16 * u + 8 * hi;
      if (!p.b1) bi[u] = u32x4{0u, 0u, 0u, 0u};
      else if (b1_vec) bi[u] = *(const u32x4*)q;
      else {
#pragma unroll
        for (int e = 0; e < 4; ++e) bi[u][e] = (unsigned)q[2 * e] | ((unsigned)q[2 * e + 1] << 16);
      }
    }
  };
  fetch(0, t1, t2, bia);
  if (nchunk > 1) fetch(1, t1b, t2b, bib);
  // Output accumulators: row `row`, ALL D columns (block nb = columns 32 nb ..), contracted over the wave's own 32
  // hidden columns of every chunk -- z then goes from the accumulator of the first product into the operand of
  // the second without leaving registers, and the two waves of a row block add their halves once, at the end.
  // The wave that writes a column block (blocks wn * NB ..) starts it at b2.
  f32x16 acc2[2 * NB];
  {
    int off[NB * 4];
    float bq[NB * 4][4];
#pragma unroll
    for (int nbi = 0; nbi < NB; ++nbi)
#pragma unroll
      for (int i = 0; i < 4; ++i) off[nbi * 4 + i] = (wn * NB + nbi) * 32 + 8 * i + 4 * hi;
    bias_quads<NB * 4>(p.b2, off, bq);
#pragma unroll
    for (int nb = 0; nb < 2 * NB; ++nb)
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc2[nb][4 * i + j] = (nb / NB) == wn ? bq[(nb % NB) * 4 + i][j] : 0.f;
  }
  // the lane's LN(h) operand fragments (its row, all of D) stay in registers for every chunk
  bf16x8 fa[D / 16];
  __syncthreads();  // sA is complete
#pragma unroll
  for (int s = 0; s < D / 16; ++s) fa[s] = frag_rows(sA, LDD, row, s * 16 + hi * 8);
  auto chunk = [&](int c, ChunkTile<D, 64>& ra, ChunkTile<64, D>& rb, u32x4 (&bi)[2]) {
    __syncthreads();  // the previous chunk's W1 and W2 tiles have been read
    ra.store(sW1, LDC, tid);
    rb.store(sW2, LDD, tid);
    f32x16 acc1;
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        acc1[8 * u + 2 * e] = __uint_as_float(bi[u][e] << 16);
        acc1[8 * u + 2 * e + 1] = __uint_as_float(bi[u][e] & 0xffff0000u);
      }
    __syncthreads();
    if (c + 2 < nchunk) fetch(c + 2, ra, rb, bi);
#pragma unroll
    for (int s = 0; s < D / 16; ++s)
      acc1 = mfma32(lds_frag_tr_perm(sW1, LDC, s * 16, wn * 32, lane), fa[s], acc1);
    bf16x8 zb[2];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      float zv[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) zv[e] = gelu_erf_f(acc1[8 * u + e]);
      zb[u] = pack8(zv);
    }
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
      for (int nb = 0; nb < 2 * NB; ++nb)
        acc2[nb] = mfma32(lds_frag_tr(sW2, LDD, wn * 32 + u * 16, nb * 32, lane), zb[u], acc2[nb]);
  };
  for (int c = 0; c < nchunk; c += 2) {
    chunk(c, t1, t2, bia);
    if (c + 1 < nchunk) chunk(c + 1, t1b, t2b, bib);
  }
  // each wave hands the NB column blocks it does not write to its neighbour (wave ^ 1: same rows, other wn);
  // wn is wave-uniform and every accumulator index below a compile-time constant
  float* const xch = (float*)sW1;
  __syncthreads();  // the last chunk's tiles have been read
  auto put = [&](const f32x16& a, int nbi) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
      *(float4*)(xch + (((wave * NB + nbi) * 4 + i) * 64 + lane) * 4) = make_float4(a[4 * i], a[4 * i + 1], a[4 * i + 2], a[4 * i + 3]);
  };
  auto get = [&](const f32x16& mine, int nbi) {
    f32x16 r;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float4 v = *(const float4*)(xch + ((((wave ^ 1) * NB + nbi) * 4 + i) * 64 + lane) * 4);
      r[4 * i] = mine[4 * i] + v.x; r[4 * i + 1] = mine[4 * i + 1] + v.y;
      r[4 * i + 2] = mine[4 * i + 2] + v.z; r[4 * i + 3] = mine[4 * i + 3] + v.w;
    }
    return r;
  };
  f32x16 accf[NB];
  if (wn == 0) {
#pragma unroll
    for (int nbi = 0; nbi < NB; ++nbi) put(acc2[NB + nbi], nbi);
    __syncthreads();
#pragma unroll
    for (int nbi = 0; nbi < NB; ++nbi) accf[nbi] = get(acc2[nbi], nbi);
  } else {
#pragma unroll
    for (int nbi = 0; nbi < NB; ++nbi) put(acc2[nbi], nbi);
    __syncthreads();
#pragma unroll
    for (int nbi = 0; nbi < NB; ++nbi) accf[nbi] = get(acc2[NB + nbi], nbi);
  }
  const int m = m0 + row;
  if (m >= p.R) return;
#pragma unroll
  for (int nb = 0; nb < NB; ++nb)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int n = wn * (D / 2) + nb * 32 + 8 * i + 4 * hi;
      // residual: the rows before the LayerNorm
      const u32x2 rv = PROJ ? *(const u32x2*)(sH + row * LDD + n) : *(const u32x2*)(p.h + (long)m * D + n);
      const u32x2 pk = {pack_bf16(accf[nb][4 * i] + __uint_as_float(rv[0] << 16), accf[nb][4 * i + 1] + __uint_as_float(rv[0] & 0xffff0000u)),
                        pack_bf16(accf[nb][4 * i + 2] + __uint_as_float(rv[1] << 16), accf[nb][4 * i + 3] + __uint_as_float(rv[1] & 0xffff0000u))};
      *(u32x2*)(p.y + (long)m * p.ldy + n) = pk;
    }
}
// Registers: 168 at D = 64 (three workgroups per CU, as the LDS allows), 256 at D = 128 (two; left to itself the
// compiler took 260 and halved the resident workgroups).
template <int D, bool PROJ>
__global__ __launch_bounds__(256, D == 64 ? 3 : 2) void mlp_tail_kernel(MlpTailArgs p) {
  mlp_tail_tile<D, PROJ>(p);
}
// the tails of two layers of the same shape (two encoders side by side) in one launch: grid y = 2
template <int D, bool PROJ>
__global__ __launch_bounds__(256, D == 64 ? 3 : 2) void mlp_tail_pair_kernel(MlpTailArgs p0, MlpTailArgs p1) {
  mlp_tail_tile<D, PROJ>(blockIdx.y == 0 ? p0 : p1);
}
bool mlp_tail_ok(int is_bf16, long d, long d_ff, const void* h, const void* ln_g, const void* ln_b, const void* w1,
                 const void* w2, const void* y) {
  const uintptr_t a = (uintptr_t)h | (uintptr_t)ln_g | (uintptr_t)ln_b | (uintptr_t)w1 | (uintptr_t)w2 | (uintptr_t)y;
  return is_bf16 && (d == 64 || d == 128) && d_ff >= 64 && d_ff % 64 == 0 && (a & 15) == 0;
}
void launch_mlp_tail(const void* h, const void* ln_g, const void* ln_b, float ln_eps, const void* w1, const void* b1,
                     const void* w2, const void* b2, void* y, int R, int d, int d_ff, hipStream_t st, const void* o,
                     const void* wo, const void* bo) {
  MlpTailArgs p = {(const bf16_t*)h, (const bf16_t*)ln_g, (const bf16_t*)ln_b, ln_eps, (const bf16_t*)w1, (const bf16_t*)b1,
                   (const bf16_t*)w2, (const bf16_t*)b2, (bf16_t*)y, R, d_ff, (const bf16_t*)o, (const bf16_t*)wo,
                   (const bf16_t*)bo, (long)d};
  const dim3 grid((R + 63) / 64), block(256);
  if (d == 64) {
    if (o) hipLaunchKernelGGL((mlp_tail_kernel<64, true>), grid, block, 0, st, p);
    else hipLaunchKernelGGL((mlp_tail_kernel<64, false>), grid, block, 0, st, p);
  } else {
    if (o) hipLaunchKernelGGL((mlp_tail_kernel<128, true>), grid, block, 0, st, p);
    else hipLaunchKernelGGL((mlp_tail_kernel<128, false>), grid, block, 0, st, p);
  }
}

void launch_mlp_tail_pair(const MlpTailPairSide& a, const MlpTailPairSide& b, float ln_eps, int R, int d, int d_ff,
                          hipStream_t st) {
  auto mk = [&](const MlpTailPairSide& s) {
    return MlpTailArgs{(const bf16_t*)s.x, (const bf16_t*)s.ln_g, (const bf16_t*)s.ln_b, ln_eps, (const bf16_t*)s.w1,
                       (const bf16_t*)s.b1, (const bf16_t*)s.w2, (const bf16_t*)s.b2, (bf16_t*)s.y, R, d_ff,
                       (const bf16_t*)s.o, (const bf16_t*)s.wo, (const bf16_t*)s.bo, s.ldy ? s.ldy : (long)d};
  };
  const dim3 grid((R + 63) / 64, 2), block(256);
  if (d == 64) hipLaunchKernelGGL((mlp_tail_pair_kernel<64, true>), grid, block, 0, st, mk(a), mk(b));
  else hipLaunchKernelGGL((mlp_tail_pair_kernel<128, true>), grid, block, 0, st, mk(a), mk(b));
}

// partial[z][M][N] -> out (fp32), z summed in fixed order; output column blocks may go to 3 matrices.
// One thread per 4 consecutive outputs (N and n_per are multiples of 4).
__global__ void mfma_splitk_reduce_kernel(const float* partial, int split_k, int M, int N, float* o0, float* o1,
                                          float* o2, int n_per) {
  const long n_out = (long)M * N;
  const long i = ((long)blockIdx.x * blockDim.x + threadIdx.x) * 4;
  if (i >= n_out) return;
  float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
  int z = 0;
  for (; z + 3 < split_k; z += 4) {   // four requests in flight; added in the same ascending order
    float4 v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) v[u] = *(const float4*)(partial + (z + u) * n_out + i);
#pragma unroll
    for (int u = 0; u < 4; ++u) { s.x += v[u].x; s.y += v[u].y; s.z += v[u].z; s.w += v[u].w; }
  }
  for (; z < split_k; ++z) {
    const float4 v = *(const float4*)(partial + z * n_out + i);
    s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
  }
  const int m = i / N, n = i % N;
  if (n_per > 0) {
    float* o = (n / n_per == 0) ? o0 : (n / n_per == 1) ? o1 : o2;
    if (o) *(float4*)(o + (long)m * n_per + n % n_per) = s;
  } else {
    *(float4*)(o0 + i) = s;
  }
}

// The same for small outputs: with few output quads the kernel above is a handful of workgroups whose
// threads each walk through split_k dependent-latency loads.  Here a block is 16 quads x 16 lanes over
// z: lane zl sums z = zl, zl + 16, ... in ascending order, then the 16 lane sums are added in a fixed
// order through LDS (deterministic; the grouping differs from the kernel above, which is why a shape
// always takes the same one of the two).
__global__ __launch_bounds__(256) void mfma_splitk_reduce_par_kernel(const float* partial, int split_k, int M, int N,
                                                                     float* o0, float* o1, float* o2, int n_per) {
  __shared__ float4 red[16][16];
  const long n_out = (long)M * N;
  const int ql = threadIdx.x & 15, zl = threadIdx.x >> 4;
  const long i = ((long)blockIdx.x * 16 + ql) * 4;
  float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
  if (i < n_out) {
    int z = zl;
    for (; z + 48 < split_k; z += 64) {   // four requests in flight; added in the same ascending order
      float4 v[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) v[u] = *(const float4*)(partial + (z + 16 * u) * n_out + i);
#pragma unroll
      for (int u = 0; u < 4; ++u) { s.x += v[u].x; s.y += v[u].y; s.z += v[u].z; s.w += v[u].w; }
    }
    for (; z < split_k; z += 16) {
      const float4 v = *(const float4*)(partial + z * n_out + i);
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
  const int m = i / N, n = i % N;
  if (n_per > 0) {
    float* o = (n / n_per == 0) ? o0 : (n / n_per == 1) ? o1 : o2;
    if (o) *(float4*)(o + (long)m * n_per + n % n_per) = s;
  } else {
    *(float4*)(o0 + i) = s;
  }
}

// Which kernel (measured on MI355X, C5 shapes):
//  - weight gradients (both operands k-major, long contraction over token rows): the asynchronous
//    256 x 256 kernel is 1.5x faster than the 128 x 128 kernel;
//  - projections with row-major activations and k-major weights (QKV, output projection; K = d):
//    the 256 x 256 kernel needs half the L1 traffic per flop and wins by 1.2-1.35x;
//  - both operands row-major (dO, dx): the 128 x 128 kernel with three workgroups per CU wins (also against
//    the large-tile kernel with 8 waves: 0.122 vs 0.142 ms for the two GEMMs).
static bool use_dma(int M, int N, int K, bool akm = true, bool bkm = true) {
  if (!(bkm && M >= DM && N >= DN && K % DK == 0 && M % 8 == 0 && N % 8 == 0)) return false;
  return akm ? K >= 64 * DK : K >= 8 * DK;
}

// true if a row-major-A, k-major-B (forward linear) or all-row-major (data gradient) GEMM of this shape runs on the
// 128 x 128 kernel, whose epilogue knows MGEMM_GELU_BOTH and MGEMM_GELU_GRAD
bool mfma_gemm_small_tile(int M, int N, int K, bool b_kmajor) { return !use_dma(M, N, K, false, b_kmajor); }

int mfma_gemm_split(int M, int N, int K) {
  if (use_dma(M, N, K)) {
    const long tiles = (long)((M + DM - 1) / DM) * ((N + DN - 1) / DN);
    const int ktiles = K / DK;
    if (tiles >= 128 || ktiles < 32) return 1;
    int s = (int)(256 / tiles);
    if (s > ktiles / 8) s = ktiles / 8;
    return s < 1 ? 1 : s;
  }
  const long tiles = (long)((M + GM - 1) / GM) * ((N + GN - 1) / GN);
  const int ktiles = (K + GK - 1) / GK;
  if (tiles >= 256 || ktiles < 16) return 1;
  int s = (int)((512 + tiles - 1) / tiles);
  if (s > ktiles / 4) s = ktiles / 4;
  if (s > 192) s = 192;  // beyond this the fixed-order reduction of the partials costs more than the GEMM gains
  return s < 1 ? 1 : s;
}

constexpr int DMA_WAVES = 8;   // waves per workgroup of the large-tile kernel
template <bool AKM, bool BKM, bool EPI>
static void launch_dma(const MGemm& p, hipStream_t st) {
  static bool configured = false;  // raise the dynamic-LDS limit once per instantiation (128 KB > the 64 KB default)
  if (!configured) {
    (void)hipFuncSetAttribute((const void*)mfma_gemm_dma_kernel<AKM, BKM, EPI, DMA_WAVES>,
                              hipFuncAttributeMaxDynamicSharedMemorySize, DMA_LDS_BYTES);
    configured = true;
  }
  dim3 grid((p.N + DN - 1) / DN, (p.M + DM - 1) / DM, p.split_k);
  hipLaunchKernelGGL((mfma_gemm_dma_kernel<AKM, BKM, EPI, DMA_WAVES>), grid, dim3(DMA_WAVES * 64), DMA_LDS_BYTES, st, p);
}
// the 288-row variant when its workgroups need fewer (weighted) rounds of the CUs than the 256-row tiles
static bool use_dma12(const MGemm& p) {
  if (p.split_k > 1 || p.partial || p.M < TM || p.b_kper > 0) return false;
  static int cus = 0;   // compute units of the device (the first device that launches; one GPU per process)
  if (cus == 0) {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) == hipSuccess && hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0) cus = n;
    else cus = 256;
  }
  const long nt = (p.N + DN - 1) / DN;
  const long t256 = (long)((p.M + DM - 1) / DM) * nt, t288 = (long)((p.M + TM - 1) / TM) * nt;
  const double r256 = (double)((t256 + cus - 1) / cus), r288 = (double)((t288 + cus - 1) / cus) * (double)TM / DM;
  return r288 < r256;
}
template <bool EPI>
static void launch_dma12(const MGemm& p, hipStream_t st) {
  static bool configured = false;
  if (!configured) {
    (void)hipFuncSetAttribute((const void*)mfma_gemm_dma12_kernel<EPI>, hipFuncAttributeMaxDynamicSharedMemorySize, T_LDS_BYTES);
    configured = true;
  }
  dim3 grid((p.N + DN - 1) / DN, (p.M + TM - 1) / TM, 1);
  hipLaunchKernelGGL((mfma_gemm_dma12_kernel<EPI>), grid, dim3(TWAVES * 64), T_LDS_BYTES, st, p);
}
template <bool AKM, bool BKM>
static void launch_layout(const MGemm& p, bool dma, hipStream_t st) {
  const bool epi = p.gelu || p.res != nullptr;
  if constexpr (!AKM && BKM) {
    if (dma && use_dma12(p)) {
      if (epi) launch_dma12<true>(p, st);
      else launch_dma12<false>(p, st);
      return;
    }
  }
  if (dma) {
    if (epi) launch_dma<AKM, BKM, true>(p, st);
    else launch_dma<AKM, BKM, false>(p, st);
    return;
  }
  const long tiles = (long)((p.N + GN - 1) / GN) * ((p.M + GM - 1) / GM);
  if constexpr (!AKM) {
    // under one workgroup per CU, or under two with an epilogue that loads a residual / evaluates GELU
    // (measured at M = 29 600: plain N = 192 11.8 -> 13.4 us, N = 64 + residual 14.6 -> 12.6, N = 256 + GELU 17.7 -> 15.8)
    if (p.split_k == 1 && !p.partial && p.M > 64 && (tiles < 256 || (epi && tiles < 512))) {
      dim3 grid((p.N + GN - 1) / GN, (p.M + 63) / 64, 1);
      if (epi) hipLaunchKernelGGL((mfma_gemm_kernel<AKM, BKM, true, 64>), grid, dim3(256), 0, st, p);
      else hipLaunchKernelGGL((mfma_gemm_kernel<AKM, BKM, false, 64>), grid, dim3(256), 0, st, p);
      return;
    }
  }
  dim3 grid((p.N + GN - 1) / GN, (p.M + GM - 1) / GM, p.split_k);
  if (epi) hipLaunchKernelGGL((mfma_gemm_kernel<AKM, BKM, true>), grid, dim3(256), 0, st, p);
  else hipLaunchKernelGGL((mfma_gemm_kernel<AKM, BKM, false>), grid, dim3(256), 0, st, p);
}

// Data gradients C = G W^T multiply by a weight stored [n][k] (an m-major B operand).  The large-tile kernels want
// k-major B, and a weight is tiny beside the activations: when they apply, the caller transposes the weights once
// per call (2 MB at d = 512) and the data gradients run on the same kernel as the forward projections.
bool mfma_dgrad_wants_transposed_weights(int M, int N, int K) { return use_dma(M, N, K, false, true) && M >= TM; }
// out[s][c][r] = w[s][r][c] for up to four square d x d matrices (d % 32 == 0); grid (d / 32, d / 32, count)
__global__ __launch_bounds__(256) void transpose_square_kernel(const bf16_t* w0, const bf16_t* w1, const bf16_t* w2,
                                                               const bf16_t* w3, int d, bf16_t* out) {
  __shared__ bf16_t t[32][33];
  const int z = blockIdx.z;
  const bf16_t* w = z == 0 ? w0 : z == 1 ? w1 : z == 2 ? w2 : w3;
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;   // 32 x 8
  const int r0 = blockIdx.y * 32, c0 = blockIdx.x * 32;
#pragma unroll
  for (int i = 0; i < 4; ++i) t[ty + 8 * i][tx] = w[(long)(r0 + ty + 8 * i) * d + c0 + tx];
  __syncthreads();
  bf16_t* o = out + (long)z * d * d;
#pragma unroll
  for (int i = 0; i < 4; ++i) o[(long)(c0 + ty + 8 * i) * d + r0 + tx] = t[tx][ty + 8 * i];
}
void launch_transpose_weights(const void* w0, const void* w1, const void* w2, const void* w3, int count, int d, void* out,
                              hipStream_t st) {
  hipLaunchKernelGGL(transpose_square_kernel, dim3(d / 32, d / 32, count), dim3(256), 0, st, (const bf16_t*)w0,
                     (const bf16_t*)w1, (const bf16_t*)w2, (const bf16_t*)w3, d, (bf16_t*)out);
}

// The Q|K|V projection shape qkv_rows_kernel serves: x [R][d] rows, three [d][d] weights, output rows [R][3d].
static bool qkv_rows_shape(const MGemm& p) {
  auto al16 = [](const void* q) { return (reinterpret_cast<uintptr_t>(q) & 15) == 0; };
  return (p.K == 64 || p.K == 128) && p.N == 3 * p.K && !p.a_kmajor && p.b_kmajor && p.b_nper == p.K && p.b_kper == 0 &&
         p.lda == p.K && p.ldb == p.K && p.ldc == p.N && p.n_per == p.K && p.split_k == 1 && !p.partial && !p.gelu &&
         !p.res && p.M >= 1 && p.B[0] && p.B[1] && p.B[2] && al16(p.A) && al16(p.B[0]) && al16(p.B[1]) && al16(p.B[2]) &&
         al16(p.C) && (!p.ln_g || (p.ln_b && al16(p.ln_g) && al16(p.ln_b)));
}
static void launch_qkv_rows(const MGemm& a, const MGemm* b, hipStream_t st) {
  QkvRows q = {};
  const MGemm* pr[2] = {&a, b};
  for (int z = 0; z < (b ? 2 : 1); ++z) {
    q.x[z] = pr[z]->A; q.qkv[z] = pr[z]->C; q.ln_g[z] = pr[z]->ln_g; q.ln_b[z] = pr[z]->ln_b;
    for (int i = 0; i < 3; ++i) { q.w[z][i] = pr[z]->B[i]; q.bias[z][i] = pr[z]->bias[i]; }
  }
  q.R = a.M; q.ln_eps = a.ln_eps; q.qscale = a.scale0_on ? a.scale0 : 1.f;
  q.groups = (a.M + 127) / 128;
  const dim3 grid((unsigned)q.groups * (b ? 2 : 1));
  static bool configured = false;
  if (!configured) {
    (void)hipFuncSetAttribute((const void*)qkv_rows_kernel<64>, hipFuncAttributeMaxDynamicSharedMemorySize, qkv_rows_lds_bytes<64>());
    (void)hipFuncSetAttribute((const void*)qkv_rows_kernel<128>, hipFuncAttributeMaxDynamicSharedMemorySize, qkv_rows_lds_bytes<128>());
    configured = true;
  }
  if (a.K == 64) hipLaunchKernelGGL(qkv_rows_kernel<64>, grid, dim3(256), qkv_rows_lds_bytes<64>(), st, q);
  else hipLaunchKernelGGL(qkv_rows_kernel<128>, grid, dim3(256), qkv_rows_lds_bytes<128>(), st, q);
}

// Two GEMMs of identical shape and layout (row-major A, k-major B, 64-row tiles, no split-K) in one launch.
bool mfma_gemm_pair_ok(const MGemm& a, const MGemm& b) {
  return !a.a_kmajor && a.b_kmajor && !b.a_kmajor && b.b_kmajor && a.M == b.M && a.N == b.N && a.K == b.K &&
         a.lda == b.lda && a.ldb == b.ldb && a.ldc == b.ldc && a.b_nper == b.b_nper && a.b_kper == b.b_kper &&
         a.n_per == b.n_per && a.scale0_on == b.scale0_on && a.scale0 == b.scale0 && a.ln_eps == b.ln_eps &&
         a.gelu == b.gelu && (a.ln_g != nullptr) == (b.ln_g != nullptr) && (a.res != nullptr) == (b.res != nullptr) &&
         (a.B[1] != nullptr) == (b.B[1] != nullptr) && (a.B[2] != nullptr) == (b.B[2] != nullptr) &&
         (a.bias[0] != nullptr) == (b.bias[0] != nullptr) && (a.bias[1] != nullptr) == (b.bias[1] != nullptr) &&
         (a.bias[2] != nullptr) == (b.bias[2] != nullptr) &&
         a.split_k == 1 && b.split_k == 1 && !a.partial && !b.partial && a.M > 64 && a.gelu <= 1;
}
void launch_mfma_gemm_pair(const MGemm& a, const MGemm& b, hipStream_t st) {
  if (qkv_rows_shape(a) && qkv_rows_shape(b)) return launch_qkv_rows(a, &b, st);   // mfma_gemm_pair_ok: same shape, scale, eps
  MGemm p = a;
  auto off = [](const void* x, const void* y) { return (long)((const char*)y - (const char*)x); };
  p.z_a = off(a.A, b.A); p.z_c = off(a.C, b.C); p.z_res = off(a.res, b.res);
  p.z_ln_g = off(a.ln_g, b.ln_g); p.z_ln_b = off(a.ln_b, b.ln_b);
  for (int i = 0; i < 3; ++i) { p.z_b[i] = off(a.B[i], b.B[i]); p.z_bias[i] = off(a.bias[i], b.bias[i]); }
  const bool epi = a.gelu || a.res != nullptr;
  // 64-row tiles when 128-row tiles would leave the chip under-filled (the rule of launch_layout, on both problems)
  const long tiles = 2L * ((a.N + GN - 1) / GN) * ((a.M + GM - 1) / GM);
  if (tiles < 256 || (epi && tiles < 512)) {
    dim3 grid((a.N + GN - 1) / GN, (a.M + 63) / 64, 2);
    if (epi) hipLaunchKernelGGL((mfma_gemm_pair_kernel<false, true, true, 64>), grid, dim3(256), 0, st, p);
    else hipLaunchKernelGGL((mfma_gemm_pair_kernel<false, true, false, 64>), grid, dim3(256), 0, st, p);
  } else {
    dim3 grid((a.N + GN - 1) / GN, (a.M + GM - 1) / GM, 2);
    if (epi) hipLaunchKernelGGL((mfma_gemm_pair_kernel<false, true, true, GM>), grid, dim3(256), 0, st, p);
    else hipLaunchKernelGGL((mfma_gemm_pair_kernel<false, true, false, GM>), grid, dim3(256), 0, st, p);
  }
}

void launch_mfma_gemm(const MGemm& p, hipStream_t st) {
  if (qkv_rows_shape(p)) return launch_qkv_rows(p, nullptr, st);
  const bool dma = use_dma(p.M, p.N, p.K, p.a_kmajor, p.b_kmajor) && (p.b_kper == 0 || p.b_kper % DK == 0) && !p.ln_g &&
                   p.gelu <= 1;   // MGEMM_GELU_BOTH / _GRAD exist in the 128 x 128 kernel only
  if (p.a_kmajor && p.b_kmajor) launch_layout<true, true>(p, dma, st);
  else if (p.b_kmajor) launch_layout<false, true>(p, dma, st);
  else if (p.a_kmajor) launch_layout<true, false>(p, dma, st);
  else launch_layout<false, false>(p, dma, st);
}
void launch_splitk_reduce(const float* partial, int split_k, int M, int N, float* o0, float* o1, float* o2, int n_per,
                          hipStream_t st) {
  const long quads = ((long)M * N + 3) / 4;
  if (quads <= 65536 && split_k >= 8)   // small output, long reduction: parallel over z as well
    hipLaunchKernelGGL(mfma_splitk_reduce_par_kernel, dim3((unsigned)((quads + 15) / 16)), dim3(256), 0, st, partial,
                       split_k, M, N, o0, o1, o2, n_per);
  else
    hipLaunchKernelGGL(mfma_splitk_reduce_kernel, dim3((unsigned)((quads + 255) / 256)), dim3(256), 0, st, partial, split_k,
                       M, N, o0, o1, o2, n_per);
}

}  // namespace imattn
