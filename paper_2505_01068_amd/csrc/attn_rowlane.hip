// Row-per-lane IM attention for small head dimensions (dh <= 16), plain fp32 ALU.
//
// The multimodal-sentiment shapes have head dimension 5..8: a contraction that
// short cannot fill an MFMA tile, so the live-block products are done as FMAs
// with one query row (forward, dQ) or one key row (dK/dV) per lane and the
// other operand broadcast from LDS.  Each workgroup owns a tile of 64 rows of
// one modality segment (1 or 4 wavefronts, which share the rows of the other
// operand between them); it visits only the key (query) segments the Interlaced
// Mask leaves live for its segment (Sec. 6 "Decomposition"), trimmed to the
// valid length, and keeps one running maximum and sum per row across all of
// them (joint row softmax, Sec. "Information Disorder").
#include "common.hpp"

namespace imattn {

constexpr int RL_ROWS = 64;    // rows per tile == lanes
constexpr int RL_CHUNK = 64;    // rows of the other operand staged in LDS at a time
static_assert(RL_CHUNK == RL_ROWS, "a lane stages exactly one per-row value (key validity, row statistics) of a chunk");
// Kernels are instantiated for the exact head dimension DH (register arrays and FMA loops have DH
// entries: at dh = 5 a padded-to-8 loop would waste 3 of every 8 FMAs); LDS rows are padded to a
// power of two for aligned broadcast reads.
__host__ __device__ constexpr int lds_row(int dh) { return dh <= 4 ? 4 : dh <= 8 ? 8 : 16; }

// Splitting one tile's work over the NW waves of a workgroup.  The rows of the other operand (keys
// for forward / dQ, queries for dK/dV) are visited in chunks of RL_CHUNK rows; the chunks of all live
// segments form one numbered sequence, and wave w takes chunks w, w + NW, ...  Each wave stages its
// chunk in its own LDS slice and keeps its own partial result; the partials are combined in wave
// order at the end (fixed order: results are reproducible).  With a single wave per tile the longest
// tile (one wave walking through every key of a long segment) set the kernel time at the small
// multimodal shapes, where the grid is only a few waves per SIMD.
//
// chunk id -> (segment, first row, rows); false once id is past the last chunk
template <class LenFn>
__device__ __forceinline__ bool locate_chunk(unsigned live, int n_seg, int id, LenFn len_of, int& seg, int& c0, int& n) {
  for (int j = 0; j < n_seg; ++j) {
    if (!((live >> j) & 1u)) continue;
    const int len = len_of(j);
    const int nch = (len + RL_CHUNK - 1) / RL_CHUNK;
    if (id < nch) {
      seg = j;
      c0 = id * RL_CHUNK;
      n = min(RL_CHUNK, len - c0);
      return true;
    }
    id -= nch;
  }
  return false;
}
template <class LenFn>
__device__ __forceinline__ int count_chunks(unsigned live, int n_seg, LenFn len_of) {
  int total = 0;
  for (int j = 0; j < n_seg; ++j)
    if ((live >> j) & 1u) total += (len_of(j) + RL_CHUNK - 1) / RL_CHUNK;
  return total;
}

// The head's dh values of one row (base = the row's first column of the head), zero beyond dh.  Every load is
// issued, none sits behind a branch on dh: a conditional load per element is a round trip per element.
template <typename T, int DH>
__device__ __forceinline__ void load_head_row(const T* base, int dh, float (&out)[DH]) {
  float v[DH];
#pragma unroll
  for (int e = 0; e < DH; ++e) v[e] = ldf(base + (e < dh ? e : 0));
#pragma unroll
  for (int e = 0; e < DH; ++e) out[e] = e < dh ? v[e] : 0.f;
}
// Rows row0 .. row0 + n - 1 (n <= RL_CHUNK) of the head's columns of two matrices into two [RL_CHUNK][LP] LDS
// tiles of one wave, zero beyond n and beyond dh; the first matrix is multiplied by scale_a.  All 2 LP loads of
// a lane are in flight before the first LDS store: written as a loop over the chunk with a store after every
// load, staging was one memory round trip per 64 elements, eight per chunk, and these kernels are latency-bound.
template <typename T, int LP>
__device__ __forceinline__ void stage_chunk(const T* A, long lda, const T* B, long ldb, long row0, int n, int hc, int dh,
                                            float scale_a, float (*sa)[LP], float (*sb)[LP], int lane) {
  constexpr int PER = RL_CHUNK * LP / RL_ROWS;
  float va[PER], vb[PER];
#pragma unroll
  for (int u = 0; u < PER; ++u) {
    const int i = lane + u * RL_ROWS, c = i / LP, e = i % LP;
    const bool ok = c < n && e < dh;
    const long r = row0 + (ok ? c : 0);
    const int col = hc + (ok ? e : 0);
    va[u] = ldf(A + r * lda + col);
    vb[u] = ldf(B + r * ldb + col);
  }
#pragma unroll
  for (int u = 0; u < PER; ++u) {
    const int i = lane + u * RL_ROWS, c = i / LP, e = i % LP;
    const bool ok = c < n && e < dh;
    sa[c][e] = ok ? va[u] * scale_a : 0.f;
    sb[c][e] = ok ? vb[u] : 0.f;
  }
}

template <typename T, int DH, int NW>
__global__ __launch_bounds__(NW * RL_ROWS) void rowlane_fwd_kernel(Geo g, const T* __restrict__ Q, const T* __restrict__ K,
                                                                   const T* __restrict__ V, long ld,
                                                                   const int32_t* __restrict__ valid_len,
                                                                   const uint8_t* __restrict__ key_pad, T* __restrict__ O,
                                                                   long ldo, float* __restrict__ lse2) {
  constexpr int LP = lds_row(DH);
  __shared__ float sKV[NW][2][RL_CHUNK][LP];  // per wave: K rows, V rows of its chunk
  __shared__ float sBias[NW][RL_CHUNK];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int tile, h, b, qs, q0;
  segment_major_index(g.q_tile_prefix, g.q_nord, g.cu != nullptr, tile, h, b);
  decode_tile(g.q_order, g.q_tile_prefix, g.q_nord, RL_ROWS, tile, qs, q0);
  const int qlen = seg_rows(g, b, qs);
  if (q0 >= qlen) return;  // packed rows: this batch element's segment ends before the tile
  const int row = q0 + lane;
  const bool active = row < qlen;
  const long t = seg_row0(g, b, qs) + (active ? row : 0);
  const int dh = g.dh, hc = h * dh;

  float q[DH], acc[DH];
  load_head_row<T, DH>(Q + t * ld + hc, dh, q);
#pragma unroll
  for (int e = 0; e < DH; ++e) {
    q[e] *= g.scale_log2e;
    acc[e] = 0.f;
  }
  float m = IM_NEG_INF, l = 0.f;

  const unsigned live = g.q_live[qs];
  auto klen_of = [&](int j) {
    int klen = seg_rows(g, b, j);
    if (valid_len) klen = min(klen, max(0, valid_len[b * g.n_seg + j]));
    return klen;
  };
  const int rounds = (count_chunks(live, g.n_seg, klen_of) + NW - 1) / NW;
  for (int r = 0; r < rounds; ++r) {
    int j = 0, c0 = 0, n = 0;
    const bool has = locate_chunk(live, g.n_seg, r * NW + wave, klen_of, j, c0, n);
    const int n4 = (n + 3) & ~3;
    __syncthreads();
    if (has) {
      const long kbase = seg_row0(g, b, j);
      // the lane's key-validity byte is requested before the chunk (RL_CHUNK == RL_ROWS: one key per lane): asked for
      // after the chunk's LDS stores it was a round trip of its own
      const unsigned char pad = key_pad ? key_pad[kbase + c0 + min(lane, n - 1)] : (unsigned char)0;
      stage_chunk<T, LP>(K, ld, V, ld, kbase + c0, n, hc, dh, 1.f, sKV[wave][0], sKV[wave][1], lane);
      sBias[wave][lane] = (lane < n && pad == 0) ? 0.f : IM_NEG_INF;
    }
    __syncthreads();
    if (!has) continue;
    for (int c = 0; c < n4; c += 4) {
      float s[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        float a = sBias[wave][c + u];
#pragma unroll
        for (int e = 0; e < DH; ++e) a = fmaf(q[e], sKV[wave][0][c + u][e], a);
        s[u] = a;
      }
      const float mn = fmaxf(fmaxf(fmaxf(s[0], s[1]), fmaxf(s[2], s[3])), m);
      const float ms = (mn == IM_NEG_INF) ? 0.f : mn;
      const float alpha = __builtin_amdgcn_exp2f(m - ms);
      l *= alpha;
#pragma unroll
      for (int e = 0; e < DH; ++e) acc[e] *= alpha;
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const float p = __builtin_amdgcn_exp2f(s[u] - ms);
        l += p;
#pragma unroll
        for (int e = 0; e < DH; ++e) acc[e] = fmaf(p, sKV[wave][1][c + u][e], acc[e]);
      }
      m = mn;
    }
  }
  if (NW > 1) {
    // combine the waves' (max, sum, accumulator) triples; wave w's LDS slice holds its partial
    constexpr int PS = DH + 2;
    static_assert(RL_ROWS * PS <= 2 * RL_CHUNK * LP, "partial results must fit in a wave's LDS slice");
    __syncthreads();
    float* part = &sKV[wave][0][0][0] + lane * PS;
    part[0] = m;
    part[1] = l;
#pragma unroll
    for (int e = 0; e < DH; ++e) part[2 + e] = acc[e];
    __syncthreads();
    if (wave != 0) return;
    for (int w = 1; w < NW; ++w) {
      const float* o = &sKV[w][0][0][0] + lane * PS;
      const float m2 = o[0];
      const float mn = fmaxf(m, m2);
      const float ms = (mn == IM_NEG_INF) ? 0.f : mn;
      const float a1 = __builtin_amdgcn_exp2f(m - ms), a2 = __builtin_amdgcn_exp2f(m2 - ms);
      l = l * a1 + o[1] * a2;
#pragma unroll
      for (int e = 0; e < DH; ++e) acc[e] = acc[e] * a1 + o[2 + e] * a2;
      m = mn;
    }
  }
  if (active) {
    const float inv = (l > 0.f) ? 1.f / l : 0.f;
#pragma unroll
    for (int e = 0; e < DH; ++e)
      if (e < dh) stf(O + t * ldo + hc + e, acc[e] * inv);
    if (lse2) lse2[seg_stat0(g, b, h, qs) + row] = (l > 0.f) ? m + log2f(l) : IM_NEG_INF;
  }
}

// dQ (and delta = rowsum(dO * O)) : one query row per lane, keys broadcast from LDS.
template <typename T, int DH, int NW>
__global__ __launch_bounds__(NW * RL_ROWS) void rowlane_dq_kernel(Geo g, const T* __restrict__ Q, const T* __restrict__ K,
                                                                  const T* __restrict__ V, long ld, const T* __restrict__ O,
                                                                  const T* __restrict__ dO, long ldo,
                                                                  const float* __restrict__ lse2,
                                                                  const int32_t* __restrict__ valid_len,
                                                                  const uint8_t* __restrict__ key_pad,
                                                                  float* __restrict__ delta, T* __restrict__ dQ, long ldg) {
  constexpr int LP = lds_row(DH);
  __shared__ float sKV[NW][2][RL_CHUNK][LP];  // per wave: K rows, V rows of its chunk
  __shared__ float sBias[NW][RL_CHUNK];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int tile, h, b, qs, q0;
  segment_major_index(g.q_tile_prefix, g.q_nord, g.cu != nullptr, tile, h, b);
  decode_tile(g.q_order, g.q_tile_prefix, g.q_nord, RL_ROWS, tile, qs, q0);
  const int qlen = seg_rows(g, b, qs);
  if (q0 >= qlen) return;  // packed rows: this batch element's segment ends before the tile
  const int row = q0 + lane;
  const bool active = row < qlen;
  const long t = seg_row0(g, b, qs) + (active ? row : 0);
  const int dh = g.dh, hc = h * dh;
  const long li = seg_stat0(g, b, h, qs) + (active ? row : 0);

  float q[DH], go[DH], acc[DH];
  float dl = 0.f;
  float oo[DH];
  load_head_row<T, DH>(Q + t * ld + hc, dh, q);
  load_head_row<T, DH>(dO + t * ldo + hc, dh, go);
  load_head_row<T, DH>(O + t * ldo + hc, dh, oo);
#pragma unroll
  for (int e = 0; e < DH; ++e) {
    q[e] *= g.scale_log2e;
    dl = fmaf(go[e], oo[e], dl);
    acc[e] = 0.f;
  }
  float ls = lse2[li];
  if (ls == IM_NEG_INF) ls = __builtin_inff();  // row with no live valid key: every p becomes 0
  if (active && wave == 0) delta[li] = dl;

  const unsigned live = g.q_live[qs];
  auto klen_of = [&](int j) {
    int klen = seg_rows(g, b, j);
    if (valid_len) klen = min(klen, max(0, valid_len[b * g.n_seg + j]));
    return klen;
  };
  const int rounds = (count_chunks(live, g.n_seg, klen_of) + NW - 1) / NW;
  for (int r = 0; r < rounds; ++r) {
    int j = 0, c0 = 0, n = 0;
    const bool has = locate_chunk(live, g.n_seg, r * NW + wave, klen_of, j, c0, n);
    __syncthreads();
    if (has) {
      const long kbase = seg_row0(g, b, j);
      const unsigned char pad = key_pad ? key_pad[kbase + c0 + min(lane, n - 1)] : (unsigned char)0;   // before the chunk
      stage_chunk<T, LP>(K, ld, V, ld, kbase + c0, n, hc, dh, 1.f, sKV[wave][0], sKV[wave][1], lane);
      sBias[wave][lane] = pad == 0 ? 0.f : IM_NEG_INF;
    }
    __syncthreads();
    if (!has) continue;
    for (int c = 0; c < n; ++c) {
      float s = sBias[wave][c], dp = 0.f;
#pragma unroll
      for (int e = 0; e < DH; ++e) {
        s = fmaf(q[e], sKV[wave][0][c][e], s);
        dp = fmaf(go[e], sKV[wave][1][c][e], dp);
      }
      const float p = __builtin_amdgcn_exp2f(s - ls);
      const float ds = p * (dp - dl);
#pragma unroll
      for (int e = 0; e < DH; ++e) acc[e] = fmaf(ds, sKV[wave][0][c][e], acc[e]);
    }
  }
  if (NW > 1) {
    // sum the waves' partial dQ rows in wave order
    static_assert(RL_ROWS * DH <= 2 * RL_CHUNK * LP, "partial results must fit in a wave's LDS slice");
    __syncthreads();
    float* part = &sKV[wave][0][0][0] + lane * DH;
#pragma unroll
    for (int e = 0; e < DH; ++e) part[e] = acc[e];
    __syncthreads();
    if (wave != 0) return;
    for (int w = 1; w < NW; ++w) {
      const float* o = &sKV[w][0][0][0] + lane * DH;
#pragma unroll
      for (int e = 0; e < DH; ++e) acc[e] += o[e];
    }
  }
  if (active) {
#pragma unroll
    for (int e = 0; e < DH; ++e)
      if (e < dh) stf(dQ + t * ldg + hc + e, acc[e] * g.scale);
  }
}

// dK, dV : one key row per lane, query rows (Q, dO, lse, delta) broadcast from LDS.
// Each key segment has a single producer workgroup per tile, so no atomics.
template <typename T, int DH, int NW>
__global__ __launch_bounds__(NW * RL_ROWS) void rowlane_dkv_kernel(Geo g, const T* __restrict__ Q, const T* __restrict__ K,
                                                                   const T* __restrict__ V, long ld,
                                                                   const T* __restrict__ dO, long ldo,
                                                                   const float* __restrict__ lse2,
                                                                   const float* __restrict__ delta,
                                                                   const int32_t* __restrict__ valid_len,
                                                                   const uint8_t* __restrict__ key_pad, T* __restrict__ dK,
                                                                   T* __restrict__ dV, long ldg) {
  constexpr int LP = lds_row(DH);
  __shared__ float sQG[NW][2][RL_CHUNK][LP];  // per wave: Q rows, dO rows of its chunk
  __shared__ float sL[NW][RL_CHUNK];
  __shared__ float sD[NW][RL_CHUNK];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int tile, h, b, ks, k0;
  segment_major_index(g.k_tile_prefix, g.k_nord, g.cu != nullptr, tile, h, b);
  decode_tile(g.k_order, g.k_tile_prefix, g.k_nord, RL_ROWS, tile, ks, k0);
  const int klen_seg = seg_rows(g, b, ks);
  if (k0 >= klen_seg) return;  // packed rows: this batch element's segment ends before the tile
  const int row = k0 + lane;
  const bool in_seg = row < klen_seg;
  bool valid = in_seg;
  if (valid && valid_len) valid = row < valid_len[b * g.n_seg + ks];
  const long t = seg_row0(g, b, ks) + (in_seg ? row : 0);
  if (valid && key_pad) valid = key_pad[t] == 0;
  const int dh = g.dh, hc = h * dh;
  // A tile that lies entirely behind the segment's valid length has no key that any query attends: zeros.
  if (valid_len && k0 >= valid_len[b * g.n_seg + ks]) {
    if (in_seg && wave == 0) {
#pragma unroll
      for (int e = 0; e < DH; ++e)
        if (e < dh) {
          stf(dK + t * ldg + hc + e, 0.f);
          stf(dV + t * ldg + hc + e, 0.f);
        }
    }
    return;
  }

  float k[DH], v[DH], ak[DH], av[DH];
  load_head_row<T, DH>(K + t * ld + hc, dh, k);
  load_head_row<T, DH>(V + t * ld + hc, dh, v);
#pragma unroll
  for (int e = 0; e < DH; ++e) {
    ak[e] = 0.f;
    av[e] = 0.f;
  }
  const unsigned live = g.k_live[ks];
  auto qlen_of = [&](int i) { return seg_rows(g, b, i); };
  const int rounds = (count_chunks(live, g.n_seg, qlen_of) + NW - 1) / NW;
  for (int rd = 0; rd < rounds; ++rd) {
    int i = 0, r0 = 0, n = 0;
    const bool has = locate_chunk(live, g.n_seg, rd * NW + wave, qlen_of, i, r0, n);
    __syncthreads();
    if (has) {
      const long qbase = seg_row0(g, b, i);
      const long lbase = seg_stat0(g, b, h, i);
      // the lane's row statistics are requested before the chunk (one row per lane), not after its LDS stores
      const long at = lbase + r0 + min(lane, n - 1);
      const float ls = lse2[at], dl = delta[at];
      stage_chunk<T, LP>(Q, ld, dO, ldo, qbase + r0, n, hc, dh, g.scale_log2e, sQG[wave][0], sQG[wave][1], lane);
      sL[wave][lane] = (ls == IM_NEG_INF) ? __builtin_inff() : ls;
      sD[wave][lane] = dl;
    }
    __syncthreads();
    if (!has) continue;
    for (int r = 0; r < n; ++r) {
      float s = 0.f, dp = 0.f;
#pragma unroll
      for (int e = 0; e < DH; ++e) {
        s = fmaf(sQG[wave][0][r][e], k[e], s);
        dp = fmaf(sQG[wave][1][r][e], v[e], dp);
      }
      const float p = __builtin_amdgcn_exp2f(s - sL[wave][r]);
      const float ds = p * (dp - sD[wave][r]);
#pragma unroll
      for (int e = 0; e < DH; ++e) {
        av[e] = fmaf(p, sQG[wave][1][r][e], av[e]);
        ak[e] = fmaf(ds, sQG[wave][0][r][e], ak[e]);
      }
    }
  }
  if (NW > 1) {
    // sum the waves' partial dK / dV rows in wave order
    static_assert(RL_ROWS * 2 * DH <= 2 * RL_CHUNK * LP, "partial results must fit in a wave's LDS slice");
    __syncthreads();
    float* part = &sQG[wave][0][0][0] + lane * 2 * DH;
#pragma unroll
    for (int e = 0; e < DH; ++e) { part[e] = ak[e]; part[DH + e] = av[e]; }
    __syncthreads();
    if (wave != 0) return;
    for (int w = 1; w < NW; ++w) {
      const float* o = &sQG[w][0][0][0] + lane * 2 * DH;
#pragma unroll
      for (int e = 0; e < DH; ++e) { ak[e] += o[e]; av[e] += o[DH + e]; }
    }
  }
  if (in_seg) {
    // sQ holds q * scale * log2(e); dK = scale * dS^T q  ==  ln(2) * dS^T (q * scale * log2 e)
    const float ln2 = 0.69314718055994530942f;
#pragma unroll
    for (int e = 0; e < DH; ++e)
      if (e < dh) {
        stf(dK + t * ldg + hc + e, valid ? ak[e] * ln2 : 0.f);
        stf(dV + t * ldg + hc + e, valid ? av[e] : 0.f);
      }
  }
}

// Zero columns col0 .. col0+ncols-1 of the rows of segment s (all batch elements): outputs of query
// segments with no live key segment, gradients of segments that no live block reads.
template <typename T>
__global__ void zero_seg_rows_kernel(Geo g, int s, T* p, long ld, int col0, int ncols) {
  const int nrows = g.seg_len[s];
  const long n = (long)g.B * nrows * ncols;
  for (long i = blockIdx.x * (long)blockDim.x + threadIdx.x; i < n; i += (long)gridDim.x * blockDim.x) {
    const int e = i % ncols;
    const long r = i / ncols;
    const int b = r / nrows, rr = r % nrows;
    if (rr < seg_rows(g, b, s)) stf(p + (seg_row0(g, b, s) + rr) * ld + col0 + e, 0.f);
  }
}
// per-row statistic (lse) of segment s, all batch elements and heads := value
__global__ void fill_seg_stat_kernel(Geo g, int s, float* stat, float value) {
  const int nrows = g.seg_len[s];
  const long n = (long)g.B * g.H * nrows;
  for (long i = blockIdx.x * (long)blockDim.x + threadIdx.x; i < n; i += (long)gridDim.x * blockDim.x) {
    const int rr = i % nrows;
    const long bh = i / nrows;
    const int b = bh / g.H, h = bh % g.H;
    if (rr < seg_rows(g, b, s)) stat[seg_stat0(g, b, h, s) + rr] = value;
  }
}
void launch_zero_seg_rows(const Geo& g, int s, int bf16, void* p, long ld, int col0, int ncols, hipStream_t st) {
  if (bf16) hipLaunchKernelGGL((zero_seg_rows_kernel<bf16_t>), dim3(64), dim3(256), 0, st, g, s, (bf16_t*)p, ld, col0, ncols);
  else hipLaunchKernelGGL((zero_seg_rows_kernel<float>), dim3(64), dim3(256), 0, st, g, s, (float*)p, ld, col0, ncols);
}
void launch_fill_seg_stat(const Geo& g, int s, float* stat, float value, hipStream_t st) {
  hipLaunchKernelGGL(fill_seg_stat_kernel, dim3(16), dim3(256), 0, st, g, s, stat, value);
}

bool rowlane_supports(int dh) { return dh >= 1 && dh <= 16; }

// smallest instantiated head dimension >= dh
#define RL_DISPATCH(dh, LAUNCH) \
  do {                          \
    if ((dh) <= 4) LAUNCH(4);   \
    else if ((dh) == 5) LAUNCH(5); \
    else if ((dh) == 6) LAUNCH(6); \
    else if ((dh) <= 8) LAUNCH(8); \
    else if ((dh) <= 12) LAUNCH(12); \
    else LAUNCH(16);            \
  } while (0)

// Waves per tile when some tile has more than one chunk of the other operand to walk through (by the maximum
// segment lengths), else 1.  Measured at B = 32, 50/500/375 rows, 8 heads of 5 (forward / dQ / dK/dV in us):
// 1 wave 63 / 74 / -, 2 waves 43 / 60 / 70, 3 waves 46 / 65 / 63, 4 waves 48 / 71 / 64.  A wave lives for three
// dependent memory round trips (indices and lengths, its rows, its chunk) around about 45 keys of arithmetic, so
// the kernels are bound by latency and by the instructions around the loop, and fewer, longer waves win until the
// longest tile (one wave walking through 500 keys) sets the time.
constexpr int RL_SPLIT = 2, RL_SPLIT_KV = 4;
static int max_chunks(const Geo& g, bool query_side) {
  int best = 0;
  for (int i = 0; i < g.n_seg; ++i) {
    const unsigned live = query_side ? g.q_live[i] : g.k_live[i];
    int n = 0;
    for (int j = 0; j < g.n_seg; ++j)
      if ((live >> j) & 1u) n += (g.seg_len[j] + RL_CHUNK - 1) / RL_CHUNK;
    best = n > best ? n : best;
  }
  return best;
}

template <typename T>
static int fwd_dispatch(const Geo& g, const T* q, const T* k, const T* v, long ld, const int32_t* vl, const uint8_t* kp,
                        T* o, long ldo, float* lse2, hipStream_t st) {
  const int ntiles = g.q_tile_prefix[g.q_nord];
  if (ntiles == 0) return IM_OK;
  dim3 grid(ntiles, g.H, g.B);
  const bool split = max_chunks(g, true) > 1;
#define RL_FWD(DHV)                                                                                                        \
  do {                                                                                                                     \
    if (split) hipLaunchKernelGGL((rowlane_fwd_kernel<T, DHV, RL_SPLIT>), grid, dim3(RL_SPLIT * RL_ROWS), 0, st, g, q, k, v, \
                                  ld, vl, kp, o, ldo, lse2);                                                               \
    else hipLaunchKernelGGL((rowlane_fwd_kernel<T, DHV, 1>), grid, dim3(RL_ROWS), 0, st, g, q, k, v, ld, vl, kp, o, ldo, lse2); \
  } while (0)
  RL_DISPATCH(g.dh, RL_FWD);
#undef RL_FWD
  return IM_OK;
}

// Rows of query segments with no live block never get written by the kernels: the
// host zero-fills them (output 0, lse -inf) before launching.
template <typename T>
static void zero_dead_rows(const Geo& g, bool query_side, T* p, long ld, hipStream_t st) {
  for (int s = 0; s < g.n_seg; ++s) {
    const unsigned live = query_side ? g.q_live[s] : g.k_live[s];
    if (live) continue;
    launch_zero_seg_rows(g, s, sizeof(T) == 2, p, ld, 0, g.d, st);
  }
}

int launch_rowlane_fwd(const Geo& g, int bf16, const void* q, const void* k, const void* v, long ld,
                       const int32_t* valid_len, const uint8_t* key_pad, void* o, long ldo, float* lse2,
                       hipStream_t st) {
  if (!rowlane_supports(g.dh)) return IM_ERR_UNSUPPORTED;
  for (int s = 0; s < g.n_seg; ++s)
    if (!g.q_live[s] && lse2)
      launch_fill_seg_stat(g, s, lse2, IM_NEG_INF, st);
  if (bf16) {
    zero_dead_rows<bf16_t>(g, true, (bf16_t*)o, ldo, st);
    return fwd_dispatch<bf16_t>(g, (const bf16_t*)q, (const bf16_t*)k, (const bf16_t*)v, ld, valid_len, key_pad,
                                (bf16_t*)o, ldo, lse2, st);
  }
  zero_dead_rows<float>(g, true, (float*)o, ldo, st);
  return fwd_dispatch<float>(g, (const float*)q, (const float*)k, (const float*)v, ld, valid_len, key_pad, (float*)o,
                             ldo, lse2, st);
}

template <typename T>
static int bwd_dispatch(const Geo& g, const T* q, const T* k, const T* v, long ld, const T* o, const T* d_o, long ldo,
                        const float* lse2, const int32_t* vl, const uint8_t* kp, float* delta, T* dq, T* dk, T* dv,
                        long ldg, hipStream_t st) {
  zero_dead_rows<T>(g, true, dq, ldg, st);
  zero_dead_rows<T>(g, false, dk, ldg, st);
  zero_dead_rows<T>(g, false, dv, ldg, st);
  const int nq = g.q_tile_prefix[g.q_nord], nk = g.k_tile_prefix[g.k_nord];
  if (nq == 0) return IM_OK;
  const bool split_q = max_chunks(g, true) > 1, split_k = max_chunks(g, false) > 1;
#define RL_DQ(DHV)                                                                                                         \
  do {                                                                                                                     \
    if (split_q) hipLaunchKernelGGL((rowlane_dq_kernel<T, DHV, RL_SPLIT>), dim3(nq, g.H, g.B), dim3(RL_SPLIT * RL_ROWS), 0, st, \
                                    g, q, k, v, ld, o, d_o, ldo, lse2, vl, kp, delta, dq, ldg);                             \
    else hipLaunchKernelGGL((rowlane_dq_kernel<T, DHV, 1>), dim3(nq, g.H, g.B), dim3(RL_ROWS), 0, st, g, q, k, v, ld, o, d_o, \
                            ldo, lse2, vl, kp, delta, dq, ldg);                                                            \
  } while (0)
#define RL_DKV(DHV)                                                                                                        \
  do {                                                                                                                     \
    if (split_k) hipLaunchKernelGGL((rowlane_dkv_kernel<T, DHV, RL_SPLIT_KV>), dim3(nk, g.H, g.B), dim3(RL_SPLIT_KV * RL_ROWS), 0,  \
                                    st, g, q, k, v, ld, d_o, ldo, lse2, delta, vl, kp, dk, dv, ldg);                        \
    else hipLaunchKernelGGL((rowlane_dkv_kernel<T, DHV, 1>), dim3(nk, g.H, g.B), dim3(RL_ROWS), 0, st, g, q, k, v, ld, d_o,  \
                            ldo, lse2, delta, vl, kp, dk, dv, ldg);                                                        \
  } while (0)
  { ProfScope ps(PF_ATTN_DQ, st); RL_DISPATCH(g.dh, RL_DQ); }
  { ProfScope ps(PF_ATTN_DKV, st); RL_DISPATCH(g.dh, RL_DKV); }
#undef RL_DQ
#undef RL_DKV
  return IM_OK;
}

int launch_rowlane_bwd(const Geo& g, int bf16, const void* q, const void* k, const void* v, long ld, const void* o,
                       const void* d_o, long ldo, const float* lse2, const int32_t* valid_len, const uint8_t* key_pad,
                       float* delta, void* dq, void* dk, void* dv, long ldg, hipStream_t st) {
  if (!rowlane_supports(g.dh)) return IM_ERR_UNSUPPORTED;
  if (bf16)
    return bwd_dispatch<bf16_t>(g, (const bf16_t*)q, (const bf16_t*)k, (const bf16_t*)v, ld, (const bf16_t*)o,
                                (const bf16_t*)d_o, ldo, lse2, valid_len, key_pad, delta, (bf16_t*)dq, (bf16_t*)dk,
                                (bf16_t*)dv, ldg, st);
  return bwd_dispatch<float>(g, (const float*)q, (const float*)k, (const float*)v, ld, (const float*)o,
                             (const float*)d_o, ldo, lse2, valid_len, key_pad, delta, (float*)dq, (float*)dk,
                             (float*)dv, ldg, st);
}

}  // namespace imattn
