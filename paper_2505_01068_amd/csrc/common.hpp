// Shared host/device definitions for the IM attention kernels (gfx950).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "imattn.h"

namespace imattn {

typedef uint16_t bf16_t;  // raw bfloat16 storage

// Geometry of one IM attention problem, passed to kernels by value.
// Activations are [B, T, ld] rows with the head h occupying columns
// [h*dh, (h+1)*dh) of each tensor's row slice.
struct Geo {
  int B, H, d, dh, T, n_seg;
  int seg_off[IM_MAX_SEG + 1];
  int seg_len[IM_MAX_SEG];
  unsigned q_live[IM_MAX_SEG];  // query segment i -> bit set of live key segments j
  unsigned k_live[IM_MAX_SEG];  // key segment j   -> bit set of query segments i that read it
  // Tile schedule (Sec. 6 "Decomposition"): segments in order of decreasing
  // work per row; tiles of one segment are consecutive.  Segments with no live
  // partner are absent.
  int q_order[IM_MAX_SEG], q_tile_prefix[IM_MAX_SEG + 1], q_nord;
  int k_order[IM_MAX_SEG], k_tile_prefix[IM_MAX_SEG + 1], k_nord;
  // Sub-head forward only: bit k set = the query tiles of the k-th segment of q_order are half as tall
  // (q_tile_prefix counts them so); see launch_mfma_fwd.
  unsigned q_half;
  float scale, scale_log2e;
  // Packed rows (im_shape_t::cu_rows): row offsets [B * n_seg + 1] on the device, and the row count.
  // cu == nullptr: padded rows, batch element b owns rows b*T .. b*T + T - 1.
  const int32_t* cu;
  long R;
  // Two problems of the same shape in one launch (pair_B > 0; forward only, padded rows): batch elements
  // b >= pair_B belong to the second problem, whose rows follow the first one's in every tensor and whose
  // mask gives the query segments the live sets / tile order below; valid_len and key_pad are shared
  // (indexed by b - pair_B).
  int pair_B;
  unsigned q_live2[IM_MAX_SEG];
  int q_order2[IM_MAX_SEG], q_tile_prefix2[IM_MAX_SEG + 1], q_nord2;
};

// First row, and number of rows, of segment s of batch element b in the [rows, .] tensors; first
// element of the per-row fp32 tensors (lse, delta) of head h for that segment: [B, H, T] padded,
// [H, R] packed.
__device__ __forceinline__ long seg_row0(const Geo& g, int b, int s) {
  return g.cu ? (long)g.cu[b * g.n_seg + s] : (long)b * g.T + g.seg_off[s];
}
__device__ __forceinline__ int seg_rows(const Geo& g, int b, int s) {
  return g.cu ? g.cu[b * g.n_seg + s + 1] - g.cu[b * g.n_seg + s] : g.seg_len[s];
}
__device__ __forceinline__ long seg_stat0(const Geo& g, int b, int h, int s) {
  return g.cu ? (long)h * g.R + g.cu[b * g.n_seg + s] : ((long)b * g.H + h) * g.T + g.seg_off[s];
}
// The same for callers whose b and s are wave-uniform (the matrix-core kernels): the row offsets
// read from memory are moved to scalar registers, so pointers derived from them stay scalar.
__device__ __forceinline__ int cu_u(const Geo& g, int i) { return __builtin_amdgcn_readfirstlane(g.cu[i]); }
__device__ __forceinline__ long useg_row0(const Geo& g, int b, int s) {
  return g.cu ? (long)cu_u(g, b * g.n_seg + s) : (long)b * g.T + g.seg_off[s];
}
__device__ __forceinline__ int useg_rows(const Geo& g, int b, int s) {
  return g.cu ? cu_u(g, b * g.n_seg + s + 1) - cu_u(g, b * g.n_seg + s) : g.seg_len[s];
}
__device__ __forceinline__ long useg_stat0(const Geo& g, int b, int h, int s) {
  return g.cu ? (long)h * g.R + cu_u(g, b * g.n_seg + s) : ((long)b * g.H + h) * g.T + g.seg_off[s];
}
// rows of the [rows, .] tensors of a shape (host)
inline long shape_rows(const im_shape_t* s) {
  if (s->cu_rows) return (long)s->total_rows;
  long T = 0;
  for (int i = 0; i < s->n_seg; ++i) T += s->seg_len[i];
  return (long)s->batch * T;
}

// tile index -> (segment, first row).  Same code on host (schedule listing)
// and device (kernels), so the listing is what the kernels execute.
__host__ __device__ inline void decode_tile(const int* order, const int* prefix, int nord, int tile_rows, int tile,
                                            int& seg, int& start) {
  int k = 0;
  while (k + 1 < nord && tile >= prefix[k + 1]) ++k;
  seg = order[k];
  start = (tile - prefix[k]) * tile_rows;
}

__device__ __forceinline__ float bf2f(bf16_t v) { return __uint_as_float(((uint32_t)v) << 16); }
__device__ __forceinline__ bf16_t f2bf(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40);  // quiet NaN
  u += 0x7fffu + ((u >> 16) & 1u);                                        // round to nearest even
  return (bf16_t)(u >> 16);
}
__device__ __forceinline__ float ldf(const float* p) { return *p; }
__device__ __forceinline__ float ldf(const bf16_t* p) { return bf2f(*p); }
__device__ __forceinline__ void stf(float* p, float v) { *p = v; }
__device__ __forceinline__ void stf(bf16_t* p, float v) { *p = f2bf(v); }

#define IM_NEG_INF (-__builtin_inff())

// XCD-aware workgroup index.  The dispatcher deals consecutive workgroup ids round-robin to the
// 8 XCDs (each with its own L2).  Remapping id -> (id % 8) * chunk + id / 8 makes every XCD work
// through one CONTIGUOUS range of logical tiles, so tiles that share an operand (the K/V of one
// (batch, head); the activation rows of one GEMM row block) meet in the same L2.
#ifdef __HIPCC__
__device__ __forceinline__ void xcd_block_index(int& bx, int& by, int& bz) {
  const unsigned gx = gridDim.x, gy = gridDim.y, gz = gridDim.z;
  const unsigned total = gx * gy * gz;
  const unsigned lin = blockIdx.x + gx * (blockIdx.y + gy * blockIdx.z);
  const unsigned xcd = lin & 7u, idx = lin >> 3;
  const unsigned q = total >> 3, r = total & 7u;
  const unsigned logical = xcd * q + (xcd < r ? xcd : r) + idx;
  bx = logical % gx;
  by = (logical / gx) % gy;
  bz = logical / (gx * gy);
}
// q = n / d and r = n % d of workgroup indices.  Below 2^22 the quotient comes from a float
// reciprocal (off by at most one, corrected), a quarter of the instructions of the exact 32-bit
// division; workgroups that find nothing to do (packed rows) spend most of their time here.
__device__ __forceinline__ void udivmod(unsigned n, unsigned d, unsigned& q, unsigned& r) {
  if (n < (1u << 22)) {
    q = (unsigned)((float)n * __builtin_amdgcn_rcpf((float)d));
    r = n - q * d;
    if ((int)r < 0) { --q; r += d; }
    else if (r >= d) { ++q; r -= d; }
  } else {
    q = n / d;
    r = n % d;
  }
}

// Workgroup -> (tile, head, batch element) for a grid (tiles, heads, batch), segment-major: all
// workgroups of the first segment of the tile order (the one with the most work per tile) come
// first, for every (batch element, head) pair, then those of the next segment.  The workgroups
// that run longest start first and the short ones fill the tail of the launch.  Inside a segment
// the order is pair, then tile (the tiles of one pair read the same keys and start together) --
// except with packed rows (tile_first), where the grid covers the longest sample and the later
// tiles of most pairs find no rows: there tile, then pair, so the tiles that have work are not
// queued behind the empty ones.
__device__ __forceinline__ void segment_major_index(const int* prefix, int nord, bool tile_first, int& tile, int& h,
                                                    int& b) {
  const unsigned gx = gridDim.x, gy = gridDim.y, npair = gy * gridDim.z;
  const unsigned lin = blockIdx.x + gx * (blockIdx.y + gy * blockIdx.z);
  int k = 0;
  while (k + 1 < nord && lin >= npair * (unsigned)prefix[k + 1]) ++k;
  const unsigned nt = (unsigned)(prefix[k + 1] - prefix[k]), j = lin - npair * (unsigned)prefix[k];
  unsigned pair, t, hh, bb;
  if (tile_first) udivmod(j, npair, t, pair);
  else udivmod(j, nt, pair, t);
  udivmod(pair, gy, bb, hh);
  tile = prefix[k] + (int)t;
  h = (int)hh;
  b = (int)bb;
}
#endif

// ---- launchers implemented in the .hip files (all enqueue on `st`, none syncs) ----

// fp32-ALU GEMM  C[m,n] = sum_k A(m,k) B(k,n) (+bias[n]) (+res[m,n]), optional GELU,
// operands addressed by strides; B / bias / C may be split over up to 3 buffers.
struct GemmDesc {
  const void* A;
  long sam, sak;            // element strides of A(m,k)
  const void* B[3];
  long sbk, sbn;            // element strides of B(k,n) inside one B buffer
  int b_split;              // 0: one B buffer; 1: B[s] holds column block s (n_per columns each); 2: row block s (k_per rows each)
  int n_per, k_per;         // block extents for the splits (n_per also blocks bias / C when those are split)
  const void* bias[3];      // bias along N; bias_split = 1: bias[s] belongs to column block s
  void* C[3];               // outputs; c_split = 1: column block s goes to the [M, n_per] matrix C[s]
  int c_split, bias_split;
  long ldc;
  const void* res;          // residual added in the epilogue (same dtype/ld as C[0]) or NULL
  int M, N, K;
  int gelu;                 // apply exact GELU after bias
  int split_k;              // >1: partial sums in `partial` [split_k, M, N] fp32, reduced in fixed order
  float* partial;
  // batched-K form (weight gradients): K runs over kb batches of kt rows; A/B advance by sab/sbb per batch
  int kb, kt;
  long sab, sbb;
};
int launch_gemm_alu(const GemmDesc& g, int a_bf16, int b_bf16, int c_bf16, hipStream_t st);
size_t gemm_alu_partial_bytes(int M, int N, int K, int* split_k);

// Second stages that a caller may postpone to ONE launch at the end of a backward pass: the fixed-order sums over
// split-K partials [nparts][M][N] (outputs as mfma_wgrad's) and over the row-block partials of column sums (M = 1).
// Each is a few microseconds of launch latency on its own.  A postponed job's partial buffer must stay untouched
// until launch_reduce_list.
struct ReduceJob { const float* partial; int nparts, M, N, n_per; float* o[3]; };
struct ReduceList { ReduceJob job[16]; int n; };
// N % 4 == 0, at most 65536 output quads and at most 8 MB of partials (a larger set is read back faster right after
// it was written, while it is still in the last-level cache): the job can go on a list
bool reduce_deferrable(int M, int N, int nparts);
void reduce_push(ReduceList* l, const float* partial, int nparts, int M, int N, float* o0, float* o1, float* o2, int n_per);
void launch_reduce_list(const ReduceList& l, hipStream_t st);
// column sums of a [R, n] matrix (bias gradients), deterministic two-stage
int launch_colsum(const void* a, long lda, int R, int n, int a_bf16, float* out, float* partial, hipStream_t st);
size_t colsum_partial_bytes(int R, int n);   // for one matrix; launch_colsum_multi (count <= 4) needs count times as much
// column sums of up to 3 [R, n] matrices (same element type) in one pair of launches; out[i] == nullptr skips matrix i
int launch_colsum_multi(const void* const* a, const long* lda, float* const* out, int count, int R, int n, int a_bf16,
                        float* partial, hipStream_t st, ReduceList* defer = nullptr);   // defer: second stage onto the list

// Zero columns col0 .. col0+ncols-1 of the rows of segment s of a [rows, ld] matrix; set a per-row
// fp32 statistic ([B,H,T] padded / [H,R] packed) of the rows of segment s.  All batch elements.
void launch_zero_seg_rows(const Geo& g, int s, int bf16, void* p, long ld, int col0, int ncols, hipStream_t st);
void launch_fill_seg_stat(const Geo& g, int s, float* stat, float value, hipStream_t st);

// row-per-lane attention for small head dims (plain ALU)
int launch_rowlane_fwd(const Geo& g, int bf16, const void* q, const void* k, const void* v, long ld,
                       const int32_t* valid_len, const uint8_t* key_pad, void* o, long ldo, float* lse2,
                       hipStream_t st);
int launch_rowlane_bwd(const Geo& g, int bf16, const void* q, const void* k, const void* v, long ld, const void* o,
                       const void* d_o, long ldo, const float* lse2, const int32_t* valid_len, const uint8_t* key_pad,
                       float* delta, void* dq, void* dk, void* dv, long ldg, hipStream_t st);
bool rowlane_supports(int dh);

// LayerNorm rows
int launch_layernorm(const void* x, const void* gamma, const void* beta, void* y, int R, int d, float eps, int bf16,
                     hipStream_t st);

// weight gradient of a narrow layer, C[M,N] = A[R,M]^T G[R,N] with M <= 64, N <= 256 (see gemm_alu.hip):
// writes and returns a number of partial [M,N] matrices that the caller sums in a fixed order
bool wgrad_small_ok(int M, int N, int n_per);
size_t wgrad_small_partial_bytes(int M, int N, int R);
void launch_wgrad_small_reduce(const float* partial, int nz, int M, int N, float* o0, float* o1, float* o2, int n_per,
                               hipStream_t st);
int launch_wgrad_small(const void* A, long lda, const void* G, long ldg, int R, int M, int N, int in_bf16, float* partial,
                       hipStream_t st);
// the same for fp32 operands of a tall matrix (R >= 1024, M <= 64, N <= 128) on the fp32 matrix instruction; sums the
// partial results itself: C into o0 (n_per == 0) or column blocks of n_per columns into o0 | o1 | o2 (NULL = dropped)
bool wgrad_mfma_ok(int M, int N, int R, int in_bf16);
size_t wgrad_mfma_partial_bytes(int M, int N, int R);
void launch_wgrad_mfma_f32(const float* A, long lda, const float* G, long ldg, int R, int M, int N, float* partial,
                           float* o0, float* o1, float* o2, int n_per, hipStream_t st);
// both weight gradients of an attention block (d <= 42: 3 d <= 128) in one pair of launches; NULL outputs are dropped;
// partial: wgrad_mfma_partial_bytes(d, 3 d, R) + wgrad_mfma_partial_bytes(d, d, R) bytes
void launch_wgrad_mfma_f32_attn(const float* X, const float* dQKV, const float* O, const float* dY, int R, int d,
                                float* partial, float* q0, float* q1, float* q2, float* dwo, hipStream_t st);

// encoder-layer backward pieces: a = GELU(z); g <- g * GELU'(z) in place; LayerNorm backward of rows
// (dx = input gradient + res (res may be NULL), t = dy * xhat for the gamma gradient)
int launch_gelu_fwd(const void* z, void* a, long n, int bf16, hipStream_t st);
int launch_gelu_bwd(const void* z, void* g, long n, int bf16, hipStream_t st);
int launch_layernorm_bwd(const void* x, const void* gamma, const void* dy, const void* res, void* dx, void* t, int R,
                         int d, float eps, int bf16, hipStream_t st);

void set_error(const char* fmt, ...);

// One layer of each of two encoders side by side (see api.hip); workspace bytes (0: shape not served)
size_t gsit_layer_pair_ws(const im_shape_t* s);
int gsit_layer_fwd_pair(const im_shape_t* s0, uint64_t mask1, int32_t d_ff, const void* x0, const void* x1,
                        const gsit_layer_params_t& p0, const gsit_layer_params_t& p1, float ln_eps,
                        const int32_t* valid_len, const uint8_t* key_pad, void* y0, void* y1, void* workspace,
                        size_t workspace_bytes, hipStream_t st, bool* done, long ldy = 0);

// Optional per-kernel-family timing (see im_profile_enable): records an event pair
// around the launches issued while the scope is alive.
enum ProfFamily { PF_PROJ_FWD = 0, PF_ATTN_FWD, PF_ATTN_DQ, PF_ATTN_DKV, PF_PROJ_BWD, PF_WGRAD, PF_MISC, PF_COUNT };
struct ProfScope {
  int slot;
  hipStream_t st;
  ProfScope(ProfFamily f, hipStream_t s);
  ~ProfScope();
};

}  // namespace imattn
