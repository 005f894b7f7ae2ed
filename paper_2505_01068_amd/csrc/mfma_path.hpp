// bf16 MFMA path (head dimension 64): projections as MFMA GEMMs and flash-style
// IM attention on the matrix cores.
#pragma once
#include "common.hpp"

namespace imattn {

// Descriptor of one bf16 MFMA GEMM  C[M,N] = sum_k A(m,k) B(n,k)  (see mfma_gemm.hip).
// Epilogue modes of the 128 x 128 kernel beyond the plain GELU (gelu = 1), for a layer's training passes:
//   BOTH: C = A B + bias (the pre-activation), C2 = GELU(C as rounded to bf16);
//   GRAD: C = (A B) * GELU'(res), res = the saved pre-activation (not added).
constexpr int MGEMM_GELU_BOTH = 2, MGEMM_GELU_GRAD = 3;
struct MGemm {
  const bf16_t* A; long lda; int a_kmajor;  // a_kmajor = 0: A is [M][K] rows; 1: A is [K][M] rows
  const bf16_t* B[3]; long ldb; int b_kmajor;  // b_kmajor = 0: B is [N][K] rows; 1: B is [K][N] rows
  int b_kper;                            // > 0 (m-major B): B[s] covers K columns [s*b_kper, (s+1)*b_kper)
  int b_nper;                            // > 0 (k-major B): B[s] covers N columns [s*b_nper, (s+1)*b_nper)
  int M, N, K;
  int split_k; float* partial;           // partial != NULL: write fp32 partial[z][M][N] instead of the epilogue
  const bf16_t* bias[3]; int n_per;      // bias[n / n_per][n % n_per] (n_per = N for a single bias), or all NULL
  int scale0_on; float scale0;           // scale0_on: columns n < n_per leave as scale0 * (A B + bias)
  const bf16_t* ln_g; const bf16_t* ln_b; float ln_eps;  // ln_g != NULL: the rows of A are LayerNorm-ed as they are
                                                         // staged (row-major A; K == 64: mfma_gemm_fuses_ln, or the Q|K|V shape: mfma_qkv_fuses_ln)
  int gelu;                              // 0, 1 = GELU epilogue, or one of the two modes below (EPI kernels)
  bf16_t* C2;                            // MGEMM_GELU_BOTH: the activation output, same ld as C
  const bf16_t* res;                     // residual rows, same ld as C
  bf16_t* C; long ldc;                   // row-major output
  // paired launch (launch_mfma_gemm_pair): byte offsets from this problem's tensors to the second problem's
  long z_a, z_b[3], z_bias[3], z_ln_g, z_ln_b, z_res, z_c;
};
void launch_mfma_gemm(const MGemm& p, hipStream_t st);
// data gradients with weights transposed once per call: see mfma_gemm.hip
bool mfma_dgrad_wants_transposed_weights(int M, int N, int K);
void launch_transpose_weights(const void* w0, const void* w1, const void* w2, const void* w3, int count, int d, void* out,
                              hipStream_t st);
// two GEMMs of identical shape (row-major A, k-major B, no split-K) in one launch, when mfma_gemm_pair_ok
bool mfma_gemm_pair_ok(const MGemm& a, const MGemm& b);
void launch_mfma_gemm_pair(const MGemm& a, const MGemm& b, hipStream_t st);
// LayerNorm over the K axis of a row-major A can run inside the GEMM when a tile row is the whole feature row
inline bool mfma_gemm_fuses_ln(int is_bf16, long K, long N) { return is_bf16 && K == 64 && N % 8 == 0 && N >= 8; }
// ... and inside the Q|K|V projection of a width-64 or width-128 model (x, the three weights, the output and
// the LayerNorm vectors 16-byte aligned)
inline bool mfma_qkv_fuses_ln(int is_bf16, long d) { return is_bf16 && (d == 64 || d == 128); }
// LayerNorm parameters for the rows of the left operand (all NULL / 0: none)
struct LnArgs { const void* g; const void* b; float eps; };
// bf16 linear layer C[M,N] = A[M,K] W + bias (+ GELU) (+ residual) with weights stored [K][N] (k-major),
// optionally three weight / bias blocks of n_per columns each.  Usable when K % 8 == 0 and N % 8 == 0.
inline bool mfma_linear_ok(int is_bf16, long K, long N) { return is_bf16 && K % 8 == 0 && N % 8 == 0 && K >= 8 && N >= 8; }
// data gradient  C[M,N] = G[M,K] W^T  with W stored [N][K'] row-major; the contraction may run over up to three
// weights of k_per columns each (K = 3 k_per, k_per % 64 == 0), as in dx = dQ Wq^T + dK Wk^T + dV Wv^T
void mfma_dgrad(const void* G, long ldg, const void* w0, const void* w1, const void* w2, long ldw, int k_per, void* C,
                long ldc, int M, int N, int K, hipStream_t st, const void* gelu_grad_of = nullptr);
// (gelu_grad_of != NULL, shapes with mfma_gemm_small_tile only: C = (G W^T) * GELU'(gelu_grad_of), same ld as C)
// weight gradient  C[M,N] (fp32) = A[R,M]^T G[R,N]  (contraction over rows), split-K with a fixed-order
// reduction; n_per > 0: column block s of n_per columns goes to the [M, n_per] output o<s> (NULL = dropped);
// n_per = 0: one [M, N] output o0.  `partial`: mfma_wgrad_partial_bytes.  M % 8 == 0 and N % 8 == 0.
size_t mfma_wgrad_partial_bytes(int M, int N, int R);
void mfma_wgrad(const void* A, long lda, const void* G, long ldg, float* o0, float* o1, float* o2, int n_per, int M,
                int N, int R, float* partial, hipStream_t st, ReduceList* defer = nullptr);
void mfma_linear(const void* A, long lda, const void* w0, const void* w1, const void* w2, long ldb, int n_per,
                 const void* b0, const void* b1, const void* b2, int gelu, const void* res, void* C, long ldc, int M,
                 int N, int K, hipStream_t st, LnArgs ln = {nullptr, nullptr, 0.f}, void* C2 = nullptr);
// (gelu = MGEMM_GELU_BOTH, shapes with mfma_gemm_small_tile only: C = the pre-activation, C2 = GELU of it)
// y = h + GELU(LayerNorm(h) W1 + b1) W2 + b2 in one kernel at model width 64 or 128 (bf16, d_ff % 64 == 0,
// 16-byte aligned pointers; b1 / b2 may be NULL)
bool mlp_tail_ok(int is_bf16, long d, long d_ff, const void* h, const void* ln_g, const void* ln_b, const void* w1,
                 const void* w2, const void* y);
// o != NULL: h is computed in the kernel as x + o Wo + bo, with x passed as `h` (o, Wo 16-byte aligned; bo may be NULL)
void launch_mlp_tail(const void* h, const void* ln_g, const void* ln_b, float ln_eps, const void* w1, const void* b1,
                     const void* w2, const void* b2, void* y, int R, int d, int d_ff, hipStream_t st,
                     const void* o = nullptr, const void* wo = nullptr, const void* bo = nullptr);
// the same for two layers of identical shape in one launch (output projection included: o, wo, bo as above)
struct MlpTailPairSide {
  const void *x, *ln_g, *ln_b, *w1, *b1, *w2, *b2, *o, *wo, *bo;
  void* y;
  long ldy;   // row stride of y in elements; 0 = d
};
void launch_mlp_tail_pair(const MlpTailPairSide& a, const MlpTailPairSide& b, float ln_eps, int R, int d, int d_ff,
                          hipStream_t st);
bool mfma_gemm_small_tile(int M, int N, int K, bool b_kmajor);
int mfma_gemm_split(int M, int N, int K);
void launch_splitk_reduce(const float* partial, int split_k, int M, int N, float* o0, float* o1, float* o2, int n_per,
                          hipStream_t st);

int mfma_fwd_tile_rows(int dh, int n_heads);
int mfma_dq_tile_rows();
int mfma_dkv_tile_rows();
void launch_mfma_fwd(const Geo& g, const bf16_t* qkv, long ld, const int32_t* valid_len, const uint8_t* key_pad,
                     bf16_t* o, long ldo, float* lse2, hipStream_t st);
bool mfma_fwd_pair_ok(const Geo& g0, const Geo& g1);
void launch_mfma_fwd_pair(const Geo& g0, const Geo& g1, const bf16_t* qkv, long ld, const int32_t* valid_len,
                          const uint8_t* key_pad, bf16_t* o, long ldo, float* lse2, hipStream_t st);
void launch_mfma_bwd(const Geo& g, const bf16_t* qkv, long ld, const bf16_t* o, const bf16_t* d_o, long ldo,
                     const float* lse2, const int32_t* valid_len, const uint8_t* key_pad, float* delta, bf16_t* dqkv,
                     long ldg, hipStream_t st);

// Geometry helper shared with api.hip
void build_geo(const im_shape_t* s, int q_tile, int k_tile, Geo* g);

bool mfma_supports(int d_model, int dh);
size_t mfma_saved_extra_bytes(const im_shape_t* s);
size_t mfma_fwd_workspace_bytes(int d);
size_t mfma_bwd_workspace_bytes(const im_shape_t* s);

// sv + off_* : Q|K|V rows [R,3d], O [R,d], lse [B,H,T], extra (transposed copies).
int mfma_attention_fwd(const im_shape_t* s, const void* x, const void* wq, const void* wk, const void* wv,
                       const void* wo, const void* bq, const void* bk, const void* bv, const void* bo,
                       const int32_t* valid_len, const uint8_t* key_pad, void* y, const void* res, char* sv,
                       size_t off_qkv, size_t off_o, size_t off_lse, size_t off_extra, char* ws, hipStream_t st,
                       LnArgs ln = {nullptr, nullptr, 0.f});   // ln: LayerNorm x inside the QKV projection
bool mfma_attention_fwd_pair(const im_shape_t* s0, uint64_t mask1, const void* x0, const void* x1,
                             const gsit_layer_params_t& p0, const gsit_layer_params_t& p1, LnArgs ln0, LnArgs ln1,
                             const int32_t* valid_len, const uint8_t* key_pad, char* sv, size_t off_qkv, size_t off_o,
                             size_t off_lse, hipStream_t st);
int mfma_attention_bwd(const im_shape_t* s, const void* x, const void* wq, const void* wk, const void* wv,
                       const void* wo, const int32_t* valid_len, const uint8_t* key_pad, const char* sv,
                       size_t off_qkv, size_t off_o, size_t off_lse, size_t off_extra, const void* dy, void* dx,
                       void* dwq, void* dwk, void* dwv, void* dwo, void* dbq, void* dbk, void* dbv, void* dbo, char* ws,
                       hipStream_t st, ReduceList* defer = nullptr);   // defer: see ReduceList (small outputs only)

}  // namespace imattn
