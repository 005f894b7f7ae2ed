// Host sequencing of the bf16 MFMA path: projections as MFMA GEMMs around the
// flash-style IM attention kernels; buffers carved from the caller's `saved`
// and `workspace`.  Every tensor exists once in HBM, row-major.
#include "mfma_path.hpp"

#include <string.h>

#include <algorithm>

#include "mfma_common.hpp"

namespace imattn {

static inline size_t al(size_t n) { return (n + 255) & ~(size_t)255; }

// head dimension 64, or 8 / 16 in sub-head mode (a head = a slice of a 64-column group)
bool mfma_supports(int d_model, int dh) { return (dh == 64 || dh == 16 || dh == 8) && d_model % 64 == 0; }

struct Dims { size_t B, T, d, R; };
static Dims dims(const im_shape_t* s) {
  Dims x;
  x.B = s->batch; x.d = s->d_model; x.T = 0;
  for (int i = 0; i < s->n_seg; ++i) x.T += s->seg_len[i];
  x.R = (size_t)shape_rows(s);
  return x;
}

size_t mfma_saved_extra_bytes(const im_shape_t*) { return 0; }
size_t mfma_fwd_workspace_bytes(int) { return 0; }

struct BwdWs { size_t d_o, delta, dqkv, partial, partial_o, cpart, wt, total; int split_w, split_o; bool tw; };
static BwdWs bwd_ws(const im_shape_t* s) {
  const Dims x = dims(s);
  BwdWs w;
  size_t off = 0;
  w.d_o = off; off += al(x.R * x.d * 2);
  w.delta = off; off += al((size_t)s->n_heads * x.R * 4);
  w.dqkv = off; off += al(x.R * 3 * x.d * 2);
  w.split_w = mfma_gemm_split((int)x.d, (int)(3 * x.d), (int)x.R);
  w.split_o = mfma_gemm_split((int)x.d, (int)x.d, (int)x.R);
  // one region per weight gradient: a postponed reduction (ReduceList) reads its partials at the end of the pass
  w.partial = off; off += al((size_t)w.split_w * x.d * 3 * x.d * 4);
  w.partial_o = off; off += al((size_t)w.split_o * x.d * x.d * 4);
  w.cpart = off; off += al(4 * colsum_partial_bytes((int)x.R, (int)x.d));   // dbo, dbq, dbk, dbv in one launch
  // Wo^T and [Wq^T; Wk^T; Wv^T] for the data gradients, where the large-tile GEMM serves them
  w.tw = x.d % 32 == 0 && mfma_dgrad_wants_transposed_weights((int)x.R, (int)x.d, (int)x.d);
  w.wt = off; off += w.tw ? al(4 * x.d * x.d * 2) : 0;
  w.total = off;
  return w;
}
size_t mfma_bwd_workspace_bytes(const im_shape_t* s) { return bwd_ws(s).total; }

static void init_gemm(MGemm* p) {
  memset(p, 0, sizeof(*p));
  p->split_k = 1;
}

void mfma_linear(const void* A, long lda, const void* w0, const void* w1, const void* w2, long ldb, int n_per,
                 const void* b0, const void* b1, const void* b2, int gelu, const void* res, void* C, long ldc, int M,
                 int N, int K, hipStream_t st, LnArgs ln, void* C2) {
  MGemm p;
  init_gemm(&p);
  p.C2 = (bf16_t*)C2;
  p.ln_g = (const bf16_t*)ln.g; p.ln_b = (const bf16_t*)ln.b; p.ln_eps = ln.eps;
  p.A = (const bf16_t*)A; p.lda = lda;
  p.B[0] = (const bf16_t*)w0; p.B[1] = (const bf16_t*)w1; p.B[2] = (const bf16_t*)w2; p.ldb = ldb;
  p.b_kmajor = 1; p.b_nper = (w1 || w2) ? n_per : 0;
  p.M = M; p.N = N; p.K = K;
  p.bias[0] = (const bf16_t*)b0; p.bias[1] = (const bf16_t*)b1; p.bias[2] = (const bf16_t*)b2; p.n_per = n_per;
  p.gelu = gelu;
  p.res = (const bf16_t*)res;
  p.C = (bf16_t*)C; p.ldc = ldc;
  launch_mfma_gemm(p, st);
}

void mfma_dgrad(const void* G, long ldg, const void* w0, const void* w1, const void* w2, long ldw, int k_per, void* C,
                long ldc, int M, int N, int K, hipStream_t st, const void* gelu_grad_of) {
  MGemm p;
  init_gemm(&p);
  if (gelu_grad_of) { p.res = (const bf16_t*)gelu_grad_of; p.gelu = MGEMM_GELU_GRAD; }
  p.A = (const bf16_t*)G; p.lda = ldg;
  p.B[0] = (const bf16_t*)w0; p.B[1] = (const bf16_t*)w1; p.B[2] = (const bf16_t*)w2; p.ldb = ldw;
  p.b_kper = (w1 || w2) ? k_per : 0;
  p.M = M; p.N = N; p.K = K;
  p.C = (bf16_t*)C; p.ldc = ldc;
  launch_mfma_gemm(p, st);
}

size_t mfma_wgrad_partial_bytes(int M, int N, int R) { return (size_t)mfma_gemm_split(M, N, R) * M * N * sizeof(float); }

void mfma_wgrad(const void* A, long lda, const void* G, long ldg, float* o0, float* o1, float* o2, int n_per, int M,
                int N, int R, float* partial, hipStream_t st, ReduceList* defer) {
  MGemm p;
  init_gemm(&p);
  p.A = (const bf16_t*)A; p.lda = lda; p.a_kmajor = 1;
  p.B[0] = (const bf16_t*)G; p.ldb = ldg; p.b_kmajor = 1;
  p.M = M; p.N = N; p.K = R;
  p.split_k = mfma_gemm_split(M, N, R); p.partial = partial;
  launch_mfma_gemm(p, st);
  if (defer && reduce_deferrable(M, N, p.split_k) && defer->n < 16) reduce_push(defer, partial, p.split_k, M, N, o0, o1, o2, n_per);
  else launch_splitk_reduce(partial, p.split_k, M, N, o0, o1, o2, n_per, st);
}

// Q|K|V = x [Wq|Wk|Wv] + [bq|bk|bv]: the weights are [d_in][d_out] = k-major B operands.
// Q is stored as scale * log2(e) * (x Wq + bq), rounded once: the attention kernels then get their
// scores in the exponent domain of exp2 straight from the matrix cores (App. B's score scaling included)
static void qkv_gemm(MGemm* p, const void* x, const void* wq, const void* wk, const void* wv, const void* bq,
                     const void* bk, const void* bv, LnArgs ln, float scale_log2e, bf16_t* qkv, int R, int d) {
  init_gemm(p);
  p->A = (const bf16_t*)x; p->lda = d;
  p->B[0] = (const bf16_t*)wq; p->B[1] = (const bf16_t*)wk; p->B[2] = (const bf16_t*)wv; p->ldb = d;
  p->b_kmajor = 1; p->b_nper = d;
  p->M = R; p->N = 3 * d; p->K = d;
  p->bias[0] = (const bf16_t*)bq; p->bias[1] = (const bf16_t*)bk; p->bias[2] = (const bf16_t*)bv; p->n_per = d;
  p->scale0_on = 1; p->scale0 = scale_log2e;
  p->ln_g = (const bf16_t*)ln.g; p->ln_b = (const bf16_t*)ln.b; p->ln_eps = ln.eps;
  p->C = qkv; p->ldc = 3 * d;
}

// The attention of two layers of the same shape (masks s0->live_mask and mask1, own weights, inputs x0 / x1) up
// to the attention output O, in two launches instead of four: one launch holds both QKV projections (the
// LayerNorm inside, model width 64), one both attention kernels.  sv: the forward's tensors for 2 B batch
// elements (rows of the second problem after the first one's).  Returns false, with nothing enqueued, when the
// shape is not one the paired kernels serve.
bool mfma_attention_fwd_pair(const im_shape_t* s0, uint64_t mask1, const void* x0, const void* x1,
                             const gsit_layer_params_t& p0, const gsit_layer_params_t& p1, LnArgs ln0, LnArgs ln1,
                             const int32_t* valid_len, const uint8_t* key_pad, char* sv, size_t off_qkv, size_t off_o,
                             size_t off_lse, hipStream_t st) {
  const int dh = s0->d_model / s0->n_heads;
  im_shape_t s1 = *s0;
  s1.live_mask = mask1;
  Geo g0, g1;
  build_geo(s0, mfma_fwd_tile_rows(dh, s0->n_heads), mfma_dkv_tile_rows(), &g0);
  build_geo(&s1, mfma_fwd_tile_rows(dh, s1.n_heads), mfma_dkv_tile_rows(), &g1);
  if (!mfma_fwd_pair_ok(g0, g1) || !ln0.g || !ln1.g) return false;
  const Dims dm = dims(s0);
  const int d = (int)dm.d, R = (int)dm.R;
  bf16_t* qkv = (bf16_t*)(sv + off_qkv);
  bf16_t* o = (bf16_t*)(sv + off_o);
  float* lse2 = (float*)(sv + off_lse);
  MGemm a, b;
  qkv_gemm(&a, x0, p0.wq, p0.wk, p0.wv, p0.bq, p0.bk, p0.bv, ln0, g0.scale_log2e, qkv, R, d);
  qkv_gemm(&b, x1, p1.wq, p1.wk, p1.wv, p1.bq, p1.bk, p1.bv, ln1, g1.scale_log2e, qkv + (size_t)R * 3 * d, R, d);
  if (!mfma_gemm_pair_ok(a, b)) return false;
  { ProfScope ps(PF_PROJ_FWD, st);
    launch_mfma_gemm_pair(a, b, st); }
  launch_mfma_fwd_pair(g0, g1, qkv, 3 * d, valid_len, key_pad, o, d, lse2, st);
  return true;
}

int mfma_attention_fwd(const im_shape_t* s, const void* x, const void* wq, const void* wk, const void* wv,
                       const void* wo, const void* bq, const void* bk, const void* bv, const void* bo,
                       const int32_t* valid_len, const uint8_t* key_pad, void* y, const void* res, char* sv,
                       size_t off_qkv, size_t off_o, size_t off_lse, size_t, char*, hipStream_t st, LnArgs ln) {
  Geo g;
  build_geo(s, mfma_fwd_tile_rows(s->d_model / s->n_heads, s->n_heads), mfma_dkv_tile_rows(), &g);
  const Dims dm = dims(s);
  const int d = (int)dm.d;
  bf16_t* qkv = (bf16_t*)(sv + off_qkv);
  bf16_t* o = (bf16_t*)(sv + off_o);
  float* lse2 = (float*)(sv + off_lse);

  MGemm p;
  {
    ProfScope ps(PF_PROJ_FWD, st);
    qkv_gemm(&p, x, wq, wk, wv, bq, bk, bv, ln, g.scale_log2e, qkv, (int)dm.R, d);
    launch_mfma_gemm(p, st);
  }

  launch_mfma_fwd(g, qkv, 3 * d, valid_len, key_pad, o, d, lse2, st);

  if (y) {   // y == NULL: the caller applies the output projection itself (to O at sv + off_o)
    ProfScope ps(PF_PROJ_FWD, st);
    init_gemm(&p);
    p.A = o; p.lda = d;
    p.B[0] = (const bf16_t*)wo; p.ldb = d; p.b_kmajor = 1;
    p.M = (int)dm.R; p.N = d; p.K = d;
    p.bias[0] = (const bf16_t*)bo; p.n_per = d;
    p.res = (const bf16_t*)res;
    p.C = (bf16_t*)y; p.ldc = d;
    launch_mfma_gemm(p, st);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) { set_error("im_attention_fwd (MFMA path) launch: %s", hipGetErrorString(e)); return IM_ERR_HIP; }
  return IM_OK;
}

int mfma_attention_bwd(const im_shape_t* s, const void* x, const void* wq, const void* wk, const void* wv,
                       const void* wo, const int32_t* valid_len, const uint8_t* key_pad, const char* sv,
                       size_t off_qkv, size_t off_o, size_t off_lse, size_t, const void* dy, void* dx, void* dwq,
                       void* dwk, void* dwv, void* dwo, void* dbq, void* dbk, void* dbv, void* dbo, char* ws,
                       hipStream_t st, ReduceList* defer) {
  Geo g;
  build_geo(s, mfma_dq_tile_rows(), mfma_dkv_tile_rows(), &g);
  const Dims dm = dims(s);
  const int d = (int)dm.d, R = (int)dm.R;
  const BwdWs w = bwd_ws(s);
  const bf16_t* qkv = (const bf16_t*)(sv + off_qkv);
  const bf16_t* o = (const bf16_t*)(sv + off_o);
  const float* lse2 = (const float*)(sv + off_lse);
  bf16_t* d_o = (bf16_t*)(ws + w.d_o);
  float* delta = (float*)(ws + w.delta);
  bf16_t* dqkv = (bf16_t*)(ws + w.dqkv);
  float* partial = (float*)(ws + w.partial);
  float* partial_o = (float*)(ws + w.partial_o);
  float* cpart = (float*)(ws + w.cpart);

  MGemm p;
  bf16_t* wt = (bf16_t*)(ws + w.wt);   // [Wo^T; Wq^T; Wk^T; Wv^T], each d x d
  {
    // dO = dy Wo^T : B(n = i, k = o) = Wo[i][o], an m-major operand as stored (or k-major after the transpose)
    ProfScope ps(PF_PROJ_BWD, st);
    if (w.tw) launch_transpose_weights(wo, wq, wk, wv, 4, d, wt, st);
    init_gemm(&p);
    p.A = (const bf16_t*)dy; p.lda = d;
    p.B[0] = (const bf16_t*)wo; p.ldb = d;
    if (w.tw) { p.B[0] = wt; p.b_kmajor = 1; }
    p.M = R; p.N = d; p.K = d;
    p.C = d_o; p.ldc = d;
    launch_mfma_gemm(p, st);
  }
  if (dwo) {
    // dWo = O^T dy : contraction over token rows, both operands k-major as stored
    ProfScope ps(PF_WGRAD, st);
    init_gemm(&p);
    p.A = o; p.lda = d; p.a_kmajor = 1;
    p.B[0] = (const bf16_t*)dy; p.ldb = d; p.b_kmajor = 1;
    p.M = d; p.N = d; p.K = R;
    p.split_k = w.split_o; p.partial = partial_o;
    launch_mfma_gemm(p, st);
    if (defer && reduce_deferrable(d, d, w.split_o) && defer->n < 16) reduce_push(defer, partial_o, w.split_o, d, d, (float*)dwo, nullptr, nullptr, 0);
    else launch_splitk_reduce(partial_o, w.split_o, d, d, (float*)dwo, nullptr, nullptr, 0, st);
  }

  launch_mfma_bwd(g, qkv, 3 * d, o, d_o, d, lse2, valid_len, key_pad, delta, dqkv, 3 * d, st);

  if (dwq || dwk || dwv) {
    // dWq | dWk | dWv = x^T [dQ | dK | dV]
    ProfScope ps(PF_WGRAD, st);
    init_gemm(&p);
    p.A = (const bf16_t*)x; p.lda = d; p.a_kmajor = 1;
    p.B[0] = dqkv; p.ldb = 3 * d; p.b_kmajor = 1;
    p.M = d; p.N = 3 * d; p.K = R;
    p.split_k = w.split_w; p.partial = partial;
    launch_mfma_gemm(p, st);
    if (defer && reduce_deferrable(d, 3 * d, w.split_w) && defer->n < 16)
      reduce_push(defer, partial, w.split_w, d, 3 * d, (float*)dwq, (float*)dwk, (float*)dwv, d);
    else launch_splitk_reduce(partial, w.split_w, d, 3 * d, (float*)dwq, (float*)dwk, (float*)dwv, d, st);
  }
  if (dbo || dbq || dbk || dbv) {  // column sums of dy and of the dQ | dK | dV column blocks, one pair of launches
    const void* src[4] = {dy, dqkv, dqkv + d, dqkv + 2 * (size_t)d};
    const long lds4[4] = {(long)d, 3 * (long)d, 3 * (long)d, 3 * (long)d};
    float* dbs[4] = {(float*)dbo, (float*)dbq, (float*)dbk, (float*)dbv};
    ProfScope ps(PF_WGRAD, st);
    launch_colsum_multi(src, lds4, dbs, 4, R, d, 1, cpart, st, defer);
  }

  if (dx) {
    // dx = dQ Wq^T + dK Wk^T + dV Wv^T : K = 3d split over the three weights, each m-major as stored
    ProfScope ps(PF_PROJ_BWD, st);
    init_gemm(&p);
    p.A = dqkv; p.lda = 3 * d;
    p.B[0] = (const bf16_t*)wq; p.B[1] = (const bf16_t*)wk; p.B[2] = (const bf16_t*)wv; p.ldb = d; p.b_kper = d;
    if (w.tw) { p.B[0] = wt + (size_t)d * d; p.B[1] = p.B[2] = nullptr; p.b_kper = 0; p.b_kmajor = 1; }   // [3d][d], k-major
    p.M = R; p.N = d; p.K = 3 * d;
    p.C = (bf16_t*)dx; p.ldc = d;
    launch_mfma_gemm(p, st);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) { set_error("im_attention_bwd (MFMA path) launch: %s", hipGetErrorString(e)); return IM_ERR_HIP; }
  return IM_OK;
}

}  // namespace imattn
