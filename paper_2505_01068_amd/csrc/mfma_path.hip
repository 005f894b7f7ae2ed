// Host sequencing of the bf16 MFMA path: projections as MFMA GEMMs around the
// flash-style IM attention kernels; buffers carved from the caller's `saved`
// and `workspace`.
#include "mfma_path.hpp"

#include <string.h>

#include <algorithm>

#include "mfma_common.hpp"

namespace imattn {

static inline size_t al(size_t n) { return (n + 255) & ~(size_t)255; }
constexpr size_t SLACK = 1024;  // tiles read up to one 16-byte vector past the last padded column

bool mfma_supports(int d_model, int dh) { return dh == 64 && d_model % 64 == 0; }

static void build_geot(const im_shape_t* s, GeoT* gt) {
  int off = 0;
  for (int i = 0; i < s->n_seg; ++i) { gt->tp_off[i] = off; off += (s->seg_len[i] + 7) & ~7; }
  for (int i = s->n_seg; i <= IM_MAX_SEG; ++i) gt->tp_off[i] = off;
  gt->Tp = off;
}

struct Dims { size_t B, T, Tp, d, R; };
static Dims dims(const im_shape_t* s) {
  GeoT gt;
  build_geot(s, &gt);
  Dims x;
  x.B = s->batch; x.d = s->d_model; x.Tp = gt.Tp; x.T = 0;
  for (int i = 0; i < s->n_seg; ++i) x.T += s->seg_len[i];
  x.R = x.B * x.T;
  return x;
}

// saved.extra = QKV^T [B][3d][Tp] | O^T [B][d][Tp]
size_t mfma_saved_extra_bytes(const im_shape_t* s) {
  const Dims x = dims(s);
  return al(x.B * 3 * x.d * x.Tp * 2 + SLACK) + al(x.B * x.d * x.Tp * 2 + SLACK);
}
// forward scratch: transposed weights
size_t mfma_fwd_workspace_bytes(int d) { return al((size_t)4 * d * d * 2); }

struct BwdWs { size_t d_o, d_ot, delta, dqkv, dqkvt, xt, dyt, partial, cpart, total; int split_w, split_o; };
static BwdWs bwd_ws(const im_shape_t* s) {
  const Dims x = dims(s);
  BwdWs w;
  size_t off = 0;
  w.d_o = off; off += al(x.R * x.d * 2);
  w.d_ot = off; off += al(x.B * x.d * x.Tp * 2 + SLACK);
  w.delta = off; off += al(x.B * s->n_heads * x.T * 4);
  w.dqkv = off; off += al(x.R * 3 * x.d * 2);
  w.dqkvt = off; off += al(x.B * 3 * x.d * x.Tp * 2 + SLACK);
  w.xt = off; off += al(x.B * x.d * x.Tp * 2 + SLACK);
  w.dyt = off; off += al(x.B * x.d * x.Tp * 2 + SLACK);
  const int ktiles = (int)(x.B * ((x.Tp + 63) / 64));
  w.split_w = mfma_gemm_split((int)x.d, (int)(3 * x.d), ktiles);
  w.split_o = mfma_gemm_split((int)x.d, (int)x.d, ktiles);
  w.partial = off;
  off += al(std::max((size_t)w.split_w * x.d * 3 * x.d, (size_t)w.split_o * x.d * x.d) * 4);
  w.cpart = off; off += al(colsum_partial_bytes((int)x.R, (int)x.d));
  w.total = off;
  return w;
}
size_t mfma_bwd_workspace_bytes(const im_shape_t* s) { return bwd_ws(s).total; }

static void init_gemm(MGemm* p, const Geo& g, const GeoT& gt) {
  memset(p, 0, sizeof(*p));
  p->kb = 1; p->split_k = 1;
  p->Tp = gt.Tp; p->T = g.T; p->n_seg = g.n_seg;
  for (int i = 0; i <= IM_MAX_SEG; ++i) { p->seg_off[i] = g.seg_off[i < g.n_seg ? i : g.n_seg]; p->tp_off[i] = gt.tp_off[i]; }
}

int mfma_attention_fwd(const im_shape_t* s, const void* x, const void* wq, const void* wk, const void* wv,
                       const void* wo, const void* bq, const void* bk, const void* bv, const void* bo,
                       const int32_t* valid_len, const uint8_t* key_pad, void* y, const void* res, char* sv,
                       size_t off_qkv, size_t off_o, size_t off_lse, size_t off_extra, char* ws, hipStream_t st) {
  Geo g;
  build_geo(s, mfma_fwd_tile_rows(), mfma_dkv_tile_rows(), &g);
  GeoT gt;
  build_geot(s, &gt);
  const Dims dm = dims(s);
  const int d = (int)dm.d;
  bf16_t* qkv = (bf16_t*)(sv + off_qkv);
  bf16_t* o = (bf16_t*)(sv + off_o);
  float* lse2 = (float*)(sv + off_lse);
  bf16_t* qkvt = (bf16_t*)(sv + off_extra);
  bf16_t* ot = (bf16_t*)(sv + off_extra + al(dm.B * 3 * dm.d * dm.Tp * 2 + SLACK));
  bf16_t* wt = (bf16_t*)ws;  // [4][d][d]: Wq^T, Wk^T, Wv^T, Wo^T

  const void* wsrc[4] = {wq, wk, wv, wo};
  MGemm p;
  {
  ProfScope ps(PF_PROJ_FWD, st);
  for (int i = 0; i < 4; ++i) launch_transpose_w((const bf16_t*)wsrc[i], d, d, wt + (size_t)i * d * d, st);

  init_gemm(&p, g, gt);
  p.A = (const bf16_t*)x; p.lda = d;
  p.B[0] = wt; p.ldb = d;  // rows n of [Wq^T; Wk^T; Wv^T] are contiguous: one [3d][d] matrix
  p.M = (int)dm.R; p.N = 3 * d; p.kt = d;
  p.bias[0] = (const bf16_t*)bq; p.bias[1] = (const bf16_t*)bk; p.bias[2] = (const bf16_t*)bv; p.n_per = d;
  p.C = qkv; p.ldc = 3 * d;
  p.Ct = qkvt; p.ct_bs = (long)3 * d * gt.Tp;
  launch_mfma_gemm(p, st);
  }

  launch_mfma_fwd(g, gt, qkv, 3 * d, qkvt, valid_len, key_pad, o, d, ot, lse2, st);

  init_gemm(&p, g, gt);
  p.A = o; p.lda = d;
  p.B[0] = wt + (size_t)3 * d * d; p.ldb = d;
  p.M = (int)dm.R; p.N = d; p.kt = d;
  p.bias[0] = (const bf16_t*)bo; p.n_per = d;
  p.res = (const bf16_t*)res;
  p.C = (bf16_t*)y; p.ldc = d;
  { ProfScope ps(PF_PROJ_FWD, st); launch_mfma_gemm(p, st); }

  hipError_t e = hipGetLastError();
  if (e != hipSuccess) { set_error("im_attention_fwd (MFMA path) launch: %s", hipGetErrorString(e)); return IM_ERR_HIP; }
  return IM_OK;
}

int mfma_attention_bwd(const im_shape_t* s, const void* x, const void* wq, const void* wk, const void* wv,
                       const void* wo, const int32_t* valid_len, const uint8_t* key_pad, const char* sv,
                       size_t off_qkv, size_t off_o, size_t off_lse, size_t off_extra, const void* dy, void* dx,
                       void* dwq, void* dwk, void* dwv, void* dwo, void* dbq, void* dbk, void* dbv, void* dbo, char* ws,
                       hipStream_t st) {
  Geo g;
  build_geo(s, mfma_dq_tile_rows(), mfma_dkv_tile_rows(), &g);
  GeoT gt;
  build_geot(s, &gt);
  const Dims dm = dims(s);
  const int d = (int)dm.d;
  const BwdWs w = bwd_ws(s);
  const bf16_t* qkv = (const bf16_t*)(sv + off_qkv);
  const bf16_t* o = (const bf16_t*)(sv + off_o);
  const float* lse2 = (const float*)(sv + off_lse);
  const bf16_t* qkvt = (const bf16_t*)(sv + off_extra);
  const bf16_t* ot = (const bf16_t*)(sv + off_extra + al(dm.B * 3 * dm.d * dm.Tp * 2 + SLACK));
  bf16_t* d_o = (bf16_t*)(ws + w.d_o);
  bf16_t* d_ot = (bf16_t*)(ws + w.d_ot);
  float* delta = (float*)(ws + w.delta);
  bf16_t* dqkv = (bf16_t*)(ws + w.dqkv);
  bf16_t* dqkvt = (bf16_t*)(ws + w.dqkvt);
  bf16_t* xt = (bf16_t*)(ws + w.xt);
  bf16_t* dyt = (bf16_t*)(ws + w.dyt);
  float* partial = (float*)(ws + w.partial);
  float* cpart = (float*)(ws + w.cpart);

  MGemm p;
  // dO = dy Wo^T  (+ transposed copy for the dK/dV kernel)
  init_gemm(&p, g, gt);
  p.A = (const bf16_t*)dy; p.lda = d;
  p.B[0] = (const bf16_t*)wo; p.ldb = d;
  p.M = (int)dm.R; p.N = d; p.kt = d;
  p.C = d_o; p.ldc = d; p.Ct = d_ot; p.ct_bs = (long)d * gt.Tp;
  { ProfScope ps(PF_PROJ_BWD, st); launch_mfma_gemm(p, st); }

  if (dwo) {
    ProfScope ps(PF_WGRAD, st);
    launch_transpose_pad((const bf16_t*)dy, d, d, g, gt, dyt, st);
    init_gemm(&p, g, gt);
    p.A = ot; p.lda = gt.Tp; p.a_bs = (long)d * gt.Tp;
    p.B[0] = dyt; p.ldb = gt.Tp; p.b_bs = (long)d * gt.Tp;
    p.M = d; p.N = d; p.kb = (int)dm.B; p.kt = gt.Tp;
    p.split_k = w.split_o; p.partial = partial;
    launch_mfma_gemm(p, st);
    launch_splitk_reduce(partial, w.split_o, d, d, (float*)dwo, nullptr, nullptr, 0, st);
  }
  if (dbo) { ProfScope ps(PF_WGRAD, st); launch_colsum(dy, d, (int)dm.R, d, 1, (float*)dbo, cpart, st); }

  launch_mfma_bwd(g, g, gt, qkv, 3 * d, qkvt, o, d_o, d, d_ot, lse2, valid_len, key_pad, delta, dqkv, 3 * d, dqkvt, st);

  if (dwq || dwk || dwv) {
    ProfScope ps(PF_WGRAD, st);
    launch_transpose_pad((const bf16_t*)x, d, d, g, gt, xt, st);
    init_gemm(&p, g, gt);
    p.A = xt; p.lda = gt.Tp; p.a_bs = (long)d * gt.Tp;
    p.B[0] = dqkvt; p.ldb = gt.Tp; p.b_bs = (long)3 * d * gt.Tp;
    p.M = d; p.N = 3 * d; p.kb = (int)dm.B; p.kt = gt.Tp;
    p.split_k = w.split_w; p.partial = partial;
    launch_mfma_gemm(p, st);
    launch_splitk_reduce(partial, w.split_w, d, 3 * d, (float*)dwq, (float*)dwk, (float*)dwv, d, st);
  }
  void* dbs[3] = {dbq, dbk, dbv};
  for (int i = 0; i < 3; ++i)
    if (dbs[i]) { ProfScope ps(PF_WGRAD, st); launch_colsum(dqkv + (size_t)i * d, 3 * d, (int)dm.R, d, 1, (float*)dbs[i], cpart, st); }

  if (dx) {
    init_gemm(&p, g, gt);
    p.A = dqkv; p.lda = 3 * d;
    p.B[0] = (const bf16_t*)wq; p.B[1] = (const bf16_t*)wk; p.B[2] = (const bf16_t*)wv; p.ldb = d; p.b_kper = d;
    p.M = (int)dm.R; p.N = d; p.kt = 3 * d;
    p.C = (bf16_t*)dx; p.ldc = d;
    ProfScope ps(PF_PROJ_BWD, st);
    launch_mfma_gemm(p, st);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) { set_error("im_attention_bwd (MFMA path) launch: %s", hipGetErrorString(e)); return IM_ERR_HIP; }
  return IM_OK;
}

}  // namespace imattn
