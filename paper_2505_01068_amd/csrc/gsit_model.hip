// The GsiT model around the encoder layers (Sec. 5, Eq. "allmodalinone fusion"):
//   F = encoder(x) under the forward IFM, B = encoder(x) under the backward IFM (own weights),
//   Vbar = F || B (width 2d), A = encoder(Vbar) under the IEM, X = f(|| last step of every segment of A).
// Host sequencing of gsit_layer_fwd plus three small kernels (feature concatenation, last-step
// gather, final linear through the ALU GEMM).
#include <math.h>
#include <string.h>

#include "common.hpp"

namespace imattn {

// c[r, 0:d) = a[r, :], c[r, d:2d) = b[r, :]   (16-bit or 32-bit elements, `es` bytes each)
template <typename T>
__global__ void concat_features_kernel(const T* __restrict__ a, const T* __restrict__ b, T* __restrict__ c, long rows, int d) {
  const long n = rows * 2L * d;
  for (long i = blockIdx.x * (long)blockDim.x + threadIdx.x; i < n; i += (long)gridDim.x * blockDim.x) {
    const long r = i / (2 * d);
    const int col = (int)(i - r * 2 * d);
    c[i] = col < d ? a[r * d + col] : b[r * d + col - d];
  }
}

// z[b, s*w : (s+1)*w) = a[b, last position of segment s, :]; the last position is the last VALID
// one when valid lengths are given (max(min(valid, T_s), 1) - 1), else T_s - 1.
template <typename T>
__global__ void gather_last_kernel(const T* __restrict__ a, T* __restrict__ z, const int32_t* __restrict__ valid_len,
                                   int B, int Tm, int w, int n_seg, Geo g) {
  const long n = (long)B * n_seg * w;
  for (long i = blockIdx.x * (long)blockDim.x + threadIdx.x; i < n; i += (long)gridDim.x * blockDim.x) {
    const int col = (int)(i % w);
    const int s = (int)((i / w) % n_seg);
    const int b = (int)(i / ((long)w * n_seg));
    int pos = g.seg_len[s] - 1;
    if (valid_len) pos = max(min(valid_len[b * n_seg + s], g.seg_len[s]), 1) - 1;
    z[i] = a[((long)b * Tm + g.seg_off[s] + pos) * w + col];
  }
}

static size_t al256(size_t n) { return (n + 255) & ~(size_t)255; }

struct ModelWs {
  size_t f, b, cat, z, layer, total;
  size_t layer_inter, layer_intra;
};

static int model_ws(const im_shape_t* s, const gsit_model_t* m, im_shape_t* intra_shape, ModelWs* w) {
  if (!s || !m) { set_error("shape and model must not be NULL"); return IM_ERR_INVALID; }
  if (s->cu_rows) { set_error("the whole-model call needs padded rows (shape->cu_rows must be NULL)"); return IM_ERR_UNSUPPORTED; }
  if (m->n_layers_inter < 1 || m->n_layers_intra < 1 || m->n_out < 1) {
    set_error("n_layers_inter, n_layers_intra and n_out must be >= 1");
    return IM_ERR_INVALID;
  }
  if (m->n_heads_intra < 1 || (2 * s->d_model) % m->n_heads_intra != 0) {
    set_error("n_heads_intra (%d) must divide 2 * d_model (%d)", m->n_heads_intra, 2 * s->d_model);
    return IM_ERR_INVALID;
  }
  if (!(m->scale_intra >= 0.f) || !isfinite(m->scale_intra)) { set_error("scale_intra must be finite and >= 0"); return IM_ERR_INVALID; }
  *intra_shape = *s;
  intra_shape->d_model = 2 * s->d_model;
  intra_shape->n_heads = m->n_heads_intra;
  intra_shape->scale = m->scale_intra;
  intra_shape->live_mask = m->mask_intra;
  im_shape_t inter = *s;
  int rc;
  inter.live_mask = m->mask_fwd;
  if ((rc = gsit_layer_sizes(&inter, m->d_ff_inter, &w->layer_inter))) return rc;
  inter.live_mask = m->mask_bwd;
  if ((rc = gsit_layer_sizes(&inter, m->d_ff_inter, &w->layer_inter))) return rc;
  if ((rc = gsit_layer_sizes(intra_shape, m->d_ff_intra, &w->layer_intra))) return rc;
  const size_t es = s->dtype == IM_DTYPE_BF16 ? 2 : 4;
  long T = 0;
  for (int i = 0; i < s->n_seg; ++i) T += s->seg_len[i];
  const size_t R = (size_t)s->batch * T, d = s->d_model;
  size_t off = 0;
  w->f = off; off += al256(R * d * es);
  w->b = off; off += al256(R * d * es);
  w->cat = off; off += al256(R * 2 * d * es);
  w->z = off; off += al256((size_t)s->batch * s->n_seg * 2 * d * es);
  size_t lw = w->layer_inter > w->layer_intra ? w->layer_inter : w->layer_intra;
  inter.live_mask = m->mask_fwd;
  const size_t pw = gsit_layer_pair_ws(&inter);   // the two inter-modal encoders layer by layer in shared launches
  if (pw > lw) lw = pw;
  w->layer = off; off += al256(lw);
  w->total = off;
  return IM_OK;
}

static int run_encoder(const im_shape_t* s, int d_ff, const gsit_layer_params_t* L, int n, float eps, const void* in,
                       void* out, const int32_t* valid_len, const uint8_t* key_pad, void* ws, size_t ws_bytes, void* st) {
  const void* cur = in;
  for (int l = 0; l < n; ++l) {
    const gsit_layer_params_t& p = L[l];
    // every layer writes `out`; from the second layer on it reads `out` as well (y may alias x)
    int rc = gsit_layer_fwd(s, d_ff, cur, p.ln1_g, p.ln1_b, p.wq, p.wk, p.wv, p.wo, p.bq, p.bk, p.bv, p.bo, p.ln2_g,
                            p.ln2_b, p.w1, p.b1, p.w2, p.b2, eps, valid_len, key_pad, out, ws, ws_bytes, st);
    if (rc) return rc;
    cur = out;
  }
  return IM_OK;
}

// out[m, n] = sum_k z[m, k] wf[k, n] + bf[n] for the few (batch x n_out) outputs of the fusion head: one
// wavefront per output, lanes stride over k, fixed-order shuffle reduction.  The tiled GEMM would walk
// the 6 d-long contraction as a serial chain of 16-deep tiles in a single workgroup.
// The gather of the last positions happens inside: z[m, s * w + c] is read from `a` where it lies
// (gather_last_kernel's indexing), one launch instead of two.
template <typename T>
__global__ __launch_bounds__(256) void head_dot_gather_kernel(const T* __restrict__ a, const int32_t* __restrict__ valid_len,
                                                              const T* __restrict__ wf, const T* __restrict__ bias,
                                                              T* __restrict__ out, int M, int N, int Tm, int w, int n_seg,
                                                              Geo g) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const long o = (long)blockIdx.x * 4 + wave;
  if (o >= (long)M * N) return;
  const int m = (int)(o / N), n = (int)(o % N), K = n_seg * w;
  float acc = 0.f;
  for (int k = lane; k < K; k += 64) {
    const int s = k / w, col = k - s * w;
    int pos = g.seg_len[s] - 1;
    if (valid_len) pos = max(min(valid_len[m * n_seg + s], g.seg_len[s]), 1) - 1;
    acc = fmaf(ldf(a + ((long)m * Tm + g.seg_off[s] + pos) * w + col), ldf(wf + (long)k * N + n), acc);
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off, 64);
  if (lane == 0) stf(out + o, acc + (bias ? ldf(bias + n) : 0.f));
}

}  // namespace imattn

using namespace imattn;

extern "C" {

int gsit_model_sizes(const im_shape_t* shape, const gsit_model_t* model, size_t* workspace_bytes) {
  im_shape_t intra;
  ModelWs w;
  int rc = model_ws(shape, model, &intra, &w);
  if (rc) return rc;
  if (workspace_bytes) *workspace_bytes = w.total;
  return IM_OK;
}

int gsit_model_fwd(const im_shape_t* shape, const gsit_model_t* model, const void* x, const int32_t* valid_len,
                   const uint8_t* key_pad, void* out, void* workspace, size_t workspace_bytes, void* hip_stream) {
  im_shape_t intra;
  ModelWs w;
  int rc = model_ws(shape, model, &intra, &w);
  if (rc) return rc;
  if (!x || !out || !model->fwd_layers || !model->bwd_layers || !model->intra_layers || !model->wf) {
    set_error("x, out, the three layer arrays and wf must not be NULL");
    return IM_ERR_INVALID;
  }
  if (!workspace || workspace_bytes < w.total) {
    set_error("gsit_model_fwd needs %zu workspace bytes, got %zu", w.total, workspace_bytes);
    return IM_ERR_WORKSPACE;
  }
  hipStream_t st = (hipStream_t)hip_stream;
  char* ws = (char*)workspace;
  const int bf = shape->dtype == IM_DTYPE_BF16;
  long T = 0;
  for (int i = 0; i < shape->n_seg; ++i) T += shape->seg_len[i];
  const long R = (long)shape->batch * T;
  const int d = shape->d_model;
  void* F = ws + w.f;
  void* Bk = ws + w.b;
  void* cat = ws + w.cat;
  void* z = ws + w.z;
  void* lws = ws + w.layer;
  const size_t lws_bytes = w.total - w.layer;

  // The two inter-modal encoders read the same V_m and are independent of each other: layer l of both runs in
  // shared launches when the shape allows (one read of x for the first layer's projections, twice the
  // workgroups per launch); otherwise, and from the first layer that is not served on, one encoder after the other.
  im_shape_t inter = *shape;
  inter.live_mask = model->mask_fwd;
  int l0 = 0;
  // The last pair of layers writes its two outputs as the column blocks of the concatenated matrix (row stride 2d):
  // no separate concatenation pass.
  bool concatenated = false;
  const size_t es = bf ? 2 : 4;
  for (; l0 < model->n_layers_inter; ++l0) {
    bool done = false;
    const bool last = l0 + 1 == model->n_layers_inter;
    void* y0 = last ? cat : F;
    void* y1 = last ? (void*)((char*)cat + (size_t)d * es) : Bk;
    if ((rc = gsit_layer_fwd_pair(&inter, model->mask_bwd, model->d_ff_inter, l0 ? F : x, l0 ? Bk : x, model->fwd_layers[l0],
                                  model->bwd_layers[l0], model->ln_eps, valid_len, key_pad, y0, y1, lws, lws_bytes, st, &done,
                                  last ? 2L * d : 0L)))
      return rc;
    if (!done) break;
    concatenated = last;
  }
  if (l0 < model->n_layers_inter) {
    if ((rc = run_encoder(&inter, model->d_ff_inter, model->fwd_layers + l0, model->n_layers_inter - l0, model->ln_eps,
                          l0 ? F : x, F, valid_len, key_pad, lws, lws_bytes, hip_stream))) return rc;
    inter.live_mask = model->mask_bwd;
    if ((rc = run_encoder(&inter, model->d_ff_inter, model->bwd_layers + l0, model->n_layers_inter - l0, model->ln_eps,
                          l0 ? Bk : x, Bk, valid_len, key_pad, lws, lws_bytes, hip_stream))) return rc;
  }
  const int blocks = (int)((R * 2 * d + 255) / 256 < 4096 ? (R * 2 * d + 255) / 256 : 4096);
  if (concatenated) {}
  else if (bf) hipLaunchKernelGGL(concat_features_kernel<uint16_t>, dim3(blocks), dim3(256), 0, st, (const uint16_t*)F, (const uint16_t*)Bk, (uint16_t*)cat, R, d);
  else hipLaunchKernelGGL(concat_features_kernel<float>, dim3(blocks), dim3(256), 0, st, (const float*)F, (const float*)Bk, (float*)cat, R, d);
  if ((rc = run_encoder(&intra, model->d_ff_intra, model->intra_layers, model->n_layers_intra, model->ln_eps, cat, cat,
                        valid_len, key_pad, lws, lws_bytes, hip_stream))) return rc;

  Geo g;
  memset(&g, 0, sizeof(g));
  g.n_seg = shape->n_seg;
  for (int i = 0; i < shape->n_seg; ++i) { g.seg_len[i] = shape->seg_len[i]; g.seg_off[i + 1] = g.seg_off[i] + shape->seg_len[i]; }
  const int wz = 2 * d, nz = shape->n_seg * wz;
  if ((long)shape->batch * model->n_out <= 16384) {
    // few outputs: one launch gathers the last positions and multiplies
    const unsigned hb = (unsigned)(((long)shape->batch * model->n_out + 3) / 4);
    if (bf) hipLaunchKernelGGL(head_dot_gather_kernel<uint16_t>, dim3(hb), dim3(256), 0, st, (const uint16_t*)cat, valid_len, (const uint16_t*)model->wf, (const uint16_t*)model->bf, (uint16_t*)out, shape->batch, model->n_out, (int)T, wz, shape->n_seg, g);
    else hipLaunchKernelGGL(head_dot_gather_kernel<float>, dim3(hb), dim3(256), 0, st, (const float*)cat, valid_len, (const float*)model->wf, (const float*)model->bf, (float*)out, shape->batch, model->n_out, (int)T, wz, shape->n_seg, g);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) { set_error("gsit_model_fwd launch: %s", hipGetErrorString(e)); return IM_ERR_HIP; }
    return IM_OK;
  }
  const int gblocks = (shape->batch * nz + 255) / 256;
  if (bf) hipLaunchKernelGGL(gather_last_kernel<uint16_t>, dim3(gblocks), dim3(256), 0, st, (const uint16_t*)cat, (uint16_t*)z, valid_len, shape->batch, (int)T, wz, shape->n_seg, g);
  else hipLaunchKernelGGL(gather_last_kernel<float>, dim3(gblocks), dim3(256), 0, st, (const float*)cat, (float*)z, valid_len, shape->batch, (int)T, wz, shape->n_seg, g);

  GemmDesc p;
  memset(&p, 0, sizeof(p));
  p.A = z; p.sam = nz; p.sak = 1;
  p.B[0] = model->wf; p.sbk = model->n_out; p.sbn = 1;
  p.bias[0] = model->bf;
  p.C[0] = out; p.ldc = model->n_out;
  p.M = shape->batch; p.N = model->n_out; p.K = nz;
  if ((rc = launch_gemm_alu(p, bf, bf, bf, st))) return rc;
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) { set_error("gsit_model_fwd launch: %s", hipGetErrorString(e)); return IM_ERR_HIP; }
  return IM_OK;
}

}  // extern "C"
