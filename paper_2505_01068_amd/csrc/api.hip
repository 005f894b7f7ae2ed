// C-ABI entry points: argument validation, the live-block schedule, workspace
// carving and kernel sequencing.  No device memory is allocated here and no call
// synchronises; everything is enqueued on the caller's stream.
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <initializer_list>
#include <mutex>

#include "common.hpp"
#include "mfma_path.hpp"

namespace imattn {

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
}

static int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

// ---- optional kernel-family timing ----
static const char* kProfNames[PF_COUNT] = {"proj_fwd", "attn_fwd", "attn_dq", "attn_dkv", "proj_bwd", "wgrad", "misc"};
constexpr int PROF_MAX = 8192;
static unsigned g_prof_mask = 0;  // bit f set: kernel family f is bracketed with events
static int g_prof_n = 0;
static hipEvent_t g_prof_ev[PROF_MAX][2];
static int g_prof_family[PROF_MAX];
static int g_prof_created = 0;

ProfScope::ProfScope(ProfFamily f, hipStream_t s) : slot(-1), st(s) {
  if (!((g_prof_mask >> f) & 1u) || g_prof_n >= PROF_MAX) return;
  if (g_prof_n >= g_prof_created) {
    if (hipEventCreate(&g_prof_ev[g_prof_n][0]) != hipSuccess || hipEventCreate(&g_prof_ev[g_prof_n][1]) != hipSuccess) return;
    g_prof_created = g_prof_n + 1;
  }
  slot = g_prof_n++;
  g_prof_family[slot] = f;
  (void)hipEventRecord(g_prof_ev[slot][0], st);
}
ProfScope::~ProfScope() {
  if (slot >= 0) (void)hipEventRecord(g_prof_ev[slot][1], st);
}

static int check_hip(const char* what) {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(IM_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
  return IM_OK;
}

static int validate_shape(const im_shape_t* s) {
  if (!s) return fail(IM_ERR_INVALID, "shape is NULL");
  if (s->batch < 1 || s->batch > 65535) return fail(IM_ERR_INVALID, "batch must be in 1..65535 (got %d)", s->batch);
  if (s->n_seg < 1 || s->n_seg > IM_MAX_SEG)
    return fail(IM_ERR_INVALID, "n_seg must be in 1..%d (got %d)", IM_MAX_SEG, s->n_seg);
  long T = 0;
  for (int i = 0; i < s->n_seg; ++i) {
    if (s->seg_len[i] < 1) return fail(IM_ERR_INVALID, "seg_len[%d] must be >= 1 (got %d)", i, s->seg_len[i]);
    T += s->seg_len[i];
  }
  if (T > (1 << 24)) return fail(IM_ERR_INVALID, "T_m = %ld too large", T);
  if (s->d_model < 1 || s->n_heads < 1 || s->d_model % s->n_heads != 0)
    return fail(IM_ERR_INVALID, "d_model (%d) must be a positive multiple of n_heads (%d)", s->d_model, s->n_heads);
  const int nb = s->n_seg * s->n_seg;
  if (nb < 64 && (s->live_mask >> nb) != 0)
    return fail(IM_ERR_INVALID, "live_mask has bits set at or above n_seg^2 = %d", nb);
  if (!(s->scale >= 0.f) || isinf(s->scale)) return fail(IM_ERR_INVALID, "scale must be finite and >= 0");
  if (s->dtype != IM_DTYPE_F32 && s->dtype != IM_DTYPE_BF16)
    return fail(IM_ERR_INVALID, "dtype must be IM_DTYPE_F32 or IM_DTYPE_BF16 (got %d)", s->dtype);
  if ((long)s->batch * T * s->d_model > (1l << 40)) return fail(IM_ERR_INVALID, "problem too large");
  if (s->cu_rows && (s->total_rows < 1 || s->total_rows > (long)s->batch * T))
    return fail(IM_ERR_INVALID, "packed rows: total_rows must be in 1..batch * T_m = %ld (got %ld)", (long)s->batch * T,
                (long)s->total_rows);
  return IM_OK;
}

// Which kernel family serves this shape.
enum Path { PATH_ROWLANE, PATH_MFMA, PATH_NONE };
static Path pick_path(const im_shape_t* s) {
  const int dh = s->d_model / s->n_heads;
  if (s->dtype == IM_DTYPE_BF16 && mfma_supports(s->d_model, dh)) {
    // the dK/dV kernel addresses one segment of one batch element with 32-bit byte offsets
    long max_seg = 0;
    for (int i = 0; i < s->n_seg; ++i) max_seg = s->seg_len[i] > max_seg ? s->seg_len[i] : max_seg;
    if (max_seg * 3L * s->d_model * 2L < (1L << 31) && 3L * s->d_model * 2L < (1L << 24)) return PATH_MFMA;
    return PATH_NONE;
  }
  if (rowlane_supports(dh)) return PATH_ROWLANE;
  return PATH_NONE;
}
static int check_supported(const im_shape_t* s) {
  if (pick_path(s) == PATH_NONE)
    return fail(IM_ERR_UNSUPPORTED,
                "no kernel for dtype %d with head dimension %d (supported: head dim <= 16 for fp32/bf16; bf16 with "
                "head dim 8, 16 or 64, d_model %% 64 == 0 and segment length * d_model < 2^28)",
                s->dtype, s->d_model / s->n_heads);
  return IM_OK;
}

// The matrix-core kernels read and write activations, weights and their scratch tensors in 16-byte
// units (vector loads, global->LDS copies): every such pointer must be 16-byte aligned.
static int check_align16(const im_shape_t* s, const char* what, std::initializer_list<const void*> ptrs) {
  if (pick_path(s) != PATH_MFMA) return IM_OK;
  for (const void* p : ptrs)
    if (((uintptr_t)p & 15) != 0)
      return fail(IM_ERR_INVALID, "%s: with bf16 and head dimension 8 / 16 / 64 every tensor pointer must be 16-byte aligned", what);
  return IM_OK;
}

// Sec. 6 "Decomposition": per query segment the set of live key segments, per key
// segment the set of query segments that read it, and the tile order (segments
// by decreasing live range, i.e. decreasing work per row).
void build_geo(const im_shape_t* s, int q_tile, int k_tile, Geo* g) {
  memset(g, 0, sizeof(*g));
  g->B = s->batch; g->H = s->n_heads; g->d = s->d_model; g->dh = s->d_model / s->n_heads; g->n_seg = s->n_seg;
  int off = 0;
  for (int i = 0; i < s->n_seg; ++i) { g->seg_off[i] = off; g->seg_len[i] = s->seg_len[i]; off += s->seg_len[i]; }
  g->seg_off[s->n_seg] = off;
  g->T = off;
  for (int i = 0; i < s->n_seg; ++i)
    for (int j = 0; j < s->n_seg; ++j)
      if ((s->live_mask >> (i * s->n_seg + j)) & 1ull) { g->q_live[i] |= 1u << j; g->k_live[j] |= 1u << i; }
  auto order = [&](const unsigned* live, int tile_rows, int* ord, int* prefix, int* nord) {
    long work[IM_MAX_SEG];
    int n = 0;
    for (int i = 0; i < s->n_seg; ++i) {
      if (!live[i]) continue;
      long w = 0;
      for (int j = 0; j < s->n_seg; ++j) if ((live[i] >> j) & 1u) w += s->seg_len[j];
      work[i] = w;
      ord[n++] = i;
    }
    std::stable_sort(ord, ord + n, [&](int a, int b) { return work[a] > work[b]; });
    prefix[0] = 0;
    for (int k = 0; k < n; ++k) prefix[k + 1] = prefix[k] + (s->seg_len[ord[k]] + tile_rows - 1) / tile_rows;
    *nord = n;
  };
  order(g->q_live, q_tile, g->q_order, g->q_tile_prefix, &g->q_nord);
  order(g->k_live, k_tile, g->k_order, g->k_tile_prefix, &g->k_nord);
  g->scale = s->scale;
  g->scale_log2e = s->scale * 1.44269504088896340736f;
  g->cu = s->cu_rows;
  g->R = shape_rows(s);
}

static inline size_t align256(size_t n) { return (n + 255) & ~(size_t)255; }

struct Bump {
  char* base; size_t off, cap;
  void* take(size_t n) { void* p = base ? base + off : nullptr; off += align256(n); return p; }
};

// Layout of the forward's saved tensors (also used from workspace when saved == NULL).
struct SavedLayout {
  size_t qkv, o, lse, extra, total;  // byte offsets; `extra` = transposed copies of the MFMA path
};
static SavedLayout saved_layout(const im_shape_t* s) {
  const size_t es = s->dtype == IM_DTYPE_BF16 ? 2 : 4;
  const size_t R = (size_t)shape_rows(s), d = s->d_model;
  SavedLayout L;
  size_t off = 0;
  L.qkv = off; off += align256(R * 3 * d * es);
  L.o = off; off += align256(R * d * es);
  L.lse = off; off += align256((size_t)s->n_heads * R * sizeof(float));
  L.extra = off;
  if (pick_path(s) == PATH_MFMA) off += align256(mfma_saved_extra_bytes(s));
  L.total = off;
  return L;
}

static size_t bwd_workspace_bytes(const im_shape_t* s) {
  const size_t es = s->dtype == IM_DTYPE_BF16 ? 2 : 4;
  const size_t R = (size_t)shape_rows(s), d = s->d_model;
  if (pick_path(s) == PATH_MFMA) return mfma_bwd_workspace_bytes(s);
  size_t n = 0;
  n += align256(R * d * es);                                          // dO
  n += align256(R * 3 * d * es);                                      // dQ | dK | dV
  n += align256((size_t)s->n_heads * R * sizeof(float));   // delta
  size_t pb = std::max(gemm_alu_partial_bytes((int)d, (int)(3 * d), (int)R, nullptr),
                       gemm_alu_partial_bytes((int)d, (int)d, (int)R, nullptr));
  if (mfma_linear_ok(s->dtype == IM_DTYPE_BF16, d, d))
    pb = std::max(pb, std::max(mfma_wgrad_partial_bytes((int)d, (int)(3 * d), (int)R), mfma_wgrad_partial_bytes((int)d, (int)d, (int)R)));
  if (wgrad_small_ok((int)d, (int)(3 * d), (int)d)) pb = std::max(pb, wgrad_small_partial_bytes((int)d, (int)(3 * d), (int)R));
  if (wgrad_mfma_ok((int)d, (int)(3 * d), (int)R, 0))
    pb = std::max(pb, wgrad_mfma_partial_bytes((int)d, (int)(3 * d), (int)R) + wgrad_mfma_partial_bytes((int)d, (int)d, (int)R));
  n += align256(pb);
  n += align256(4 * colsum_partial_bytes((int)R, (int)d));            // dbo, dbq, dbk, dbv in one launch
  n += align256(3 * d * d * sizeof(float));                           // sinks for unwanted weight gradients
  return n;
}

static hipStream_t as_stream(void* p) { return (hipStream_t)p; }

// ---- scratch memory of the allocation-free entry point ----
// One file-scope device array per GPU the library is loaded on (held until the process ends).  In host
// code the array's NAME is only a stand-in for the symbol: the device address is looked up once per
// device with hipGetSymbolAddress and that pointer is what kernels and copies receive.
static __device__ __align__(256) unsigned char scratch[IM_NOALLOC_MAX_BYTES];
constexpr int kMaxDevices = 64;
static void* g_scratch_ptr[kMaxDevices];
static std::mutex g_scratch_mu;

static int scratch_of_current_device(char** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return fail(IM_ERR_HIP, "hipGetDevice: %s", hipGetErrorString(e));
  if (dev < 0 || dev >= kMaxDevices) return fail(IM_ERR_UNSUPPORTED, "device index %d outside 0..%d", dev, kMaxDevices - 1);
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) return fail(IM_ERR_HIP, "hipGetSymbolAddress(scratch) on device %d: %s", dev, hipGetErrorString(e));
    g_scratch_ptr[dev] = p;
  }
  *out = (char*)g_scratch_ptr[dev];
  return IM_OK;
}

// ---------------------------------------------------------------------------------------------
// forward on the ALU path; `res` (same layout as y) is added to y when not NULL.
static int fwd_rowlane(const im_shape_t* s, const void* x, const void* wq, const void* wk, const void* wv,
                       const void* wo, const void* bq, const void* bk, const void* bv, const void* bo,
                       const int32_t* valid_len, const uint8_t* key_pad, void* y, const void* res, char* sv,
                       hipStream_t st) {
  const int bf = s->dtype == IM_DTYPE_BF16;
  const size_t es = bf ? 2 : 4;
  Geo g;
  build_geo(s, 64, 64, &g);
  const SavedLayout L = saved_layout(s);
  const long R = g.R, d = g.d;
  char* qkv = sv + L.qkv;
  void* o = sv + L.o;
  float* lse2 = (float*)(sv + L.lse);

  GemmDesc p;
  memset(&p, 0, sizeof(p));
  p.A = x; p.sam = d; p.sak = 1;
  p.B[0] = wq; p.B[1] = wk; p.B[2] = wv; p.sbk = d; p.sbn = 1; p.b_split = 1; p.n_per = (int)d;
  p.bias[0] = bq; p.bias[1] = bk; p.bias[2] = bv; p.bias_split = 1;
  p.C[0] = qkv; p.ldc = 3 * d; p.M = (int)R; p.N = (int)(3 * d); p.K = (int)d;
  int rc = IM_OK;
  // bf16 projections go to the matrix cores whenever the widths allow 16-byte chunks
  const bool mm = mfma_linear_ok(bf, d, d);
  { ProfScope ps(PF_PROJ_FWD, st);
    if (mm) mfma_linear(x, d, wq, wk, wv, d, (int)d, bq, bk, bv, 0, nullptr, qkv, 3 * d, (int)R, (int)(3 * d), (int)d, st);
    else rc = launch_gemm_alu(p, bf, bf, bf, st); }
  if (rc) return rc;

  { ProfScope ps(PF_ATTN_FWD, st);
  rc = launch_rowlane_fwd(g, bf, qkv, qkv + d * es, qkv + 2 * d * es, 3 * d, valid_len, key_pad, o, d, lse2, st); }
  if (rc) return rc;

  ProfScope ps2(PF_PROJ_FWD, st);
  memset(&p, 0, sizeof(p));
  p.A = o; p.sam = d; p.sak = 1;
  p.B[0] = wo; p.sbk = d; p.sbn = 1;
  p.bias[0] = bo; p.C[0] = y; p.ldc = d; p.res = res; p.M = (int)R; p.N = (int)d; p.K = (int)d;
  if (mm) mfma_linear(o, d, wo, nullptr, nullptr, d, (int)d, bo, nullptr, nullptr, 0, res, y, d, (int)R, (int)d, (int)d, st);
  else rc = launch_gemm_alu(p, bf, bf, bf, st);
  if (rc) return rc;
  return check_hip("im_attention_fwd launch");
}

static int bwd_rowlane(const im_shape_t* s, const void* x, const void* wq, const void* wk, const void* wv,
                       const void* wo, const int32_t* valid_len, const uint8_t* key_pad, const char* sv,
                       const void* dy, void* dx, void* dwq, void* dwk, void* dwv, void* dwo, void* dbq, void* dbk,
                       void* dbv, void* dbo, char* ws, hipStream_t st) {
  const int bf = s->dtype == IM_DTYPE_BF16;
  const size_t es = bf ? 2 : 4;
  Geo g;
  build_geo(s, 64, 64, &g);
  const SavedLayout L = saved_layout(s);
  const long R = g.R, d = g.d;
  const char* qkv = sv + L.qkv;
  const void* o = sv + L.o;
  const float* lse2 = (const float*)(sv + L.lse);

  Bump b{ws, 0, 0};
  char* d_o = (char*)b.take(R * d * es);
  char* dqkv = (char*)b.take(R * 3 * d * es);
  float* delta = (float*)b.take((size_t)g.H * R * sizeof(float));
  int split = 1;
  size_t pbytes = std::max(gemm_alu_partial_bytes((int)d, (int)(3 * d), (int)R, &split),
                           gemm_alu_partial_bytes((int)d, (int)d, (int)R, nullptr));
  // bf16 GEMMs go to the matrix cores whenever the widths allow 16-byte chunks
  const bool mm = mfma_linear_ok(bf, d, d);
  if (mm) pbytes = std::max(pbytes, std::max(mfma_wgrad_partial_bytes((int)d, (int)(3 * d), (int)R), mfma_wgrad_partial_bytes((int)d, (int)d, (int)R)));
  // narrow models (d <= 64) off the matrix cores: the dedicated tall-skinny weight-gradient kernel
  const bool ws_small = !mm && wgrad_small_ok((int)d, (int)(3 * d), (int)d);
  if (ws_small) pbytes = std::max(pbytes, wgrad_small_partial_bytes((int)d, (int)(3 * d), (int)R));
  // ... and tall fp32 inputs on the fp32 matrix instruction
  const bool ws_mfma = !mm && wgrad_mfma_ok((int)d, (int)(3 * d), (int)R, bf);
  if (ws_mfma) pbytes = std::max(pbytes, wgrad_mfma_partial_bytes((int)d, (int)(3 * d), (int)R) + wgrad_mfma_partial_bytes((int)d, (int)d, (int)R));
  float* partial = (float*)b.take(pbytes);
  float* cpart = (float*)b.take(4 * colsum_partial_bytes((int)R, (int)d));
  float* sink = (float*)b.take(3 * d * d * sizeof(float));

  GemmDesc p;
  int rc;
  // dO = dy Wo^T
  memset(&p, 0, sizeof(p));
  p.A = dy; p.sam = d; p.sak = 1;
  p.B[0] = wo; p.sbk = 1; p.sbn = d;
  p.C[0] = d_o; p.ldc = d; p.M = (int)R; p.N = (int)d; p.K = (int)d;
  { ProfScope ps(PF_PROJ_BWD, st);
    if (mm) mfma_dgrad(dy, d, wo, nullptr, nullptr, d, 0, d_o, d, (int)R, (int)d, (int)d, st);
    else if ((rc = launch_gemm_alu(p, bf, bf, bf, st))) return rc; }
  // dWo = O^T dy
  if (dwo && mm) {
    ProfScope ps(PF_WGRAD, st);
    mfma_wgrad(o, d, dy, d, (float*)dwo, nullptr, nullptr, 0, (int)d, (int)d, (int)R, partial, st);
  } else if (dwo && ws_mfma) {
    // with dWq | dWk | dWv below when those are wanted too (one pair of launches for both), else alone
    if (!(dwq || dwk || dwv)) {
      ProfScope ps(PF_WGRAD, st);
      launch_wgrad_mfma_f32((const float*)o, d, (const float*)dy, d, (int)R, (int)d, (int)d, partial, (float*)dwo, nullptr,
                            nullptr, 0, st);
    }
  } else if (dwo && ws_small) {
    ProfScope ps(PF_WGRAD, st);
    const int nb = launch_wgrad_small(o, d, dy, d, (int)R, (int)d, (int)d, bf, partial, st);
    launch_wgrad_small_reduce(partial, nb, (int)d, (int)d, (float*)dwo, nullptr, nullptr, 0, st);
  } else if (dwo) {
    memset(&p, 0, sizeof(p));
    p.A = o; p.sam = 1; p.sak = d;
    p.B[0] = dy; p.sbk = d; p.sbn = 1;
    p.C[0] = dwo; p.ldc = d; p.M = (int)d; p.N = (int)d; p.K = (int)R;
    gemm_alu_partial_bytes((int)d, (int)d, (int)R, &p.split_k);
    p.partial = partial;
    ProfScope ps(PF_WGRAD, st);
    if ((rc = launch_gemm_alu(p, bf, bf, 0, st))) return rc;
  }
  rc = launch_rowlane_bwd(g, bf, qkv, qkv + d * es, qkv + 2 * d * es, 3 * d, o, d_o, d, lse2, valid_len, key_pad,
                          delta, dqkv, dqkv + d * es, dqkv + 2 * d * es, 3 * d, st);
  if (rc) return rc;

  // dWq | dWk | dWv = x^T [dQ | dK | dV]
  if ((dwq || dwk || dwv) && mm) {
    ProfScope ps(PF_WGRAD, st);
    mfma_wgrad(x, d, dqkv, 3 * d, (float*)dwq, (float*)dwk, (float*)dwv, (int)d, (int)d, (int)(3 * d), (int)R, partial, st);
  } else if ((dwq || dwk || dwv) && ws_mfma) {
    ProfScope ps(PF_WGRAD, st);
    if (dwo) launch_wgrad_mfma_f32_attn((const float*)x, (const float*)dqkv, (const float*)o, (const float*)dy, (int)R, (int)d,
                                        partial, (float*)dwq, (float*)dwk, (float*)dwv, (float*)dwo, st);
    else launch_wgrad_mfma_f32((const float*)x, d, (const float*)dqkv, 3 * d, (int)R, (int)d, (int)(3 * d), partial,
                               (float*)dwq, (float*)dwk, (float*)dwv, (int)d, st);
  } else if ((dwq || dwk || dwv) && ws_small) {
    ProfScope ps(PF_WGRAD, st);
    const int nb = launch_wgrad_small(x, d, dqkv, 3 * d, (int)R, (int)d, (int)(3 * d), bf, partial, st);
    launch_wgrad_small_reduce(partial, nb, (int)d, (int)(3 * d), (float*)dwq, (float*)dwk, (float*)dwv, (int)d, st);
  } else if (dwq || dwk || dwv) {
    memset(&p, 0, sizeof(p));
    p.A = x; p.sam = 1; p.sak = d;
    p.B[0] = dqkv; p.sbk = 3 * d; p.sbn = 1;
    p.C[0] = dwq ? dwq : sink; p.C[1] = dwk ? dwk : sink + d * d; p.C[2] = dwv ? dwv : sink + 2 * d * d;
    p.c_split = 1; p.n_per = (int)d; p.ldc = d; p.M = (int)d; p.N = (int)(3 * d); p.K = (int)R;
    p.split_k = split; p.partial = partial;
    ProfScope ps(PF_WGRAD, st);
    if ((rc = launch_gemm_alu(p, bf, bf, 0, st))) return rc;
  }
  if (dbo || dbq || dbk || dbv) {  // column sums of dy and of the dQ | dK | dV column blocks, one pair of launches
    const void* src[4] = {dy, dqkv, dqkv + d * es, dqkv + 2 * d * es};
    const long lds4[4] = {d, 3 * d, 3 * d, 3 * d};
    float* dbs[4] = {(float*)dbo, (float*)dbq, (float*)dbk, (float*)dbv};
    ProfScope ps(PF_WGRAD, st);
    if ((rc = launch_colsum_multi(src, lds4, dbs, 4, (int)R, (int)d, bf, cpart, st))) return rc;
  }
  // dx = dQ Wq^T + dK Wk^T + dV Wv^T
  if (dx && mm && d % 64 == 0) {  // the contraction is split over three weights: whole 64-deep k-tiles per weight
    ProfScope ps(PF_PROJ_BWD, st);
    mfma_dgrad(dqkv, 3 * d, wq, wk, wv, d, (int)d, dx, d, (int)R, (int)d, (int)(3 * d), st);
  } else if (dx) {
    memset(&p, 0, sizeof(p));
    p.A = dqkv; p.sam = 3 * d; p.sak = 1;
    p.B[0] = wq; p.B[1] = wk; p.B[2] = wv; p.sbk = 1; p.sbn = d; p.b_split = 2; p.k_per = (int)d;
    p.C[0] = dx; p.ldc = d; p.M = (int)R; p.N = (int)d; p.K = (int)(3 * d);
    ProfScope ps(PF_PROJ_BWD, st);
    if ((rc = launch_gemm_alu(p, bf, bf, bf, st))) return rc;
  }
  return check_hip("im_attention_bwd launch");
}

}  // namespace imattn

using namespace imattn;

extern "C" {

const char* im_last_error(void) { return g_err; }

int im_profile_enable(int on) {
  g_prof_mask = on == 1 ? ~0u : on > 1 ? (unsigned)on >> 1 : 0u;
  if (on) g_prof_n = 0;
  return IM_OK;
}

int im_profile_get(int idx, const char** name, double* total_ms, int64_t* launches) {
  if (idx < 0 || idx >= PF_COUNT) return PF_COUNT;
  double ms = 0.0;
  int64_t n = 0;
  for (int i = 0; i < g_prof_n; ++i) {
    if (g_prof_family[i] != idx) continue;
    float t = 0.f;
    if (hipEventSynchronize(g_prof_ev[i][1]) == hipSuccess &&
        hipEventElapsedTime(&t, g_prof_ev[i][0], g_prof_ev[i][1]) == hipSuccess) { ms += t; ++n; }
  }
  if (name) *name = kProfNames[idx];
  if (total_ms) *total_ms = ms;
  if (launches) *launches = n;
  return PF_COUNT;
}
const char* im_version(void) { return "imattn 0.1 gfx950"; }

int im_schedule_build(const im_shape_t* shape, int32_t tile_rows, im_work_item_t* items, int32_t max_items,
                      int32_t* n_items, int64_t* n_pairs) {
  int rc = validate_shape(shape);
  if (rc) return rc;
  if (tile_rows < 1) return fail(IM_ERR_INVALID, "tile_rows must be >= 1");
  Geo g;
  build_geo(shape, tile_rows, tile_rows, &g);
  const int n = g.q_tile_prefix[g.q_nord];
  int64_t pairs = 0;
  if (items && max_items < n) return fail(IM_ERR_INVALID, "max_items (%d) < number of work items (%d)", max_items, n);
  for (int t = 0; t < n; ++t) {
    int seg, start;
    decode_tile(g.q_order, g.q_tile_prefix, g.q_nord, tile_rows, t, seg, start);
    im_work_item_t it;
    memset(&it, 0, sizeof(it));
    it.q_seg = seg; it.q_start = start; it.q_rows = std::min(tile_rows, g.seg_len[seg] - start);
    long klen = 0;
    for (int j = 0; j < g.n_seg; ++j)
      if ((g.q_live[seg] >> j) & 1u) { it.key_seg[it.n_key_seg++] = j; klen += g.seg_len[j]; }
    it.pairs = (int64_t)it.q_rows * klen;
    pairs += it.pairs;
    if (items) items[t] = it;
  }
  if (n_items) *n_items = n;
  if (n_pairs) *n_pairs = pairs;
  return IM_OK;
}

int im_attention_sizes(const im_shape_t* shape, size_t* saved_bytes, size_t* workspace_bytes) {
  int rc = validate_shape(shape);
  if (rc) return rc;
  if ((rc = check_supported(shape))) return rc;
  const SavedLayout L = saved_layout(shape);
  if (saved_bytes) *saved_bytes = L.total;
  if (workspace_bytes) {
    size_t fwd = L.total;  // inference keeps Q, K, V, O, LSE in the workspace
    if (pick_path(shape) == PATH_MFMA) fwd += mfma_fwd_workspace_bytes(shape->d_model);
    *workspace_bytes = std::max(fwd, bwd_workspace_bytes(shape));
  }
  return IM_OK;
}

int im_attention_fwd(const im_shape_t* shape, const void* x, const void* wq, const void* wk, const void* wv,
                     const void* wo, const void* bq, const void* bk, const void* bv, const void* bo,
                     const int32_t* valid_len, const uint8_t* key_pad, void* y, void* saved, void* workspace,
                     size_t workspace_bytes, void* hip_stream) {
  int rc = validate_shape(shape);
  if (rc) return rc;
  if ((rc = check_supported(shape))) return rc;
  if (shape->cu_rows && valid_len) return fail(IM_ERR_INVALID, "packed rows carry the lengths in cu_rows: valid_len must be NULL");
  if (!x || !wq || !wk || !wv || !wo || !y) return fail(IM_ERR_INVALID, "x, wq, wk, wv, wo and y must not be NULL");
  if ((rc = check_align16(shape, "im_attention_fwd", {x, wq, wk, wv, wo, y, saved, workspace}))) return rc;
  const SavedLayout L = saved_layout(shape);
  const Path path = pick_path(shape);
  size_t need = saved ? 0 : L.total;
  if (path == PATH_MFMA) need += mfma_fwd_workspace_bytes(shape->d_model);
  if (need > 0 && (!workspace || workspace_bytes < need))
    return fail(IM_ERR_WORKSPACE, "im_attention_fwd needs %zu workspace bytes, got %zu", need, workspace_bytes);
  char* sv = saved ? (char*)saved : (char*)workspace;
  char* ws = saved ? (char*)workspace : (char*)workspace + L.total;
  if (path == PATH_MFMA)
    return mfma_attention_fwd(shape, x, wq, wk, wv, wo, bq, bk, bv, bo, valid_len, key_pad, y, nullptr, sv, L.qkv,
                              L.o, L.lse, L.extra, ws, as_stream(hip_stream));
  return fwd_rowlane(shape, x, wq, wk, wv, wo, bq, bk, bv, bo, valid_len, key_pad, y, nullptr, sv,
                     as_stream(hip_stream));
}

int im_attention_bwd(const im_shape_t* shape, const void* x, const void* wq, const void* wk, const void* wv,
                     const void* wo, const int32_t* valid_len, const uint8_t* key_pad, const void* saved,
                     const void* dy, void* dx, void* dwq, void* dwk, void* dwv, void* dwo, void* dbq, void* dbk,
                     void* dbv, void* dbo, void* workspace, size_t workspace_bytes, void* hip_stream) {
  int rc = validate_shape(shape);
  if (rc) return rc;
  if ((rc = check_supported(shape))) return rc;
  if (shape->cu_rows && valid_len) return fail(IM_ERR_INVALID, "packed rows carry the lengths in cu_rows: valid_len must be NULL");
  if (!x || !wq || !wk || !wv || !wo || !saved || !dy)
    return fail(IM_ERR_INVALID, "x, wq, wk, wv, wo, saved and dy must not be NULL");
  if ((rc = check_align16(shape, "im_attention_bwd", {x, wq, wk, wv, wo, saved, dy, dx, workspace}))) return rc;
  const size_t need = bwd_workspace_bytes(shape);
  if (!workspace || workspace_bytes < need)
    return fail(IM_ERR_WORKSPACE, "im_attention_bwd needs %zu workspace bytes, got %zu", need, workspace_bytes);
  const SavedLayout L = saved_layout(shape);
  if (pick_path(shape) == PATH_MFMA) {
    ReduceList later;   // at small widths the second-stage sums of the gradients run as one launch at the end
    later.n = 0;
    if ((rc = mfma_attention_bwd(shape, x, wq, wk, wv, wo, valid_len, key_pad, (const char*)saved, L.qkv, L.o, L.lse,
                                 L.extra, dy, dx, dwq, dwk, dwv, dwo, dbq, dbk, dbv, dbo, (char*)workspace,
                                 as_stream(hip_stream), &later)))
      return rc;
    launch_reduce_list(later, as_stream(hip_stream));
    return check_hip("im_attention_bwd launch");
  }
  return bwd_rowlane(shape, x, wq, wk, wv, wo, valid_len, key_pad, (const char*)saved, dy, dx, dwq, dwk, dwv, dwo, dbq,
                     dbk, dbv, dbo, (char*)workspace, as_stream(hip_stream));
}

int im_noalloc_init(void) {
  char* p = nullptr;
  return scratch_of_current_device(&p);
}

int im_attention_fwd_noalloc(const im_shape_t* shape, const void* x, const void* wq, const void* wk, const void* wv,
                             const void* wo, const void* bq, const void* bk, const void* bv, const void* bo,
                             const int32_t* valid_len, const uint8_t* key_pad, void* y, void* hip_stream) {
  int rc = validate_shape(shape);
  if (rc) return rc;
  if ((rc = check_supported(shape))) return rc;
  if (shape->cu_rows && valid_len) return fail(IM_ERR_INVALID, "packed rows carry the lengths in cu_rows: valid_len must be NULL");
  if (!x || !wq || !wk || !wv || !wo || !y) return fail(IM_ERR_INVALID, "x, wq, wk, wv, wo and y must not be NULL");
  if ((rc = check_align16(shape, "im_attention_fwd_noalloc", {x, wq, wk, wv, wo, y}))) return rc;
  const SavedLayout L = saved_layout(shape);
  const Path path = pick_path(shape);
  size_t need = L.total;
  if (path == PATH_MFMA) need += mfma_fwd_workspace_bytes(shape->d_model);
  if (need > (size_t)IM_NOALLOC_MAX_BYTES)
    return fail(IM_ERR_WORKSPACE,
                "im_attention_fwd_noalloc: this shape needs %zu bytes of scratch, the built-in buffer holds %zu "
                "(IM_NOALLOC_MAX_BYTES); use im_attention_fwd with a caller workspace",
                need, (size_t)IM_NOALLOC_MAX_BYTES);
  char* sv = nullptr;
  if ((rc = scratch_of_current_device(&sv))) return rc;
  // Q|K|V, O and the row statistics are all written before they are read (query segments without a live
  // block are zero-filled by a kernel), so nothing left in the buffer by an earlier call matters.
  if (path == PATH_MFMA)
    return mfma_attention_fwd(shape, x, wq, wk, wv, wo, bq, bk, bv, bo, valid_len, key_pad, y, nullptr, sv, L.qkv,
                              L.o, L.lse, L.extra, sv + L.total, as_stream(hip_stream));
  return fwd_rowlane(shape, x, wq, wk, wv, wo, bq, bk, bv, bo, valid_len, key_pad, y, nullptr, sv,
                     as_stream(hip_stream));
}

static int layer_check(const im_shape_t* shape, int32_t d_ff) {
  int rc = validate_shape(shape);
  if (rc) return rc;
  if ((rc = check_supported(shape))) return rc;
  if (d_ff < 1) return fail(IM_ERR_INVALID, "d_ff must be >= 1 (got %d)", d_ff);
  return IM_OK;
}

static size_t layer_ws(const im_shape_t* s, int32_t d_ff, size_t* attn_ws_bytes) {
  const size_t es = s->dtype == IM_DTYPE_BF16 ? 2 : 4;
  const size_t R = (size_t)shape_rows(s), d = s->d_model;
  size_t aws = saved_layout(s).total;
  if (pick_path(s) == PATH_MFMA) aws += mfma_fwd_workspace_bytes(s->d_model);
  if (attn_ws_bytes) *attn_ws_bytes = aws;
  return align256(R * d * es) /* LN out */ + align256(R * d * es) /* h */ + align256(R * (size_t)d_ff * es) + align256(aws);
}

int gsit_layer_sizes(const im_shape_t* shape, int32_t d_ff, size_t* workspace_bytes) {
  int rc = layer_check(shape, d_ff);
  if (rc) return rc;
  if (workspace_bytes) *workspace_bytes = layer_ws(shape, d_ff, nullptr);
  return IM_OK;
}

int gsit_layer_fwd(const im_shape_t* shape, int32_t d_ff, const void* x, const void* ln1_g, const void* ln1_b,
                   const void* wq, const void* wk, const void* wv, const void* wo, const void* bq, const void* bk,
                   const void* bv, const void* bo, const void* ln2_g, const void* ln2_b, const void* w1,
                   const void* b1, const void* w2, const void* b2, float ln_eps, const int32_t* valid_len,
                   const uint8_t* key_pad, void* y, void* workspace, size_t workspace_bytes, void* hip_stream) {
  int rc = layer_check(shape, d_ff);
  if (rc) return rc;
  if (shape->cu_rows && valid_len) return fail(IM_ERR_INVALID, "packed rows carry the lengths in cu_rows: valid_len must be NULL");
  if (!x || !ln1_g || !ln1_b || !wq || !wk || !wv || !wo || !ln2_g || !ln2_b || !w1 || !w2 || !y)
    return fail(IM_ERR_INVALID, "x, LayerNorm parameters, wq, wk, wv, wo, w1, w2 and y must not be NULL");
  if (!(ln_eps >= 0.f)) return fail(IM_ERR_INVALID, "ln_eps must be >= 0");
  if ((rc = check_align16(shape, "gsit_layer_fwd", {x, wq, wk, wv, wo, w1, w2, y, workspace}))) return rc;
  size_t aws = 0;
  const size_t need = layer_ws(shape, d_ff, &aws);
  if (!workspace || workspace_bytes < need)
    return fail(IM_ERR_WORKSPACE, "gsit_layer_fwd needs %zu workspace bytes, got %zu", need, workspace_bytes);
  hipStream_t st = as_stream(hip_stream);
  const int bf = shape->dtype == IM_DTYPE_BF16;
  const size_t es = bf ? 2 : 4;
  const long R = shape_rows(shape), d = shape->d_model;
  Bump b{(char*)workspace, 0, 0};
  void* u = b.take(R * d * es);
  void* h = b.take(R * d * es);
  void* z = b.take(R * (size_t)d_ff * es);
  char* aw = (char*)b.take(aws);

  // At d = 64 a GEMM tile row is the whole feature row: both LayerNorms then run inside the GEMM that consumes
  // them (the QKV projection, the first MLP GEMM) and u is never written.  The QKV projection of a width-128
  // model normalises its rows too.
  const bool mfma = pick_path(shape) == PATH_MFMA;
  auto al16 = [](const void* a, const void* b2) { return (((uintptr_t)a | (uintptr_t)b2) & 15) == 0; };
  const bool ln1_fused = mfma && mfma_qkv_fuses_ln(bf, d) && al16(ln1_g, ln1_b);
  const bool mlp_mfma = mfma_linear_ok(bf, d, d_ff) && mfma_linear_ok(bf, d_ff, d);
  const bool ln2_fused = mlp_mfma && mfma_gemm_fuses_ln(bf, d, d_ff) && al16(ln2_g, ln2_b);
  if (!ln1_fused && (rc = launch_layernorm(x, ln1_g, ln1_b, u, (int)R, (int)d, ln_eps, bf, st))) return rc;
  // h = x + IMAttention(u)
  const SavedLayout L = saved_layout(shape);
  // At d = 64 / 128 on the matrix-core path the rest of the layer after the attention kernel -- output projection,
  // residual, LayerNorm, MLP, residual -- is row-local and runs as ONE kernel on the attention's O rows.
  const bool tail_fused = mfma && mlp_tail_ok(bf, d, d_ff, x, ln2_g, ln2_b, w1, w2, y) && (((uintptr_t)wo | (uintptr_t)aw) & 15) == 0;
  if (mfma)
    rc = mfma_attention_fwd(shape, ln1_fused ? x : u, wq, wk, wv, wo, bq, bk, bv, bo, valid_len, key_pad,
                            tail_fused ? nullptr : h, x, aw, L.qkv, L.o, L.lse, L.extra, aw + L.total, st,
                            ln1_fused ? LnArgs{ln1_g, ln1_b, ln_eps} : LnArgs{nullptr, nullptr, 0.f});
  else
    rc = fwd_rowlane(shape, u, wq, wk, wv, wo, bq, bk, bv, bo, valid_len, key_pad, h, x, aw, st);
  if (rc) return rc;
  if (tail_fused) {
    ProfScope ps(PF_MISC, st);
    launch_mlp_tail(x, ln2_g, ln2_b, ln_eps, w1, b1, w2, b2, y, (int)R, (int)d, d_ff, st, aw + L.o, wo, bo);
    return check_hip("gsit_layer_fwd launch");
  }
  if (mlp_tail_ok(bf, d, d_ff, h, ln2_g, ln2_b, w1, w2, y)) {   // the whole MLP sub-block in one kernel
    ProfScope ps(PF_MISC, st);
    launch_mlp_tail(h, ln2_g, ln2_b, ln_eps, w1, b1, w2, b2, y, (int)R, (int)d, d_ff, st);
    return check_hip("gsit_layer_fwd launch");
  }
  if (!ln2_fused && (rc = launch_layernorm(h, ln2_g, ln2_b, u, (int)R, (int)d, ln_eps, bf, st))) return rc;
  // z = GELU(u W1 + b1);  y = h + z W2 + b2
  if (mlp_mfma) {
    ProfScope ps(PF_MISC, st);
    mfma_linear(ln2_fused ? h : u, d, w1, nullptr, nullptr, d_ff, d_ff, b1, nullptr, nullptr, 1, nullptr, z, d_ff, (int)R,
                d_ff, (int)d, st, ln2_fused ? LnArgs{ln2_g, ln2_b, ln_eps} : LnArgs{nullptr, nullptr, 0.f});
    mfma_linear(z, d_ff, w2, nullptr, nullptr, d, (int)d, b2, nullptr, nullptr, 0, h, y, d, (int)R, (int)d, d_ff, st);
    return check_hip("gsit_layer_fwd launch");
  }
  GemmDesc p;
  memset(&p, 0, sizeof(p));
  p.A = u; p.sam = d; p.sak = 1; p.B[0] = w1; p.sbk = d_ff; p.sbn = 1; p.bias[0] = b1;
  p.C[0] = z; p.ldc = d_ff; p.M = (int)R; p.N = d_ff; p.K = (int)d; p.gelu = 1;
  if ((rc = launch_gemm_alu(p, bf, bf, bf, st))) return rc;
  memset(&p, 0, sizeof(p));
  p.A = z; p.sam = d_ff; p.sak = 1; p.B[0] = w2; p.sbk = d; p.sbn = 1; p.bias[0] = b2;
  p.C[0] = y; p.ldc = d; p.res = h; p.M = (int)R; p.N = (int)d; p.K = d_ff;
  if ((rc = launch_gemm_alu(p, bf, bf, bf, st))) return rc;
  return check_hip("gsit_layer_fwd launch");
}


}  // extern "C"

namespace imattn {

// Workspace of gsit_layer_fwd_pair; 0 when the shape is not one the paired kernels serve.
size_t gsit_layer_pair_ws(const im_shape_t* s) {
  if (s->cu_rows || 2L * s->batch > 65535 || pick_path(s) != PATH_MFMA || s->d_model / s->n_heads == 64) return 0;
  im_shape_t s2 = *s;
  s2.batch = 2 * s->batch;
  return align256(saved_layout(&s2).total);
}

// One layer of each of two encoders that run side by side on inputs of the same shape (the forward- and the
// backward-IFM encoder over the same V_m, Sec. 5 Eq. "allmodalinone fusion"): y0 = layer(x0; p0, mask of s0),
// y1 = layer(x1; p1, mask1), in three launches (both QKV projections with their LayerNorms, both attention
// kernels, both fused tails) instead of six, so that each launch fills the chip.  *done = false with nothing
// enqueued when the shape or the parameters are not served (the caller then runs the layers one by one).
// ldy: row stride of y0 and y1 in elements (0 = d_model; wider: the outputs are column blocks of one matrix).
int gsit_layer_fwd_pair(const im_shape_t* s0, uint64_t mask1, int32_t d_ff, const void* x0, const void* x1,
                        const gsit_layer_params_t& p0, const gsit_layer_params_t& p1, float ln_eps,
                        const int32_t* valid_len, const uint8_t* key_pad, void* y0, void* y1, void* workspace,
                        size_t workspace_bytes, hipStream_t st, bool* done, long ldy) {
  *done = false;
  const size_t need = gsit_layer_pair_ws(s0);
  if (!need || !workspace || workspace_bytes < need) return IM_OK;
  const int bf = s0->dtype == IM_DTYPE_BF16;
  const long R = shape_rows(s0), d = s0->d_model;
  auto al16 = [](std::initializer_list<const void*> ps) {
    uintptr_t a = 0;
    for (const void* q : ps) a |= (uintptr_t)q;
    return (a & 15) == 0;
  };
  auto side_ok = [&](const gsit_layer_params_t& p, const void* x, const void* y) {
    return p.ln1_g && p.ln1_b && p.wq && p.wk && p.wv && p.wo && p.ln2_g && p.ln2_b && p.w1 && p.w2 &&
           mfma_gemm_fuses_ln(bf, d, 3 * d) && mlp_tail_ok(bf, d, d_ff, x, p.ln2_g, p.ln2_b, p.w1, p.w2, y) &&
           al16({p.ln1_g, p.ln1_b, p.wq, p.wk, p.wv, p.wo, x, y, workspace});
  };
  if (!side_ok(p0, x0, y0) || !side_ok(p1, x1, y1)) return IM_OK;
  im_shape_t s2 = *s0;
  s2.batch = 2 * s0->batch;
  const SavedLayout L = saved_layout(&s2);
  char* sv = (char*)workspace;
  if (!mfma_attention_fwd_pair(s0, mask1, x0, x1, p0, p1, LnArgs{p0.ln1_g, p0.ln1_b, ln_eps}, LnArgs{p1.ln1_g, p1.ln1_b, ln_eps},
                               valid_len, key_pad, sv, L.qkv, L.o, L.lse, st))
    return IM_OK;
  {
    ProfScope ps(PF_MISC, st);
    const size_t es = 2;
    const MlpTailPairSide a = {x0, p0.ln2_g, p0.ln2_b, p0.w1, p0.b1, p0.w2, p0.b2, sv + L.o, p0.wo, p0.bo, y0, ldy};
    const MlpTailPairSide b = {x1, p1.ln2_g, p1.ln2_b, p1.w1, p1.b1, p1.w2, p1.b2, sv + L.o + (size_t)R * d * es, p1.wo, p1.bo, y1, ldy};
    launch_mlp_tail_pair(a, b, ln_eps, (int)R, (int)d, d_ff, st);
  }
  *done = true;
  return check_hip("gsit_layer_fwd_pair launch");
}

}  // namespace imattn

extern "C" {

// ---- encoder layer, training: forward that saves what the backward needs, and the backward ----

struct LayerTrain {
  size_t att, h, zpre, a, saved_total;                                   // saved
  size_t u, v, dz, dv, dh, t, partial, partial1, cpart, cpart2, cpart3, attws, ws_total;   // backward workspace
  size_t fwd_ws_total;                                                   // forward workspace: u
  int split_w1, split_w2;
  size_t aws_bytes;
};
static LayerTrain layer_train_layout(const im_shape_t* s, int32_t d_ff) {
  LayerTrain L;
  const size_t es = s->dtype == IM_DTYPE_BF16 ? 2 : 4;
  const size_t R = (size_t)shape_rows(s), d = s->d_model, f = (size_t)d_ff;
  size_t off = 0;
  L.att = off; off += align256(saved_layout(s).total);
  L.h = off; off += align256(R * d * es);
  L.zpre = off; off += align256(R * f * es);
  L.a = off; off += align256(R * f * es);
  L.saved_total = off;
  off = 0;
  L.u = off; off += align256(R * d * es);
  L.fwd_ws_total = off + align256(pick_path(s) == PATH_MFMA ? mfma_fwd_workspace_bytes(s->d_model) : 0);
  L.v = off; off += align256(R * d * es);
  L.dz = off; off += align256(R * f * es);
  L.dv = off; off += align256(R * d * es);
  L.dh = off; off += align256(R * d * es);
  L.t = off; off += align256(R * d * es);
  L.split_w1 = L.split_w2 = 1;
  size_t p1 = gemm_alu_partial_bytes((int)d, d_ff, (int)R, &L.split_w1);
  size_t p2 = gemm_alu_partial_bytes(d_ff, (int)d, (int)R, &L.split_w2);
  if (mfma_linear_ok(s->dtype == IM_DTYPE_BF16, d, d_ff) && mfma_linear_ok(1, d_ff, d)) {
    p1 = std::max(p1, mfma_wgrad_partial_bytes((int)d, d_ff, (int)R));
    p2 = std::max(p2, mfma_wgrad_partial_bytes(d_ff, (int)d, (int)R));
  }
  // every second-stage sum of the backward may be postponed to one launch at its end (ReduceList): each set of
  // partials keeps a region of its own
  L.partial = off; off += align256(p2);     // dW2
  L.partial1 = off; off += align256(p1);    // dW1
  L.cpart = off; off += align256(colsum_partial_bytes((int)R, (int)f));         // db1
  L.cpart2 = off; off += align256(colsum_partial_bytes((int)R, (int)(3 * d)));  // second LayerNorm's two sums and db2
  L.cpart3 = off; off += align256(colsum_partial_bytes((int)R, (int)(2 * d)));  // first LayerNorm's two sums
  L.aws_bytes = bwd_workspace_bytes(s);
  L.attws = off; off += align256(L.aws_bytes);
  L.ws_total = off;
  return L;
}

int gsit_layer_train_sizes(const im_shape_t* shape, int32_t d_ff, size_t* saved_bytes, size_t* workspace_bytes) {
  int rc = layer_check(shape, d_ff);
  if (rc) return rc;
  const LayerTrain L = layer_train_layout(shape, d_ff);
  if (saved_bytes) *saved_bytes = L.saved_total;
  if (workspace_bytes) *workspace_bytes = std::max(L.ws_total, L.fwd_ws_total);
  return IM_OK;
}

int gsit_layer_fwd_train(const im_shape_t* shape, int32_t d_ff, const void* x, const gsit_layer_params_t* p, float ln_eps,
                         const int32_t* valid_len, const uint8_t* key_pad, void* y, void* saved, void* workspace,
                         size_t workspace_bytes, void* hip_stream) {
  int rc = layer_check(shape, d_ff);
  if (rc) return rc;
  if (shape->cu_rows && valid_len) return fail(IM_ERR_INVALID, "packed rows carry the lengths in cu_rows: valid_len must be NULL");
  if (!x || !p || !y || !saved) return fail(IM_ERR_INVALID, "x, params, y and saved must not be NULL");
  if (!p->ln1_g || !p->ln1_b || !p->wq || !p->wk || !p->wv || !p->wo || !p->ln2_g || !p->ln2_b || !p->w1 || !p->w2)
    return fail(IM_ERR_INVALID, "LayerNorm parameters, wq, wk, wv, wo, w1 and w2 must not be NULL");
  if (!(ln_eps >= 0.f)) return fail(IM_ERR_INVALID, "ln_eps must be >= 0");
  if ((rc = check_align16(shape, "gsit_layer_fwd_train", {x, p->wq, p->wk, p->wv, p->wo, p->w1, p->w2, y, saved, workspace}))) return rc;
  const LayerTrain L = layer_train_layout(shape, d_ff);
  if (!workspace || workspace_bytes < L.fwd_ws_total)
    return fail(IM_ERR_WORKSPACE, "gsit_layer_fwd_train needs %zu workspace bytes, got %zu", L.fwd_ws_total, workspace_bytes);
  hipStream_t st = as_stream(hip_stream);
  const int bf = shape->dtype == IM_DTYPE_BF16;
  const long R = shape_rows(shape), d = shape->d_model;
  char* sv = (char*)saved;
  char* ws = (char*)workspace;
  void* u = ws + L.u;
  void* h = sv + L.h;
  void* zpre = sv + L.zpre;
  void* a = sv + L.a;

  // the LayerNorms run inside the GEMMs that consume them where those can (see gsit_layer_fwd)
  auto al16 = [](const void* a0, const void* a1) { return (((uintptr_t)a0 | (uintptr_t)a1) & 15) == 0; };
  const bool mfma = pick_path(shape) == PATH_MFMA;
  const bool ln1_fused = mfma && mfma_qkv_fuses_ln(bf, d) && al16(p->ln1_g, p->ln1_b);
  const bool mlp_mfma = mfma_linear_ok(bf, d, d_ff) && mfma_linear_ok(bf, d_ff, d);
  const bool ln2_fused = mlp_mfma && mfma_gemm_fuses_ln(bf, d, d_ff) && al16(p->ln2_g, p->ln2_b);
  if (!ln1_fused && (rc = launch_layernorm(x, p->ln1_g, p->ln1_b, u, (int)R, (int)d, ln_eps, bf, st))) return rc;
  const SavedLayout A = saved_layout(shape);
  if (mfma)
    rc = mfma_attention_fwd(shape, ln1_fused ? x : u, p->wq, p->wk, p->wv, p->wo, p->bq, p->bk, p->bv, p->bo, valid_len,
                            key_pad, h, x, sv + L.att, A.qkv, A.o, A.lse, A.extra,
                            ws + L.u + align256((size_t)R * d * (bf ? 2 : 4)), st,
                            ln1_fused ? LnArgs{p->ln1_g, p->ln1_b, ln_eps} : LnArgs{nullptr, nullptr, 0.f});
  else
    rc = fwd_rowlane(shape, u, p->wq, p->wk, p->wv, p->wo, p->bq, p->bk, p->bv, p->bo, valid_len, key_pad, h, x,
                     sv + L.att, st);
  if (rc) return rc;
  if (!ln2_fused && (rc = launch_layernorm(h, p->ln2_g, p->ln2_b, u, (int)R, (int)d, ln_eps, bf, st))) return rc;
  if (mlp_mfma) {
    // at the small shapes the first GEMM writes the pre-activation and its GELU in one epilogue
    const bool both = mfma_gemm_small_tile((int)R, d_ff, (int)d, true);
    mfma_linear(ln2_fused ? h : u, d, p->w1, nullptr, nullptr, d_ff, d_ff, p->b1, nullptr, nullptr, both ? MGEMM_GELU_BOTH : 0,
                nullptr, zpre, d_ff, (int)R, d_ff, (int)d, st,
                ln2_fused ? LnArgs{p->ln2_g, p->ln2_b, ln_eps} : LnArgs{nullptr, nullptr, 0.f}, both ? a : nullptr);
    if (!both && (rc = launch_gelu_fwd(zpre, a, R * (long)d_ff, bf, st))) return rc;
    mfma_linear(a, d_ff, p->w2, nullptr, nullptr, d, (int)d, p->b2, nullptr, nullptr, 0, h, y, d, (int)R, (int)d, d_ff, st);
    return check_hip("gsit_layer_fwd_train launch");
  }
  GemmDesc g;
  memset(&g, 0, sizeof(g));
  g.A = u; g.sam = d; g.sak = 1; g.B[0] = p->w1; g.sbk = d_ff; g.sbn = 1; g.bias[0] = p->b1;
  g.C[0] = zpre; g.ldc = d_ff; g.M = (int)R; g.N = d_ff; g.K = (int)d;
  if ((rc = launch_gemm_alu(g, bf, bf, bf, st))) return rc;
  if ((rc = launch_gelu_fwd(zpre, a, R * (long)d_ff, bf, st))) return rc;
  memset(&g, 0, sizeof(g));
  g.A = a; g.sam = d_ff; g.sak = 1; g.B[0] = p->w2; g.sbk = d; g.sbn = 1; g.bias[0] = p->b2;
  g.C[0] = y; g.ldc = d; g.res = h; g.M = (int)R; g.N = (int)d; g.K = d_ff;
  if ((rc = launch_gemm_alu(g, bf, bf, bf, st))) return rc;
  return check_hip("gsit_layer_fwd_train launch");
}

int gsit_layer_bwd(const im_shape_t* shape, int32_t d_ff, const void* x, const gsit_layer_params_t* p, float ln_eps,
                   const int32_t* valid_len, const uint8_t* key_pad, const void* saved, const void* dy, void* dx,
                   const gsit_layer_grads_t* gr, void* workspace, size_t workspace_bytes, void* hip_stream) {
  int rc = layer_check(shape, d_ff);
  if (rc) return rc;
  if (shape->cu_rows && valid_len) return fail(IM_ERR_INVALID, "packed rows carry the lengths in cu_rows: valid_len must be NULL");
  if (!x || !p || !saved || !dy || !dx || !gr) return fail(IM_ERR_INVALID, "x, params, saved, dy, dx and grads must not be NULL");
  if (!p->ln1_g || !p->ln1_b || !p->wq || !p->wk || !p->wv || !p->wo || !p->ln2_g || !p->ln2_b || !p->w1 || !p->w2)
    return fail(IM_ERR_INVALID, "LayerNorm parameters, wq, wk, wv, wo, w1 and w2 must not be NULL");
  if (!(ln_eps >= 0.f)) return fail(IM_ERR_INVALID, "ln_eps must be >= 0");
  if ((rc = check_align16(shape, "gsit_layer_bwd", {x, p->wq, p->wk, p->wv, p->wo, p->w1, p->w2, saved, dy, dx, workspace}))) return rc;
  const LayerTrain L = layer_train_layout(shape, d_ff);
  if (!workspace || workspace_bytes < L.ws_total)
    return fail(IM_ERR_WORKSPACE, "gsit_layer_bwd needs %zu workspace bytes, got %zu", L.ws_total, workspace_bytes);
  hipStream_t st = as_stream(hip_stream);
  const int bf = shape->dtype == IM_DTYPE_BF16;
  const long R = shape_rows(shape), d = shape->d_model;
  const char* sv = (const char*)saved;
  char* ws = (char*)workspace;
  const void* h = sv + L.h;
  const void* zpre = sv + L.zpre;
  const void* a = sv + L.a;
  void* u = ws + L.u;
  void* v = ws + L.v;
  void* dz = ws + L.dz;
  void* dv = ws + L.dv;
  void* dh = ws + L.dh;
  void* t = ws + L.t;
  float* partial = (float*)(ws + L.partial);
  float* partial1 = (float*)(ws + L.partial1);
  float* cpart = (float*)(ws + L.cpart);
  float* cpart2 = (float*)(ws + L.cpart2);
  float* cpart3 = (float*)(ws + L.cpart3);
  ReduceList later;   // second-stage sums postponed to one launch at the end (matrix-core path, small outputs)
  later.n = 0;
  GemmDesc g;
  const bool mm = mfma_linear_ok(bf, d, d_ff) && mfma_linear_ok(bf, d_ff, d);  // bf16 GEMMs on the matrix cores

  // y = h + a W2 + b2
  if (gr->w2 && mm) {
    mfma_wgrad(a, d_ff, dy, d, (float*)gr->w2, nullptr, nullptr, 0, d_ff, (int)d, (int)R, partial, st, &later);
  } else if (gr->w2) {  // dW2 = a^T dy
    memset(&g, 0, sizeof(g));
    g.A = a; g.sam = 1; g.sak = d_ff; g.B[0] = dy; g.sbk = d; g.sbn = 1;
    g.C[0] = gr->w2; g.ldc = d; g.M = d_ff; g.N = (int)d; g.K = (int)R; g.split_k = L.split_w2; g.partial = partial;
    if ((rc = launch_gemm_alu(g, bf, bf, 0, st))) return rc;
  }
  // (db2 = column sums of dy: taken further down, together with the second LayerNorm's parameter gradients)
  // dz = (dy W2^T) * GELU'(z)
  const bool dz_fused = mm && mfma_gemm_small_tile((int)R, d_ff, (int)d, false);   // GELU' in the GEMM's epilogue
  if (mm) {
    mfma_dgrad(dy, d, p->w2, nullptr, nullptr, d, 0, dz, d_ff, (int)R, d_ff, (int)d, st, dz_fused ? zpre : nullptr);
  } else {
    memset(&g, 0, sizeof(g));
    g.A = dy; g.sam = d; g.sak = 1; g.B[0] = p->w2; g.sbk = 1; g.sbn = d;
    g.C[0] = dz; g.ldc = d_ff; g.M = (int)R; g.N = d_ff; g.K = (int)d;
    if ((rc = launch_gemm_alu(g, bf, bf, bf, st))) return rc;
  }
  if (!dz_fused && (rc = launch_gelu_bwd(zpre, dz, R * (long)d_ff, bf, st))) return rc;
  // z = v W1 + b1 with v = LN(h; ln2)
  if ((rc = launch_layernorm(h, p->ln2_g, p->ln2_b, v, (int)R, (int)d, ln_eps, bf, st))) return rc;
  if (gr->w1 && mm) {
    mfma_wgrad(v, d, dz, d_ff, (float*)gr->w1, nullptr, nullptr, 0, (int)d, d_ff, (int)R, partial1, st, &later);
  } else if (gr->w1) {  // dW1 = v^T dz
    memset(&g, 0, sizeof(g));
    g.A = v; g.sam = 1; g.sak = d; g.B[0] = dz; g.sbk = d_ff; g.sbn = 1;
    g.C[0] = gr->w1; g.ldc = d_ff; g.M = (int)d; g.N = d_ff; g.K = (int)R; g.split_k = L.split_w1; g.partial = partial1;
    if ((rc = launch_gemm_alu(g, bf, bf, 0, st))) return rc;
  }
  if (gr->b1) {
    const void* src1[1] = {dz};
    const long ld1[1] = {d_ff};
    float* out1[1] = {(float*)gr->b1};
    if ((rc = launch_colsum_multi(src1, ld1, out1, 1, (int)R, d_ff, bf, cpart, st, mm ? &later : nullptr))) return rc;
  }
  if (mm) {  // dv = dz W1^T
    mfma_dgrad(dz, d_ff, p->w1, nullptr, nullptr, d_ff, 0, dv, d, (int)R, (int)d, d_ff, st);
  } else {
    memset(&g, 0, sizeof(g));
    g.A = dz; g.sam = d_ff; g.sak = 1; g.B[0] = p->w1; g.sbk = 1; g.sbn = d_ff;
    g.C[0] = dv; g.ldc = d; g.M = (int)R; g.N = (int)d; g.K = d_ff;
    if ((rc = launch_gemm_alu(g, bf, bf, bf, st))) return rc;
  }
  // dh = dy + LN2 backward(dv)
  if ((rc = launch_layernorm_bwd(h, p->ln2_g, dv, dy, dh, t, (int)R, (int)d, ln_eps, bf, st))) return rc;
  {  // gradients of the LayerNorm gain and bias: column sums of dy * xhat and of dy; and db2 = column sums of dy
    const void* src[3] = {t, dv, dy};
    const long ld3[3] = {d, d, d};
    float* out3[3] = {(float*)gr->ln2_g, (float*)gr->ln2_b, (float*)gr->b2};
    if ((rc = launch_colsum_multi(src, ld3, out3, 3, (int)R, (int)d, bf, cpart2, st, mm ? &later : nullptr))) return rc;
  }
  // h = x + IMAttention(u), u = LN(x; ln1): attention backward with upstream gradient dh; its dx is du (into dv)
  if ((rc = launch_layernorm(x, p->ln1_g, p->ln1_b, u, (int)R, (int)d, ln_eps, bf, st))) return rc;
  const SavedLayout A = saved_layout(shape);
  if (pick_path(shape) == PATH_MFMA)
    rc = mfma_attention_bwd(shape, u, p->wq, p->wk, p->wv, p->wo, valid_len, key_pad, sv + L.att, A.qkv, A.o, A.lse, A.extra,
                            dh, dv, gr->wq, gr->wk, gr->wv, gr->wo, gr->bq, gr->bk, gr->bv, gr->bo, ws + L.attws, st,
                            mm ? &later : nullptr);
  else
    rc = bwd_rowlane(shape, u, p->wq, p->wk, p->wv, p->wo, valid_len, key_pad, sv + L.att, dh, dv, gr->wq, gr->wk, gr->wv,
                     gr->wo, gr->bq, gr->bk, gr->bv, gr->bo, ws + L.attws, st);
  if (rc) return rc;
  // dx = dh + LN1 backward(du)
  if ((rc = launch_layernorm_bwd(x, p->ln1_g, dv, dh, dx, t, (int)R, (int)d, ln_eps, bf, st))) return rc;
  {
    const void* src[2] = {t, dv};
    const long ld2[2] = {d, d};
    float* out2[2] = {(float*)gr->ln1_g, (float*)gr->ln1_b};
    if ((rc = launch_colsum_multi(src, ld2, out2, 2, (int)R, (int)d, bf, cpart3, st, mm ? &later : nullptr))) return rc;
  }
  launch_reduce_list(later, st);
  return check_hip("gsit_layer_bwd launch");
}

}  // extern "C"
