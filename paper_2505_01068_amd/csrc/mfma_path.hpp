// bf16 MFMA path (head dimension 64): projections as MFMA GEMMs and flash-style
// IM attention on the matrix cores.
#pragma once
#include "common.hpp"

namespace imattn {

bool mfma_supports(int d_model, int dh);
size_t mfma_saved_extra_bytes(int B, int T, int d);
size_t mfma_fwd_workspace_bytes(int d);
size_t mfma_bwd_workspace_bytes(int B, int T, int d, int H);

// sv + off_* : Q|K|V rows [R,3d], O [R,d], lse [B,H,T], extra (transposed copies).
int mfma_attention_fwd(const im_shape_t* s, const void* x, const void* wq, const void* wk, const void* wv,
                       const void* wo, const void* bq, const void* bk, const void* bv, const void* bo,
                       const int32_t* valid_len, const uint8_t* key_pad, void* y, const void* res, char* sv,
                       size_t off_qkv, size_t off_o, size_t off_lse, size_t off_extra, char* ws, hipStream_t st);
int mfma_attention_bwd(const im_shape_t* s, const void* x, const void* wq, const void* wk, const void* wv,
                       const void* wo, const int32_t* valid_len, const uint8_t* key_pad, const char* sv,
                       size_t off_qkv, size_t off_o, size_t off_lse, size_t off_extra, const void* dy, void* dx,
                       void* dwq, void* dwk, void* dwv, void* dwo, void* dbq, void* dbk, void* dbv, void* dbo, char* ws,
                       hipStream_t st);

}  // namespace imattn
