#include "mfma_path.hpp"
namespace imattn {
bool mfma_supports(int, int) { return false; }
size_t mfma_saved_extra_bytes(int, int, int) { return 0; }
size_t mfma_fwd_workspace_bytes(int) { return 0; }
size_t mfma_bwd_workspace_bytes(int, int, int, int) { return 0; }
int mfma_attention_fwd(const im_shape_t*, const void*, const void*, const void*, const void*, const void*, const void*,
                       const void*, const void*, const void*, const int32_t*, const uint8_t*, void*, const void*, char*,
                       size_t, size_t, size_t, size_t, char*, hipStream_t) { return IM_ERR_UNSUPPORTED; }
int mfma_attention_bwd(const im_shape_t*, const void*, const void*, const void*, const void*, const void*,
                       const int32_t*, const uint8_t*, const char*, size_t, size_t, size_t, size_t, const void*, void*,
                       void*, void*, void*, void*, void*, void*, void*, void*, char*, hipStream_t) { return IM_ERR_UNSUPPORTED; }
}
