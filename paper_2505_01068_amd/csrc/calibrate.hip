// Two micro-benchmarks that measure what this GPU sustains, for the "fraction of the measured
// achievable peak" a benchmark reports next to the fraction of the published peak:
//   - a register-resident MFMA loop (v_mfma_f32_32x32x16_bf16, the instruction of the attention and
//     GEMM kernels; four independent accumulators per wave, no memory traffic), and
//   - a streaming copy (16-byte loads and stores, grid-stride) for the HBM rate.
// Both only enqueue on the caller's stream; the caller times them with events.
#include "mfma_common.hpp"

namespace imattn {

constexpr int CAL_WAVES = 4;        // waves per workgroup
constexpr int CAL_WGS_PER_CU = 2;   // 8 waves per CU, two per SIMD
constexpr int CAL_CHAINS = 4;       // independent accumulator chains per wave

__global__ __launch_bounds__(64 * CAL_WAVES) void calibrate_mfma_kernel(int iters, float* sink) {
  const int lane = threadIdx.x & 63;
  // operands that the compiler cannot fold: they depend on the lane and on a kernel argument
  u32x4 av, bv;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    av[i] = 0x3c003c00u + (unsigned)(lane + i);            // small bf16 values
    bv[i] = 0x3b803b80u + (unsigned)(lane * 3 + i + (iters & 1));
  }
  const bf16x8 a = as_bf16x8(av), b = as_bf16x8(bv);
  f32x16 acc[CAL_CHAINS];
#pragma unroll
  for (int c = 0; c < CAL_CHAINS; ++c)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[c][r] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int c = 0; c < CAL_CHAINS; ++c) acc[c] = mfma32(a, b, acc[c]);
  }
  float s = 0.f;
#pragma unroll
  for (int c = 0; c < CAL_CHAINS; ++c)
#pragma unroll
    for (int r = 0; r < 16; ++r) s += acc[c][r];
  if (s == 12345.678f) sink[0] = s;   // keeps the loop alive; practically never true
}

__global__ __launch_bounds__(256) void calibrate_copy_kernel(u32x4* __restrict__ dst, const u32x4* __restrict__ src,
                                                          size_t n16) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

}  // namespace imattn

using namespace imattn;

extern "C" {

int im_calibrate_mfma(int32_t iters, void* sink, double* flops, void* hip_stream) {
  if (iters < 1 || !sink) { set_error("im_calibrate_mfma: iters must be >= 1 and sink a device pointer"); return IM_ERR_INVALID; }
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) {
    set_error("im_calibrate_mfma: cannot query the device");
    return IM_ERR_HIP;
  }
  const int grid = cus * CAL_WGS_PER_CU;
  hipLaunchKernelGGL(calibrate_mfma_kernel, dim3(grid), dim3(64 * CAL_WAVES), 0, (hipStream_t)hip_stream, iters, (float*)sink);
  if (flops) *flops = (double)grid * CAL_WAVES * (double)iters * 4.0 * CAL_CHAINS * (2.0 * 32 * 32 * 16);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) { set_error("im_calibrate_mfma launch: %s", hipGetErrorString(e)); return IM_ERR_HIP; }
  return IM_OK;
}

int im_calibrate_copy(void* dst, const void* src, size_t bytes, void* hip_stream) {
  if (!dst || !src || bytes < 16 || (bytes & 15) || (((uintptr_t)dst | (uintptr_t)src) & 15)) {
    set_error("im_calibrate_copy: dst and src must be 16-byte aligned device pointers, bytes a positive multiple of 16");
    return IM_ERR_INVALID;
  }
  hipLaunchKernelGGL(calibrate_copy_kernel, dim3(256 * 8), dim3(256), 0, (hipStream_t)hip_stream, (u32x4*)dst,
                     (const u32x4*)src, bytes / 16);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) { set_error("im_calibrate_copy launch: %s", hipGetErrorString(e)); return IM_ERR_HIP; }
  return IM_OK;
}

}  // extern "C"
