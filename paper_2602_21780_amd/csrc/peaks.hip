// Two yardsticks measured on the device the library runs on: the rate of a loop of nothing but
// v_mfma_f32_32x32x16_bf16 (the instruction the attention kernel computes with) and the rate of a plain
// streaming copy.  The published peaks (2.5 PFLOP/s dense bf16, 8 TB/s) are what the benchmark's
// roofline is priced against; these say how much of them any kernel can reach on this chip and clock.
#include "../../include/xsv_tune.h"
#include "xsv_internal.h"

namespace xsv {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;

// 256 threads; every wave issues 8 * iters MFMAs on four independent accumulators
__global__ __launch_bounds__(256) void mfma_loop_kernel(float* out, int iters) {
  const bf16x8_t a = __builtin_bit_cast(bf16x8_t, make_uint4(threadIdx.x, 1u, 2u, 3u));
  const bf16x8_t b = __builtin_bit_cast(bf16x8_t, make_uint4(5u, threadIdx.x, 7u, 8u));
  f32x16_t acc[4];
  for (int i = 0; i < 4; ++i)
    for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i % 4] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[i % 4], 0, 0, 0);
  }
  float s = 0.f;
  for (int i = 0; i < 4; ++i)
    for (int r = 0; r < 16; ++r) s += acc[i][r];
  out[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
}

__global__ __launch_bounds__(256) void stream_copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n16) {
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (size_t)gridDim.x * 256) dst[i] = src[i];
}

}  // namespace xsv

extern "C" int xsv_measure_peaks(void* hip_stream, float* mfma_bf16_tflops, float* copy_gbs) {
  using namespace xsv;
  if (!mfma_bf16_tflops || !copy_gbs) return XSV_ERR_ARG;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  constexpr int kWgs = 2048, kIters = 4096;
  constexpr size_t kBytes = (size_t)512 << 20;  // per buffer
  float* out = nullptr;
  uint4 *src = nullptr, *dst = nullptr;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  int rc = XSV_OK;
  auto cleanup = [&]() {
    if (out) (void)hipFree(out);
    if (src) (void)hipFree(src);
    if (dst) (void)hipFree(dst);
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
  };
  if (hipMalloc(&out, (size_t)kWgs * 256 * 4) != hipSuccess || hipMalloc(&src, kBytes) != hipSuccess ||
      hipMalloc(&dst, kBytes) != hipSuccess) {
    (void)hipGetLastError();
    cleanup();
    return XSV_ERR_OOM;
  }
  bool ok = hipEventCreate(&e0) == hipSuccess && hipEventCreate(&e1) == hipSuccess &&
            hipMemsetAsync(src, 1, kBytes, stream) == hipSuccess;
  float ms = 0.f;
  if (ok) {
    hipLaunchKernelGGL(mfma_loop_kernel, dim3(kWgs), dim3(256), 0, stream, out, 64);  // warm-up
    ok = hipEventRecord(e0, stream) == hipSuccess;
    hipLaunchKernelGGL(mfma_loop_kernel, dim3(kWgs), dim3(256), 0, stream, out, kIters);
    ok = ok && hipEventRecord(e1, stream) == hipSuccess && hipEventSynchronize(e1) == hipSuccess &&
         hipEventElapsedTime(&ms, e0, e1) == hipSuccess && ms > 0.f;
    // waves * MFMAs per wave * 32 x 32 x 16 multiply-adds
    if (ok) *mfma_bf16_tflops = (float)((double)kWgs * 4 * kIters * 8 * (2.0 * 32 * 32 * 16) / (ms * 1e-3) / 1e12);
  }
  if (ok) {
    const size_t n16 = kBytes / 16;
    hipLaunchKernelGGL(stream_copy_kernel, dim3(8192), dim3(256), 0, stream, src, dst, n16);  // warm-up
    ok = hipEventRecord(e0, stream) == hipSuccess;
    for (int rep = 0; rep < 4; ++rep) hipLaunchKernelGGL(stream_copy_kernel, dim3(8192), dim3(256), 0, stream, src, dst, n16);
    ok = ok && hipEventRecord(e1, stream) == hipSuccess && hipEventSynchronize(e1) == hipSuccess &&
         hipEventElapsedTime(&ms, e0, e1) == hipSuccess && ms > 0.f;
    if (ok) *copy_gbs = (float)(4.0 * 2.0 * (double)kBytes / (ms * 1e-3) / 1e9);  // bytes read + bytes written
  }
  if (!ok || hipGetLastError() != hipSuccess) rc = XSV_ERR_HIP;
  cleanup();
  return rc;
}
