// Benchmark aid: measured ceilings of the device, to set the kernels' rates against
// something other than the data-sheet peaks.
//   matrix: every SIMD of the chip issues independent v_mfma_f32_32x32x16_bf16 back to back, once on
//           constant operands (1 and 0/1) and once on operands with random signs and mantissas that
//           change from one instruction to the next: the part lowers its clock with the switching
//           activity of the matrix units, so the second figure is the ceiling of a kernel that
//           multiplies real data
//   copy:   a streaming kernel reads the first half of a buffer and writes the second half
#include "mfma_common.h"

namespace oomb {

__global__ __launch_bounds__(512) void calib_mfma_kernel(float* sink, int iters) {
  bf16x8 a, b;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    a[e] = (__bf16)1.0f;
    b[e] = (__bf16)(float)(threadIdx.x & 1);
  }
  f32x16 acc[4];
#pragma unroll
  for (int n = 0; n < 4; ++n)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[n][r] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int n = 0; n < 4; ++n) acc[n] = mfma32(a, b, acc[n]);
  }
  float s = 0.f;
#pragma unroll
  for (int n = 0; n < 4; ++n) s += acc[n][0];
  if (s == 123.f) sink[0] = s;  // never true: keeps the loop alive
}

// same instruction stream on operands that differ per lane, per element and per instruction
__global__ __launch_bounds__(512) void calib_mfma_random_kernel(float* sink, int iters) {
  bf16x8 a[4], b[4];
  uint32_t h = (blockIdx.x * 512u + threadIdx.x) * 2654435761u + 12345u;
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    uint32_t wa[4], wb[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      // two bf16 values each: random sign and mantissa, exponent of 0.5 .. 2
      h ^= h >> 15; h *= 2246822519u; h ^= h >> 13; h += 0x9e3779b9u;
      wa[e] = ((h & 0x80ff80ffu) | 0x3f003f00u) ^ ((h >> 3) & 0x00800080u);
      h ^= h >> 15; h *= 2246822519u; h ^= h >> 13; h += 0x9e3779b9u;
      wb[e] = ((h & 0x80ff80ffu) | 0x3f003f00u) ^ ((h >> 3) & 0x00800080u);
    }
    a[q] = as_bf16x8(make_uint4(wa[0], wa[1], wa[2], wa[3]));
    b[q] = as_bf16x8(make_uint4(wb[0], wb[1], wb[2], wb[3]));
  }
  f32x16 acc[4];
#pragma unroll
  for (int n = 0; n < 4; ++n)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[n][r] = 0.f;
  for (int it = 0; it < iters; it += 4) {
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int n = 0; n < 4; ++n) acc[n] = mfma32(a[(n + j) & 3], b[(n + 2 * j + 1) & 3], acc[n]);
  }
  float s = 0.f;
#pragma unroll
  for (int n = 0; n < 4; ++n) s += acc[n][0];
  if (s == 123.f) sink[0] = s;  // keeps the loop alive
}

__global__ __launch_bounds__(256) void calib_copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n16) {
  const size_t stride = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

}  // namespace oomb

extern "C" oomb_status oomb_calibrate(int32_t which, void* buf, size_t bytes, double* result, void* hip_stream) {
  using namespace oomb;
  if (!result || !buf || bytes < 4096 || ((uintptr_t)buf & 15)) return OOMB_ERR_INVALID_ARG;
  hipStream_t st = (hipStream_t)hip_stream;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return OOMB_ERR_LAUNCH;
  oomb_status rc = OOMB_OK;
  float ms = 0.f;
  if (which == 0 || which == 2) {
    const int blocks = 2048, iters = 20000;
    auto kernel = which == 0 ? calib_mfma_kernel : calib_mfma_random_kernel;
    kernel<<<dim3(blocks), dim3(512), 0, st>>>((float*)buf, 200);  // warm-up
    (void)hipEventRecord(e0, st);
    kernel<<<dim3(blocks), dim3(512), 0, st>>>((float*)buf, iters);
    (void)hipEventRecord(e1, st);
    if (hipEventSynchronize(e1) != hipSuccess || hipEventElapsedTime(&ms, e0, e1) != hipSuccess || hipGetLastError() != hipSuccess)
      rc = OOMB_ERR_LAUNCH;
    else
      *result = (double)blocks * 8 * iters * 4 * (2.0 * 32 * 32 * 16) / (ms * 1e-3) / 1e12;  // TFLOP/s
  } else if (which == 1) {
    const size_t n16 = bytes / 32;  // 16-byte words per half
    const uint4* src = (const uint4*)buf;
    uint4* dst = (uint4*)buf + n16;
    calib_copy_kernel<<<dim3(4096), dim3(256), 0, st>>>(src, dst, n16);  // warm-up
    (void)hipEventRecord(e0, st);
    calib_copy_kernel<<<dim3(4096), dim3(256), 0, st>>>(src, dst, n16);
    (void)hipEventRecord(e1, st);
    if (hipEventSynchronize(e1) != hipSuccess || hipEventElapsedTime(&ms, e0, e1) != hipSuccess || hipGetLastError() != hipSuccess)
      rc = OOMB_ERR_LAUNCH;
    else
      *result = 2.0 * (double)n16 * 16 / (ms * 1e-3) / 1e9;  // GB/s, read + write
  } else {
    rc = OOMB_ERR_INVALID_ARG;
  }
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  return rc;
}
