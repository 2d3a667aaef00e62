// Measured ceilings of the device the library runs on, next to the published peaks: a pure issue loop of the
// matrix-core instruction the exact GEMM uses (V_MFMA_F32_16X16X32_F16, operands in registers, every compute
// unit busy) and a streaming copy.  Neither touches a model; the caller passes the stream and, for the copy,
// a scratch buffer.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "../../include/pahq.h"
#include "mma_util.h"
#include "device_util.h"

namespace pahq {

// 8 waves per workgroup, 16 independent accumulator tiles per wave, two dependent MFMAs per tile and step (the
// shape of the GEMM's inner loop without its loads, converts and waits)
__global__ __launch_bounds__(512, 1) void mfma_issue_k(float* out, int iters) {
  const int lane = threadIdx.x & 63;
  v4f acc[4][4];
  v8h a[4], b[4];
#pragma unroll
  for (int i = 0; i < 4; i++) {
#pragma unroll
    for (int e = 0; e < 8; e++) { a[i][e] = (_Float16)(0.001f * (float)(lane + i + e)); b[i][e] = (_Float16)(0.002f * (float)(lane - i + e)); }
#pragma unroll
    for (int j = 0; j < 4; j++) acc[i][j] = (v4f){0.f, 0.f, 0.f, 0.f};
  }
  for (int it = 0; it < iters; it++) {
#pragma unroll
    for (int j = 0; j < 4; j++)
#pragma unroll
      for (int i = 0; i < 4; i++) {
        acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[i], b[j], acc[i][j], 0, 0, 0);
        acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(b[j], a[i], acc[i][j], 0, 0, 0);
      }
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 4; i++)
#pragma unroll
    for (int j = 0; j < 4; j++) s += acc[i][j][0] + acc[i][j][1] + acc[i][j][2] + acc[i][j][3];
  out[blockIdx.x * 512 + threadIdx.x] = s;
}

__global__ __launch_bounds__(256) void stream_copy_k(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n16) {
  const size_t stride = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

// Every binary32 pattern with the given upper 16 bits (one workgroup each): the code the kernels take (hardware
// conversion) against the encoder on the bit pattern that defines it.  out[0] counts mismatches, out[1] keeps one.
__global__ __launch_bounds__(256) void encoder_compare_k(unsigned long long* out) {
  const uint32_t hi = blockIdx.x;
  for (uint32_t lo = threadIdx.x; lo < 65536u; lo += 256u) {
    const uint32_t u = (hi << 16) | lo;
    const float y = __uint_as_float(u);
    if (!(fabsf(y) <= 3.0e38f)) continue;                       // finite
    if ((e4m3_encode(y) & 0xFFu) != (e4m3_encode_bits(y) & 0xFFu) ||
        e4m3_encode4(y, -y, y, -y) != ((e4m3_encode_bits(y) & 0xFFu) * 0x00010001u | (e4m3_encode_bits(-y) & 0xFFu) * 0x01000100u)) {
      atomicAdd(out, 1ull);
      out[1] = u;
    }
  }
}

}  // namespace pahq

extern "C" int pahq_compare_encoders(void* hip_stream, void* scratch, uint64_t* mismatches, uint32_t* example) {
  using namespace pahq;
  if (!scratch || !mismatches || (((uintptr_t)scratch) & 15)) return PAHQ_EINVAL;
  hipStream_t st = (hipStream_t)hip_stream;
  unsigned long long* out = (unsigned long long*)scratch;
  unsigned long long h[2] = {0, 0};
  if (hipMemcpyAsync(out, h, sizeof(h), hipMemcpyHostToDevice, st) != hipSuccess) return PAHQ_EHIP;
  hipLaunchKernelGGL(encoder_compare_k, dim3(65536), dim3(256), 0, st, out);
  if (hipMemcpyAsync(h, out, sizeof(h), hipMemcpyDeviceToHost, st) != hipSuccess || hipStreamSynchronize(st) != hipSuccess) return PAHQ_EHIP;
  *mismatches = h[0];
  if (example) *example = (uint32_t)h[1];
  return hipGetLastError() == hipSuccess ? PAHQ_OK : PAHQ_EHIP;
}

extern "C" int pahq_measure_ceilings(void* hip_stream, void* scratch, size_t scratch_bytes, double* mfma_f16_tflops,
                                     double* copy_gbs) {
  using namespace pahq;
  if (!scratch || !mfma_f16_tflops || !copy_gbs || scratch_bytes < ((size_t)64 << 20) || (((uintptr_t)scratch) & 255)) return PAHQ_EINVAL;
  hipStream_t st = (hipStream_t)hip_stream;
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return PAHQ_EHIP;
  int rc = PAHQ_OK;
  float ms = 0.f;
  // ---- matrix cores: 256 workgroups x 8 waves x iters x 32 MFMAs of 16 x 16 x 32 (2 * 16 * 16 * 32 flops each)
  const int grid = 256, iters = 80000;
  float* out = (float*)scratch;                       // 256 * 512 floats
  hipLaunchKernelGGL(mfma_issue_k, dim3(grid), dim3(512), 0, st, out, 200);
  hipEventRecord(e0, st);
  hipLaunchKernelGGL(mfma_issue_k, dim3(grid), dim3(512), 0, st, out, iters);
  hipEventRecord(e1, st);
  if (hipEventSynchronize(e1) != hipSuccess || hipEventElapsedTime(&ms, e0, e1) != hipSuccess) rc = PAHQ_EHIP;
  else *mfma_f16_tflops = (double)grid * 8 * (double)iters * 32.0 * 16384.0 / (ms * 1e-3) / 1e12;
  // ---- copy: half of the scratch to the other half, three times
  if (rc == PAHQ_OK) {
    const size_t half = scratch_bytes / 2 / 4096 * 4096, n16 = half / 16;
    const uint4* src = (const uint4*)scratch;
    uint4* dst = (uint4*)((char*)scratch + half);
    hipLaunchKernelGGL(stream_copy_k, dim3(4096), dim3(256), 0, st, src, dst, n16);
    hipEventRecord(e0, st);
    for (int r = 0; r < 3; r++) hipLaunchKernelGGL(stream_copy_k, dim3(4096), dim3(256), 0, st, src, dst, n16);
    hipEventRecord(e1, st);
    if (hipEventSynchronize(e1) != hipSuccess || hipEventElapsedTime(&ms, e0, e1) != hipSuccess) rc = PAHQ_EHIP;
    else *copy_gbs = 3.0 * 2.0 * (double)half / (ms * 1e-3) / 1e9;      // bytes read + written
  }
  hipEventDestroy(e0); hipEventDestroy(e1);
  if (rc == PAHQ_OK && hipGetLastError() != hipSuccess) rc = PAHQ_EHIP;
  return rc;
}
