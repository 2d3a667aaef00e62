// The activation quantiser as a function that allocates nothing: device rows in, E4M3 codes and
// one scale per row out, any row length.  A row is split over workgroups; the per-row absolute
// maxima they combine live in a file-scope device array, so the call needs no model, no
// workspace and no allocation of any kind (callers under HIP graph capture, serving loops and
// harnesses that may not allocate).
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <mutex>
#include "../../include/pahq.h"
#include "device_util.h"

namespace pahq {

// One word per row: the bit pattern of max |x| over the row (non-negative floats order like
// unsigned integers, so atomicMax on the bits is exact and independent of the order of arrival).
// Every GPU the library runs on holds its own copy of this array until the process ends.
static __device__ __align__(256) unsigned scratch[PAHQ_NOALLOC_MAX_ROWS];

constexpr int CHUNK = 4096;          // elements of a row per workgroup (256 threads x 16)

__global__ __launch_bounds__(256) void noalloc_clear_k(unsigned* amax, int rows) {
  int i = blockIdx.x * 256 + threadIdx.x;
  if (i < rows) amax[i] = 0u;
}

__global__ __launch_bounds__(256) void noalloc_amax_k(const float* x, int cols, unsigned* amax) {
  const int row = blockIdx.y;
  const float* p = x + (long long)row * cols;
  const int e0 = blockIdx.x * CHUNK, e1 = min(cols, e0 + CHUNK);
  float m = 0.f;
  for (int e = e0 + threadIdx.x; e < e1; e += 256) m = fmaxf(m, fabsf(p[e]));
  m = wave_max(m);
  if ((threadIdx.x & 63) == 0) atomicMax(&amax[row], __float_as_uint(m));
}

__global__ __launch_bounds__(256) void noalloc_encode_k(const float* x, int cols, const unsigned* amax,
                                                        uint8_t* codes, float* scales) {
  const int row = blockIdx.y;
  const float am = __uint_as_float(amax[row]);
  const float scale = (am == 0.f) ? 1.0f : am / 448.0f;
  const float inv = 1.0f / scale;
  const float* p = x + (long long)row * cols;
  uint8_t* o = codes + (long long)row * cols;
  const int e0 = blockIdx.x * CHUNK, e1 = min(cols, e0 + CHUNK);
  for (int e = e0 + threadIdx.x; e < e1; e += 256) o[e] = (uint8_t)e4m3_encode(p[e] * inv);
  if (blockIdx.x == 0 && threadIdx.x == 0) scales[row] = scale;
}

namespace {
constexpr int MAX_DEVICES = 64;
unsigned* scratch_ptr[MAX_DEVICES];      // device address of `scratch` on each GPU (its name is a host-side stand-in)
std::mutex scratch_mu;

// Address of this device's copy of the array, looked up once per device with that device current.
int scratch_of_current_device(unsigned** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return PAHQ_EHIP;
  std::lock_guard<std::mutex> lock(scratch_mu);
  if (!scratch_ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return PAHQ_EHIP;
    scratch_ptr[dev] = (unsigned*)p;
  }
  *out = scratch_ptr[dev];
  return PAHQ_OK;
}
}  // namespace

}  // namespace pahq

extern "C" int pahq_quantize_rows_noalloc(void* hip_stream, const float* x, int32_t rows, int32_t cols,
                                          uint8_t* codes, float* scales) {
  using namespace pahq;
  if (rows < 0 || cols < 1) return PAHQ_EINVAL;
  if (rows > PAHQ_NOALLOC_MAX_ROWS) return PAHQ_ETOOBIG;
  if (rows == 0) return PAHQ_OK;
  if (!x || !codes || !scales) return PAHQ_EINVAL;
  unsigned* amax = nullptr;
  int rc = scratch_of_current_device(&amax);
  if (rc != PAHQ_OK) return rc;
  hipStream_t st = (hipStream_t)hip_stream;
  // the array keeps the last call's maxima: the rows of this call start from zero (a fill kernel,
  // not a memset, so that the sequence can be captured into a graph)
  hipLaunchKernelGGL(noalloc_clear_k, dim3((rows + 255) / 256), dim3(256), 0, st, amax, rows);
  const dim3 grid((cols + CHUNK - 1) / CHUNK, rows);
  hipLaunchKernelGGL(noalloc_amax_k, grid, dim3(256), 0, st, x, cols, amax);
  hipLaunchKernelGGL(noalloc_encode_k, grid, dim3(256), 0, st, x, cols, amax, codes, scales);
  return hipGetLastError() == hipSuccess ? PAHQ_OK : PAHQ_EHIP;
}
