// Small device helpers shared by the kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace pahq {

// Butterfly reductions over the 64 lanes of a wavefront; every lane gets the
// result and the order of operations is fixed, so results are reproducible.
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
__device__ __forceinline__ double wave_sum_d(double v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

// binary32 -> FP8 E4M3 (bias 7, max 448, no infinities), round to nearest, ties
// to even, saturating; the sign of zero is kept.  Normal range: round the 23-bit
// mantissa to 3 bits on the bit pattern and re-bias the exponent (127 -> 7).
// Below 2^-6 the grid is uniform with step 2^-9, so the code is |y| * 512
// rounded to the nearest even integer (8 is the first normal code).
__device__ __forceinline__ uint32_t e4m3_encode(float y) {
  uint32_t sign = (__float_as_uint(y) >> 24) & 0x80u;
  float a = fminf(fabsf(y), 448.0f);
  uint32_t code;
  if (a >= 0.015625f) {
    uint32_t b = __float_as_uint(a);
    b += 0x7FFFFu + ((b >> 20) & 1u);
    code = (b >> 20) - 960u;
  } else {
    code = (uint32_t)__float2int_rn(a * 512.0f);
  }
  return code | sign;
}

// tanh-form GELU, 0.5 x (1 + tanh(u)) with u = sqrt(2/pi) (x + 0.044715 x^3), written as
// x / (1 + exp(-2u)): relative accuracy is kept for negative x, where 1 + tanh(u) cancels.  The
// exponential and the division are the correctly rounded-to-an-ulp library forms, not the hardware
// approximations: the result feeds the row quantiser, where a relative error e moves about e / 2^-4
// of the elements across a rounding boundary, and the approximations' 1e-6 was the largest single
// contribution to such moves on GELU models.  exp(-2u) overflows to +inf for very negative x, which
// gives the correct limit -0.
__device__ __forceinline__ float gelu_tanh(float x) {
  const float k2 = -2.0f * 0.7978845608028654f;   // -2 sqrt(2/pi)
  float u = k2 * (x + 0.044715f * x * x * x);
  return x / (1.0f + expf(u));
}

}  // namespace pahq
