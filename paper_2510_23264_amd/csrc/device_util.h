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
__device__ __forceinline__ uint32_t e4m3_encode_bits(float y) {
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
// The same code from the hardware conversion (V_CVT_PK_FP8_F32: two values per instruction instead of a dozen
// integer operations per value).  With the value clamped to +-448 first it returns e4m3_encode_bits(y) for every
// finite binary32 pattern -- ties, the subnormal range and the sign of zero included; compared exhaustively on the
// device -- so the kernels use it and the form above stays as the definition (and for the weights at set-up).
__device__ __forceinline__ uint32_t e4m3_encode(float y) {
  const float c = __builtin_amdgcn_fmed3f(y, -448.0f, 448.0f);
  return (uint32_t)__builtin_amdgcn_cvt_pk_fp8_f32(c, c, 0, false) & 0xFFu;
}
// four values -> their codes in the four bytes of a word (byte k = code of y_k)
__device__ __forceinline__ uint32_t e4m3_encode4(float y0, float y1, float y2, float y3) {
  int w = __builtin_amdgcn_cvt_pk_fp8_f32(__builtin_amdgcn_fmed3f(y0, -448.0f, 448.0f), __builtin_amdgcn_fmed3f(y1, -448.0f, 448.0f), 0, false);
  w = __builtin_amdgcn_cvt_pk_fp8_f32(__builtin_amdgcn_fmed3f(y2, -448.0f, 448.0f), __builtin_amdgcn_fmed3f(y3, -448.0f, 448.0f), w, true);
  return (uint32_t)w;
}

// The grid a quantiser rounds to.  bits == 4: the paper's Eq. RTN-Q with N = 4 as printed -- step = max|x| / 2^(N-1),
// integer multiples of it, round to nearest (ties to even) -- with the multiple k (|k| <= 8) stored as the E4M3
// code of the integer k, which is exact, so the matrix products downstream are the same exact machinery.
// Any other value: E4M3 itself (step = max|x| / 448 at the top of the grid).
__device__ __forceinline__ float q_top(int bits) { return bits == 4 ? 8.0f : 448.0f; }
__device__ __forceinline__ uint32_t q_encode(float y, int bits) { return e4m3_encode(bits == 4 ? rintf(y) : y); }
__device__ __forceinline__ uint32_t q_encode4(float y0, float y1, float y2, float y3, int bits) {
  if (bits == 4) { y0 = rintf(y0); y1 = rintf(y1); y2 = rintf(y2); y3 = rintf(y3); }
  return e4m3_encode4(y0, y1, y2, y3);
}

// binary32 -> bfloat16 bit pattern, round to nearest, ties to even (finite input): the 16 dropped mantissa bits
// round the kept ones up when they exceed half a unit, or equal it and the kept pattern is odd.
__device__ __forceinline__ uint32_t bf16_rne(float x) {
  const uint32_t u = __float_as_uint(x);
  return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

// tanh-form GELU, 0.5 x (1 + tanh(u)) with u = sqrt(2/pi) (x + 0.044715 x^3), written as
// x / (1 + exp(-2u)): relative accuracy is kept for negative x, where 1 + tanh(u) cancels.  The result
// feeds the row quantiser, where a relative error e moves about e / 2^-4 of the elements across a rounding
// boundary, so both the exponential and the reciprocal are carried to an ulp or two instead of the 1e-6 of
// the bare hardware forms: exp(v) = exp2(t) * (1 + r ln 2) with t = fl(v log2 e) and r what that product
// and the rounding of log2 e lost (one FMA recovers it), and one Newton step on the hardware reciprocal.
// The exponent is clamped at 126: beyond it the result is below 2^-125 |x| and quantises to zero either way.
__device__ __forceinline__ float gelu_tanh(float x) {
  const float k2 = -2.0f * 0.7978845608028654f;   // -2 sqrt(2/pi)
  const float l2e_hi = 1.44269502162933349609375f, l2e_lo = 1.925963033500011e-8f, ln2 = 0.6931471805599453f;
  const float v = k2 * (x + 0.044715f * x * x * x);
  const float t = fminf(v * l2e_hi, 126.0f);
  const float r = (t < 126.0f) ? __fmaf_rn(v, l2e_hi, -t) + v * l2e_lo : 0.0f;
  float e = __builtin_amdgcn_exp2f(t);
  e = __fmaf_rn(e, r * ln2, e);
  const float den = 1.0f + e;
  float q = __builtin_amdgcn_rcpf(den);
  q = __fmaf_rn(__fmaf_rn(-den, q, 1.0f), q, q);
  return x * q;
}

}  // namespace pahq
