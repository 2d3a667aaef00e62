// Row-wise kernels: receiver-input gather + norm + e4m3 row quantisation, the
// edge-batched patch, hidden-activation quantisation, tile arithmetic,
// embedding lookup and weight quantisation.  All are HBM-bound streaming
// kernels: one 64-lane wavefront owns one row of d_model floats, loads are
// coalesced along the row, reductions are wave shuffles in a fixed order.
#include <algorithm>
#include "kernels.h"
#include "device_util.h"
#include "mma_util.h"

namespace pahq {

// ------------------------------------------------------------------ fill
__global__ void fill_zero_k(uint4* p, size_t n16) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  size_t stride = (size_t)gridDim.x * blockDim.x;
  uint4 z = {0, 0, 0, 0};
  for (; i < n16; i += stride) p[i] = z;
}
hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t s) {
  size_t n16 = bytes / 16;          // callers pass 16-byte multiples
  if (n16 == 0) return hipSuccess;
  int blocks = (int)((n16 + 255) / 256 < 65535 ? (n16 + 255) / 256 : 65535);
  hipLaunchKernelGGL(fill_zero_k, dim3(blocks), dim3(256), 0, s, (uint4*)p, n16);
  return hipGetLastError();
}

// ------------------------------------------------------------------ weight quantisation
// amax over each contiguous slice, as the bit pattern of a non-negative float
// (unsigned integer order = float order, so atomicMax is exact and order-free).
__global__ void slice_absmax_k(const float* w, long long slice_elems, unsigned* amax_bits, int* nonfinite) {
  int sl = blockIdx.y;
  const float* p = w + (long long)sl * slice_elems;
  float m = 0.f;
  int bad = 0;
  for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < slice_elems;
       i += (long long)gridDim.x * blockDim.x) {
    float v = p[i];
    if (!(fabsf(v) <= 3.0e38f)) bad = 1;     // catches NaN and infinities
    m = fmaxf(m, fabsf(v));
  }
  m = wave_max(m);
  if ((threadIdx.x & 63) == 0) atomicMax(&amax_bits[sl], __float_as_uint(m));
  if (bad) atomicOr(nonfinite, 1);
}
hipError_t launch_slice_absmax(const float* w, long long slice_elems, int n_slices, unsigned* amax_bits,
                               int* nonfinite_flag, hipStream_t s) {
  long long per = (slice_elems + 255) / 256;
  int bx = (int)(per < 1024 ? (per < 1 ? 1 : per) : 1024);
  hipLaunchKernelGGL(slice_absmax_k, dim3(bx, n_slices), dim3(256), 0, s, w, slice_elems, amax_bits,
                     nonfinite_flag);
  return hipGetLastError();
}

// W slice [K][N] row-major -> codes [N][ldq] (K contiguous), through a 32x32 LDS transpose.
__global__ void quant_transpose_k(const float* w, int K, int N, const unsigned* amax_bits, float* scale_out,
                                  uint8_t* codes, int ldq, int qbits) {
  __shared__ float tile[32][33];
  float amax = __uint_as_float(*amax_bits);
  float scale = (amax == 0.f || qbits == 16) ? 1.0f : amax / q_top(qbits);      // bfloat16 has no scale
  float inv = 1.0f / scale;
  if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0 && threadIdx.y == 0) *scale_out = scale;
  int k0 = blockIdx.y * 32, n0 = blockIdx.x * 32;
  for (int r = threadIdx.y; r < 32; r += 8) {
    int k = k0 + r, n = n0 + threadIdx.x;
    tile[r][threadIdx.x] = (k < K && n < N) ? w[(long long)k * N + n] : 0.f;
  }
  __syncthreads();
  for (int r = threadIdx.y; r < 32; r += 8) {
    int n = n0 + r, k = k0 + threadIdx.x;
    if (n < N && k < K) {
      if (qbits == 16) *(uint16_t*)(codes + (long long)n * ldq + 2 * k) = (uint16_t)bf16_rne(tile[threadIdx.x][r]);     // ldq in bytes
      else codes[(long long)n * ldq + k] = (uint8_t)e4m3_encode_bits(qbits == 4 ? rintf(tile[threadIdx.x][r] * inv) : tile[threadIdx.x][r] * inv);
    }
  }
}
hipError_t launch_quant_transpose(const float* w, int K, int N, const unsigned* amax_bits, float* scale_out,
                                  uint8_t* codes_out, int ldq, int qbits, hipStream_t s) {
  hipLaunchKernelGGL(quant_transpose_k, dim3((N + 31) / 32, (K + 31) / 32), dim3(32, 8), 0, s, w, K, N,
                     amax_bits, scale_out, codes_out, ldq, qbits);
  return hipGetLastError();
}

// ------------------------------------------------------------------ embedding
__global__ void embed_k(const int* tok, const float* W_E, const float* W_pos, float* out, int T, int S, int d) {
  long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (long long)T * d) return;
  int t = (int)(i / d), e = (int)(i % d);
  float v = W_E[(long long)tok[t] * d + e];
  if (W_pos) v += W_pos[(long long)(t % S) * d + e];
  out[i] = v;
}
hipError_t launch_embed(const int* tok, const float* W_E, const float* W_pos, float* out, int T, int S, int d,
                        hipStream_t s) {
  long long n = (long long)T * d;
  hipLaunchKernelGGL(embed_k, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, tok, W_E, W_pos, out, T, S, d);
  return hipGetLastError();
}

// ------------------------------------------------------------------ norm + quantise of one row held by a wave
// A wavefront holds one row of d = 64 E floats in registers x[0 .. E).  Two
// element-to-lane maps: the plain one (x[j] = element lane + 64 j, any E) and
// the vector one for E % 4 == 0 (x[4q + c] = element 4 (64 q + lane) + c), where
// every access is a 16-byte load or store and four codes leave as one word.
// All kernels of a launch family use the same map, so a row that enters two of
// them with the same values leaves with the same bits.
template <int MAXE, bool VEC>
__device__ __forceinline__ void row_load(float (&x)[MAXE], const float* p, int E, int lane) {
  if (VEC) {
#pragma unroll
    for (int q = 0; q < MAXE / 4; q++) if (4 * q < E) {
      float4 v = *(const float4*)(p + (q * 64 + lane) * 4);
      x[4 * q] = v.x; x[4 * q + 1] = v.y; x[4 * q + 2] = v.z; x[4 * q + 3] = v.w;
    }
  } else {
#pragma unroll
    for (int j = 0; j < MAXE; j++) if (j < E) x[j] = p[lane + 64 * j];
  }
}
// x += sign * p   (sign = +-1: the product is exact)
template <int MAXE, bool VEC>
__device__ __forceinline__ void row_axpy(float (&x)[MAXE], float sign, const float* p, int E, int lane) {
  if (VEC) {
#pragma unroll
    for (int q = 0; q < MAXE / 4; q++) if (4 * q < E) {
      float4 v = *(const float4*)(p + (q * 64 + lane) * 4);
      x[4 * q] += sign * v.x; x[4 * q + 1] += sign * v.y; x[4 * q + 2] += sign * v.z; x[4 * q + 3] += sign * v.w;
    }
  } else {
#pragma unroll
    for (int j = 0; j < MAXE; j++) if (j < E) x[j] += sign * p[lane + 64 * j];
  }
}
// y = a - p
template <int MAXE, bool VEC>
__device__ __forceinline__ void row_sub(float (&y)[MAXE], const float (&a)[MAXE], const float* p, int E, int lane) {
  if (VEC) {
#pragma unroll
    for (int q = 0; q < MAXE / 4; q++) if (4 * q < E) {
      float4 v = *(const float4*)(p + (q * 64 + lane) * 4);
      y[4 * q] = a[4 * q] - v.x; y[4 * q + 1] = a[4 * q + 1] - v.y;
      y[4 * q + 2] = a[4 * q + 2] - v.z; y[4 * q + 3] = a[4 * q + 3] - v.w;
    }
  } else {
#pragma unroll
    for (int j = 0; j < MAXE; j++) if (j < E) y[j] = a[j] - p[lane + 64 * j];
  }
}

// gain and offset of a norm, in the element map of the rows (offset only for LayerNorm)
template <int MAXE, bool VEC>
__device__ __forceinline__ void norm_params_load(float (&gn)[MAXE], float (&of)[MAXE], int E, int lane, int norm_kind,
                                                 const float* gain, const float* offset) {
  row_load<MAXE, VEC>(gn, gain, E, lane);
  if (norm_kind == 0) row_load<MAXE, VEC>(of, offset, E, lane);
}
template <int MAXE, bool VEC>
__device__ __forceinline__ void norm_row(float (&x)[MAXE], int E, int d, int lane, int norm_kind, float eps,
                                         const float (&gn)[MAXE], const float (&of)[MAXE]) {
  float inv_d = 1.0f / (float)d;
  float rstd;
  if (norm_kind == 0) {
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < MAXE; j++) if (j < E) s += x[j];
    float mean = wave_sum(s) * inv_d;
    float v = 0.f;
#pragma unroll
    for (int j = 0; j < MAXE; j++) if (j < E) { x[j] -= mean; v += x[j] * x[j]; }
    rstd = 1.0f / sqrtf(wave_sum(v) * inv_d + eps);
  } else {
    float v = 0.f;
#pragma unroll
    for (int j = 0; j < MAXE; j++) if (j < E) v += x[j] * x[j];
    rstd = 1.0f / sqrtf(wave_sum(v) * inv_d + eps);
  }
  if (norm_kind == 0) {
#pragma unroll
    for (int j = 0; j < MAXE; j++) if (j < E) x[j] = x[j] * rstd * gn[j] + of[j];
  } else {
#pragma unroll
    for (int j = 0; j < MAXE; j++) if (j < E) x[j] = x[j] * rstd * gn[j];
  }
}
template <int MAXE, bool VEC>
__device__ __forceinline__ void norm_row(float (&x)[MAXE], int E, int d, int lane, int norm_kind, float eps,
                                         const float* gain, const float* offset) {
  float gn[MAXE], of[MAXE];
  norm_params_load<MAXE, VEC>(gn, of, E, lane, norm_kind, gain, offset);
  norm_row<MAXE, VEC>(x, E, d, lane, norm_kind, eps, gn, of);
}

template <int MAXE, bool VEC>
__device__ __forceinline__ void emit_row(const float (&y)[MAXE], int E, int d, int lane, const GroupDesc& g,
                                         int inst, int row, int ldq) {
  if (g.out_f32) {
    float* o = g.out_f32 + inst * g.out_f32_is + (long long)row * d;
    if (VEC) {
#pragma unroll
      for (int q = 0; q < MAXE / 4; q++) if (4 * q < E)
        *(float4*)(o + (q * 64 + lane) * 4) = make_float4(y[4 * q], y[4 * q + 1], y[4 * q + 2], y[4 * q + 3]);
    } else {
#pragma unroll
      for (int j = 0; j < MAXE; j++) if (j < E) o[lane + 64 * j] = y[j];
    }
  }
  if (g.out_codes && g.qbits == 16) {
    // bfloat16 rows: two bytes per element, rows of exactly 2 d bytes (d is a multiple of 64: no padding; ldq is the
    // launch's stride for one-byte codes), no scale (the scale array gets 1 so that the product's epilogue is the same)
    uint8_t* o = g.out_codes + inst * g.out_codes_is + (long long)row * (2 * d);
    if (VEC) {
#pragma unroll
      for (int q = 0; q < MAXE / 4; q++) if (4 * q < E) {
        uint2 w;
        w.x = bf16_rne(y[4 * q]) | (bf16_rne(y[4 * q + 1]) << 16);
        w.y = bf16_rne(y[4 * q + 2]) | (bf16_rne(y[4 * q + 3]) << 16);
        *(uint2*)(o + (q * 64 + lane) * 8) = w;
      }
    } else {
#pragma unroll
      for (int j = 0; j < MAXE; j++) if (j < E) *(uint16_t*)(o + (lane + 64 * j) * 2) = (uint16_t)bf16_rne(y[j]);
    }
    if (lane == 0) g.out_scale[inst * g.out_scale_is + row] = 1.0f;
  } else if (g.out_codes) {
    float am = 0.f;
#pragma unroll
    for (int j = 0; j < MAXE; j++) if (j < E) am = fmaxf(am, fabsf(y[j]));
    am = wave_max(am);
    const int qb = g.qbits;
    float scale = (am == 0.f) ? 1.0f : am / q_top(qb);
    float inv = 1.0f / scale;
    uint8_t* o = g.out_codes + inst * g.out_codes_is + (long long)row * ldq;
    if (VEC) {
#pragma unroll
      for (int q = 0; q < MAXE / 4; q++) if (4 * q < E) {
        uint32_t w = q_encode4(y[4 * q] * inv, y[4 * q + 1] * inv, y[4 * q + 2] * inv, y[4 * q + 3] * inv, qb);
        *(uint32_t*)(o + (q * 64 + lane) * 4) = w;
      }
    } else {
#pragma unroll
      for (int j = 0; j < MAXE; j++) if (j < E) o[lane + 64 * j] = (uint8_t)q_encode(y[j] * inv, qb);
    }
    if (lane == 0) g.out_scale[inst * g.out_scale_is + row] = scale;
  }
}

// One wavefront per (group, row), blockIdx.z = a chunk of instances.  Everything that is the same for every
// instance -- a base without instance stride and the terms without one (cached sender tiles, senders
// recomputed once for all candidates) -- is summed once per row into x0 and reused for the instances of the
// chunk; with most edges removed that is the larger part of what a receiver's input is gathered from.  The
// arithmetic of an instance does not depend on the chunk size or on its place in the chunk.
template <int MAXE, bool VEC>
__global__ __launch_bounds__(256) void build_inputs_k(const GroupDesc* groups, const Term* terms, int T, int B,
                                                       int S, int d, int ldq, int norm_kind, float eps) {
  GroupDesc g = groups[blockIdx.y];
  int inst = blockIdx.z;
  int lane = threadIdx.x & 63;
  int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  int rows = g.last_only ? B : T;
  if (row >= rows) return;
  long long src = (long long)(g.last_only ? row * S + S - 1 : row) * d;
  // the vector forms with up to 16 values per lane are launched for exactly that width (PAHQ_DISPATCH_E): the width is
  // then a constant and every `j < E` below folds away
  const int E = (VEC && MAXE <= 16) ? MAXE : (d >> 6);
  float x[MAXE];
#pragma unroll
  for (int j = 0; j < MAXE; j++) x[j] = 0.f;
  // order of the sum: what every instance shares (a base without instance stride, terms without one), then the
  // instance's own base / stream, then its own terms -- the order build_inputs_shared_k takes, so that a group
  // gets the same bits from either kernel
  const Term* tt = terms + g.term_begin;
  const bool base_shared = g.base && g.base_is == 0;
  if (base_shared) row_load<MAXE, VEC>(x, g.base + src, E, lane);
  int n_dyn = 0;
  for (int t = 0; t < g.term_count; t++) {
    Term tm = tt[t];
    if (tm.inst_stride == 0) row_axpy<MAXE, VEC>(x, tm.sign, tm.p + src, E, lane);
    else n_dyn++;
  }
  if (g.base && !base_shared) row_axpy<MAXE, VEC>(x, 1.0f, g.base + inst * g.base_is + src, E, lane);
  if (g.run) row_axpy<MAXE, VEC>(x, 1.0f, g.run + inst * g.run_is + src, E, lane);
  if (n_dyn)
    for (int t = 0; t < g.term_count; t++) {
      Term tm = tt[t];
      if (tm.inst_stride != 0) row_axpy<MAXE, VEC>(x, tm.sign, tm.p + inst * tm.inst_stride + src, E, lane);
    }
  norm_row<MAXE, VEC>(x, E, d, lane, norm_kind, eps, g.gain, g.offset);
  emit_row<MAXE, VEC>(x, E, d, lane, g, inst, row, ldq);
}

// The same for groups that have terms every instance reads from the same tile (cached sender outputs, senders
// recomputed once for all candidates), blockIdx.z = a chunk of instances: those terms and a base without
// instance stride are summed once per row into x0 and reused for the instances of the chunk.  With most edges
// removed that is the larger part of what a receiver's input is gathered from.  The arithmetic of an instance
// does not depend on the chunk size or on its place in the chunk, and is that of the kernel above.
template <int MAXE, bool VEC>
__global__ __launch_bounds__(256) void build_inputs_shared_k(const GroupDesc* groups, const Term* terms, int T, int B,
                                                              int S, int d, int ldq, int norm_kind, float eps,
                                                              int n_inst, int chunk, int n_groups) {
  // Workgroup -> (row quad, group): all groups of a row quad run back to back on one XCD (workgroup id mod 8), so
  // that a sender row several receivers of the layer gather is fetched into that XCD's L2 once.
  const int xcd = blockIdx.x & 7, t_ = blockIdx.x >> 3;
  const int gi = t_ % n_groups, rq = (t_ / n_groups) * 8 + xcd;
  GroupDesc g = groups[gi];
  int lane = threadIdx.x & 63;
  int row = rq * 4 + (threadIdx.x >> 6);
  int rows = g.last_only ? B : T;
  if (row >= rows) return;
  long long src = (long long)(g.last_only ? row * S + S - 1 : row) * d;
  // the vector forms with up to 16 values per lane are launched for exactly that width (PAHQ_DISPATCH_E): the width is
  // then a constant and every `j < E` below folds away
  const int E = (VEC && MAXE <= 16) ? MAXE : (d >> 6);
  const Term* tt = terms + g.term_begin;
  const bool base_shared = g.base && g.base_is == 0;
  float x0[MAXE];
#pragma unroll
  for (int j = 0; j < MAXE; j++) x0[j] = 0.f;
  if (base_shared) row_load<MAXE, VEC>(x0, g.base + src, E, lane);
  int n_dyn = 0;
  for (int t = 0; t < g.term_count; t++) {
    Term tm = tt[t];
    if (tm.inst_stride == 0) row_axpy<MAXE, VEC>(x0, tm.sign, tm.p + src, E, lane);
    else n_dyn++;
  }
  float gn[MAXE], of[MAXE];               // read once for the chunk, not once per instance
  norm_params_load<MAXE, VEC>(gn, of, E, lane, norm_kind, g.gain, g.offset);
  const int i_end = min(n_inst, ((int)blockIdx.z + 1) * chunk);
  for (int inst = blockIdx.z * chunk; inst < i_end; inst++) {
    float x[MAXE];
#pragma unroll
    for (int j = 0; j < MAXE; j++) x[j] = x0[j];
    if (g.base && !base_shared) row_axpy<MAXE, VEC>(x, 1.0f, g.base + inst * g.base_is + src, E, lane);
    if (g.run) row_axpy<MAXE, VEC>(x, 1.0f, g.run + inst * g.run_is + src, E, lane);
    if (n_dyn)
      for (int t = 0; t < g.term_count; t++) {
        Term tm = tt[t];
        if (tm.inst_stride != 0) row_axpy<MAXE, VEC>(x, tm.sign, tm.p + inst * tm.inst_stride + src, E, lane);
      }
    norm_row<MAXE, VEC>(x, E, d, lane, norm_kind, eps, gn, of);
    emit_row<MAXE, VEC>(x, E, d, lane, g, inst, row, ldq);
  }
}

template <int MAXE, bool VEC>
__global__ __launch_bounds__(256) void patch_build_k(const GroupDesc* gp, const float* xv, const float* delta0,
                                                      long long delta_stride, const int* send, int n_inst, int mode,
                                                      int T, int B, int S, int d, int ldq, int norm_kind,
                                                      float eps) {
  GroupDesc g = *gp;
  int lane = threadIdx.x & 63;
  int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  int rows = g.last_only ? B : T;
  if (row >= rows) return;
  long long src = (long long)(g.last_only ? row * S + S - 1 : row) * d;
  // the vector forms with up to 16 values per lane are launched for exactly that width (PAHQ_DISPATCH_E): the width is
  // then a constant and every `j < E` below folds away
  const int E = (VEC && MAXE <= 16) ? MAXE : (d >> 6);
  float x0[MAXE], y[MAXE];
#pragma unroll
  for (int j = 0; j < MAXE; j++) x0[j] = 0.f;
  row_load<MAXE, VEC>(x0, xv + src, E, lane);
  for (int i = 0; i < n_inst; i++) {
#pragma unroll
    for (int j = 0; j < MAXE; j++) y[j] = 0.f;
    row_sub<MAXE, VEC>(y, x0, delta0 + (long long)send[i] * delta_stride + src, E, lane);
    if (mode == 2) {
#pragma unroll
      for (int j = 0; j < MAXE; j++) x0[j] = y[j];
    }
    norm_row<MAXE, VEC>(y, E, d, lane, norm_kind, eps, g.gain, g.offset);
    emit_row<MAXE, VEC>(y, E, d, lane, g, i, row, ldq);
  }
}

// Independent candidates (x_i = xv - delta[send[i]]): one wavefront per (row, instance).
template <int MAXE, bool VEC>
__global__ __launch_bounds__(256) void patch_indep_k(const GroupDesc* gp, const float* xv, const float* delta0,
                                                      long long delta_stride, const int* send, int T, int B, int S,
                                                      int d, int ldq, int norm_kind, float eps) {
  GroupDesc g = *gp;
  int lane = threadIdx.x & 63;
  int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  int inst = blockIdx.y;
  int rows = g.last_only ? B : T;
  if (row >= rows) return;
  long long src = (long long)(g.last_only ? row * S + S - 1 : row) * d;
  // the vector forms with up to 16 values per lane are launched for exactly that width (PAHQ_DISPATCH_E): the width is
  // then a constant and every `j < E` below folds away
  const int E = (VEC && MAXE <= 16) ? MAXE : (d >> 6);
  float x0[MAXE], y[MAXE];
#pragma unroll
  for (int j = 0; j < MAXE; j++) { x0[j] = 0.f; y[j] = 0.f; }
  row_load<MAXE, VEC>(x0, xv + src, E, lane);
  row_sub<MAXE, VEC>(y, x0, delta0 + (long long)send[inst] * delta_stride + src, E, lane);
  norm_row<MAXE, VEC>(y, E, d, lane, norm_kind, eps, g.gain, g.offset);
  emit_row<MAXE, VEC>(y, E, d, lane, g, inst, row, ldq);
}

// E % 4 == 0 takes the vector element map (all tiles, gains and code rows are 16-byte aligned
// there: d is a multiple of 256 floats and every buffer starts on a 256-byte boundary).
#define PAHQ_DISPATCH_E(E, CALL)                                    \
  do {                                                              \
    if ((E) == 4) { CALL(4, true); }                                \
    else if ((E) == 8) { CALL(8, true); }                           \
    else if ((E) == 12) { CALL(12, true); }                         \
    else if ((E) == 16) { CALL(16, true); }                         \
    else if ((E) % 4 == 0 && (E) <= 32) { CALL(32, true); }         \
    else if ((E) % 4 == 0) { CALL(64, true); }                      \
    else if ((E) <= 1) { CALL(1, false); }                          \
    else if ((E) <= 4) { CALL(4, false); }                          \
    else if ((E) <= 8) { CALL(8, false); }                          \
    else if ((E) <= 12) { CALL(12, false); }                        \
    else if ((E) <= 16) { CALL(16, false); }                        \
    else if ((E) <= 32) { CALL(32, false); }                        \
    else { CALL(64, false); }                                       \
  } while (0)

hipError_t launch_build_inputs(const GroupDesc* groups, int n_groups, const Term* terms, int n_inst, int T, int B,
                               int S, int d, int ldq, int norm_kind, float eps, int shared_terms, hipStream_t s) {
  if (n_groups == 0 || n_inst == 0) return hipSuccess;
  // Groups with instance-independent terms go to the kernel that sums those once per chunk of instances (wide
  // rows, more than 16 values per lane, have no registers to spare for the shared sum and stay with the plain
  // kernel).  Both kernels give a group the same bits.
  if (shared_terms > 0 && d / 64 <= 16) {
    long long blocks = (long long)((T + 3) / 4) * n_groups * n_inst;
    int chunk = (int)std::min<long long>(8, std::max<long long>(1, blocks / 16384));
    const int rq8 = ((T + 3) / 4 + 7) / 8 * 8;        // row quads, padded to the 8 XCDs (the padding exits at once)
    dim3 grid(rq8 * n_groups, 1, (n_inst + chunk - 1) / chunk);
#define CALL(M, V) hipLaunchKernelGGL((build_inputs_shared_k<M, V>), grid, dim3(256), 0, s, groups, terms, T, B, S, d, ldq, norm_kind, eps, n_inst, chunk, n_groups)
    PAHQ_DISPATCH_E(d / 64, CALL);
#undef CALL
    return hipGetLastError();
  }
  dim3 grid((T + 3) / 4, n_groups, n_inst);
#define CALL(M, V) hipLaunchKernelGGL((build_inputs_k<M, V>), grid, dim3(256), 0, s, groups, terms, T, B, S, d, ldq, norm_kind, eps)
  PAHQ_DISPATCH_E(d / 64, CALL);
#undef CALL
  return hipGetLastError();
}

hipError_t launch_patch_build(const GroupDesc* g, const float* xv, const float* delta0, long long delta_stride,
                              const int* send, int n_inst, int mode, int T, int B, int S, int d, int ldq,
                              int norm_kind, float eps, hipStream_t s) {
  if (n_inst == 0) return hipSuccess;
  if (mode == 1) {
    dim3 grid2((T + 3) / 4, n_inst);
#define CALL(M, V) hipLaunchKernelGGL((patch_indep_k<M, V>), grid2, dim3(256), 0, s, g, xv, delta0, delta_stride, send, T, B, S, d, ldq, norm_kind, eps)
    PAHQ_DISPATCH_E(d / 64, CALL);
#undef CALL
    return hipGetLastError();
  }
  dim3 grid((T + 3) / 4);
#define CALL(M, V) hipLaunchKernelGGL((patch_build_k<M, V>), grid, dim3(256), 0, s, g, xv, delta0, delta_stride, send, n_inst, mode, T, B, S, d, ldq, norm_kind, eps)
  PAHQ_DISPATCH_E(d / 64, CALL);
#undef CALL
  return hipGetLastError();
}

// ------------------------------------------------------------------ tile arithmetic
// Four senders' loads are in flight together; the subtractions keep the senders' order.
__global__ void xv_advance_k(float4* xv, const float* delta0, long long delta_stride, const int* send, int k,
                             long long n4) {
  long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n4) return;
  float4 x = xv[i];
  auto ld = [&](int j) { return *(const float4*)(delta0 + (long long)send[j] * delta_stride + i * 4); };
  auto sub = [&](const float4& v) { x.x -= v.x; x.y -= v.y; x.z -= v.z; x.w -= v.w; };
  int j = 0;
  for (; j + 4 <= k; j += 4) {
    const float4 v0 = ld(j), v1 = ld(j + 1), v2 = ld(j + 2), v3 = ld(j + 3);
    sub(v0); sub(v1); sub(v2); sub(v3);
  }
  for (; j < k; j++) sub(ld(j));
  xv[i] = x;
}
hipError_t launch_xv_advance(float* xv, const float* delta0, long long delta_stride, const int* send, int k,
                             long long n_elem, hipStream_t s) {
  if (k == 0) return hipSuccess;
  if (n_elem % 4 != 0 || delta_stride % 4 != 0) return hipErrorInvalidValue;
  const long long n4 = n_elem / 4;
  hipLaunchKernelGGL(xv_advance_k, dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, s, (float4*)xv, delta0,
                     delta_stride, send, k, n4);
  return hipGetLastError();
}

// out = base + sum of terms, or (sum of terms) + base when base_last: the two orders in which build_inputs_k
// adds a group's shared base (first) and an instance's stream (after the shared terms), so that a receiver's
// input built here has the bits the row kernels give the same sum.
__global__ void tile_lincomb_k(float* out, const float* base, const Term* terms, int n_terms, long long n,
                               int base_last) {
  long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  float x = (base && !base_last) ? base[i] : 0.f;
  for (int t = 0; t < n_terms; t++) x += terms[t].sign * terms[t].p[i];
  if (base && base_last) x += base[i];
  out[i] = x;
}
hipError_t launch_tile_lincomb(float* out, const float* base, const Term* terms, int n_terms, long long n_elem,
                               int base_last, hipStream_t s) {
  hipLaunchKernelGGL(tile_lincomb_k, dim3((unsigned)((n_elem + 255) / 256)), dim3(256), 0, s, out, base, terms,
                     n_terms, n_elem, base_last);
  return hipGetLastError();
}

__global__ void tile_sub_k(float4* out, const float4* a, const float4* b, long long n4) {
  long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n4) return;
  float4 x = a[i], y = b[i];
  out[i] = make_float4(x.x - y.x, x.y - y.y, x.z - y.z, x.w - y.w);
}
hipError_t launch_tile_sub(float* out, const float* a, const float* b, long long n_elem, hipStream_t s) {
  long long n4 = n_elem / 4;
  hipLaunchKernelGGL(tile_sub_k, dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, s, (float4*)out,
                     (const float4*)a, (const float4*)b, n4);
  return hipGetLastError();
}

// run_out = run_in + bias + sum_k src_k ; slot_k = src_k - sub_k
// A thread owns four values of up to four instances.  A dead layer's stand-ins arrive as tens of sources that are
// the same tile for every instance: each is loaded once for the thread's instances, four sources' loads are in
// flight together, and every instance's sum keeps the order of the sources.
__global__ void combine_k(const CombineDesc* descs, int di, const CombineSrc* srcs, long long n4, int d, int n_inst) {
  constexpr int IPT = 4;
  CombineDesc D = descs[di];
  const int inst0 = blockIdx.y * IPT, ni = min(IPT, n_inst - inst0);
  long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n4) return;
  long long e = i * 4;
  float4 acc[IPT];
  float4 b = make_float4(0.f, 0.f, 0.f, 0.f);
  if (D.bias) b = *(const float4*)(D.bias + (e % d));
#pragma unroll
  for (int q = 0; q < IPT; q++) {
    acc[q] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (q >= ni) continue;
    acc[q] = *(const float4*)(D.run_in + (inst0 + q) * D.run_in_is + e);
    if (D.bias) { acc[q].x += b.x; acc[q].y += b.y; acc[q].z += b.z; acc[q].w += b.w; }
  }
  auto shared = [&](const CombineSrc& s) { return (s.bcast || s.src_is == 0) && !s.slot; };
  auto ld = [&](const CombineSrc& s, int inst) {
    return s.bcast ? *(const float4*)(s.src + (e % d)) : *(const float4*)(s.src + inst * s.src_is + e);
  };
  auto add_all = [&](const float4& v) {
#pragma unroll
    for (int q = 0; q < IPT; q++) { acc[q].x += v.x; acc[q].y += v.y; acc[q].z += v.z; acc[q].w += v.w; }
  };
  const CombineSrc* sp = srcs + D.src_begin;
  int k = 0;
  while (k < D.n_src) {
    if (k + 4 <= D.n_src) {
      const CombineSrc s0 = sp[k], s1 = sp[k + 1], s2 = sp[k + 2], s3 = sp[k + 3];
      if (shared(s0) && shared(s1) && shared(s2) && shared(s3)) {
        const float4 v0 = ld(s0, 0), v1 = ld(s1, 0), v2 = ld(s2, 0), v3 = ld(s3, 0);
        add_all(v0); add_all(v1); add_all(v2); add_all(v3);
        k += 4;
        continue;
      }
    }
    const CombineSrc s0 = sp[k++];
    if (shared(s0)) { add_all(ld(s0, 0)); continue; }
#pragma unroll
    for (int q = 0; q < IPT; q++) {
      if (q >= ni) continue;
      float4 v = ld(s0, inst0 + q);
      acc[q].x += v.x; acc[q].y += v.y; acc[q].z += v.z; acc[q].w += v.w;
      if (s0.slot) {
        if (s0.sub) {
          float4 u = *(const float4*)(s0.sub + e);
          v.x -= u.x; v.y -= u.y; v.z -= u.z; v.w -= u.w;
        }
        *(float4*)(s0.slot + (inst0 + q) * s0.slot_is + e) = v;
      }
    }
  }
#pragma unroll
  for (int q = 0; q < IPT; q++)
    if (q < ni) *(float4*)(D.run_out + (inst0 + q) * D.run_out_is + e) = acc[q];
}
hipError_t launch_combine(const CombineDesc* descs, int desc_index, const CombineSrc* srcs, int n_inst,
                          long long n_elem, int d, hipStream_t s) {
  long long n4 = n_elem / 4;
  hipLaunchKernelGGL(combine_k, dim3((unsigned)((n4 + 255) / 256), (n_inst + 3) / 4), dim3(256), 0, s, descs,
                     desc_index, srcs, n4, d, n_inst);
  return hipGetLastError();
}

// ------------------------------------------------------------------ generic row quantiser (one block per row)
// act: 0 the value as it is, 1 tanh-GELU of it, 2 SwiGLU (silu(gate) * value)
__device__ __forceinline__ float hidden_act(float u, float g, int act) {
  if (act == 1) return gelu_tanh(u);
  if (act == 2) return g / (1.0f + expf(-g)) * u;
  return u;
}
__device__ __forceinline__ float hidden_value(const float* up, const float* gate, long long i, int act) {
  return hidden_act(up[i], act == 2 ? gate[i] : 0.f, act);
}

__global__ __launch_bounds__(256) void hidden_quant_k(const float* up, const float* gate, long long h_is,
                                                      uint8_t* codes, long long c_is, float* scale, long long s_is,
                                                      int T, int m, int ldq, int act, int qbits) {
  __shared__ float red[4];
  int inst = blockIdx.y, row = blockIdx.x;
  const float* pu = up + inst * h_is + (long long)row * m;
  const float* pg = gate ? gate + inst * h_is + (long long)row * m : nullptr;
  float am = 0.f;
  for (int i = threadIdx.x; i < m; i += 256) am = fmaxf(am, fabsf(hidden_value(pu, pg, i, act)));
  am = wave_max(am);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = am;
  __syncthreads();
  am = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
  float sc = (am == 0.f || qbits == 16) ? 1.0f : am / q_top(qbits);
  float inv = 1.0f / sc;
  uint8_t* o = codes + inst * c_is + (long long)row * ldq;
  if (qbits == 16) { for (int i = threadIdx.x; i < m; i += 256) *(uint16_t*)(o + 2 * i) = (uint16_t)bf16_rne(hidden_value(pu, pg, i, act)); }
  else
  for (int i = threadIdx.x; i < m; i += 256) o[i] = (uint8_t)q_encode(hidden_value(pu, pg, i, act) * inv, qbits);
  if (threadIdx.x == 0) scale[inst * s_is + row] = sc;
}
// The same quantiser for rows of 4-float multiples: TPR threads own a row (a wavefront, or the
// whole block for long rows), the row is read once with 16-byte loads and stays in registers
// between the abs-max and the encode, and four codes leave as one 32-bit store.
// The activation is a template parameter: as a run-time argument it costs a scalar branch per value.
template <int TPR, int NV, int ACT>
__global__ __launch_bounds__(256) void hidden_quant_vec_k(const float* up, const float* gate, long long h_is,
                                                          uint8_t* codes, long long c_is, float* scale,
                                                          long long s_is, int T, int m, int ldq, int qbits) {
  constexpr int act = ACT;
  constexpr int RPB = 256 / TPR;
  __shared__ float red[4];
  const int inst = blockIdx.y;
  const int row = blockIdx.x * RPB + (TPR == 64 ? (int)(threadIdx.x >> 6) : 0);
  const int t = (TPR == 64) ? (int)(threadIdx.x & 63) : (int)threadIdx.x;
  const bool live = row < T;
  // loads are unconditional so that all of a row's loads are in flight together: a row past the end re-reads
  // the last row, a group of four past the end of the row re-reads the last group; neither is stored
  const long long ro = (long long)min(row, T - 1) * m;
  const float* pu = up + inst * h_is + ro;
  const float* pg = (act == 2) ? gate + inst * h_is + ro : nullptr;
  float4 v[NV], g[NV];
#pragma unroll
  for (int j = 0; j < NV; j++) {
    const int e = min((j * TPR + t) * 4, m - 4);
    v[j] = gload4_nt(pu + e);
    if (act == 2) g[j] = gload4_nt(pg + e);
  }
  float am = 0.f;
#pragma unroll
  for (int j = 0; j < NV; j++) {
    if (act) {
      const float4 gg = (act == 2) ? g[j] : make_float4(0.f, 0.f, 0.f, 0.f);
      v[j].x = hidden_act(v[j].x, gg.x, act);
      v[j].y = hidden_act(v[j].y, gg.y, act);
      v[j].z = hidden_act(v[j].z, gg.z, act);
      v[j].w = hidden_act(v[j].w, gg.w, act);
    }
    if ((j * TPR + t) * 4 >= m) v[j] = make_float4(0.f, 0.f, 0.f, 0.f);
    am = fmaxf(fmaxf(am, fmaxf(fabsf(v[j].x), fabsf(v[j].y))), fmaxf(fabsf(v[j].z), fabsf(v[j].w)));
  }
  am = wave_max(am);
  if (TPR == 256) {
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = am;
    __syncthreads();
    am = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
  }
  if (!live) return;
  const float sc = (am == 0.f || qbits == 16) ? 1.0f : am / q_top(qbits);
  const float inv = 1.0f / sc;
  uint8_t* o = codes + inst * c_is + (long long)row * ldq;
  if (qbits == 16) {
#pragma unroll
    for (int j = 0; j < NV; j++) {
      int e = (j * TPR + t) * 4;
      if (e < m) {
        uint2 w;
        w.x = bf16_rne(v[j].x) | (bf16_rne(v[j].y) << 16);
        w.y = bf16_rne(v[j].z) | (bf16_rne(v[j].w) << 16);
        *(uint2*)(o + 2 * e) = w;
      }
    }
    if (t == 0) scale[inst * s_is + row] = 1.0f;
    return;
  }
#pragma unroll
  for (int j = 0; j < NV; j++) {
    int e = (j * TPR + t) * 4;
    if (e < m) {
      uint32_t w = q_encode4(v[j].x * inv, v[j].y * inv, v[j].z * inv, v[j].w * inv, qbits);
      *(uint32_t*)(o + e) = w;
    }
  }
  if (t == 0) scale[inst * s_is + row] = sc;
}

hipError_t launch_hidden_quant(const float* up, const float* gate, long long h_is, uint8_t* codes, long long c_is,
                               float* scale, long long s_is, int n_inst, int T, int m, int ldq, int act, int qbits,
                               hipStream_t s) {
  const int ca = qbits == 16 ? 8 : 4;       // bytes four codes take
  const bool vec = (m % 4 == 0) && (ldq % ca == 0) && (h_is % 4 == 0) && (c_is % ca == 0) &&
                   ((((uintptr_t)up) | ((uintptr_t)gate)) % 16 == 0) && (((uintptr_t)codes) % ca == 0);
#define HQV_(TPR_, NV_, ACT_)                                                                                    \
  hipLaunchKernelGGL((hidden_quant_vec_k<TPR_, NV_, ACT_>), dim3((T + 256 / TPR_ - 1) / (256 / TPR_), n_inst),   \
                     dim3(256), 0, s, up, gate, h_is, codes, c_is, scale, s_is, T, m, ldq, qbits)
#define HQV(TPR_, NV_)                                                                                           \
  do {                                                                                                           \
    if (act == 1) HQV_(TPR_, NV_, 1); else if (act == 2) HQV_(TPR_, NV_, 2); else HQV_(TPR_, NV_, 0);            \
  } while (0)
  if (vec && m <= 64 * 4 * 8) HQV(64, 8);
  else if (vec && m <= 64 * 4 * 12) HQV(64, 12);
  else if (vec && m <= 64 * 4 * 16) HQV(64, 16);
  else if (vec && m <= 256 * 4 * 8) HQV(256, 8);
  else if (vec && m <= 256 * 4 * 12) HQV(256, 12);
  else
    hipLaunchKernelGGL(hidden_quant_k, dim3(T, n_inst), dim3(256), 0, s, up, gate, h_is, codes, c_is, scale, s_is,
                       T, m, ldq, act, qbits);
#undef HQV
#undef HQV_
  return hipGetLastError();
}

__global__ void swiglu_f32_k(float* up, const float* gate, long long n) {
  long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  const float g = gate[i];
  up[i] = g / (1.0f + expf(-g)) * up[i];
}
hipError_t launch_swiglu_f32(float* up, const float* gate, long long n_elem, hipStream_t s) {
  if (n_elem == 0) return hipSuccess;
  hipLaunchKernelGGL(swiglu_f32_k, dim3((unsigned)((n_elem + 255) / 256)), dim3(256), 0, s, up, gate, n_elem);
  return hipGetLastError();
}

// The quantiser at the end of the gather / patch kernels (emit_row) on given rows: one wavefront per row, the
// row in the element map those kernels use.  cols a multiple of 64, at most 4096.
template <int MAXE, bool VEC>
__global__ __launch_bounds__(256) void emit_rows_k(const float* x, int rows, int d, uint8_t* codes, float* scales, int qbits) {
  const int lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  // the vector forms with up to 16 values per lane are launched for exactly that width (PAHQ_DISPATCH_E): the width is
  // then a constant and every `j < E` below folds away
  const int E = (VEC && MAXE <= 16) ? MAXE : (d >> 6);
  float y[MAXE];
#pragma unroll
  for (int j = 0; j < MAXE; j++) y[j] = 0.f;
  row_load<MAXE, VEC>(y, x + (long long)row * d, E, lane);
  GroupDesc g;
  g.out_f32 = nullptr; g.out_codes = codes; g.out_codes_is = 0; g.out_scale = scales; g.out_scale_is = 0; g.qbits = qbits;
  emit_row<MAXE, VEC>(y, E, d, lane, g, 0, row, d);
}
hipError_t launch_emit_rows(const float* x, int rows, int cols, uint8_t* codes, float* scales, int qbits, hipStream_t s) {
  if (rows == 0) return hipSuccess;
  if (cols % 64 != 0 || cols > 4096) return hipErrorInvalidValue;
  dim3 grid((rows + 3) / 4);
#define CALL(M, V) hipLaunchKernelGGL((emit_rows_k<M, V>), grid, dim3(256), 0, s, x, rows, cols, codes, scales, qbits)
  PAHQ_DISPATCH_E(cols / 64, CALL);
#undef CALL
  return hipGetLastError();
}

hipError_t launch_quant_rows_plain(const float* x, int rows, int cols, uint8_t* codes, float* scales, int qbits,
                                   hipStream_t s) {
  return launch_hidden_quant(x, nullptr, 0LL, codes, 0LL, scales, 0LL, 1, rows, cols, cols, 0, qbits, s);
}

}  // namespace pahq
