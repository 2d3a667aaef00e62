// Grouped GEMMs on the CDNA4 matrix cores.
//
// gemm_fp8: C = (A_codes * W_codes^T) * row_scale * col_scale (+ bias, GELU).
//   Both operands are FP8 E4M3 codes with K contiguous; the products are
//   formed by V_MFMA_SCALE_F32_16X16X128_F8F6F4 with both block scales fixed
//   at 2^0, accumulating in fp32.  One workgroup (4 wavefronts) owns a BM x BN
//   output tile; K advances in slabs of 128 bytes staged through LDS (rows
//   padded to 144 bytes so that the 16 rows a quarter-wave reads fall into
//   distinct banks); the next slab is prefetched into registers while the
//   current one feeds the MFMAs.
//   Lane layout of the instruction (64 lanes, lane = 16*g + i): the A operand
//   of lane (i, g) is row i, bytes [32g, 32g+32) of the slab; B likewise for
//   column i; the result lane (i, g) holds C[4g + r][i], r = 0..3.
//   Only the pairing of A's and B's k positions matters for the product, and
//   both operands are loaded with the same byte -> (g, position) map.
//
// gemm_f32: plain fp32 C = A * W (+ bias) with V_MFMA_F32_16X16X4_F32 (true
//   fp32 multiply-accumulate) for the investigated head.
#include "kernels.h"
#include "device_util.h"

namespace pahq {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef _Float16 v8h __attribute__((ext_vector_type(8)));
typedef _Float16 v2h __attribute__((ext_vector_type(2)));

// Eight e4m3 codes (two 32-bit words) -> eight fp16 values, exactly.  Moving
// the 7 magnitude bits of a code to bits 13..7 of a half gives value * 2^-8 for
// normal and subnormal codes alike (both formats have the same subnormal
// structure); the multiplication by 256 is exact in fp16.
__device__ __forceinline__ v8h decode8(uint32_t w0, uint32_t w1) {
  union { v8h h; uint32_t u[4]; v2h p[4]; } r;
  uint32_t w[2] = {w0, w1};
#pragma unroll
  for (int q = 0; q < 2; q++) {
    uint32_t x = w[q];
    uint32_t b0 = x & 0xFFu, b1 = (x >> 8) & 0xFFu, b2 = (x >> 16) & 0xFFu, b3 = x >> 24;
    r.u[2 * q] = (((b0 & 0x7Fu) << 7) | ((b0 & 0x80u) << 8)) | ((((b1 & 0x7Fu) << 7) | ((b1 & 0x80u) << 8)) << 16);
    r.u[2 * q + 1] = (((b2 & 0x7Fu) << 7) | ((b2 & 0x80u) << 8)) | ((((b3 & 0x7Fu) << 7) | ((b3 & 0x80u) << 8)) << 16);
  }
  const v2h k256 = {(_Float16)256.0f, (_Float16)256.0f};
#pragma unroll
  for (int q = 0; q < 4; q++) r.p[q] = r.p[q] * k256;
  return r.h;
}

#define LDS_ROW 144   // 128 data bytes + 16 pad

// EXACT = false: FP8 matrix-core instruction (its adder keeps a fixed-point
// window below the largest product, about 2^-13 of sum|a*w| in the worst case).
// EXACT = true: the same codes decoded to fp16 and multiplied by
// V_MFMA_F32_16X16X32_F16: products exact, sums in fp32.
template <int BM, int BN, bool EXACT>
__global__ __launch_bounds__(256) void gemm_fp8_k(const GemmProb* probs, int n_inst) {
  constexpr int WM = BM / 4;            // rows per wave (4 waves stacked along M)
  constexpr int TM = WM / 16;           // 16-row MFMA tiles per wave
  constexpr int TN = BN / 16;
  constexpr int A_CH = BM * 8 / 256;    // 16-byte chunks per thread
  constexpr int B_CH = BN * 8 / 256;
  __shared__ __attribute__((aligned(16))) uint8_t sA[BM * LDS_ROW];
  __shared__ __attribute__((aligned(16))) uint8_t sB[BN * LDS_ROW];

  const int pi = blockIdx.z / n_inst, inst = blockIdx.z % n_inst;
  const GemmProb P = probs[pi];
  const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
  if (m0 >= P.M || n0 >= P.N) return;
  const uint8_t* A = (const uint8_t*)P.A + inst * P.a_is;
  const uint8_t* W = (const uint8_t*)P.W;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int li = lane & 15, lg = lane >> 4;

  uint4 ra[A_CH], rb[B_CH];
  auto load_slab = [&](int k0) {
#pragma unroll
    for (int c = 0; c < A_CH; c++) {
      int ch = tid + c * 256, r = ch >> 3, kc = ch & 7;
      int m = m0 + r;
      ra[c] = (m < P.M) ? *(const uint4*)(A + (long long)m * P.lda + k0 + kc * 16) : make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int c = 0; c < B_CH; c++) {
      int ch = tid + c * 256, r = ch >> 3, kc = ch & 7;
      int n = n0 + r;
      rb[c] = (n < P.N) ? *(const uint4*)(W + (long long)n * P.ldw + k0 + kc * 16) : make_uint4(0, 0, 0, 0);
    }
  };
  auto store_slab = [&]() {
#pragma unroll
    for (int c = 0; c < A_CH; c++) {
      int ch = tid + c * 256, r = ch >> 3, kc = ch & 7;
      *(uint4*)(sA + r * LDS_ROW + kc * 16) = ra[c];
    }
#pragma unroll
    for (int c = 0; c < B_CH; c++) {
      int ch = tid + c * 256, r = ch >> 3, kc = ch & 7;
      *(uint4*)(sB + r * LDS_ROW + kc * 16) = rb[c];
    }
  };

  v4f acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; i++)
#pragma unroll
    for (int j = 0; j < TN; j++) acc[i][j] = (v4f){0.f, 0.f, 0.f, 0.f};

  load_slab(0);
  for (int k0 = 0; k0 < P.K; k0 += 128) {
    __syncthreads();                 // previous slab fully consumed
    store_slab();
    __syncthreads();
    if (k0 + 128 < P.K) load_slab(k0 + 128);
    if (EXACT) {
#pragma unroll
      for (int kk = 0; kk < 4; kk++) {
        v8h ha[TM], hb[TN];
#pragma unroll
        for (int i = 0; i < TM; i++) {
          uint2 w = *(const uint2*)(sA + (wave * WM + i * 16 + li) * LDS_ROW + kk * 32 + lg * 8);
          ha[i] = decode8(w.x, w.y);
        }
#pragma unroll
        for (int j = 0; j < TN; j++) {
          uint2 w = *(const uint2*)(sB + (j * 16 + li) * LDS_ROW + kk * 32 + lg * 8);
          hb[j] = decode8(w.x, w.y);
        }
#pragma unroll
        for (int i = 0; i < TM; i++)
#pragma unroll
          for (int j = 0; j < TN; j++)
            acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(ha[i], hb[j], acc[i][j], 0, 0, 0);
      }
      continue;
    }
    v8i fa[TM], fb[TN];
#pragma unroll
    for (int i = 0; i < TM; i++) {
      const uint8_t* p = sA + (wave * WM + i * 16 + li) * LDS_ROW + lg * 32;
      uint4 lo = *(const uint4*)p, hi = *(const uint4*)(p + 16);
      fa[i] = (v8i){(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w, (int)hi.x, (int)hi.y, (int)hi.z, (int)hi.w};
    }
#pragma unroll
    for (int j = 0; j < TN; j++) {
      const uint8_t* p = sB + (j * 16 + li) * LDS_ROW + lg * 32;
      uint4 lo = *(const uint4*)p, hi = *(const uint4*)(p + 16);
      fb[j] = (v8i){(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w, (int)hi.x, (int)hi.y, (int)hi.z, (int)hi.w};
    }
#pragma unroll
    for (int i = 0; i < TM; i++)
#pragma unroll
      for (int j = 0; j < TN; j++)
        acc[i][j] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(fa[i], fb[j], acc[i][j], 0, 0, 0, 0x7F7F7F7F,
                                                                     0, 0x7F7F7F7F);
  }

  float* C = P.C + inst * P.c_is;
  const float* as = P.ascale + inst * P.as_is;
#pragma unroll
  for (int i = 0; i < TM; i++) {
#pragma unroll
    for (int r = 0; r < 4; r++) {
      int m = m0 + wave * WM + i * 16 + lg * 4 + r;
      if (m >= P.M) continue;
      float sa = as[(long long)m * P.as_stride];
#pragma unroll
      for (int j = 0; j < TN; j++) {
        int n = n0 + j * 16 + li;
        if (n >= P.N) continue;
        float v = acc[i][j][r] * sa * P.wscale[n / P.wscale_block];
        if (P.bias) v += P.bias[n];
        if (P.act == 1) v = gelu_tanh(v);
        C[(long long)m * P.ldc + n] = v;
      }
    }
  }
}

hipError_t launch_gemm_fp8(const GemmProb* probs, int n_probs, int n_inst, int max_M, int max_N, int exact,
                           hipStream_t s) {
  if (n_probs == 0 || n_inst == 0) return hipSuccess;
  constexpr int BM = 128, BN = 64;
  dim3 grid((max_N + BN - 1) / BN, (max_M + BM - 1) / BM, n_probs * n_inst);
  if (exact) hipLaunchKernelGGL((gemm_fp8_k<BM, BN, true>), grid, dim3(256), 0, s, probs, n_inst);
  else hipLaunchKernelGGL((gemm_fp8_k<BM, BN, false>), grid, dim3(256), 0, s, probs, n_inst);
  return hipGetLastError();
}

// ------------------------------------------------------------------ fp32
// 64 x 64 tile, K slabs of 16, four waves as 2 x 2, each 32 x 32 (2 x 2 MFMA tiles).
// MFMA 16x16x4 f32: A operand of lane (i, g) = A[i][g], B operand = B[g][i],
// result lane (i, g) holds C[4g + r][i].
__global__ __launch_bounds__(256) void gemm_f32_k(const GemmProb* probs, int n_inst) {
  __shared__ float sA[64][17];
  __shared__ float sB[16][65];
  const int pi = blockIdx.z / n_inst, inst = blockIdx.z % n_inst;
  const GemmProb P = probs[pi];
  const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
  if (m0 >= P.M || n0 >= P.N) return;
  const float* A = (const float*)P.A + inst * P.a_is;
  const float* W = (const float*)P.W;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int li = lane & 15, lg = lane >> 4;
  const int wm = wave >> 1, wn = wave & 1;
  v4f acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; i++)
#pragma unroll
    for (int j = 0; j < 2; j++) acc[i][j] = (v4f){0.f, 0.f, 0.f, 0.f};

  for (int k0 = 0; k0 < P.K; k0 += 16) {
    __syncthreads();
#pragma unroll
    for (int c = 0; c < 4; c++) {               // A tile 64 x 16
      int idx = tid + c * 256, r = idx >> 4, k = idx & 15;
      int m = m0 + r;
      sA[r][k] = (m < P.M && k0 + k < P.K) ? A[(long long)m * P.lda + k0 + k] : 0.f;
    }
#pragma unroll
    for (int c = 0; c < 4; c++) {               // B tile 16 x 64
      int idx = tid + c * 256, k = idx >> 6, n = idx & 63;
      sB[k][n] = (n0 + n < P.N && k0 + k < P.K) ? W[(long long)(k0 + k) * P.ldw + n0 + n] : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < 16; kk += 4) {
      float fa[2], fb[2];
#pragma unroll
      for (int i = 0; i < 2; i++) fa[i] = sA[wm * 32 + i * 16 + li][kk + lg];
#pragma unroll
      for (int j = 0; j < 2; j++) fb[j] = sB[kk + lg][wn * 32 + j * 16 + li];
#pragma unroll
      for (int i = 0; i < 2; i++)
#pragma unroll
        for (int j = 0; j < 2; j++) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x4f32(fa[i], fb[j], acc[i][j], 0, 0, 0);
    }
  }
  float* C = P.C + inst * P.c_is;
#pragma unroll
  for (int i = 0; i < 2; i++)
#pragma unroll
    for (int r = 0; r < 4; r++) {
      int m = m0 + wm * 32 + i * 16 + lg * 4 + r;
      if (m >= P.M) continue;
#pragma unroll
      for (int j = 0; j < 2; j++) {
        int n = n0 + wn * 32 + j * 16 + li;
        if (n >= P.N) continue;
        float v = acc[i][j][r];
        if (P.bias) v += P.bias[n];
        C[(long long)m * P.ldc + n] = v;
      }
    }
}

hipError_t launch_gemm_f32(const GemmProb* probs, int n_probs, int n_inst, int max_M, int max_N, hipStream_t s) {
  if (n_probs == 0 || n_inst == 0) return hipSuccess;
  dim3 grid((max_N + 63) / 64, (max_M + 63) / 64, n_probs * n_inst);
  hipLaunchKernelGGL(gemm_f32_k, grid, dim3(256), 0, s, probs, n_inst);
  return hipGetLastError();
}

}  // namespace pahq
