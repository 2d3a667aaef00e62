// Grouped GEMMs on the CDNA4 matrix cores.
//
// gemm_fp8: val = (A_codes * W_codes^T) * row_scale * col_scale, then the
//   epilogue of GemmProb (bias, GELU, residual add, second output).  Both
//   operands are FP8 E4M3 codes with K contiguous, K padded with zero codes to
//   a multiple of 128.  Two kernels:
//
//   gemm_x_k (exact sums, the default): codes are decoded to fp16 in registers
//   (V_CVT_SCALEF32_PK_F16_FP8, exact) and multiplied by V_MFMA_F32_16X16X32_F16:
//   exact products, fp32 sums.  Slabs of 128 K-bytes go from global memory
//   straight into LDS (GLOBAL_LOAD_LDS_DWORDX4), two stages, one barrier per
//   slab.  128 x 128 tile, four wavefronts of 64 x 64 (two decodes per MFMA; a
//   smaller wave tile is bound by instruction issue, not by the matrix cores).
//
//   gemm_fp8_k (PAHQ_MMA_FP8): V_MFMA_SCALE_F32_16X16X128_F8F6F4 with unit block
//   scales; its adder keeps a fixed-point window below the largest product of
//   an instruction (about 2^-13 of sum |a w| in the worst case).  128 x 64 tile,
//   slabs staged through registers into LDS rows padded to 144 bytes.
//
//   In both, W is the first MFMA operand, so a lane owns one output row of a
//   16 x 16 tile and four consecutive columns (16-byte stores); row scales,
//   column scales and the instance / row split are fetched before the K loop so
//   that the epilogue does not wait on them.  The workgroup -> tile map gives
//   each XCD (workgroup id mod 8) a contiguous range of tiles, column tiles
//   innermost, so the A rows of a tile are fetched into one L2 only.
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

// Eight e4m3 codes (two 32-bit words) -> eight fp16 values with the hardware
// converter (V_CVT_SCALEF32_PK_F16_FP8, scale 1): exact for every finite code,
// subnormals and signed zero included (checked over all 254 codes on gfx950).
__device__ __forceinline__ v8h decode8(uint32_t w0, uint32_t w1) {
  union { v8h h; v2h p[4]; } r;
  r.p[0] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(w0, 1.0f, false);
  r.p[1] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(w0, 1.0f, true);
  r.p[2] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(w1, 1.0f, false);
  r.p[3] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(w1, 1.0f, true);
  return r.h;
}

#define LDS_ROW 144   // gemm_fp8_k: 128 data bytes + 16 pad

// XCD-aware tile order: workgroup id w runs on XCD w % 8; that XCD gets the
// contiguous range [x * chunk, (x+1) * chunk) of the linear tile index.
__device__ __forceinline__ int xcd_tile(int wg, int total) {
  int chunk = (total + 7) >> 3;
  return (wg & 7) * chunk + (wg >> 3);
}

// One result element (the slow path: ragged column tail or unaligned rows).
__device__ __forceinline__ void epilogue_store(const GemmProb& P, int n, float acc, float sa, float sw, int inst,
                                               int r) {
  float val = acc * (sa * sw);
  float v = val;
  if (P.bias) v += P.bias[n];
  if (P.act == 1) v = gelu_tanh(v);
  long long off = (long long)r * P.ldc + n;
  if (P.add) v += P.add[inst * P.add_is + off];
  P.C[inst * P.c_is + off] = v;
  if (P.aux) {
    float x = val;
    if (P.aux_sub) x -= P.aux_sub[off];
    P.aux[inst * P.aux_is + off] = x;
  }
}

// What the epilogue needs besides the accumulators: fetched before the K loop.
template <int TM, int TN>
struct EpiPre {
  float sa[TM];      // row scale of row (mbase + 16 i + li)
  int inst[TM];      // its instance and row within the instance
  int row[TM];
  float sw[TN];      // column scale of columns nbase + 16 j + 4 lg .. + 3 (one slice when the fast path applies)
};
template <int TM, int TN>
__device__ __forceinline__ void epi_prefetch(EpiPre<TM, TN>& E, const GemmProb& P, int mbase, int nbase, int li,
                                             int lg) {
#pragma unroll
  for (int i = 0; i < TM; i++) {
    int m = min(mbase + i * 16 + li, P.M - 1);
    E.inst[i] = m / P.rpi;
    E.row[i] = m - E.inst[i] * P.rpi;
    E.sa[i] = P.ascale[E.inst[i] * P.as_is + (long long)E.row[i] * P.as_stride];
  }
#pragma unroll
  for (int j = 0; j < TN; j++) {
    int nb = min(nbase + j * 16 + lg * 4, P.N - 1);
    E.sw[j] = P.wscale[nb / P.wscale_block];
  }
}
// acc[i][j] holds, for lane (li, lg), row mbase + 16 i + li and columns nbase + 16 j + 4 lg .. + 3.
template <int TM, int TN>
__device__ __forceinline__ void epi_store(const EpiPre<TM, TN>& E, const GemmProb& P, const v4f (&acc)[TM][TN],
                                          int mbase, int nbase, int li, int lg) {
  const bool vec = ((P.ldc & 3) == 0) && ((P.wscale_block & 3) == 0) && (((P.c_is | P.add_is | P.aux_is) & 3) == 0) &&
                   ((((uintptr_t)P.C | (uintptr_t)P.add | (uintptr_t)P.aux | (uintptr_t)P.aux_sub | (uintptr_t)P.bias) & 15) == 0);
  float4 bias[TN];
#pragma unroll
  for (int j = 0; j < TN; j++) {
    int nb = nbase + j * 16 + lg * 4;
    bias[j] = (P.bias && vec && nb + 3 < P.N) ? *(const float4*)(P.bias + nb) : make_float4(0.f, 0.f, 0.f, 0.f);
  }
#pragma unroll
  for (int i = 0; i < TM; i++) {
    if (mbase + i * 16 + li >= P.M) continue;
    const int inst = E.inst[i], row = E.row[i];
    const float sa = E.sa[i];
#pragma unroll
    for (int j = 0; j < TN; j++) {
      int nb = nbase + j * 16 + lg * 4;
      if (nb >= P.N) continue;
      if (vec && nb + 3 < P.N) {
        float s2 = sa * E.sw[j];
        float4 val = make_float4(acc[i][j][0] * s2, acc[i][j][1] * s2, acc[i][j][2] * s2, acc[i][j][3] * s2);
        float4 v = make_float4(val.x + bias[j].x, val.y + bias[j].y, val.z + bias[j].z, val.w + bias[j].w);
        if (!P.bias) v = val;                  // keeps the sign of a zero result when there is no bias
        if (P.act == 1) { v.x = gelu_tanh(v.x); v.y = gelu_tanh(v.y); v.z = gelu_tanh(v.z); v.w = gelu_tanh(v.w); }
        long long off = (long long)row * P.ldc + nb;
        if (P.add) { float4 a = *(const float4*)(P.add + inst * P.add_is + off); v.x += a.x; v.y += a.y; v.z += a.z; v.w += a.w; }
        *(float4*)(P.C + inst * P.c_is + off) = v;
        if (P.aux) {
          if (P.aux_sub) { float4 u = *(const float4*)(P.aux_sub + off); val.x -= u.x; val.y -= u.y; val.z -= u.z; val.w -= u.w; }
          *(float4*)(P.aux + inst * P.aux_is + off) = val;
        }
      } else {
#pragma unroll
        for (int r = 0; r < 4; r++)
          if (nb + r < P.N)
            epilogue_store(P, nb + r, acc[i][j][r], sa, P.wscale[(nb + r) / P.wscale_block], inst, row);
      }
    }
  }
}

// ------------------------------------------------------------------ exact sums (fp16 matrix cores)
// LDS rows are 128 bytes without padding; the 16-byte chunk c of row r sits at chunk position
// c ^ (r & 7), so the 16-byte operand reads of 8 consecutive rows cover all 32 banks.  A load
// instruction fills 8 rows: lane l writes LDS bytes [16 l, 16 l + 16) behind a wave-uniform base,
// i.e. row l >> 3, position l & 7, and therefore fetches chunk (l & 7) ^ (l >> 3) of its row.
// Rows past M or N are clamped to the last valid row: they feed only results that are never stored.
// One 16-byte operand read feeds two MFMA steps: step 2 q + s takes bytes [64 q + 16 g + 8 s, + 8)
// of every row, the same k positions for both operands.
typedef __attribute__((address_space(1))) const void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;

template <int WAVES_M, int WAVES_N, int TM, int TN>
__global__ __launch_bounds__(WAVES_M* WAVES_N * 64, 2) void gemm_x_k(const GemmProb* probs) {
  constexpr int NW = WAVES_M * WAVES_N;
  constexpr int BM = WAVES_M * TM * 16, BN = WAVES_N * TN * 16, ROWS = BM + BN;
  constexpr int NI = ROWS / 8 / NW;            // load instructions per wave and slab (8 rows each)
  constexpr int STAGE = ROWS * 128;
  static_assert(ROWS % (8 * NW) == 0, "rows must split evenly over the waves");
  // two arrays, always addressed statically: the compiler then knows that the loads in flight
  // into one stage cannot alias the operand reads of the other and does not wait for them
  __shared__ __attribute__((aligned(1024))) uint8_t st0[STAGE];
  __shared__ __attribute__((aligned(1024))) uint8_t st1[STAGE];

  const GemmProb P = probs[blockIdx.y];
  const int mt = (P.M + BM - 1) / BM, nt = (P.N + BN - 1) / BN;
  const int lin = xcd_tile(blockIdx.x, mt * nt);
  if (lin >= mt * nt) return;
  const int m0 = (lin / nt) * BM, n0 = (lin % nt) * BN;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / WAVES_N, wn = wave % WAVES_N;
  const int li = lane & 15, lg = lane >> 4;

  const uint8_t* src[NI];
  const int cg = ((lane & 7) ^ (lane >> 3)) * 16;
#pragma unroll
  for (int t = 0; t < NI; t++) {
    int r = 8 * (wave * NI + t) + (lane >> 3);
    if (r < BM) {
      int m = min(m0 + r, P.M - 1);
      src[t] = (const uint8_t*)P.A + (long long)(m / P.rpi) * P.a_is + (long long)(m % P.rpi) * P.lda + cg;
    } else {
      int n = min(n0 + r - BM, P.N - 1);
      src[t] = (const uint8_t*)P.W + (long long)n * P.ldw + cg;
    }
  }
  auto issue = [&](uint8_t* st, int k0) {
#pragma unroll
    for (int t = 0; t < NI; t++)
      __builtin_amdgcn_global_load_lds((gptr_t)(src[t] + k0), (lptr_t)(st + (wave * NI + t) * 1024), 16, 0, 0);
  };
  issue(st0, 0);

  const int mbase = m0 + wm * TM * 16, nbase = n0 + wn * TN * 16;
  EpiPre<TM, TN> E;
  epi_prefetch<TM, TN>(E, P, mbase, nbase, li, lg);

  const int offA = (wm * TM * 16 + li) * 128, offB = (BM + wn * TN * 16 + li) * 128;
  const int sw0 = (lg ^ (li & 7)) * 16, sw1 = ((4 + lg) ^ (li & 7)) * 16;

  v4f acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; i++)
#pragma unroll
    for (int j = 0; j < TN; j++) acc[i][j] = (v4f){0.f, 0.f, 0.f, 0.f};

  auto compute = [&](const uint8_t* st) {
    const uint8_t* sA = st + offA;
    const uint8_t* sB = st + offB;
#pragma unroll
    for (int q = 0; q < 2; q++) {
      const int sw = q ? sw1 : sw0;
      v8h ha[TM][2];
#pragma unroll
      for (int i = 0; i < TM; i++) {
        uint4 w = *(const uint4*)(sA + i * 2048 + sw);
        ha[i][0] = decode8(w.x, w.y);
        ha[i][1] = decode8(w.z, w.w);
      }
#pragma unroll
      for (int j = 0; j < TN; j++) {
        uint4 w = *(const uint4*)(sB + j * 2048 + sw);
        v8h hb0 = decode8(w.x, w.y), hb1 = decode8(w.z, w.w);
#pragma unroll
        for (int i = 0; i < TM; i++) {
          acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(hb0, ha[i][0], acc[i][j], 0, 0, 0);
          acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(hb1, ha[i][1], acc[i][j], 0, 0, 0);
        }
      }
    }
  };

  // vmcnt(0) also covers the scale loads above; 0x0F70 = vmcnt 0, expcnt and lgkmcnt left alone
  for (int k0 = 0; k0 < P.K; k0 += 256) {
    __builtin_amdgcn_s_waitcnt(0x0F70);          // this wave's part of the slab has landed
    __syncthreads();                             // ... everyone's has, and the other stage is free
    if (k0 + 128 < P.K) issue(st1, k0 + 128);
    compute(st0);
    if (k0 + 128 >= P.K) break;
    __builtin_amdgcn_s_waitcnt(0x0F70);
    __syncthreads();
    if (k0 + 256 < P.K) issue(st0, k0 + 256);
    compute(st1);
  }
  epi_store<TM, TN>(E, P, acc, mbase, nbase, li, lg);
}

// ------------------------------------------------------------------ FP8 matrix-core instruction
// Lane layout of the instruction (lane = 16*g + i): the operand of lane (i, g) is row i, bytes
// [32g, 32g+32) of the slab.  WAVES_M x WAVES_N wavefronts; each owns a (BM / WAVES_M) x
// (BN / WAVES_N) sub-tile.
template <int BM, int BN, int WAVES_M, int WAVES_N>
__global__ __launch_bounds__(WAVES_M* WAVES_N * 64) void gemm_fp8_k(const GemmProb* probs) {
  constexpr int NT = WAVES_M * WAVES_N * 64;
  constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
  constexpr int TM = WM / 16, TN = WN / 16;
  constexpr int A_CH = BM * 8 / NT;     // 16-byte chunks per thread
  constexpr int B_CH = BN * 8 / NT;
  __shared__ __attribute__((aligned(16))) uint8_t sA[BM * LDS_ROW];
  __shared__ __attribute__((aligned(16))) uint8_t sB[BN * LDS_ROW];

  const GemmProb P = probs[blockIdx.y];
  const int mt = (P.M + BM - 1) / BM, nt = (P.N + BN - 1) / BN;
  const int lin = xcd_tile(blockIdx.x, mt * nt);
  if (lin >= mt * nt) return;
  const int m0 = (lin / nt) * BM, n0 = (lin % nt) * BN;
  const uint8_t* W = (const uint8_t*)P.W;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WAVES_N, wn = wave % WAVES_N;
  const int li = lane & 15, lg = lane >> 4;

  // global row pointers of this thread's chunks (rows of A may straddle instances)
  const uint8_t* pa[A_CH];
  const uint8_t* pb[B_CH];
#pragma unroll
  for (int c = 0; c < A_CH; c++) {
    int ch = tid + c * NT, r = ch >> 3, kc = ch & 7;
    int m = m0 + r;
    pa[c] = (m < P.M) ? (const uint8_t*)P.A + (long long)(m / P.rpi) * P.a_is + (long long)(m % P.rpi) * P.lda + kc * 16
                      : nullptr;
  }
#pragma unroll
  for (int c = 0; c < B_CH; c++) {
    int ch = tid + c * NT, r = ch >> 3, kc = ch & 7;
    int n = n0 + r;
    pb[c] = (n < P.N) ? W + (long long)n * P.ldw + kc * 16 : nullptr;
  }
  uint4 ra[A_CH], rb[B_CH];
  auto load_slab = [&](int k0) {
#pragma unroll
    for (int c = 0; c < A_CH; c++) ra[c] = pa[c] ? *(const uint4*)(pa[c] + k0) : make_uint4(0, 0, 0, 0);
#pragma unroll
    for (int c = 0; c < B_CH; c++) rb[c] = pb[c] ? *(const uint4*)(pb[c] + k0) : make_uint4(0, 0, 0, 0);
  };
  auto store_slab = [&]() {
#pragma unroll
    for (int c = 0; c < A_CH; c++) {
      int ch = tid + c * NT, r = ch >> 3, kc = ch & 7;
      *(uint4*)(sA + r * LDS_ROW + kc * 16) = ra[c];
    }
#pragma unroll
    for (int c = 0; c < B_CH; c++) {
      int ch = tid + c * NT, r = ch >> 3, kc = ch & 7;
      *(uint4*)(sB + r * LDS_ROW + kc * 16) = rb[c];
    }
  };

  v4f acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; i++)
#pragma unroll
    for (int j = 0; j < TN; j++) acc[i][j] = (v4f){0.f, 0.f, 0.f, 0.f};

  load_slab(0);
  const int mbase = m0 + wm * WM, nbase = n0 + wn * WN;
  EpiPre<TM, TN> E;
  epi_prefetch<TM, TN>(E, P, mbase, nbase, li, lg);
  for (int k0 = 0; k0 < P.K; k0 += 128) {
    __syncthreads();                 // previous slab fully consumed
    store_slab();
    __syncthreads();
    if (k0 + 128 < P.K) load_slab(k0 + 128);
    v8i fa[TM];
#pragma unroll
    for (int i = 0; i < TM; i++) {
      const uint8_t* p = sA + (wm * WM + i * 16 + li) * LDS_ROW + lg * 32;
      uint4 lo = *(const uint4*)p, hi = *(const uint4*)(p + 16);
      fa[i] = (v8i){(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w, (int)hi.x, (int)hi.y, (int)hi.z, (int)hi.w};
    }
#pragma unroll
    for (int j = 0; j < TN; j++) {
      const uint8_t* p = sB + (wn * WN + j * 16 + li) * LDS_ROW + lg * 32;
      uint4 lo = *(const uint4*)p, hi = *(const uint4*)(p + 16);
      v8i fb = (v8i){(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w, (int)hi.x, (int)hi.y, (int)hi.z, (int)hi.w};
#pragma unroll
      for (int i = 0; i < TM; i++)
        acc[i][j] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(fb, fa[i], acc[i][j], 0, 0, 0, 0x7F7F7F7F, 0,
                                                                     0x7F7F7F7F);
    }
  }
  epi_store<TM, TN>(E, P, acc, mbase, nbase, li, lg);
}

hipError_t launch_gemm_fp8(const GemmProb* probs, int n_probs, int max_M, int max_N, int exact, hipStream_t s) {
  if (n_probs == 0 || max_M == 0 || max_N == 0) return hipSuccess;
  if (exact && max_N > 64) {
    int tiles = ((max_M + 127) / 128) * ((max_N + 127) / 128);
    dim3 grid((tiles + 7) / 8 * 8, n_probs);
    hipLaunchKernelGGL((gemm_x_k<2, 2, 4, 4>), grid, dim3(256), 0, s, probs);
  } else {
    int tiles = ((max_M + 127) / 128) * ((max_N + 63) / 64);
    dim3 grid((tiles + 7) / 8 * 8, n_probs);
    if (exact) hipLaunchKernelGGL((gemm_x_k<4, 1, 2, 4>), grid, dim3(256), 0, s, probs);
    else hipLaunchKernelGGL((gemm_fp8_k<128, 64, 4, 1>), grid, dim3(256), 0, s, probs);
  }
  return hipGetLastError();
}

// ------------------------------------------------------------------ fp32
// 64 x 64 tile, K slabs of 32, four waves as 2 x 2, each 32 x 32 (2 x 2 MFMA tiles).
// MFMA 16x16x4 f32: A operand of lane (i, g) = A[i][g], B operand = B[g][i],
// result lane (i, g) holds C[4g + r][i].  Requires K % 4 == 0 and 16-byte aligned rows
// (true for d_model and d_head here); global loads are 16 bytes per lane.
__global__ __launch_bounds__(256) void gemm_f32_k(const GemmProb* probs) {
  __shared__ float sA[64][33];
  __shared__ float sB[32][65];
  const GemmProb P = probs[blockIdx.z];
  const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
  if (m0 >= P.M || n0 >= P.N) return;
  const float* W = (const float*)P.W;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int li = lane & 15, lg = lane >> 4;
  const int wm = wave >> 1, wn = wave & 1;
  // A tile 64 x 32 floats = 512 float4: thread -> rows (tid >> 3) and (tid >> 3) + 32, float4 column tid & 7
  const float* pa[2];
#pragma unroll
  for (int c = 0; c < 2; c++) {
    int m = m0 + (tid >> 3) + 32 * c;
    pa[c] = (m < P.M) ? (const float*)P.A + (long long)(m / P.rpi) * P.a_is + (long long)(m % P.rpi) * P.lda + (tid & 7) * 4
                      : nullptr;
  }
  // B tile 32 x 64 floats = 512 float4: thread -> k rows (tid >> 4) and (tid >> 4) + 16, float4 column tid & 15
  const int bn = n0 + (tid & 15) * 4;
  v4f acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; i++)
#pragma unroll
    for (int j = 0; j < 2; j++) acc[i][j] = (v4f){0.f, 0.f, 0.f, 0.f};

  for (int k0 = 0; k0 < P.K; k0 += 32) {
    float4 va[2], vb[2];
#pragma unroll
    for (int c = 0; c < 2; c++) {
      int k = k0 + (tid & 7) * 4;
      va[c] = (pa[c] && k + 3 < P.K) ? *(const float4*)(pa[c] + k0) : make_float4(0, 0, 0, 0);
      if (pa[c] && k < P.K && k + 3 >= P.K) {             // ragged K tail
        float t[4] = {0, 0, 0, 0};
        for (int q = 0; q < 4 && k + q < P.K; q++) t[q] = pa[c][k0 + q];
        va[c] = make_float4(t[0], t[1], t[2], t[3]);
      }
      int kb = k0 + (tid >> 4) + 16 * c;
      if (kb < P.K && bn + 3 < P.N && ((P.ldw & 3) == 0)) vb[c] = *(const float4*)(W + (long long)kb * P.ldw + bn);
      else {
        float t[4] = {0, 0, 0, 0};
        if (kb < P.K) for (int q = 0; q < 4 && bn + q < P.N; q++) t[q] = W[(long long)kb * P.ldw + bn + q];
        vb[c] = make_float4(t[0], t[1], t[2], t[3]);
      }
    }
    __syncthreads();
#pragma unroll
    for (int c = 0; c < 2; c++) {
      int r = (tid >> 3) + 32 * c, k = (tid & 7) * 4;
      sA[r][k] = va[c].x; sA[r][k + 1] = va[c].y; sA[r][k + 2] = va[c].z; sA[r][k + 3] = va[c].w;
      int kb = (tid >> 4) + 16 * c, n = (tid & 15) * 4;
      sB[kb][n] = vb[c].x; sB[kb][n + 1] = vb[c].y; sB[kb][n + 2] = vb[c].z; sB[kb][n + 3] = vb[c].w;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < 32; kk += 4) {
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
#pragma unroll
  for (int i = 0; i < 2; i++)
#pragma unroll
    for (int r = 0; r < 4; r++) {
      int m = m0 + wm * 32 + i * 16 + lg * 4 + r;
      if (m >= P.M) continue;
      int inst = m / P.rpi, row = m % P.rpi;
#pragma unroll
      for (int j = 0; j < 2; j++) {
        int n = n0 + wn * 32 + j * 16 + li;
        if (n >= P.N) continue;
        epilogue_store(P, n, acc[i][j][r], 1.0f, 1.0f, inst, row);
      }
    }
}

hipError_t launch_gemm_f32(const GemmProb* probs, int n_probs, int max_M, int max_N, hipStream_t s) {
  if (n_probs == 0 || max_M == 0 || max_N == 0) return hipSuccess;
  dim3 grid((max_N + 63) / 64, (max_M + 63) / 64, n_probs);
  hipLaunchKernelGGL(gemm_f32_k, grid, dim3(256), 0, s, probs);
  return hipGetLastError();
}

}  // namespace pahq
