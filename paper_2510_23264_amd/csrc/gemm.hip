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
#include <atomic>
#include "kernels.h"
#include "device_util.h"
#include "mma_util.h"

namespace pahq {

#define LDS_ROW 144   // gemm_fp8_k: 128 data bytes + 16 pad

// One result element (the slow path: ragged column tail or unaligned rows).
__device__ __forceinline__ void epilogue_store(const GemmProb& P, int n, float acc, float sa, float sw, int inst,
                                               int r) {
  float val = acc * (sa * sw);
  float v = val;
  if (P.bias) v += GCF(P.bias)[n];
  if (P.act == 1) v = gelu_tanh(v);
  long long off = (long long)r * P.ldc + n;
  if (P.add) v += GCF(P.add)[inst * P.add_is + off];
  GF(P.C)[inst * P.c_is + off] = v;
  if (P.aux) {
    float x = val;
    if (P.aux_sub) x -= GCF(P.aux_sub)[off];
    GF(P.aux)[inst * P.aux_is + off] = x;
  }
}

// What the epilogue needs besides the accumulators: fetched before the K loop.
template <int TM, int TN>
struct EpiPre {
  float sa[TM];      // row scale of row (mbase + 16 i + li)
  int inst[TM];      // its instance and row within the instance
  int row[TM];
  float sw[TN];      // column scale of columns nbase + 16 j + 4 lg .. + 3 (they share one weight slice)
  float4 bias[TN];   // bias of those columns (zero without a bias)
};
// Row m0 + r of a problem whose instances have rpi rows each: (instance, row in the instance), from the
// split (i0, r0) of m0.  One wrap covers tiles that are not taller than an instance; shorter
// instances take the loop.
__device__ __forceinline__ void split_row(int i0, int r0, int r, int rpi, int& inst, int& row) {
  inst = i0; row = r0 + r;
  while (row >= rpi) { row -= rpi; inst++; }
}
__device__ __forceinline__ int wscale_index(const GemmProb& P, int n) {
  if (P.wscale_block >= P.N) return 0;
  return P.ws_shift >= 0 ? (n >> P.ws_shift) : n / P.wscale_block;
}
template <int TM, int TN>
__device__ __forceinline__ void epi_prefetch(EpiPre<TM, TN>& E, const GemmProb& P, int m0, int i0, int r0, int mbase,
                                             int nbase, int li, int lg) {
#pragma unroll
  for (int i = 0; i < TM; i++) {
    int m = min(mbase + i * 16 + li, P.M - 1);
    split_row(i0, r0, m - m0, P.rpi, E.inst[i], E.row[i]);
    E.sa[i] = GCF(P.ascale)[E.inst[i] * P.as_is + (long long)E.row[i] * P.as_stride];
  }
#pragma unroll
  for (int j = 0; j < TN; j++) {
    int nb = nbase + j * 16 + lg * 4;
    E.sw[j] = GCF(P.wscale)[wscale_index(P, min(nb, P.N - 1))];
    // one 16-byte load, no divergence: a group past the last one re-reads the last one (its results are
    // never stored), and the last group may read up to three floats behind bias[N - 1] (the bias
    // arrays of this library are followed by padding; the values land in the padding of the C row)
    E.bias[j] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (P.bias) E.bias[j] = gload4(P.bias + min(nb, (P.N - 1) & ~3));
  }
}
// acc[i][j] holds, for lane (li, lg), row mbase + 16 i + li and columns nbase + 16 j + 4 lg .. + 3.
// Every store is 16 bytes: rows, instance strides and pointers are 16-byte aligned and a last,
// partial group of columns is written whole into the padding the row has behind column N
// (gemm8_prob_ok on the host guarantees all of this).
template <int TM, int TN>
__device__ __forceinline__ void epi_store(const EpiPre<TM, TN>& E, const GemmProb& P, const v4f (&acc)[TM][TN],
                                          int mbase, int nbase, int li, int lg) {
#pragma unroll
  for (int i = 0; i < TM; i++) {
    if (mbase + i * 16 + li >= P.M) continue;
    const int inst = E.inst[i], row = E.row[i];
    const float sa = E.sa[i];
#pragma unroll
    for (int j = 0; j < TN; j++) {
      int nb = nbase + j * 16 + lg * 4;
      if (nb >= P.N) continue;
      float s2 = sa * E.sw[j];
      float4 val = make_float4(acc[i][j][0] * s2, acc[i][j][1] * s2, acc[i][j][2] * s2, acc[i][j][3] * s2);
      float4 v = val;
      if (P.bias) { v.x += E.bias[j].x; v.y += E.bias[j].y; v.z += E.bias[j].z; v.w += E.bias[j].w; }
      if (P.act == 1) { v.x = gelu_tanh(v.x); v.y = gelu_tanh(v.y); v.z = gelu_tanh(v.z); v.w = gelu_tanh(v.w); }
      long long off = (long long)row * P.ldc + nb;
      if (P.add) { float4 a = gload4(P.add + inst * P.add_is + off); v.x += a.x; v.y += a.y; v.z += a.z; v.w += a.w; }
      gstore4(P.C + inst * P.c_is + off, v);
      if (P.aux) {
        if (P.aux_sub) { float4 u = gload4(P.aux_sub + off); val.x -= u.x; val.y -= u.y; val.z -= u.z; val.w -= u.w; }
        gstore4(P.aux + inst * P.aux_is + off, val);
      }
    }
  }
}

// The log-softmax / KL epilogue (the unembedding of a scored pass): nothing of a row has to reach
// memory but, per 64-column part of it, the running maximum, the sum of exponentials against it and
// the part's share of sum_v p_ref[v] (ref[v] - x[v]), p_ref[v] = exp(ref[v] - logz_ref).  A lane holds 16 values of a row (four groups
// of four columns); the four lanes that share the row combine through two shuffles.  Columns past N
// count as -3e38 (their exponentials vanish) and have p_ref = 0.  The order of every sum is fixed by the lane layout alone, so equal
// logits give equal parts whatever the problem's number of rows.
template <int TM, int TN>
__device__ __forceinline__ void epi_kl(const EpiPre<TM, TN>& E, const GemmProb& P, const v4f (&acc)[TM][TN],
                                       int mbase, int nbase, int li, int lg, int part) {
  const float NEG = -3.0e38f;
#pragma unroll
  for (int i = 0; i < TM; i++) {
    const int m = mbase + i * 16 + li;
    const bool row_on = m < P.M;
    const int inst = E.inst[i], row = E.row[i];
    float c[TN][4];
    float mx = NEG;
    const float lzr = P.kl_ref ? (float)P.kl_ref_logz[row] : 0.f;
#pragma unroll
    for (int j = 0; j < TN; j++) {
      const int nb = nbase + j * 16 + lg * 4;
      const float s2 = E.sa[i] * E.sw[j];
      float4 v = make_float4(acc[i][j][0] * s2, acc[i][j][1] * s2, acc[i][j][2] * s2, acc[i][j][3] * s2);
      if (P.bias) { v.x += E.bias[j].x; v.y += E.bias[j].y; v.z += E.bias[j].z; v.w += E.bias[j].w; }
      if (P.C && row_on && nb < P.N) gstore4(P.C + inst * P.c_is + (long long)row * P.ldc + nb, v);
      c[j][0] = nb + 0 < P.N ? v.x : NEG; c[j][1] = nb + 1 < P.N ? v.y : NEG;
      c[j][2] = nb + 2 < P.N ? v.z : NEG; c[j][3] = nb + 3 < P.N ? v.w : NEG;
      mx = fmaxf(fmaxf(mx, fmaxf(c[j][0], c[j][1])), fmaxf(c[j][2], c[j][3]));
    }
    float se = 0.f, a = 0.f;
#pragma unroll
    for (int j = 0; j < TN; j++) {
      const int nb = nbase + j * 16 + lg * 4;
#pragma unroll
      for (int r = 0; r < 4; r++) se += (c[j][r] > -1.0e38f) ? __expf(c[j][r] - mx) : 0.f;
      if (P.kl_ref && row_on && nb < P.N) {
        // reference probabilities from the reference logits (one fast exponential each, relative error 1e-6,
        // instead of a second load); a column past N has p = 0 exactly through the select
        const float4 rr = gload4(P.kl_ref + (long long)row * P.ldc + nb);
        const float p0 = __expf(rr.x - lzr), p1 = nb + 1 < P.N ? __expf(rr.y - lzr) : 0.f,
                    p2 = nb + 2 < P.N ? __expf(rr.z - lzr) : 0.f, p3 = nb + 3 < P.N ? __expf(rr.w - lzr) : 0.f;
        a += p0 * (rr.x - c[j][0]) + p1 * (rr.y - c[j][1]) + p2 * (rr.z - c[j][2]) + p3 * (rr.w - c[j][3]);
      }
    }
    float ma = fmaxf(mx, __shfl_xor(mx, 16, 64));
    ma = fmaxf(ma, __shfl_xor(ma, 32, 64));
    se *= __expf(mx - ma);                 // 0 * exp(0) for a lane whose columns are all past N
    se += __shfl_xor(se, 16, 64); se += __shfl_xor(se, 32, 64);
    a += __shfl_xor(a, 16, 64); a += __shfl_xor(a, 32, 64);
    if (lg == 0 && row_on) gstore4(P.kl_part + ((long long)m * P.kl_npart + part) * 4, make_float4(ma, se, a, 0.f));
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
//
// Workgroups are persistent: the gridDim.x / 8 workgroups of an XCD walk that XCD's tile range
// round-robin, so that the first slab of the next tile, its scales and its bias can be requested
// while the last slab of this tile is multiplied, and the next K loop starts while the stores of
// this tile are still in flight.

// B16: the rows hold bfloat16 patterns instead of e4m3 codes.  Nothing changes on the way into LDS (rows of 128
// bytes, K counted in bytes); a 16-byte operand read is then eight elements, one step of V_MFMA_F32_16X16X32_BF16,
// with no conversion (products of two bfloat16 numbers are exact in binary32, as those of two e4m3 codes are).
template <int WAVES_M, int WAVES_N, int TM, int TN, bool B16 = false>
__global__ __launch_bounds__(WAVES_M* WAVES_N * 64, 2) void gemm_x_k(const GemmProb* probs) {
  constexpr int NW = WAVES_M * WAVES_N;
  constexpr int BM = WAVES_M * TM * 16, BN = WAVES_N * TN * 16, ROWS = BM + BN;
  constexpr int NI = ROWS / 8 / NW;            // load instructions per wave and slab (8 rows each)
  constexpr int STAGE = ROWS * 128;
  static_assert(ROWS % (8 * NW) == 0, "rows must split evenly over the waves");
  static_assert(TM * TN < 64, "vmcnt has six bits");
  __shared__ __attribute__((aligned(1024))) uint8_t st0[STAGE];
  __shared__ __attribute__((aligned(1024))) uint8_t st1[STAGE];

  const GemmProb P = probs[blockIdx.y];
  const int mt = (P.M + BM - 1) / BM, nt = (P.N + BN - 1) / BN, total = mt * nt;
  const int chunk = (total + 7) >> 3, xcd = blockIdx.x & 7, per = gridDim.x >> 3;
  const int jend = min(chunk, total - xcd * chunk);
  int j = blockIdx.x >> 3;
  if (j >= jend) return;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / WAVES_N, wn = wave % WAVES_N;
  const int li = lane & 15, lg = lane >> 4;

  const uint8_t* src[NI];
  const int cg = ((lane & 7) ^ (lane >> 3)) * 16;
  auto set_src = [&](int m0, int n0) {
    const int i0 = m0 / P.rpi, r0 = m0 - i0 * P.rpi;
#pragma unroll
    for (int t = 0; t < NI; t++) {
      int r = 8 * (wave * NI + t) + (lane >> 3);
      if (r < BM) {
        int m = min(m0 + r, P.M - 1), inst, row;
        split_row(i0, r0, m - m0, P.rpi, inst, row);
        src[t] = (const uint8_t*)P.A + (long long)inst * P.a_is + (long long)row * P.lda + cg;
      } else {
        int n = min(n0 + r - BM, P.N - 1);
        src[t] = (const uint8_t*)P.W + (long long)n * P.ldw + cg;
      }
    }
  };
  auto issue = [&](const uint8_t* st, int k0) {
    const uint32_t base = __builtin_amdgcn_readfirstlane(lds_addr_of(st) + wave * NI * 1024);
#pragma unroll
    for (int t = 0; t < NI; t++) slab_load16(src[t] + k0, base + t * 1024);
  };

  const int offA = (wm * TM * 16 + li) * 128, offB = (BM + wn * TN * 16 + li) * 128;
  const int sw0 = (lg ^ (li & 7)) * 16, sw1 = ((4 + lg) ^ (li & 7)) * 16;
  v4f acc[TM][TN];
  auto compute = [&](const uint8_t* st) {
    const uint8_t* sA = st + offA;
    const uint8_t* sB = st + offB;
    if constexpr (B16) {
#pragma unroll
      for (int q = 0; q < 2; q++) {
        const int sw = q ? sw1 : sw0;
        union U { uint4 u; v8bf h; };
        U ha[TM];
#pragma unroll
        for (int i = 0; i < TM; i++) ha[i].u = *(const uint4*)(sA + i * 2048 + sw);
#pragma unroll
        for (int jj = 0; jj < TN; jj++) {
          U hb; hb.u = *(const uint4*)(sB + jj * 2048 + sw);
#pragma unroll
          for (int i = 0; i < TM; i++) acc[i][jj] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(hb.h, ha[i].h, acc[i][jj], 0, 0, 0);
        }
      }
      return;
    }
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
      for (int jj = 0; jj < TN; jj++) {
        uint4 w = *(const uint4*)(sB + jj * 2048 + sw);
        v8h hb0 = decode8(w.x, w.y), hb1 = decode8(w.z, w.w);
#pragma unroll
        for (int i = 0; i < TM; i++) {
          acc[i][jj] = __builtin_amdgcn_mfma_f32_16x16x32_f16(hb0, ha[i][0], acc[i][jj], 0, 0, 0);
          acc[i][jj] = __builtin_amdgcn_mfma_f32_16x16x32_f16(hb1, ha[i][1], acc[i][jj], 0, 0, 0);
        }
      }
    }
  };

  int lin = xcd * chunk + j;
  // Order of an XCD's tiles: neighbours share the larger operand.  With more weight rows than activation rows (the
  // unembedding: 50 257 columns against a few thousand rows) consecutive tiles walk down the rows of one column tile, so
  // that the weights cross HBM once and the small activation block is what the L2 re-serves; otherwise row tile first.
  const bool col_first = P.N > P.M;
  auto origin = [&](int t, int& mo, int& no) {
    if (col_first) { mo = (t % mt) * BM; no = (t / mt) * BN; } else { mo = (t / nt) * BM; no = (t % nt) * BN; }
  };
  int m0, n0;
  origin(lin, m0, n0);
  set_src(m0, n0);
  issue(st0, 0);
  // With an even number of slabs the last slab of a tile sits in st1 while st0 is idle: the first
  // slab of the next tile is requested there, a whole slab of MFMAs before it is needed, and the
  // K loop of the next tile starts with nothing but a barrier while the stores of this tile are
  // still in flight.  Row scales, column scales and bias of a tile are requested when its K loop
  // starts and are waited for together with its second slab.
  const bool even = (P.K & 255) == 0;
  bool slab0_here = false;           // this wave's part of slab 0 of the current tile has been waited for

  for (;;) {
#pragma unroll
    for (int i = 0; i < TM; i++)
#pragma unroll
      for (int jj = 0; jj < TN; jj++) acc[i][jj] = (v4f){0.f, 0.f, 0.f, 0.f};

    const int mbase = m0 + wm * TM * 16, nbase = n0 + wn * TN * 16;
    const int jn = j + per;
    const bool more = jn < jend;
    int m0n = 0, n0n = 0;
    if (more) origin(xcd * chunk + jn, m0n, n0n);
    const bool early = even && more;

    // slab 0 has landed for every wave; st1 is free
    if (slab0_here) wg_barrier();
    else wait_all_then_barrier();
    if (128 < P.K) issue(st1, 128);
    EpiPre<TM, TN> E;
    { const int i0 = m0 / P.rpi; epi_prefetch<TM, TN>(E, P, m0, i0, m0 - i0 * P.rpi, mbase, nbase, li, lg); }
    compute(st0);
    for (int k0 = 128; k0 < P.K; k0 += 256) {        // slabs k0 (in st1) and k0 + 128 (in st0)
      wait_all_then_barrier();                       // the slab has landed for everyone, the other stage is free
      const bool last = k0 + 128 >= P.K;
      if (!last) issue(st0, k0 + 128);
      else if (early) { set_src(m0n, n0n); issue(st0, 0); }
      compute(st1);
      if (last) break;
      wait_all_then_barrier();
      if (k0 + 256 < P.K) issue(st1, k0 + 256);
      compute(st0);
    }

    if (!early) {
      wg_barrier();                                  // every wave is done with both stages
      if (more) { set_src(m0n, n0n); issue(st0, 0); }
    }
    // scales, bias and this wave's part of the next slab 0: requested at least a slab ago when
    // `early`; after this wait nothing the wave has to wait for precedes the stores
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt(0x0F70);
    if (P.kl_part) epi_kl<TM, TN>(E, P, acc, mbase, nbase, li, lg, (n0 / BN) * WAVES_N + wn);
    else epi_store<TM, TN>(E, P, acc, mbase, nbase, li, lg);
    if (!more) break;
    slab0_here = true;       // the barrier at the top publishes slab 0
    j = jn; m0 = m0n; n0 = n0n;
  }
}

// ------------------------------------------------------------------ exact sums, three-stage pipeline
// The large problems.  What bounds gemm_x_k is the distance between requesting a slab and needing
// it: one slab of MFMAs, less than the latency of the loads under load.  Here one workgroup of
// eight wavefronts (4 x 2, 64 x 64 each) owns a 256 x 128 tile per compute unit, LDS holds three
// stages of 48 KB, and a slab is requested two slabs before it is multiplied.  The slabs of all
// tiles a workgroup walks form one stream: the request side runs two slabs ahead of the compute
// side across tile boundaries, so a tile's stores drain while the next tile is multiplied.
// Everything that is loaded goes through LDS, also the scales and the bias of a tile (one
// GLOBAL_LOAD_LDS_DWORD per wave when the tile's first slab is multiplied; read back by the
// epilogue), so that the only vector-memory operations the compiler knows of are stores and the
// residual loads of the epilogue, and the waits can be counted: a wave waits for slab c with
// "at most (6 if slab c+1 is requested) + (stores issued since) operations outstanding".
template <int UNUSED>
__global__ __launch_bounds__(512, 1) void gemm_p_k(const GemmProb* probs) {
  constexpr int BM = 256, BN = 128, TM = 4, TN = 4, NW = 8;
  constexpr int ROWS = BM + BN, NI = ROWS / 8 / NW, STAGE = ROWS * 128, NS = 3;
  static_assert(NI == 6, "six slab loads per wave: the wait counts below assume it");
  extern __shared__ __attribute__((aligned(1024))) uint8_t smem[];
  float* const e_rs = (float*)(smem + NS * STAGE);      // row scales of the tile [BM]
  float* const e_cs = e_rs + BM;                        // column scales [BN]
  float* const e_bi = e_cs + BN;                        // bias [BN]

  const GemmProb P = probs[blockIdx.y];
  const int mt = (P.M + BM - 1) / BM, nt = (P.N + BN - 1) / BN, total = mt * nt;
  const int chunk = (total + 7) >> 3, xcd = blockIdx.x & 7, per = gridDim.x >> 3;
  const int jend = min(chunk, total - xcd * chunk);
  int j = blockIdx.x >> 3;
  if (j >= jend) return;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;
  const int li = lane & 15, lg = lane >> 4;
  const int nslab = P.K >> 7;
  const uint32_t lds0 = lds_addr_of(smem);

  // ---- request side
  const uint8_t* src[NI];
  const int cg = ((lane & 7) ^ (lane >> 3)) * 16;
  auto set_src = [&](int m0, int n0) {
    const int i0 = m0 / P.rpi, r0 = m0 - i0 * P.rpi;
#pragma unroll
    for (int t = 0; t < NI; t++) {
      int r = 8 * (wave * NI + t) + (lane >> 3);
      if (r < BM) {
        int m = min(m0 + r, P.M - 1), inst, row;
        split_row(i0, r0, m - m0, P.rpi, inst, row);
        src[t] = (const uint8_t*)P.A + (long long)inst * P.a_is + (long long)row * P.lda + cg;
      } else {
        // LDS row 16 jj + li of a wave's 64-column block holds column 4 li + jj of the block, so that a lane's four
        // accumulators of one tile row are four neighbouring columns (see the epilogue)
        const int q = r - BM;
        int n = min(n0 + (q & 64) + (q & 15) * 4 + ((q >> 4) & 3), P.N - 1);
        src[t] = (const uint8_t*)P.W + (long long)n * P.ldw + cg;
      }
    }
  };
  auto tile_origin = [&](int jj, int& m0, int& n0) {
    int lin = xcd * chunk + jj;
    m0 = (lin / nt) * BM; n0 = (lin % nt) * BN;
  };
  int ji = j, ki = 0, si = 0;          // tile, slab and stage of the next request
  bool requesting = true;
  auto request = [&]() -> bool {
    if (!requesting) return false;
    const uint32_t base = __builtin_amdgcn_readfirstlane(lds0 + si * STAGE + wave * NI * 1024);
#pragma unroll
    for (int t = 0; t < NI; t++) slab_load16(src[t] + ki * 128, base + t * 1024);
    si = (si == NS - 1) ? 0 : si + 1;
    if (++ki == nslab) {
      ki = 0; ji += per;
      if (ji < jend) { int a, b; tile_origin(ji, a, b); set_src(a, b); }
      else requesting = false;
    }
    return true;
  };
  // scales and bias of a tile: one dword per lane and wave
  auto request_scales = [&](int m0, int n0) {
    const float* g;
    float* dst;
    if (wave < 4) {
      const int i0 = m0 / P.rpi;
      int m = min(m0 + wave * 64 + lane, P.M - 1), inst, row;
      split_row(i0, m0 - i0 * P.rpi, m - m0, P.rpi, inst, row);
      g = P.ascale + inst * P.as_is + (long long)row * P.as_stride;
      dst = e_rs + wave * 64;
    } else {
      int n = min(n0 + (wave & 1) * 64 + lane, P.N - 1);
      if (wave >= 6 && P.bias) { g = P.bias + n; dst = e_bi + (wave & 1) * 64; }
      else { g = P.wscale + wscale_index(P, n); dst = ((wave >= 6) ? e_bi : e_cs) + (wave & 1) * 64; }
    }
    lds_load4(g, __builtin_amdgcn_readfirstlane(lds_addr_of(dst)));
  };

  // ---- compute side
  const int offA = (wm * 64 + li) * 128, offB = (BM + wn * 64 + li) * 128;
  const int sw0 = (lg ^ (li & 7)) * 16, sw1 = ((4 + lg) ^ (li & 7)) * 16;
  v4f acc[TM][TN];
  auto compute = [&](const uint8_t* st) {
    const uint8_t* sA = st + offA;
    const uint8_t* sB = st + offB;
    // all operand reads of the slab are issued before the first convert, so that the reads of the
    // second half are in flight while the first half is multiplied
    uint4 ra[2][TM], rb[2][TN];
#pragma unroll
    for (int q = 0; q < 2; q++) {
      const int sw = q ? sw1 : sw0;
#pragma unroll
      for (int i = 0; i < TM; i++) ra[q][i] = *(const uint4*)(sA + i * 2048 + sw);
#pragma unroll
      for (int jj = 0; jj < TN; jj++) rb[q][jj] = *(const uint4*)(sB + jj * 2048 + sw);
    }
    __builtin_amdgcn_sched_barrier(0);       // keep the scheduler from sinking the reads to their uses
#pragma unroll
    for (int q = 0; q < 2; q++) {
      v8h ha[TM][2];
#pragma unroll
      for (int i = 0; i < TM; i++) {
        ha[i][0] = decode8(ra[q][i].x, ra[q][i].y);
        ha[i][1] = decode8(ra[q][i].z, ra[q][i].w);
      }
#pragma unroll
      for (int jj = 0; jj < TN; jj++) {
        v8h hb0 = decode8(rb[q][jj].x, rb[q][jj].y), hb1 = decode8(rb[q][jj].z, rb[q][jj].w);
#pragma unroll
        for (int i = 0; i < TM; i++) {
          acc[i][jj] = __builtin_amdgcn_mfma_f32_16x16x32_f16(ha[i][0], hb0, acc[i][jj], 0, 0, 0);
          acc[i][jj] = __builtin_amdgcn_mfma_f32_16x16x32_f16(ha[i][1], hb1, acc[i][jj], 0, 0, 0);
        }
      }
    }
  };

  int m0, n0;
  tile_origin(j, m0, n0);
  set_src(m0, n0);
  request();
  bool next_requested = request();      // is the slab after the one about to be multiplied on its way?
  int stores = 0;                       // stores this wave issued since that slab was requested (0, 16 or 32)
  int sc = 0;                           // stage of the slab about to be multiplied

  for (;;) {
#pragma unroll
    for (int i = 0; i < TM; i++)
#pragma unroll
      for (int jj = 0; jj < TN; jj++) acc[i][jj] = (v4f){0.f, 0.f, 0.f, 0.f};

    for (int k = 0; k < nslab; k++) {
      // this wave's part of the slab has landed: everything but what was issued after it is complete
      if (next_requested) {
        if (stores == 0) wait_vm<6>(); else if (stores == 16) wait_vm<22>(); else wait_vm<38>();
      } else {
        if (stores == 0) wait_vm<0>(); else if (stores == 16) wait_vm<16>(); else wait_vm<32>();
      }
      stores = 0;
      wg_barrier();                     // everyone's part has; the stage of the previous slab is free
      if (k == 0) request_scales(m0, n0);
      next_requested = request();       // two slabs ahead, into the stage just freed
      compute(smem + sc * STAGE);
      sc = (sc == NS - 1) ? 0 : sc + 1;
    }
    if (nslab == 1) { wait_vm<0>(); wg_barrier(); }     // the scales were requested in this very slab

    // ---- epilogue: scales and bias from LDS, 16-byte stores
    // Accumulator acc[i][jj][r] of lane (li, lg) is tile row 16 i + 4 lg + r and, with the column order the
    // request side gave the W rows, column 4 li + jj of the wave's block: a lane stores the four jj values of one
    // row as 16 bytes, and the 16 lanes of a group cover 256 contiguous bytes of that row.  Neighbouring lanes
    // writing neighbouring addresses is what the store path wants: the same bytes stored as 16 rows x 64 bytes
    // per instruction take a fifth longer end to end.
    const int nbase = n0 + wn * 64 + li * 4;
    const bool interior = (m0 + BM <= P.M) && (n0 + BN <= P.N);
    const bool col_on = interior || nbase < P.N;
    const int i0 = m0 / P.rpi, r0 = m0 - i0 * P.rpi;
    const float cs = e_cs[wn * 64 + li * 4];
    const float4 bias = *(const float4*)(e_bi + wn * 64 + li * 4);
    int inst[TM][4];
    int roff[TM][4];           // within one instance's block: far below 2^31 elements
    bool live[TM][4];
    float4 sa[TM];
#pragma unroll
    for (int i = 0; i < TM; i++) {
      sa[i] = *(const float4*)(e_rs + wm * 64 + i * 16 + lg * 4);
#pragma unroll
      for (int r = 0; r < 4; r++) {
        const int m = m0 + wm * 64 + i * 16 + lg * 4 + r;
        live[i][r] = col_on && (interior || m < P.M);
        int row;
        split_row(i0, r0, min(m, P.M - 1) - m0, P.rpi, inst[i][r], row);
        roff[i][r] = row * (int)P.ldc + nbase;
      }
    }
    // the residual tile first, all of it, so that its loads are in flight together
    float4 addv[TM][4];
    if (P.add) {
#pragma unroll
      for (int i = 0; i < TM; i++)
#pragma unroll
        for (int r = 0; r < 4; r++)
          addv[i][r] = live[i][r] ? gload4_nt(P.add + inst[i][r] * P.add_is + roff[i][r]) : make_float4(0.f, 0.f, 0.f, 0.f);
    }
#pragma unroll
    for (int i = 0; i < TM; i++) {
      const float sar[4] = {sa[i].x, sa[i].y, sa[i].z, sa[i].w};
#pragma unroll
      for (int r = 0; r < 4; r++) {
        if (!live[i][r]) continue;
        const float s2 = sar[r] * cs;
        float4 val = make_float4(acc[i][0][r] * s2, acc[i][1][r] * s2, acc[i][2][r] * s2, acc[i][3][r] * s2);
        float4 v = val;
        if (P.bias) { v.x += bias.x; v.y += bias.y; v.z += bias.z; v.w += bias.w; }
        // (no activation here: problems that ask for one are refused for this kernel's sizes by gemm8_prob_ok; the code
        // of 64 inlined GELUs cost every tile's epilogue 1.5-2 % of a K = 768 product although no problem used it)
        if (P.add) { v.x += addv[i][r].x; v.y += addv[i][r].y; v.z += addv[i][r].z; v.w += addv[i][r].w; }
        gstore4_nt(P.C + inst[i][r] * P.c_is + roff[i][r], v);
        if (P.aux) {
          if (P.aux_sub) { float4 u = gload4(P.aux_sub + roff[i][r]); val.x -= u.x; val.y -= u.y; val.z -= u.z; val.w -= u.w; }
          gstore4_nt(P.aux + inst[i][r] * P.aux_is + roff[i][r], val);
        }
      }
    }
    if (interior) stores = P.aux ? 32 : 16;     // every wave issued exactly that many
    else {                                      // ragged tile: the count is not uniform, so drain
      asm volatile("" ::: "memory");
      __builtin_amdgcn_s_waitcnt(0x0F70);
      stores = 0;
    }
    j += per;
    if (j >= jend) break;
    tile_origin(j, m0, n0);
  }
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
  { const int i0 = m0 / P.rpi; epi_prefetch<TM, TN>(E, P, m0, i0, m0 - i0 * P.rpi, mbase, nbase, li, lg); }
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

// Problems with the log-softmax / KL epilogue: always the 128 x 128 kernel, whose column tiling the number
// of parts per row (kl_parts_per_row) is derived from.
hipError_t launch_gemm_fp8_kl(const GemmProb* probs, int n_probs, int max_M, int max_N, int b16, hipStream_t s) {
  if (n_probs == 0 || max_M == 0 || max_N == 0) return hipSuccess;
  int tiles = ((max_M + 127) / 128) * ((max_N + 127) / 128);
  int gx = (tiles + 7) / 8 * 8;
  if (gx > 512) gx = 512;
  if (b16) hipLaunchKernelGGL((gemm_x_k<2, 2, 4, 4, true>), dim3(gx, n_probs), dim3(256), 0, s, probs);
  else hipLaunchKernelGGL((gemm_x_k<2, 2, 4, 4>), dim3(gx, n_probs), dim3(256), 0, s, probs);
  return hipGetLastError();
}

hipError_t launch_gemm_fp8(const GemmProb* probs, int n_probs, int max_M, int max_N, int exact, int b16, hipStream_t s) {
  if (n_probs == 0 || max_M == 0 || max_N == 0) return hipSuccess;
  if (b16) {
    // bfloat16 operands: the two-stage kernel at every size (the three-stage kernel has no such form)
    if (!exact) return hipErrorInvalidValue;
    const bool wide = max_N > 64;
    int tiles = ((max_M + 127) / 128) * (wide ? (max_N + 127) / 128 : (max_N + 63) / 64);
    int gx = (tiles + 7) / 8 * 8;
    if (gx > 512) gx = 512;
    dim3 grid(gx, n_probs);
    if (wide) hipLaunchKernelGGL((gemm_x_k<2, 2, 4, 4, true>), grid, dim3(256), 0, s, probs);
    else hipLaunchKernelGGL((gemm_x_k<4, 1, 2, 4, true>), grid, dim3(256), 0, s, probs);
    return hipGetLastError();
  }
  if (exact) {
    // persistent: at most two workgroups per compute unit (64 KB of LDS each), 256 compute units
    const bool wide = max_N > 64;
    if (wide && max_M >= 8192 && max_N >= 128) {
      // one 512-thread workgroup per compute unit, three 48 KB stages + 2 KB of scales
      const int lds_bytes = 3 * 384 * 128 + 2048;
      // the attribute belongs to the kernel's code object on one device: set once per device (atomically, so that
      // models on several streams or host threads may launch concurrently)
      static std::atomic<bool> attr_set[64];
      int dev = 0;
      if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return hipErrorInvalidDevice;
      if (!attr_set[dev].load(std::memory_order_acquire)) {
        hipError_t e = hipFuncSetAttribute((const void*)gemm_p_k<0>, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
        if (e != hipSuccess) return e;
        attr_set[dev].store(true, std::memory_order_release);
      }
      int tiles = ((max_M + 255) / 256) * ((max_N + 127) / 128);
      int gx = (tiles + 7) / 8 * 8;
      if (gx > 256) gx = 256;
      hipLaunchKernelGGL((gemm_p_k<0>), dim3(gx, n_probs), dim3(512), lds_bytes, s, probs);
      return hipGetLastError();
    }
    int tiles = ((max_M + 127) / 128) * (wide ? (max_N + 127) / 128 : (max_N + 63) / 64);
    int gx = (tiles + 7) / 8 * 8;
    if (gx > 512) gx = 512;
    dim3 grid(gx, n_probs);
    if (wide) hipLaunchKernelGGL((gemm_x_k<2, 2, 4, 4>), grid, dim3(256), 0, s, probs);
    else hipLaunchKernelGGL((gemm_x_k<4, 1, 2, 4>), grid, dim3(256), 0, s, probs);
  } else {
    int tiles = ((max_M + 127) / 128) * ((max_N + 63) / 64);
    dim3 grid((tiles + 7) / 8 * 8, n_probs);
    hipLaunchKernelGGL((gemm_fp8_k<128, 64, 4, 1>), grid, dim3(256), 0, s, probs);
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
