// Output projection of all heads of a layer fused with the stream update:
//   next[m][:] = run[m][:] + b_O + extra[m][:] + sum_h (z_h[m] W_O^h) * s_z[m][h] * s_w[h]
// Each head is one K slab (d_head <= 128 codes, zero padded to 128) with its
// own row and weight scale, so the MFMA result of a head is scaled and added to
// the running total in registers; the per-head sender outputs never go to HBM
// unless a receiver needs one (HeadAux: the head's output, optionally minus the
// corrupted run's, is written next to the total).  `extra` carries the fp32
// head's contribution, computed by the fp32 GEMM.
// Tile 128 x 64, four wavefronts of 32 x 64; operands staged through LDS as in
// the fp8 GEMM (144-byte rows), next head prefetched into registers.
#include "kernels.h"
#include "device_util.h"
#include "mma_util.h"
#include <atomic>
#include <type_traits>

namespace pahq {

#define LDS_ROW 144

template <bool EXACT>
__global__ __launch_bounds__(256) void oproj_fused_k(const OprojDesc* descs, int di, const HeadAux* auxs) {
  constexpr int BM = 128, BN = 64, TM = 2, TN = 4;
  __shared__ __attribute__((aligned(16))) uint8_t sA[BM * LDS_ROW];
  __shared__ __attribute__((aligned(16))) uint8_t sB[BN * LDS_ROW];
  const OprojDesc D = descs[di];
  const int mt = (D.M + BM - 1) / BM, nt = (D.N + BN - 1) / BN;
  const int chunk = (mt * nt + 7) >> 3;
  const int lin = (blockIdx.x & 7) * chunk + (blockIdx.x >> 3);
  if (lin >= mt * nt) return;
  const int m0 = (lin / nt) * BM, n0 = (lin % nt) * BN;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int li = lane & 15, lg = lane >> 4;

  // this thread's chunks: A rows (tid>>3) + 32c, B rows (tid>>3) + 32c; 16-byte column kc
  const int kc = tid & 7;
  const uint8_t* pa[4];
  const uint8_t* pb[2];
#pragma unroll
  for (int c = 0; c < 4; c++) {
    int m = m0 + (tid >> 3) + 32 * c;
    pa[c] = (m < D.M) ? D.zc + (long long)(m / D.rpi) * D.zc_is + (long long)(m % D.rpi) * D.H * D.Kh + kc * 16 : nullptr;
  }
#pragma unroll
  for (int c = 0; c < 2; c++) {
    int n = n0 + (tid >> 3) + 32 * c;
    pb[c] = (n < D.N) ? D.W + (long long)n * D.Kh + kc * 16 : nullptr;
  }
  uint4 ra[4], rb[2];
  // codes beyond d_head are zero padding: neither loaded nor (with the fp16 matrix cores) multiplied
  const bool real_chunk = kc * 16 < D.dh;
  const int nkk = (D.dh + 31) >> 5;
  auto load_head = [&](int h) {
#pragma unroll
    for (int c = 0; c < 4; c++)
      ra[c] = (pa[c] && real_chunk) ? *(const uint4*)(pa[c] + (long long)h * D.Kh) : make_uint4(0, 0, 0, 0);
#pragma unroll
    for (int c = 0; c < 2; c++)
      rb[c] = (pb[c] && real_chunk) ? *(const uint4*)(pb[c] + (long long)h * D.N * D.Kh) : make_uint4(0, 0, 0, 0);
  };
  auto skipped = [&](int h) { return ((D.skip_mask >> h) & 1ull) != 0; };
  auto next_head = [&](int h) { h++; while (h < D.H && skipped(h)) h++; return h; };

  // W is the first MFMA operand, so lane (i, g) owns row i of a 16-row tile and columns 4g .. 4g+3
  int row_m[TM];
  const float* zs_p[TM];
#pragma unroll
  for (int i = 0; i < TM; i++) {
    int m = m0 + wave * 32 + i * 16 + li;
    row_m[i] = m;
    int mm = m < D.M ? m : D.M - 1;
    zs_p[i] = D.zs + (long long)(mm / D.rpi) * D.zs_is + (long long)(mm % D.rpi) * D.H;
  }

  v4f tot[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; i++)
#pragma unroll
    for (int j = 0; j < TN; j++) tot[i][j] = (v4f){0.f, 0.f, 0.f, 0.f};

  int h = next_head(-1);
  if (h < D.H) load_head(h);
  for (; h < D.H; h = next_head(h)) {
    __syncthreads();
#pragma unroll
    for (int c = 0; c < 4; c++) *(uint4*)(sA + ((tid >> 3) + 32 * c) * LDS_ROW + kc * 16) = ra[c];
#pragma unroll
    for (int c = 0; c < 2; c++) *(uint4*)(sB + ((tid >> 3) + 32 * c) * LDS_ROW + kc * 16) = rb[c];
    __syncthreads();
    int hn = next_head(h);
    if (hn < D.H) load_head(hn);

    v4f acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; i++)
#pragma unroll
      for (int j = 0; j < TN; j++) acc[i][j] = (v4f){0.f, 0.f, 0.f, 0.f};
    if (EXACT) {
#pragma unroll
      for (int kk = 0; kk < 4; kk++) {
        if (kk >= nkk) break;
        v8h ha[TM];
#pragma unroll
        for (int i = 0; i < TM; i++) {
          uint2 w = *(const uint2*)(sA + (wave * 32 + i * 16 + li) * LDS_ROW + kk * 32 + lg * 8);
          ha[i] = decode8(w.x, w.y);
        }
#pragma unroll
        for (int j = 0; j < TN; j++) {
          uint2 w = *(const uint2*)(sB + (j * 16 + li) * LDS_ROW + kk * 32 + lg * 8);
          v8h hb = decode8(w.x, w.y);
#pragma unroll
          for (int i = 0; i < TM; i++) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(hb, ha[i], acc[i][j], 0, 0, 0);
        }
      }
    } else {
      v8i fa[TM];
#pragma unroll
      for (int i = 0; i < TM; i++) {
        const uint8_t* p = sA + (wave * 32 + i * 16 + li) * LDS_ROW + lg * 32;
        uint4 lo = *(const uint4*)p, hi = *(const uint4*)(p + 16);
        fa[i] = (v8i){(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w, (int)hi.x, (int)hi.y, (int)hi.z, (int)hi.w};
      }
#pragma unroll
      for (int j = 0; j < TN; j++) {
        const uint8_t* p = sB + (j * 16 + li) * LDS_ROW + lg * 32;
        uint4 lo = *(const uint4*)p, hi = *(const uint4*)(p + 16);
        v8i fb = (v8i){(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w, (int)hi.x, (int)hi.y, (int)hi.z, (int)hi.w};
#pragma unroll
        for (int i = 0; i < TM; i++)
          acc[i][j] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(fb, fa[i], acc[i][j], 0, 0, 0, 0x7F7F7F7F, 0,
                                                                       0x7F7F7F7F);
      }
    }
    // scale this head's result, add it to the total, and hand it out if some receiver needs it
    const float sw = D.ws[h];
    HeadAux ax; ax.dst = nullptr; ax.dst_is = 0; ax.sub = nullptr;
    if (D.aux_begin >= 0) ax = auxs[D.aux_begin + h];
#pragma unroll
    for (int i = 0; i < TM; i++) {
      float sc = zs_p[i][h] * sw;
      int m = row_m[i];
#pragma unroll
      for (int j = 0; j < TN; j++) {
        float4 val = make_float4(acc[i][j][0] * sc, acc[i][j][1] * sc, acc[i][j][2] * sc, acc[i][j][3] * sc);
        tot[i][j][0] += val.x; tot[i][j][1] += val.y; tot[i][j][2] += val.z; tot[i][j][3] += val.w;
        if (ax.dst) {
          int nb = n0 + j * 16 + lg * 4;
          if (m < D.M && nb < D.N) {
            long long off = (long long)(m % D.rpi) * D.N + nb;
            if (ax.sub) { float4 u = *(const float4*)(ax.sub + off); val.x -= u.x; val.y -= u.y; val.z -= u.z; val.w -= u.w; }
            *(float4*)(ax.dst + (long long)(m / D.rpi) * ax.dst_is + off) = val;
          }
        }
      }
    }
  }

#pragma unroll
  for (int i = 0; i < TM; i++) {
    int m = row_m[i];
    if (m >= D.M) continue;
    int inst = m / D.rpi;
    long long roff = (long long)(m % D.rpi) * D.N;
#pragma unroll
    for (int j = 0; j < TN; j++) {
      int nb = n0 + j * 16 + lg * 4;
      if (nb >= D.N) continue;
      float4 v = *(const float4*)(D.run_in + inst * D.run_in_is + roff + nb);
      if (D.bias) { float4 b = *(const float4*)(D.bias + nb); v.x += b.x; v.y += b.y; v.z += b.z; v.w += b.w; }
      v.x += tot[i][j][0]; v.y += tot[i][j][1]; v.z += tot[i][j][2]; v.w += tot[i][j][3];
      // the fp32 head goes in last: (stream + bias + other heads) + fp32 head, the same association
      // the candidate path uses when it adds that head to a precomputed sum of the others
      if (D.extra) { float4 e = *(const float4*)(D.extra + inst * D.extra_is + roff + nb); v.x += e.x; v.y += e.y; v.z += e.z; v.w += e.w; }
      *(float4*)(D.run_out + inst * D.run_out_is + roff + nb) = v;
    }
  }
}

// ------------------------------------------------------------------ exact sums, d_head 64 or 128
// The same projection with the slab pipeline of the exact GEMM: slabs of 128 code bytes (one head
// of 128, or two heads of 64: only the real codes are fetched, the padding of the stored rows is
// skipped) go straight into swizzled LDS.  128 x 64 tile, eight wavefronts of 32 x 32 (two workgroups
// per compute unit, four waves per SIMD: a tile is a chain of short dependent steps - six slabs of 16
// matrix instructions per wave, then the stream tile - and it is the number of waves in flight that
// hides their latencies; four waves of 32 x 64 took a tenth longer).  A head's
// partial result is complete after one (d_head 64) or two (d_head 128) 64-byte halves of a slab;
// it is scaled by z-scale[row][head] * w-scale[head] and added to the running total in registers.
// A head that is computed in fp32 elsewhere (skip mask) is multiplied like the others and left out of the sum.
// Three stages of 25 KB, a slab requested two slabs before it is multiplied: with one slab of
// look-ahead a workgroup waits for memory at every slab (a slab is far less work than the latency
// of its loads under load).  For the waits to be countable every
// load inside the loop goes into LDS by the same path, also the row scales of a slab's heads (one
// dword per lane and wave with each slab) and the weight scales (once, before slab 0): a wave
// waits for slab s with "at most the four operations of slab s + 1 outstanding".  A layer that
// hands out per-head results issues stores and loads of its own inside the loop; it drains
// instead of counting.
// DH: bytes of a head's row of codes (64 or 128).  B16: they are bfloat16 patterns (d_head = DH / 2), multiplied
// without conversion by V_MFMA_F32_16X16X32_BF16, one step per 16-byte operand read; everything else is the same.
constexpr int OPX_STAGES = 3;
constexpr int OPX_OPER = (128 + 64) * 128;                 // operand bytes of a stage
constexpr int OPX_STAGE = OPX_OPER + 1024;                 // + row scales [heads of the slab][128]
constexpr int OPX_LDS = OPX_STAGES * OPX_STAGE + 256;      // + weight scales [64]
template <int DH, bool B16 = false>
__global__ __launch_bounds__(512, 4) void oproj_x_k(const OprojDesc* descs, int di, const HeadAux* auxs) {
  constexpr int BM = 128, BN = 64, TM = 2, TN = 2, NI = 3, NS = OPX_STAGES, STAGE = OPX_STAGE;
  constexpr int HPS = 128 / DH;            // heads per slab
  constexpr int CPH = 8 / HPS;             // 16-byte chunks per head
  static_assert(NI + 1 == 4, "four loads per slab and wave: the wait counts below assume it");
  extern __shared__ __attribute__((aligned(1024))) uint8_t smem[];
  const float* const e_ws = (const float*)(smem + NS * STAGE);
  const OprojDesc D = descs[di];
  const int mt = (D.M + BM - 1) / BM, nt = (D.N + BN - 1) / BN;
  const int lin = xcd_tile(blockIdx.x, mt * nt);
  if (lin >= mt * nt) return;
  const int m0 = (lin / nt) * BM, n0 = (lin % nt) * BN;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;
  const int li = lane & 15, lg = lane >> 4;
  const int nslab = D.H / HPS;
  const uint32_t lds0 = lds_addr_of(smem);

  // lane l of a load instruction fills LDS row l >> 3, chunk position l & 7, i.e. logical chunk
  // c = (l & 7) ^ (l >> 3) of the slab: head c / CPH of the slab, bytes 16 (c % CPH) of that head
  const int c = (lane & 7) ^ (lane >> 3);
  const uint8_t* src[NI];
  long long stride[NI];                    // bytes from one slab to the next: activation or weight rows
#pragma unroll
  for (int t = 0; t < NI; t++) {
    int r = 8 * (wave * NI + t) + (lane >> 3);
    if (r < BM) {
      int m = min(m0 + r, D.M - 1);
      src[t] = D.zc + (long long)(m / D.rpi) * D.zc_is + (long long)(m % D.rpi) * D.H * D.Kh +
               (long long)(c / CPH) * D.Kh + (c % CPH) * 16;
      stride[t] = (long long)HPS * D.Kh;
    } else {
      int n = min(n0 + r - BM, D.N - 1);
      src[t] = D.W + (long long)n * D.Kh + (long long)(c / CPH) * D.N * D.Kh + (c % CPH) * 16;
      stride[t] = (long long)HPS * D.N * D.Kh;
    }
  }
  // row scales of a slab: entry [q][r] (head q of the slab, tile row r) is lane's if 64 wave + lane = 128 q + r;
  // waves 4 .. 7 repeat what waves 0 .. 3 fetch (so that all waves count alike), and with one head per slab waves 2
  // and 3 repeat rows 0 .. 127 into the unused half
  const float* zsrc;
  {
    const int q = (HPS == 2) ? ((wave & 3) >> 1) : 0;
    const int m = min(m0 + (wave & 1) * 64 + lane, D.M - 1);
    zsrc = D.zs + (long long)(m / D.rpi) * D.zs_is + (long long)(m % D.rpi) * D.H + q;
  }
  int si = 0;                              // stage of the next request
  auto issue = [&]() {                     // fetches the next slab and advances
    const uint32_t st = lds0 + si * STAGE;
    const uint32_t base = __builtin_amdgcn_readfirstlane(st + wave * NI * 1024);
#pragma unroll
    for (int t = 0; t < NI; t++) { slab_load16(src[t], base + t * 1024); src[t] += stride[t]; }
    lds_load4(zsrc, __builtin_amdgcn_readfirstlane(st + OPX_OPER + (wave & 3) * 256));
    zsrc += HPS;
    si = (si == NS - 1) ? 0 : si + 1;
  };
  const int mbase = m0 + wm * 32, nbase = n0 + wn * 32;
  // weight scales of all heads, the same 64 dwords from every wave (so that all waves count alike)
  lds_load4(D.ws + min(lane, D.H - 1), __builtin_amdgcn_readfirstlane(lds0 + NS * STAGE));
  issue();
  if (1 < nslab) issue();

  const int offA = (wm * 32 + li) * 128, offB = (BM + wn * 32 + li) * 128;
  const int sw0 = (lg ^ (li & 7)) * 16, sw1 = ((4 + lg) ^ (li & 7)) * 16;
  v4f tot[TM][TN], acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; i++)
#pragma unroll
    for (int j = 0; j < TN; j++) tot[i][j] = (v4f){0.f, 0.f, 0.f, 0.f};

  // adds head h's finished partial result to the total and hands it out if some receiver needs it
  auto fold = [&](auto aux_tag, int h, const float (&zsc)[TM]) {
    constexpr bool AUX = decltype(aux_tag)::value;
    // a head computed in fp32 elsewhere adds nothing here: its codes and scales are whatever an earlier pass left
    // (the total starts at +0 and so never is -0: leaving the head out gives the bits of adding zeros)
    if ((D.skip_mask >> h) & 1ull) return;
    const float sw = e_ws[h];
    HeadAux ax; ax.dst = nullptr; ax.dst_is = 0; ax.sub = nullptr;
    if constexpr (AUX) ax = auxs[D.aux_begin + h];
#pragma unroll
    for (int i = 0; i < TM; i++) {
      const float sc = zsc[i] * sw;
#pragma unroll
      for (int j = 0; j < TN; j++) {
        float4 val = make_float4(acc[i][j][0] * sc, acc[i][j][1] * sc, acc[i][j][2] * sc, acc[i][j][3] * sc);
        tot[i][j][0] += val.x; tot[i][j][1] += val.y; tot[i][j][2] += val.z; tot[i][j][3] += val.w;
        if constexpr (AUX) if (ax.dst) {
          int m = mbase + i * 16 + li, nb = nbase + j * 16 + lg * 4;
          if (m < D.M && nb < D.N) {
            long long off = (long long)(m % D.rpi) * D.N + nb;
            if (ax.sub) { float4 u = gload4(ax.sub + off); val.x -= u.x; val.y -= u.y; val.z -= u.z; val.w -= u.w; }
            gstore4(ax.dst + (long long)(m / D.rpi) * ax.dst_is + off, val);
          }
        }
      }
    }
  };
  auto compute = [&](auto aux_tag, const uint8_t* st, int s) {
    const uint8_t* sA = st + offA;
    const uint8_t* sB = st + offB;
    const float* zrow = (const float*)(st + OPX_OPER) + wm * 32 + li;
    float zsc[HPS][TM];                      // requested now, used after the MFMAs of the half
#pragma unroll
    for (int q = 0; q < HPS; q++)
#pragma unroll
      for (int i = 0; i < TM; i++) zsc[q][i] = zrow[q * BM + i * 16];
    // all operand reads of the slab first (the scheduler would otherwise sink them to their uses)
    uint4 ra[2][TM], rb[2][TN];
#pragma unroll
    for (int q = 0; q < 2; q++) {
      const int sw = q ? sw1 : sw0;
#pragma unroll
      for (int i = 0; i < TM; i++) ra[q][i] = *(const uint4*)(sA + i * 2048 + sw);
#pragma unroll
      for (int j = 0; j < TN; j++) rb[q][j] = *(const uint4*)(sB + j * 2048 + sw);
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int q = 0; q < 2; q++) {
      if (HPS == 2 || q == 0) {
#pragma unroll
        for (int i = 0; i < TM; i++)
#pragma unroll
          for (int j = 0; j < TN; j++) acc[i][j] = (v4f){0.f, 0.f, 0.f, 0.f};
      }
      if constexpr (B16) {
        union U { uint4 u; v8bf h; };
#pragma unroll
        for (int j = 0; j < TN; j++) {
          U hb; hb.u = rb[q][j];
#pragma unroll
          for (int i = 0; i < TM; i++) {
            U ha; ha.u = ra[q][i];
            acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(hb.h, ha.h, acc[i][j], 0, 0, 0);
          }
        }
      } else {
      v8h ha[TM][2];
#pragma unroll
      for (int i = 0; i < TM; i++) {
        ha[i][0] = decode8(ra[q][i].x, ra[q][i].y);
        ha[i][1] = decode8(ra[q][i].z, ra[q][i].w);
      }
#pragma unroll
      for (int j = 0; j < TN; j++) {
        v8h hb0 = decode8(rb[q][j].x, rb[q][j].y), hb1 = decode8(rb[q][j].z, rb[q][j].w);
#pragma unroll
        for (int i = 0; i < TM; i++) {
          acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(hb0, ha[i][0], acc[i][j], 0, 0, 0);
          acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(hb1, ha[i][1], acc[i][j], 0, 0, 0);
        }
      }
      }
      if (HPS == 2) fold(aux_tag, 2 * s + q, zsc[q]);
      else if (q == 1) fold(aux_tag, s, zsc[0]);
    }
  };

  int sc = 0;                                // stage of the slab about to be multiplied
  if (D.aux_begin < 0) {
    // no vector-memory operation inside the loop but the slab requests (the code that hands out per-head results is
    // not even compiled into this loop: the wait for its descriptor would sit where the two paths merge)
    for (int s = 0; s < nslab; s++) {
      // this wave's part of slab s has landed: all but the four operations of slab s + 1 are complete
      if (s + 1 < nslab) wait_vm<4>(); else wait_vm<0>();
      wg_barrier();                          // everyone's part has; the stage of slab s - 1 is free
      if (s + 2 < nslab) issue();
      compute(std::false_type{}, smem + sc * STAGE, s);
      sc = (sc == NS - 1) ? 0 : sc + 1;
    }
  } else {
    for (int s = 0; s < nslab; s++) {
      wait_all_then_barrier();
      if (s + 2 < nslab) issue();
      compute(std::true_type{}, smem + sc * STAGE, s);
      sc = (sc == NS - 1) ? 0 : sc + 1;
    }
  }
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_waitcnt(0x0F70);        // nothing is outstanding; said with the builtin so that the compiler knows

#pragma unroll
  for (int i = 0; i < TM; i++) {
    const int m = mbase + i * 16 + li;
    if (m >= D.M) continue;
    const int inst_i = m / D.rpi;
    const long long roff = (long long)(m - inst_i * D.rpi) * D.N;
#pragma unroll
    for (int j = 0; j < TN; j++) {
      int nb = nbase + j * 16 + lg * 4;
      if (nb >= D.N) continue;
      float4 v = gload4(D.run_in + inst_i * D.run_in_is + roff + nb);
      if (D.bias) { float4 b = gload4(D.bias + nb); v.x += b.x; v.y += b.y; v.z += b.z; v.w += b.w; }
      v.x += tot[i][j][0]; v.y += tot[i][j][1]; v.z += tot[i][j][2]; v.w += tot[i][j][3];
      // the fp32 head goes in last, as in oproj_fused_k
      if (D.extra) { const float4 e = gload4(D.extra + inst_i * D.extra_is + roff + nb); v.x += e.x; v.y += e.y; v.z += e.z; v.w += e.w; }
      gstore4(D.run_out + inst_i * D.run_out_is + roff + nb, v);
    }
  }
}

// The kernel's 75 KB of dynamic LDS need the attribute, which belongs to the kernel's code object on one device:
// set once per device and instantiation (atomically: models on several streams or host threads may launch at once).
template <int DH, bool B16>
static hipError_t launch_oproj_x(dim3 grid, hipStream_t s, const OprojDesc* descs, int desc_index, const HeadAux* auxs) {
  static std::atomic<bool> attr_set[64];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return hipErrorInvalidDevice;
  if (!attr_set[dev].load(std::memory_order_acquire)) {
    hipError_t e = hipFuncSetAttribute((const void*)oproj_x_k<DH, B16>, hipFuncAttributeMaxDynamicSharedMemorySize, OPX_LDS);
    if (e != hipSuccess) return e;
    attr_set[dev].store(true, std::memory_order_release);
  }
  hipLaunchKernelGGL((oproj_x_k<DH, B16>), grid, dim3(512), OPX_LDS, s, descs, desc_index, auxs);
  return hipGetLastError();
}

hipError_t launch_oproj_fused(const OprojDesc* descs, int desc_index, const HeadAux* auxs, int M, int N, int H, int dh,
                              int exact, int b16, hipStream_t s) {
  if (M == 0) return hipSuccess;
  int tiles = ((M + 127) / 128) * ((N + 63) / 64);
  dim3 grid((tiles + 7) / 8 * 8);
  if (b16) {
    // bfloat16 attention outputs: heads of 32 or 64 values (64 or 128 bytes)
    if (!exact || (dh != 32 && dh != 64) || N % 4 != 0 || H % (64 / dh) != 0) return hipErrorInvalidValue;
    if (H > 64) return hipErrorInvalidValue;
    if (dh == 32) return launch_oproj_x<64, true>(grid, s, descs, desc_index, auxs);
    return launch_oproj_x<128, true>(grid, s, descs, desc_index, auxs);
  }
  if (exact && (dh == 64 || dh == 128) && N % 4 == 0 && H % (128 / dh) == 0 && H <= 64) {
    if (dh == 64) return launch_oproj_x<64, false>(grid, s, descs, desc_index, auxs);
    return launch_oproj_x<128, false>(grid, s, descs, desc_index, auxs);
  } else if (exact) hipLaunchKernelGGL(oproj_fused_k<true>, grid, dim3(256), 0, s, descs, desc_index, auxs);
  else hipLaunchKernelGGL(oproj_fused_k<false>, grid, dim3(256), 0, s, descs, desc_index, auxs);
  return hipGetLastError();
}

}  // namespace pahq
