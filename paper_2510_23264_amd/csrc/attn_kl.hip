// Short-sequence causal attention (one wavefront per sequence and head, fp32
// matrix cores) and the fused log-softmax + KL reduction.
#include "kernels.h"
#include "device_util.h"
#include "mma_util.h"

namespace pahq {

// Causal attention on the fp32 matrix cores, one wavefront per (instance,
// sequence, head), no LDS.  S <= 64 is covered by ST = 1 .. 4 tiles of 16
// positions (longer sequences: attention_qtile_k below); lane = 16*g + i.
//   scores  S^T = K Q^T with V_MFMA_F32_16X16X4_F32: lane (i, g) feeds row i of a
//           K tile and of a Q tile (its own d_head/4 consecutive columns, the
//           same k order for both operands) and receives S[query i][key 4g + r].
//   softmax per query: over the lane's registers and the four lanes i, i+16, i+32, i+48.
//   output  Z = P V: the score registers are exactly the A operand (query i, key
//           4g + r); lane (i, g) loads V[key 4g + r][16t + i] as B and receives
//           Z[query 4g + r][16t + i].
// Rotary embedding pairs column c with c + d_head/2, which lives in lane g ^ 2.
// Output rows are either written in fp32 (investigated head) or row-quantised
// to e4m3 (one scale per token and head) for the fp8 output projection.
typedef float v4f_a __attribute__((ext_vector_type(4)));

// q, k and v each come with their own base pointer, instance stride and row
// stride (AttnSrc), so one head can take a per-candidate query, key or value
// while the other two are shared by all instances.
template <int ST, int DH, bool ROPE, bool STG>
__global__ __launch_bounds__(256) void attention_mfma_k(AttnSrc src, uint8_t* zcodes,
                                                         long long zc_is, float* zscale, long long zs_is, float* zf32,
                                                         long long zf_is, unsigned long long f32_mask, unsigned long long dead_mask,
                                                         int n_pairs, int B, int S, int H,
                                                         int ldz, int rope, const float2* rope_tab) {
  constexpr int CH = DH / 4;        // columns of q / k per lane
  constexpr int NT = DH / 16;       // output column tiles
  const int pair = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (pair >= n_pairs) return;
  const int hl = pair % src.n_heads, sb = pair / src.n_heads;          // sb = inst * B + b
  const int h = src.h0 + hl;                                           // head index in the outputs
  if ((dead_mask >> h) & 1ull) return;                                 // this head is not computed (a wave owns a pair: no barrier follows)
  const int inst = sb / B, b = sb % B;
  const int lane = threadIdx.x & 63, i = lane & 15, g = lane >> 4;
  const float* qb = src.q + inst * src.q_is + (long long)b * S * src.q_ld + hl * src.head_cols;
  const float* kb = src.k + inst * src.k_is + (long long)b * S * src.k_ld + hl * src.head_cols;
  const float* vb = src.v + inst * src.v_is + (long long)b * S * src.v_ld + hl * src.head_cols;

  float q[ST][CH], k[ST][CH];
  // STG (one 16-position tile, d_head 64): the three 16 x 64 blocks go from global memory straight into this
  // wave's 8 KB of LDS (q and k first; v takes q's place once q is in registers), four rows of 256 contiguous bytes per load instruction (lane l writes bytes [16 l, 16 l +
  // 16) behind the base: row l >> 4, chunk position l & 15), and are read back in the operand layouts.  Position p
  // of row r holds chunk p ^ r of the row, so that the 16 rows a 16-byte operand read touches lie in 16 different
  // bank groups.  Loading each lane's operand directly costs the same bytes as 16-byte pieces of 16 different rows.
  __shared__ __attribute__((aligned(1024))) float stage[STG ? 4 * 2 * 1024 : 4];
  float* const sq = stage + (STG ? (threadIdx.x >> 6) * 2048 : 0);
  if (STG) {
    const float* mats[2] = {qb, kb};
    const int lds_[2] = {src.q_ld, src.k_ld};
#pragma unroll
    for (int mtx = 0; mtx < 2; mtx++)
#pragma unroll
      for (int t = 0; t < 4; t++) {
        const int r = 4 * t + (lane >> 4);
        const float* gp = mats[mtx] + (long long)min(r, S - 1) * lds_[mtx] + (((lane & 15) ^ r) * 4);
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)gp,
                                         (__attribute__((address_space(3))) void*)(sq + mtx * 1024 + t * 256), 16, 0, 2);
      }
    __builtin_amdgcn_s_waitcnt(0x0F70);       // vmcnt(0): this wave's blocks are in LDS
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int cc = 0; cc < 4; cc++) {
      const int pos4 = ((4 * g + cc) ^ i) * 4;
      const float4 vq = *(const float4*)(sq + i * 64 + pos4), vk = *(const float4*)(sq + 1024 + i * 64 + pos4);
      const bool on = i < S;
      q[0][4 * cc] = on ? vq.x : 0.f; q[0][4 * cc + 1] = on ? vq.y : 0.f; q[0][4 * cc + 2] = on ? vq.z : 0.f; q[0][4 * cc + 3] = on ? vq.w : 0.f;
      k[0][4 * cc] = on ? vk.x : 0.f; k[0][4 * cc + 1] = on ? vk.y : 0.f; k[0][4 * cc + 2] = on ? vk.z : 0.f; k[0][4 * cc + 3] = on ? vk.w : 0.f;
    }
    __builtin_amdgcn_s_waitcnt(0xC07F);       // lgkmcnt(0): q and k are in registers
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int t = 0; t < 4; t++) {             // v into q's place; waited for after the softmax
      const int r = 4 * t + (lane >> 4);
      const float* gp = vb + (long long)min(r, S - 1) * src.v_ld + (((lane & 15) ^ r) * 4);
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)gp,
                                       (__attribute__((address_space(3))) void*)(sq + t * 256), 16, 0, 2);
    }
  } else {
#pragma unroll
  for (int a = 0; a < ST; a++) {
    int pos = 16 * a + i;
    const float* qrow = qb + (long long)pos * src.q_ld + CH * g;
    const float* krow = kb + (long long)pos * src.k_ld + CH * g;
#pragma unroll
    for (int c = 0; c < CH; c += 4) {
      float4 vq = make_float4(0, 0, 0, 0), vk = vq;
      if (pos < S) { vq = *(const float4*)(qrow + c); vk = *(const float4*)(krow + c); }
      q[a][c] = vq.x; q[a][c + 1] = vq.y; q[a][c + 2] = vq.z; q[a][c + 3] = vq.w;
      k[a][c] = vk.x; k[a][c + 1] = vk.y; k[a][c + 2] = vk.z; k[a][c + 3] = vk.w;
    }
  }
  }
  if (ROPE) {
#pragma unroll
    for (int a = 0; a < ST; a++) {
      int pos = 16 * a + i;
#pragma unroll
      for (int c = 0; c < CH; c++) {
        int col = (CH * g + c) % (DH / 2);
        // (cos, sin) of pos * theta^(-2 col / d_head), from the table rope_table_k filled once
        const float2 t2 = rope_tab[pos * (DH / 2) + col];
        float sn = t2.y, cs = t2.x;
        float pq = __shfl_xor(q[a][c], 32, 64), pk = __shfl_xor(k[a][c], 32, 64);
        // first half: x cos - y sin ; second half: x cos + y sin (y = the partner column)
        float sg = (g < 2) ? -sn : sn;
        q[a][c] = q[a][c] * cs + pq * sg;
        k[a][c] = k[a][c] * cs + pk * sg;
      }
    }
  }

  // scores[a][bk][r] = S[query 16a + i][key 16bk + 4g + r]
  v4f_a sc[ST][ST];
  const float scl = 1.0f / sqrtf((float)DH);
#pragma unroll
  for (int a = 0; a < ST; a++)
#pragma unroll
    for (int bk = 0; bk <= a; bk++) {
      v4f_a acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int c = 0; c < CH; c++) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(k[bk][c], q[a][c], acc, 0, 0, 0);
      sc[a][bk] = acc;
    }
#pragma unroll
  for (int a = 0; a < ST; a++) {
    const int qpos = 16 * a + i;
    float mx = -3.0e38f;
#pragma unroll
    for (int bk = 0; bk <= a; bk++)
#pragma unroll
      for (int r = 0; r < 4; r++) {
        int kpos = 16 * bk + 4 * g + r;
        float v = sc[a][bk][r] * scl;
        bool ok = kpos <= qpos && kpos < S;
        sc[a][bk][r] = ok ? v : -3.0e38f;
        if (ok) mx = fmaxf(mx, v);
      }
    mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    float sum = 0.f;
#pragma unroll
    for (int bk = 0; bk <= a; bk++)
#pragma unroll
      for (int r = 0; r < 4; r++) {
        float e = (sc[a][bk][r] > -1.0e38f) ? expf(sc[a][bk][r] - mx) : 0.f;
        sc[a][bk][r] = e;
        sum += e;
      }
    sum += __shfl_xor(sum, 16, 64);
    sum += __shfl_xor(sum, 32, 64);
    float rs = (sum > 0.f) ? 1.0f / sum : 0.f;
#pragma unroll
    for (int bk = 0; bk <= a; bk++)
#pragma unroll
      for (int r = 0; r < 4; r++) sc[a][bk][r] *= rs;
  }

  // values: vv[bk][r][t] = V[key 16bk + 4g + r][16t + i]
  float vv[ST][4][NT];
  if (STG) { __builtin_amdgcn_s_waitcnt(0x0F70); __builtin_amdgcn_wave_barrier(); }
#pragma unroll
  for (int bk = 0; bk < ST; bk++)
#pragma unroll
    for (int r = 0; r < 4; r++) {
      int kpos = 16 * bk + 4 * g + r;
      if (STG) {
        // V[kpos][16 t + i]: chunk 4 t + (i >> 2) of row kpos, word i & 3 of it
#pragma unroll
        for (int t = 0; t < NT; t++)
          vv[bk][r][t] = (kpos < S) ? sq[kpos * 64 + (((4 * t + (i >> 2)) ^ kpos) * 4) + (i & 3)] : 0.f;
      } else {
        const float* row = vb + (long long)kpos * src.v_ld + i;
#pragma unroll
        for (int t = 0; t < NT; t++) vv[bk][r][t] = (kpos < S) ? row[16 * t] : 0.f;
      }
    }

  const bool f32 = (f32_mask >> h) & 1ull;
  // place of this head among the fp32 heads, and their number
  const int f32_slot = __popcll(f32_mask & ((1ull << h) - 1ull)), f32_n = __popcll(f32_mask);
#pragma unroll
  for (int a = 0; a < ST; a++) {
    v4f_a z[NT];
#pragma unroll
    for (int t = 0; t < NT; t++) {
      v4f_a acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int bk = 0; bk <= a; bk++)
#pragma unroll
        for (int r = 0; r < 4; r++) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(sc[a][bk][r], vv[bk][r][t], acc, 0, 0, 0);
      z[t] = acc;
    }
    // lane (i, g) holds Z[query 16a + 4g + rr][16t + i]
#pragma unroll
    for (int rr = 0; rr < 4; rr++) {
      int pos = 16 * a + 4 * g + rr;
      long long tok = (long long)b * S + pos;
      if (f32) {
        if (pos < S) {
          float* o = zf32 + inst * zf_is + (tok * f32_n + f32_slot) * DH + i;
#pragma unroll
          for (int t = 0; t < NT; t++) o[16 * t] = z[t][rr];
        }
      } else {
        float am = 0.f;
#pragma unroll
        for (int t = 0; t < NT; t++) am = fmaxf(am, fabsf(z[t][rr]));
#pragma unroll
        for (int o = 8; o > 0; o >>= 1) am = fmaxf(am, __shfl_xor(am, o, 64));
        float scale = (am == 0.f || src.qbits == 16) ? 1.0f : am / q_top(src.qbits);
        float inv = 1.0f / scale;
        if (!STG && src.qbits == 16) {
          // bfloat16 patterns, two bytes per value, no scale
          if (pos < S) {
            uint8_t* o = zcodes + inst * zc_is + (tok * H + h) * ldz + 2 * i;
#pragma unroll
            for (int t = 0; t < NT; t++) *(uint16_t*)(o + 32 * t) = (uint16_t)bf16_rne(z[t][rr]);
            if (i == 0) zscale[inst * zs_is + tok * H + h] = 1.0f;
          }
        } else if (STG) {
          // codes of the 16 x 64 block are collected in this wave's LDS (the k block is no longer needed) and
          // leave as one 16-byte store per lane below, instead of one byte per lane and column tile here
          uint8_t* zb = (uint8_t*)(sq + 1024) + pos * 64 + i;
#pragma unroll
          for (int t = 0; t < NT; t++) zb[16 * t] = (uint8_t)q_encode(z[t][rr] * inv, src.qbits);
          if (pos < S && i == 0) zscale[inst * zs_is + tok * H + h] = scale;
        } else if (pos < S) {
          uint8_t* o = zcodes + inst * zc_is + (tok * H + h) * ldz + i;
#pragma unroll
          for (int t = 0; t < NT; t++) o[16 * t] = (uint8_t)q_encode(z[t][rr] * inv, src.qbits);
          if (i == 0) zscale[inst * zs_is + tok * H + h] = scale;
        }
      }
    }
  }
  if (STG && !f32) {
    __builtin_amdgcn_s_waitcnt(0xC07F);       // lgkmcnt(0): the byte writes above
    __builtin_amdgcn_wave_barrier();
    const int pos = lane >> 2;                // token of the block, 16-byte piece lane & 3 of its 64 codes
    if (pos < S) {
      const uint4 w = *(const uint4*)((const uint8_t*)(sq + 1024) + lane * 16);
      *(uint4*)(zcodes + inst * zc_is + (((long long)b * S + pos) * H + h) * ldz + (lane & 3) * 16) = w;
    }
  }
}

// The same attention for longer sequences: one wavefront per (instance, sequence, head, tile of 16 queries).  The
// whole-sequence kernel above keeps every tile of q, k, the scores and v of a sequence in registers, which ends at
// four tiles (two with 128-wide heads); here a wave holds one query tile and its row of score tiles (up to STM key
// tiles) and fetches the key and value tiles one after the other.  Per output element the products are formed and
// added in the order of the kernel above -- scores over the head's columns in ascending order, softmax over the key
// tiles then the lane's four keys then the four lanes, P V over key tiles and keys ascending -- so that for a
// sequence both kernels accept they give the same bits.
template <int STM, int DH, bool ROPE>
__global__ __launch_bounds__(256) void attention_qtile_k(AttnSrc src, uint8_t* zcodes, long long zc_is, float* zscale,
                                                          long long zs_is, float* zf32, long long zf_is,
                                                          unsigned long long f32_mask, unsigned long long dead_mask,
                                                          int n_pairs, int B, int S, int H, int ldz, const float2* rope_tab) {
  constexpr int CH = DH / 4, NT = DH / 16;
  const int ST = (S + 15) >> 4;
  const int job = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (job >= n_pairs * ST) return;
  const int a = job % ST, pair = job / ST;                             // query tile, (instance, sequence, head)
  const int hl = pair % src.n_heads, sb = pair / src.n_heads;
  const int h = src.h0 + hl;
  if ((dead_mask >> h) & 1ull) return;
  const int inst = sb / B, b = sb % B;
  const int lane = threadIdx.x & 63, i = lane & 15, g = lane >> 4;
  const float* qb = src.q + inst * src.q_is + (long long)b * S * src.q_ld + hl * src.head_cols;
  const float* kb = src.k + inst * src.k_is + (long long)b * S * src.k_ld + hl * src.head_cols;
  const float* vb = src.v + inst * src.v_is + (long long)b * S * src.v_ld + hl * src.head_cols;
  // row `pos` of a matrix: this lane's CH consecutive columns, rotated when the model has rotary positions
  auto load_rows = [&](float (&x)[CH], const float* base, int ld, int pos) {
    const float* row = base + (long long)pos * ld + CH * g;
#pragma unroll
    for (int c = 0; c < CH; c += 4) {
      float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
      if (pos < S) v = *(const float4*)(row + c);
      x[c] = v.x; x[c + 1] = v.y; x[c + 2] = v.z; x[c + 3] = v.w;
    }
    if (ROPE) {
#pragma unroll
      for (int c = 0; c < CH; c++) {
        const int col = (CH * g + c) % (DH / 2);
        const float2 t2 = rope_tab[pos * (DH / 2) + col];
        const float px = __shfl_xor(x[c], 32, 64);
        const float sg = (g < 2) ? -t2.y : t2.y;
        x[c] = x[c] * t2.x + px * sg;
      }
    }
  };
  float q[CH];
  load_rows(q, qb, src.q_ld, 16 * a + i);
  v4f_a sc[STM];
  const float scl = 1.0f / sqrtf((float)DH);
#pragma unroll
  for (int bk = 0; bk < STM; bk++) {
    if (bk > a) continue;                                              // (wave-uniform)
    float kk[CH];
    load_rows(kk, kb, src.k_ld, 16 * bk + i);
    v4f_a acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int c = 0; c < CH; c++) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(kk[c], q[c], acc, 0, 0, 0);
    sc[bk] = acc;
  }
  {
    const int qpos = 16 * a + i;
    float mx = -3.0e38f;
#pragma unroll
    for (int bk = 0; bk < STM; bk++) {
      if (bk > a) continue;
#pragma unroll
      for (int r = 0; r < 4; r++) {
        const int kpos = 16 * bk + 4 * g + r;
        const float v = sc[bk][r] * scl;
        const bool ok = kpos <= qpos && kpos < S;
        sc[bk][r] = ok ? v : -3.0e38f;
        if (ok) mx = fmaxf(mx, v);
      }
    }
    mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    float sum = 0.f;
#pragma unroll
    for (int bk = 0; bk < STM; bk++) {
      if (bk > a) continue;
#pragma unroll
      for (int r = 0; r < 4; r++) {
        const float e = (sc[bk][r] > -1.0e38f) ? expf(sc[bk][r] - mx) : 0.f;
        sc[bk][r] = e;
        sum += e;
      }
    }
    sum += __shfl_xor(sum, 16, 64);
    sum += __shfl_xor(sum, 32, 64);
    const float rs = (sum > 0.f) ? 1.0f / sum : 0.f;
#pragma unroll
    for (int bk = 0; bk < STM; bk++) {
      if (bk > a) continue;
#pragma unroll
      for (int r = 0; r < 4; r++) sc[bk][r] *= rs;
    }
  }
  v4f_a z[NT];
#pragma unroll
  for (int t = 0; t < NT; t++) z[t] = (v4f_a){0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int bk = 0; bk < STM; bk++) {
    if (bk > a) continue;
#pragma unroll
    for (int r = 0; r < 4; r++) {
      const int kpos = 16 * bk + 4 * g + r;
      const float* row = vb + (long long)kpos * src.v_ld + i;
#pragma unroll
      for (int t = 0; t < NT; t++) {
        const float vv = (kpos < S) ? row[16 * t] : 0.f;
        z[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(sc[bk][r], vv, z[t], 0, 0, 0);
      }
    }
  }
  const bool f32 = (f32_mask >> h) & 1ull;
  const int f32_slot = __popcll(f32_mask & ((1ull << h) - 1ull)), f32_n = __popcll(f32_mask);
  // lane (i, g) holds Z[query 16a + 4g + rr][16t + i]
#pragma unroll
  for (int rr = 0; rr < 4; rr++) {
    const int pos = 16 * a + 4 * g + rr;
    const long long tok = (long long)b * S + pos;
    if (f32) {
      if (pos < S) {
        float* o = zf32 + inst * zf_is + (tok * f32_n + f32_slot) * DH + i;
#pragma unroll
        for (int t = 0; t < NT; t++) o[16 * t] = z[t][rr];
      }
    } else {
      float am = 0.f;
#pragma unroll
      for (int t = 0; t < NT; t++) am = fmaxf(am, fabsf(z[t][rr]));
#pragma unroll
      for (int o = 8; o > 0; o >>= 1) am = fmaxf(am, __shfl_xor(am, o, 64));
      const float scale = (am == 0.f || src.qbits == 16) ? 1.0f : am / q_top(src.qbits);
      const float inv = 1.0f / scale;
      if (pos < S) {
        if (src.qbits == 16) {
          uint8_t* o = zcodes + inst * zc_is + (tok * H + h) * ldz + 2 * i;
#pragma unroll
          for (int t = 0; t < NT; t++) *(uint16_t*)(o + 32 * t) = (uint16_t)bf16_rne(z[t][rr]);
          if (i == 0) zscale[inst * zs_is + tok * H + h] = 1.0f;
        } else {
          uint8_t* o = zcodes + inst * zc_is + (tok * H + h) * ldz + i;
#pragma unroll
          for (int t = 0; t < NT; t++) o[16 * t] = (uint8_t)q_encode(z[t][rr] * inv, src.qbits);
          if (i == 0) zscale[inst * zs_is + tok * H + h] = scale;
        }
      }
    }
  }
}

// tab[pos][col] = (cos, sin) of pos * theta^(-2 col / d_head) for col < d_head / 2: the angle in fp64, rounded
// once, as the attention kernel used to compute it per element
__global__ void rope_table_k(float2* tab, int n_pos, int dh, float theta) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n_pos * (dh / 2)) return;
  int pos = i / (dh / 2), col = i % (dh / 2);
  double ang = (double)pos * pow((double)theta, -2.0 * (double)col / (double)dh);
  tab[i] = make_float2((float)cos(ang), (float)sin(ang));
}
hipError_t launch_rope_table(float* tab, int n_pos, int dh, float theta, hipStream_t s) {
  int n = n_pos * (dh / 2);
  if (n <= 0) return hipSuccess;
  hipLaunchKernelGGL(rope_table_k, dim3((n + 255) / 256), dim3(256), 0, s, (float2*)tab, n_pos, dh, theta);
  return hipGetLastError();
}

hipError_t launch_attention(const AttnSrc& src, uint8_t* zcodes, long long zc_is, float* zscale,
                            long long zs_is, float* zf32, long long zf_is, unsigned long long f32_mask, unsigned long long dead_mask, int n_inst, int B, int S,
                            int H, int dh, int ldz, int rope, const float* rope_tab, hipStream_t s) {
  if (n_inst == 0) return hipSuccess;
  if (S > 128) return hipErrorInvalidValue;
  int n_pairs = n_inst * B * src.n_heads;
  if (src.form == 1 || S > 64 || (S > 32 && dh == 128)) {
    // one wave per tile of 16 queries, up to eight key tiles
    const long long jobs = (long long)n_pairs * ((S + 15) / 16);
    if (jobs > 0x7fffffffLL) return hipErrorInvalidValue;
    dim3 qgrid((unsigned)((jobs + 3) / 4));
#define ATQ(DH_) do { if (rope) hipLaunchKernelGGL((attention_qtile_k<8, DH_, true>), qgrid, dim3(256), 0, s, src, zcodes, zc_is, zscale, zs_is, zf32, \
                                                  zf_is, f32_mask, dead_mask, n_pairs, B, S, H, ldz, (const float2*)rope_tab); \
                      else hipLaunchKernelGGL((attention_qtile_k<8, DH_, false>), qgrid, dim3(256), 0, s, src, zcodes, zc_is, zscale, zs_is, zf32, \
                                              zf_is, f32_mask, dead_mask, n_pairs, B, S, H, ldz, (const float2*)rope_tab); } while (0)
    if (dh == 16) ATQ(16); else if (dh == 32) ATQ(32); else if (dh == 64) ATQ(64); else if (dh == 128) ATQ(128);
    else return hipErrorInvalidValue;
#undef ATQ
    return hipGetLastError();
  }
  dim3 grid((n_pairs + 3) / 4);
  // the staged form (one tile, d_head 64, no rotation) collects one-byte codes in LDS: bfloat16 outputs take the plain form
#define ATT0(ST_, DH_, R_, G_) hipLaunchKernelGGL((attention_mfma_k<ST_, DH_, R_, G_>), grid, dim3(256), 0, s, src, zcodes, \
                                              zc_is, zscale, zs_is, zf32, zf_is, f32_mask, dead_mask, n_pairs, B, S, H, ldz, rope, (const float2*)rope_tab)
#define ATT1(ST_, DH_, R_) do { if ((ST_ == 1 && DH_ == 64 && !R_) && src.qbits != 16) ATT0(ST_, DH_, R_, (ST_ == 1 && DH_ == 64 && !R_)); \
                                else ATT0(ST_, DH_, R_, false); } while (0)
#define ATT(ST_, DH_) do { if (rope) ATT1(ST_, DH_, true); else ATT1(ST_, DH_, false); } while (0)
  if (S <= 16) {
    if (dh == 16) ATT(1, 16); else if (dh == 32) ATT(1, 32); else if (dh == 64) ATT(1, 64);
    else if (dh == 128) ATT(1, 128); else return hipErrorInvalidValue;
  } else if (S <= 32) {
    if (dh == 16) ATT(2, 16); else if (dh == 32) ATT(2, 32); else if (dh == 64) ATT(2, 64);
    else if (dh == 128) ATT(2, 128); else return hipErrorInvalidValue;
  } else if (S <= 48) {
    // three and four tiles of positions: the same kernel with more of a sequence's scores and values in registers
    // (d_head up to 64: with 128 they no longer fit)
    if (dh == 16) ATT(3, 16); else if (dh == 32) ATT(3, 32); else if (dh == 64) ATT(3, 64); else return hipErrorInvalidValue;
  } else {
    if (dh == 16) ATT(4, 16); else if (dh == 32) ATT(4, 32); else if (dh == 64) ATT(4, 64); else return hipErrorInvalidValue;
  }
#undef ATT
#undef ATT1
#undef ATT0
  return hipGetLastError();
}

// ------------------------------------------------------------------ log-sum-exp and KL
__device__ __forceinline__ double block_sum_d(double v, double* red) {
  v = wave_sum_d(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  return (red[0] + red[1]) + (red[2] + red[3]);
}
__device__ __forceinline__ float block_max_f(float v, float* red) {
  v = wave_max(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  return fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
}

// log-sum-exp of one row in a single sweep: every thread keeps a running maximum
// and a sum rescaled to it; the partial (max, sum) pairs are merged in a fixed order.
__device__ __forceinline__ double row_logz(const float* x, int V, float* redf, double* redd) {
  float mx = -3.0e38f;
  float s = 0.f;
  int i = threadIdx.x * 4;
  if ((((uintptr_t)x) & 15) == 0) {
    for (; i + 3 < V; i += 1024) {
      float4 v = *(const float4*)(x + i);
      float m4 = fmaxf(fmaxf(v.x, v.y), fmaxf(v.z, v.w));
      if (m4 > mx) { s *= expf(mx - m4); mx = m4; }
      s += expf(v.x - mx) + expf(v.y - mx) + expf(v.z - mx) + expf(v.w - mx);
    }
  }
  for (int e = i; e < V && e < i + 4; e++) {           // ragged tail of the strided sweep (or unaligned rows)
    float v = x[e];
    if (v > mx) { s *= expf(mx - v); mx = v; }
    s += expf(v - mx);
  }
  if ((((uintptr_t)x) & 15) != 0)
    for (int e = i + 1024; e < V; e += 1024)
      for (int q = e; q < V && q < e + 4; q++) {
        float v = x[q];
        if (v > mx) { s *= expf(mx - v); mx = v; }
        s += expf(v - mx);
      }
  float gm = block_max_f(mx, redf);
  double sd = (double)s * (double)expf(mx - gm);
  sd = block_sum_d(sd, redd);
  return (double)gm + log(sd);
}

__global__ __launch_bounds__(256) void logz_k(const float* logits, int V, int ldv, double* logz) {
  __shared__ float redf[4];
  __shared__ double redd[4];
  double z = row_logz(logits + (long long)blockIdx.x * ldv, V, redf, redd);
  if (threadIdx.x == 0) logz[blockIdx.x] = z;
}
hipError_t launch_logz(const float* logits, int rows, int V, int ldv, double* logz, hipStream_t s) {
  hipLaunchKernelGGL(logz_k, dim3(rows), dim3(256), 0, s, logits, V, ldv, logz);
  return hipGetLastError();
}

// row_kl[inst][b] = sum_v p_ref[v] * ((xr[v] - x[v]) - (logz_ref - logz)),  p_ref = exp(xr - logz_ref).
// Differences of logits (O(1) numbers) are taken before anything of the size
// of log V enters, and the sums run in fp64, so identical logits give exactly 0.
__global__ __launch_bounds__(256) void kl_rows_k(const float* logits, long long l_is, const float* ref_logits,
                                                  const double* ref_logz, double* row_kl, int B, int V, int ldv) {
  __shared__ float redf[4];
  __shared__ double redd[4];
  int b = blockIdx.x, inst = blockIdx.y;
  const float* x = logits + inst * l_is + (long long)b * ldv;
  const float* xr = ref_logits + (long long)b * ldv;
  const double lzr = ref_logz[b];
  const float lzr_f = (float)lzr;
  // one sweep over the candidate's row: the running (max, rescaled sum) of its log-sum-exp and the
  // two KL sums advance together, so the row is read once
  float mx = -3.0e38f, se = 0.f;
  double a = 0.0, psum = 0.0;
  auto step = [&](float r, float c) {
    if (c > mx) { se *= expf(mx - c); mx = c; }
    se += expf(c - mx);
    double p = (double)expf(r - lzr_f);
    a += p * (double)(r - c);
    psum += p;
  };
  if (((((uintptr_t)x) | ((uintptr_t)xr)) & 15) == 0) {
    int i = threadIdx.x * 4;
    for (; i + 3 < V; i += 1024) {
      float4 r = *(const float4*)(xr + i), c = *(const float4*)(x + i);
      float m4 = fmaxf(fmaxf(c.x, c.y), fmaxf(c.z, c.w));
      if (m4 > mx) { se *= expf(mx - m4); mx = m4; }
      se += expf(c.x - mx) + expf(c.y - mx) + expf(c.z - mx) + expf(c.w - mx);
      float p0 = expf(r.x - lzr_f), p1 = expf(r.y - lzr_f), p2 = expf(r.z - lzr_f), p3 = expf(r.w - lzr_f);
      a += (double)p0 * (double)(r.x - c.x) + (double)p1 * (double)(r.y - c.y) + (double)p2 * (double)(r.z - c.z) +
           (double)p3 * (double)(r.w - c.w);
      psum += (double)p0 + (double)p1 + (double)p2 + (double)p3;
    }
    for (int e = i; e < V && e < i + 4; e++) step(xr[e], x[e]);
  } else {
    for (int i = threadIdx.x; i < V; i += 256) step(xr[i], x[i]);
  }
  float gm = block_max_f(mx, redf);
  double sd = block_sum_d((double)se * (double)expf(mx - gm), redd);
  const double lz = (double)gm + log(sd);
  a = block_sum_d(a, redd);
  psum = block_sum_d(psum, redd);
  if (threadIdx.x == 0) row_kl[inst * B + b] = a - (lzr - lz) * psum;
}
__global__ void kl_mean_k(const double* row_kl, double* kl, int n_inst, int B) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n_inst) return;
  double s = 0.0;
  for (int b = 0; b < B; b++) s += row_kl[i * B + b];
  kl[i] = s / (double)B;
}
hipError_t launch_kl(const float* logits, long long l_is, const float* ref_logits, const double* ref_logz,
                     double* row_kl, double* kl, int n_inst, int B, int V, int ldv, hipStream_t s) {
  if (n_inst == 0) return hipSuccess;
  hipLaunchKernelGGL(kl_rows_k, dim3(B, n_inst), dim3(256), 0, s, logits, l_is, ref_logits, ref_logz, row_kl, B, V, ldv);
  hipLaunchKernelGGL(kl_mean_k, dim3((n_inst + 63) / 64), dim3(64), 0, s, row_kl, kl, n_inst, B);
  return hipGetLastError();
}

// ------------------------------------------------------------------ KL from the parts the unembedding left
// One wavefront per row.  The row's log-sum-exp from its (max, sum) parts: global maximum first, then
// the rescaled sums in fp64, lanes striding over the parts and a butterfly at the end -- an order
// that depends on nothing but the number of parts, so the reference row and a candidate row with the
// same logits get the same bits and their difference is an exact zero.
__global__ __launch_bounds__(64) void kl_reduce_k(const float* part, int npart, int B, const double* ref_logz,
                                                  const double* ref_psum, double* logz, double* row_kl) {
  const int row = blockIdx.x, lane = threadIdx.x;
  const float4* p = (const float4*)part + (long long)row * npart;
  float mx = -3.0e38f;
  for (int t = lane; t < npart; t += 64) mx = fmaxf(mx, p[t].x);
  mx = wave_max(mx);
  double se = 0.0, a = 0.0;
  for (int t = lane; t < npart; t += 64) {
    const float4 q = p[t];
    se += (double)q.y * (double)expf(q.x - mx);
    a += (double)q.z;
  }
  se = wave_sum_d(se);
  a = wave_sum_d(a);
  const double lz = (double)mx + log(se);
  if (lane == 0) {
    if (logz) logz[row] = lz;
    if (row_kl) { const int b = row % B; row_kl[row] = a - (ref_logz[b] - lz) * ref_psum[b]; }
  }
}
hipError_t launch_kl_reduce(const float* kl_part, int npart, int rows, int B, const double* ref_logz,
                            const double* ref_psum, double* logz, double* row_kl, double* kl, hipStream_t s) {
  if (rows == 0) return hipSuccess;
  hipLaunchKernelGGL(kl_reduce_k, dim3(rows), dim3(64), 0, s, kl_part, npart, B, ref_logz, ref_psum, logz, row_kl);
  if (kl) hipLaunchKernelGGL(kl_mean_k, dim3((rows / B + 63) / 64), dim3(64), 0, s, row_kl, kl, rows / B, B);
  return hipGetLastError();
}

// ------------------------------------------------------------------ logit-difference task metric
// One wavefront per (instance, sequence): the two logits the metric needs -- the answer's and the
// distractor's -- each the product of the row's e4m3 codes with one column of the unembedding codes
// (exact products, fp32 sum in an order fixed by the lane layout), scaled and biased like the GEMM's
// result.  The unembedding itself is not computed for this metric.
__global__ __launch_bounds__(64) void logit_pair_k(const uint8_t* codes, long long c_is, const float* scale, long long s_is,
                                                   int ldq, int K, const uint8_t* wcodes, int ldw, const float* wscale,
                                                   const float* bias, const int* ans, const int* dis, int B, double* ld, int b16) {
  const int row = blockIdx.x, inst = row / B, b = row % B, lane = threadIdx.x;
  const uint8_t* a = codes + inst * c_is + (long long)b * ldq;
  const float s2 = scale[inst * s_is + b] * wscale[0];
  float out[2];
#pragma unroll
  for (int which = 0; which < 2; which++) {
    const int col = which ? dis[b] : ans[b];
    const uint8_t* wv = wcodes + (long long)col * ldw;
    float acc = 0.f;
    if (b16) {
      // bfloat16 patterns (K in bytes): a pattern shifted into the upper half of a word is the binary32 value
      for (int k = lane * 8; k < K; k += 512) {
        const uint2 av = *(const uint2*)(a + k), bv = *(const uint2*)(wv + k);
        acc += __uint_as_float(av.x << 16) * __uint_as_float(bv.x << 16);
        acc += __uint_as_float(av.x & 0xFFFF0000u) * __uint_as_float(bv.x & 0xFFFF0000u);
        acc += __uint_as_float(av.y << 16) * __uint_as_float(bv.y << 16);
        acc += __uint_as_float(av.y & 0xFFFF0000u) * __uint_as_float(bv.y & 0xFFFF0000u);
      }
    } else
    for (int k = lane * 8; k < K; k += 512) {
      const uint2 av = *(const uint2*)(a + k), bv = *(const uint2*)(wv + k);
      const v8h ha = decode8(av.x, av.y), hb = decode8(bv.x, bv.y);
#pragma unroll
      for (int e = 0; e < 8; e++) acc += (float)ha[e] * (float)hb[e];
    }
    acc = wave_sum(acc);
    out[which] = acc * s2 + bias[col];
  }
  if (lane == 0) ld[row] = (double)out[0] - (double)out[1];
}
// The same from unquantised rows and the fp32 unembedding (all-fp32 mode): x [inst][B][d], W [d][ldw].
__global__ __launch_bounds__(64) void logit_pair_f32_k(const float* x, long long x_is, int d, const float* W, int ldw,
                                                       const float* bias, const int* ans, const int* dis, int B, double* ld) {
  const int row = blockIdx.x, inst = row / B, b = row % B, lane = threadIdx.x;
  const float* a = x + inst * x_is + (long long)b * d;
  float out[2];
#pragma unroll
  for (int which = 0; which < 2; which++) {
    const int col = which ? dis[b] : ans[b];
    float acc = 0.f;
    for (int k = lane; k < d; k += 64) acc += a[k] * W[(long long)k * ldw + col];
    out[which] = wave_sum(acc) + bias[col];
  }
  if (lane == 0) ld[row] = (double)out[0] - (double)out[1];
}
// score[i] = mean over the B sequences of (ref_ld[b] - ld[i][b]): how far the logit difference dropped
__global__ void metric_mean_k(const double* ld, const double* ref_ld, double* score, int n_inst, int B) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n_inst) return;
  double s = 0.0;
  for (int b = 0; b < B; b++) s += ref_ld[b] - ld[i * B + b];
  score[i] = s / (double)B;
}
hipError_t launch_logit_pair(const uint8_t* codes, long long c_is, const float* scale, long long s_is, int ldq, int K,
                             const uint8_t* wcodes, int ldw, const float* wscale, const float* bias, const int* ans,
                             const int* dis, int n_inst, int B, double* ld, int b16, hipStream_t s) {
  if (n_inst == 0) return hipSuccess;
  hipLaunchKernelGGL(logit_pair_k, dim3(n_inst * B), dim3(64), 0, s, codes, c_is, scale, s_is, ldq, K, wcodes, ldw, wscale, bias,
                     ans, dis, B, ld, b16);
  return hipGetLastError();
}
hipError_t launch_logit_pair_f32(const float* x, long long x_is, int d, const float* W, int ldw, const float* bias,
                                 const int* ans, const int* dis, int n_inst, int B, double* ld, hipStream_t s) {
  if (n_inst == 0) return hipSuccess;
  hipLaunchKernelGGL(logit_pair_f32_k, dim3(n_inst * B), dim3(64), 0, s, x, x_is, d, W, ldw, bias, ans, dis, B, ld);
  return hipGetLastError();
}
hipError_t launch_metric_mean(const double* ld, const double* ref_ld, double* score, int n_inst, int B, hipStream_t s) {
  if (n_inst == 0) return hipSuccess;
  hipLaunchKernelGGL(metric_mean_k, dim3((n_inst + 63) / 64), dim3(64), 0, s, ld, ref_ld, score, n_inst, B);
  return hipGetLastError();
}

// Sum of a reference row's probabilities (1 up to rounding; the KL uses the sum it gets).
__global__ __launch_bounds__(256) void ref_probs_k(const float* logits, const double* logz, double* psum, int V,
                                                   int ldv) {
  __shared__ double redd[4];
  const int b = blockIdx.x;
  const float* x = logits + (long long)b * ldv;
  const float lz = (float)logz[b];
  double s = 0.0;
  for (int v = threadIdx.x; v < V; v += 256) s += (double)expf(x[v] - lz);
  s = block_sum_d(s, redd);
  if (threadIdx.x == 0) psum[b] = s;
}
hipError_t launch_ref_probs(const float* logits, const double* logz, double* psum, int B, int V, int ldv,
                            hipStream_t s) {
  hipLaunchKernelGGL(ref_probs_k, dim3(B), dim3(256), 0, s, logits, logz, psum, V, ldv);
  return hipGetLastError();
}

}  // namespace pahq
