// Short-sequence causal attention (one wavefront per sequence and head) and the
// fused log-softmax + KL reduction.
#include "kernels.h"
#include "device_util.h"

namespace pahq {

// One wavefront handles one (instance, sequence, head): S <= 32 rows of d_head
// <= 128.  q, k, v are staged in LDS; lane c owns output columns c, c + 64;
// scores and the softmax are fp32, reductions are over LDS rows in a fixed
// order.  The head's output rows are either written in fp32 (investigated
// head) or row-quantised to e4m3 (one scale per token and head) for the fp8
// output projection.
template <int MAXS, int MAXD>
__global__ __launch_bounds__(64) void attention_k(const float* qkv, long long qkv_is, uint8_t* zcodes,
                                                   long long zc_is, float* zscale, long long zs_is, float* zf32,
                                                   long long zf_is, int f32_head, int B, int S, int H, int dh,
                                                   int ldz, int rope, float rope_theta) {
  __shared__ float sq[MAXS][MAXD + 1], sk[MAXS][MAXD + 1], sv[MAXS][MAXD + 1];
  __shared__ float sp[MAXS][MAXS + 1];
  const int inst = blockIdx.x / B, b = blockIdx.x % B, h = blockIdx.y;
  const int lane = threadIdx.x;
  const int ld = 3 * H * dh;
  const float* base = qkv + inst * qkv_is + (long long)b * S * ld;
  for (int idx = lane; idx < S * dh; idx += 64) {
    int i = idx / dh, c = idx % dh;
    const float* row = base + (long long)i * ld + h * dh + c;
    sq[i][c] = row[0];
    sk[i][c] = row[H * dh];
    sv[i][c] = row[2 * H * dh];
  }
  __syncthreads();
  if (rope) {
    int half = dh >> 1;
    for (int idx = lane; idx < S * half; idx += 64) {
      int i = idx / half, c = idx % half;
      double ang = (double)i * pow((double)rope_theta, -2.0 * (double)c / (double)dh);
      float sn = (float)sin(ang), cs = (float)cos(ang);
      float a = sq[i][c], bq = sq[i][c + half];
      sq[i][c] = a * cs - bq * sn;
      sq[i][c + half] = bq * cs + a * sn;
      a = sk[i][c]; bq = sk[i][c + half];
      sk[i][c] = a * cs - bq * sn;
      sk[i][c + half] = bq * cs + a * sn;
    }
    __syncthreads();
  }
  const float scl = 1.0f / sqrtf((float)dh);
  for (int idx = lane; idx < S * S; idx += 64) {
    int i = idx / S, j = idx % S;
    float a = 0.f;
    if (j <= i) {
      for (int c = 0; c < dh; c++) a += sq[i][c] * sk[j][c];
      a *= scl;
    }
    sp[i][j] = a;
  }
  __syncthreads();
  if (lane < S) {                 // softmax of row `lane` over j <= lane
    int i = lane;
    float mx = sp[i][0];
    for (int j = 1; j <= i; j++) mx = fmaxf(mx, sp[i][j]);
    float sum = 0.f;
    for (int j = 0; j <= i; j++) { float e = expf(sp[i][j] - mx); sp[i][j] = e; sum += e; }
    float r = 1.0f / sum;
    for (int j = 0; j <= i; j++) sp[i][j] *= r;
  }
  __syncthreads();
  const bool f32 = (h == f32_head);
  for (int i = 0; i < S; i++) {
    float z0 = 0.f, z1 = 0.f;
    const int c0 = lane, c1 = lane + 64;
    for (int j = 0; j <= i; j++) {
      float p = sp[i][j];
      if (c0 < dh) z0 += p * sv[j][c0];
      if (c1 < dh) z1 += p * sv[j][c1];
    }
    long long t = (long long)b * S + i;
    if (f32) {
      float* o = zf32 + inst * zf_is + t * dh;
      if (c0 < dh) o[c0] = z0;
      if (c1 < dh) o[c1] = z1;
    } else {
      float am = fmaxf(c0 < dh ? fabsf(z0) : 0.f, c1 < dh ? fabsf(z1) : 0.f);
      am = wave_max(am);
      float sc = (am == 0.f) ? 1.0f : am / 448.0f;
      float inv = 1.0f / sc;
      uint8_t* o = zcodes + inst * zc_is + (t * H + h) * ldz;
      if (c0 < dh) o[c0] = (uint8_t)e4m3_encode(z0 * inv);
      if (c1 < dh) o[c1] = (uint8_t)e4m3_encode(z1 * inv);
      if (lane == 0) zscale[inst * zs_is + t * H + h] = sc;
    }
  }
}

hipError_t launch_attention(const float* qkv, long long qkv_is, uint8_t* zcodes, long long zc_is, float* zscale,
                            long long zs_is, float* zf32, long long zf_is, int f32_head, int n_inst, int B, int S,
                            int H, int dh, int ldz, int rope, float rope_theta, hipStream_t s) {
  if (n_inst == 0) return hipSuccess;
  if (S > 32 || dh > 128) return hipErrorInvalidValue;
  dim3 grid(n_inst * B, H);
  if (dh <= 64)
    hipLaunchKernelGGL((attention_k<32, 64>), grid, dim3(64), 0, s, qkv, qkv_is, zcodes, zc_is, zscale, zs_is, zf32,
                       zf_is, f32_head, B, S, H, dh, ldz, rope, rope_theta);
  else
    hipLaunchKernelGGL((attention_k<32, 128>), grid, dim3(64), 0, s, qkv, qkv_is, zcodes, zc_is, zscale, zs_is,
                       zf32, zf_is, f32_head, B, S, H, dh, ldz, rope, rope_theta);
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

__device__ __forceinline__ double row_logz(const float* x, int V, float* redf, double* redd) {
  float mx = -3.0e38f;
  for (int i = threadIdx.x; i < V; i += 256) mx = fmaxf(mx, x[i]);
  mx = block_max_f(mx, redf);
  double s = 0.0;
  for (int i = threadIdx.x; i < V; i += 256) s += (double)expf(x[i] - mx);
  s = block_sum_d(s, redd);
  return (double)mx + log(s);
}

__global__ __launch_bounds__(256) void logz_k(const float* logits, int V, double* logz) {
  __shared__ float redf[4];
  __shared__ double redd[4];
  double z = row_logz(logits + (long long)blockIdx.x * V, V, redf, redd);
  if (threadIdx.x == 0) logz[blockIdx.x] = z;
}
hipError_t launch_logz(const float* logits, int rows, int V, double* logz, hipStream_t s) {
  hipLaunchKernelGGL(logz_k, dim3(rows), dim3(256), 0, s, logits, V, logz);
  return hipGetLastError();
}

// row_kl[inst][b] = sum_v p_ref[v] * ((xr[v] - x[v]) - (logz_ref - logz)),  p_ref = exp(xr - logz_ref).
// Differences of logits (O(1) numbers) are taken before anything of the size
// of log V enters, and the sums run in fp64, so identical logits give exactly 0.
__global__ __launch_bounds__(256) void kl_rows_k(const float* logits, long long l_is, const float* ref_logits,
                                                  const double* ref_logz, double* row_kl, int B, int V) {
  __shared__ float redf[4];
  __shared__ double redd[4];
  int b = blockIdx.x, inst = blockIdx.y;
  const float* x = logits + inst * l_is + (long long)b * V;
  const float* xr = ref_logits + (long long)b * V;
  double lz = row_logz(x, V, redf, redd);
  double lzr = ref_logz[b];
  float lzr_f = (float)lzr;
  double a = 0.0, psum = 0.0;
  for (int i = threadIdx.x; i < V; i += 256) {
    float r = xr[i];
    double p = (double)expf(r - lzr_f);
    a += p * (double)(r - x[i]);
    psum += p;
  }
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
                     double* row_kl, double* kl, int n_inst, int B, int V, hipStream_t s) {
  if (n_inst == 0) return hipSuccess;
  hipLaunchKernelGGL(kl_rows_k, dim3(B, n_inst), dim3(256), 0, s, logits, l_is, ref_logits, ref_logz, row_kl, B, V);
  hipLaunchKernelGGL(kl_mean_k, dim3((n_inst + 63) / 64), dim3(64), 0, s, row_kl, kl, n_inst, B);
  return hipGetLastError();
}

}  // namespace pahq
