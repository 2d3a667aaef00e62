// Device-side building blocks of libpahq (gfx950 only).  Every launcher
// enqueues on the given stream and returns the hipError_t of the launch.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace pahq {

// One additive term of a receiver input: sign * tile[instance][row][col].
struct Term {
  const float* p;
  long long inst_stride;   // elements between instances (0 = shared by all instances)
  float sign;
  int pad_;
};

// A receiver-input group: every receiver of one layer whose input is the same
// sum shares one normalised / quantised copy of it.
//   x = base + run + sum(terms);  y = norm(x) * gain + offset
struct GroupDesc {
  const float* base;  long long base_is;
  const float* run;   long long run_is;
  int term_begin, term_count;
  const float* gain;  const float* offset;      // norm parameters [d]
  float* out_f32;     long long out_f32_is;     // normalised rows, stride d (may be null)
  uint8_t* out_codes; long long out_codes_is;   // e4m3 codes, row stride ldq (may be null)
  float* out_scale;   long long out_scale_is;   // one scale per row
  int last_only;      // 1: only the last position of each sequence (B rows per instance)
  int qbits;          // grid of the codes: 4 = 4-bit round-to-nearest, anything else E4M3 (device_util.h, q_encode)
};

// One GEMM problem.  Rows are numbered 0 .. M-1 over all instances: row m belongs
// to instance m / rpi and is row m % rpi of it, so a launch needs no instance
// dimension and row tiles may straddle instances.
//   val[m][n] = (sum_k A[m][k] * W[n][k]) * ascale[m] * wscale[n / wscale_block]
//   C[m][n]   = act(val + bias[n]) + add[m][n]
//   aux[m][n] = val - aux_sub[m % rpi][n]            (optional second output)
// A, W: e4m3 codes, K contiguous, K a multiple of 128 (zero padded).
struct GemmProb {
  const void* A;       long long a_is;  int lda;  int rpi;          // rows per instance
  const float* ascale; long long as_is; int as_stride; int k_real;  // unpadded K (for flop counts)
  const void* W;       int ldw;  int wscale_block;
  const float* wscale;
  const float* bias;
  float* C;            long long c_is;  int ldc;  int act;   // act: 0 none, 1 tanh-GELU
  const float* add;    long long add_is;                     // row stride ldc; may be null
  float* aux;          long long aux_is;                     // row stride ldc; may be null
  const float* aux_sub;                                      // instance-independent, row stride ldc; may be null
  int M, N, K;
  int ws_shift;        // log2(wscale_block) when it is a power of two, else -1 (the kernels then divide)
  // Log-softmax / KL epilogue (launch_gemm_fp8_kl only; kl_part == null: none).  Instead of, or next to, the
  // result rows the kernel leaves, per row and per 64-column part p of the row, (max, sum exp(x - max),
  // sum p_ref * (kl_ref - x), 0) in kl_part[row][p] with p_ref = exp(kl_ref - kl_ref_logz); kl_ref is [rpi][ldc]
  // (reference logits), kl_ref_logz [rpi]; both may be null (then the third value is 0).  C may be null.
  const float* kl_ref; const double* kl_ref_logz; float* kl_part; int kl_npart;
  int b16;             // operands are bfloat16 patterns, two bytes per element (lda, ldw, K stay in bytes), not e4m3 codes
};
// Parts per row of the log-softmax / KL epilogue (128-column tiles, two wavefronts across).
inline int kl_parts_per_row(int N) { return (N + 127) / 128 * 2; }
// What the fp8 GEMM kernels assume of a problem (checked on the host before a launch): 16-byte
// aligned operands and outputs, K a multiple of 128, groups of four columns that share one weight
// scale, a row of C that has room for a last partial group of four columns, and an instance's
// block of C (rows per instance x row stride) that 32-bit element offsets can address.
inline bool gemm8_prob_ok(const GemmProb& p) {
  auto a16 = [](const void* q) { return (((uintptr_t)q) & 15) == 0; };
  return p.M >= 0 && p.N >= 1 && p.K >= 128 && p.K % 128 == 0 && p.rpi >= 1 && p.lda % 16 == 0 && p.ldw % 16 == 0 &&
         p.a_is % 16 == 0 && a16(p.A) && a16(p.W) && p.ldc % 4 == 0 && p.c_is % 4 == 0 && p.add_is % 4 == 0 &&
         p.aux_is % 4 == 0 && (p.wscale_block % 4 == 0 || p.wscale_block >= p.N) && a16(p.C) && a16(p.add) && a16(p.aux) && a16(p.aux_sub) &&
         a16(p.bias) && (p.N + 3) / 4 * 4 <= p.ldc && p.lda >= p.K && p.ldw >= p.K &&
         (long long)p.rpi * p.ldc < (1ll << 31) && (p.C || p.kl_part) &&
         (p.act == 0 || p.M < 8192) &&      // the kernel of the large problems applies no activation (the path asks for none)
         (!p.kl_part || (p.kl_npart == kl_parts_per_row(p.N) && a16(p.kl_part) && a16(p.kl_ref) &&
                         (!p.kl_ref == !p.kl_ref_logz) && !p.add && !p.aux && p.act == 0));
}
// For the fp32 GEMM the same struct is used with A = float [..][lda], W = float
// [K][ldw] (row-major, K rows), ascale / wscale unused (null).

struct CombineSrc {
  const float* src;  long long src_is;
  float* slot;       long long slot_is;   // optional: slot = src - sub
  const float* sub;                       // instance-independent tile (may be null -> slot = src)
  long long bcast;                        // nonzero: src is one row of d values added to every row (a bias)
};
// run_out = run_in + bias + sum(src), element-wise over T*d
struct CombineDesc {
  const float* run_in; long long run_in_is;
  float* run_out;      long long run_out_is;
  const float* bias;   // [d] or null
  int src_begin, n_src;
};

// Fused output projection + stream update of one layer (see oproj.hip).
struct HeadAux { float* dst; long long dst_is; const float* sub; };   // per head: dst = out_h - sub (sub may be null)
struct OprojDesc {
  const uint8_t* zc;  long long zc_is;      // attention outputs, codes [inst][rpi][H][Kh]
  const float* zs;    long long zs_is;      // their scales [inst][rpi][H]
  const uint8_t* W;   const float* ws;      // W_O codes [H][N][Kh], scales [H]
  const float* extra; long long extra_is;   // fp32 head's output [inst][rpi][N] or null
  const float* run_in; long long run_in_is;
  float* run_out;      long long run_out_is;
  const float* bias;                        // [N] or null
  int H, Kh, rpi, pad_;
  int M, N, aux_begin, dh;                  // M = rows over all instances; aux_begin: first of H HeadAux, or -1; dh = d_head (Kh = dh padded to 128)
  unsigned long long skip_mask;             // bit h set: head h is computed in fp32 elsewhere (it arrives in `extra`)
};

// ---- launchers ---------------------------------------------------------------
hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t s);

hipError_t launch_slice_absmax(const float* w, long long slice_elems, int n_slices, unsigned* amax_bits,
                               int* nonfinite_flag, hipStream_t s);
// codes_out[(n_off + n) * ldq + k] = e4m3(W[slice][k][n] / scale[slice]),  W slice is [K][N] row-major
hipError_t launch_quant_transpose(const float* w, int K, int N, const unsigned* amax_bits, float* scale_out,
                                  uint8_t* codes_out, int ldq, int qbits, hipStream_t s);

hipError_t launch_embed(const int* tok, const float* W_E, const float* W_pos, float* out, int T, int S, int d,
                        hipStream_t s);

// shared_terms: the largest number of terms without instance stride in any of the groups (0: none)
hipError_t launch_build_inputs(const GroupDesc* groups, int n_groups, const Term* terms, int n_inst, int T, int B,
                               int S, int d, int ldq, int norm_kind, float eps, int shared_terms, hipStream_t s);

// Edge-batched patch: instance i reads x_i = xv - delta[send[i]] (mode 1) or
// x_i = x_{i-1} - delta[send[i]] with x_{-1} = xv (mode 2), then norm and
// fp32 / e4m3 output as in GroupDesc (base/run/terms of g are ignored).
hipError_t launch_patch_build(const GroupDesc* g, const float* xv, const float* delta0, long long delta_stride,
                              const int* send, int n_inst, int mode, int T, int B, int S, int d, int ldq,
                              int norm_kind, float eps, hipStream_t s);
// xv -= delta[send[0]]; xv -= delta[send[1]]; ... (k terms, same order as mode 2 above)
hipError_t launch_xv_advance(float* xv, const float* delta0, long long delta_stride, const int* send, int k,
                             long long n_elem, hipStream_t s);
// out = base + sum(terms) over n_elem elements (instance 0 of every term)
hipError_t launch_gemm_fp8_kl(const GemmProb* probs, int n_probs, int max_M, int max_N, int b16, hipStream_t s);
// One wavefront per row of kl_part: logz[row] = log sum exp of the row from its parts (if logz != null);
// row_kl[row] = a - (ref_logz[row % B] - logz) * ref_psum[row % B] with a = the sum of the parts' third values
// (if row_kl != null); then kl[i] = mean over the B rows of instance i (if kl != null).
hipError_t launch_kl_reduce(const float* kl_part, int npart, int rows, int B, const double* ref_logz,
                            const double* ref_psum, double* logz, double* row_kl, double* kl, hipStream_t s);
// psum[b] = sum over v < V of exp(logits[b][v] - logz[b])
hipError_t launch_ref_probs(const float* logits, const double* logz, double* psum, int B, int V, int ldv,
                            hipStream_t s);
hipError_t launch_tile_lincomb(float* out, const float* base, const Term* terms, int n_terms, long long n_elem,
                               int base_last, hipStream_t s);
hipError_t launch_tile_sub(float* out, const float* a, const float* b, long long n_elem, hipStream_t s);

// exact = 0: FP8 matrix-core instruction; exact = 1: codes decoded to fp16, fp16 matrix cores (exact
// products, fp32 sums).
// b16: the problems' operands are bfloat16 patterns (exact products on the bf16 matrix cores, fp32 sums)
hipError_t launch_gemm_fp8(const GemmProb* probs, int n_probs, int max_M, int max_N, int exact, int b16, hipStream_t s);
hipError_t launch_gemm_f32(const GemmProb* probs, int n_probs, int max_M, int max_N, hipStream_t s);
hipError_t launch_oproj_fused(const OprojDesc* descs, int desc_index, const HeadAux* auxs, int M, int N, int H, int dh,
                              int exact, int b16, hipStream_t s);

// Causal attention per (instance, sequence, head).  q, k, v: fp32 rows [inst][T][..]; head hl of the
// launch reads columns hl * head_cols .. + dh of each and writes output head h0 + hl (of H).
// Heads whose bit is clear in f32_mask: z rows quantised per head -> zcodes [inst][T][H][ldz], zscale [inst][T][H].
// Heads whose bit is set: z written unquantised to zf32 [inst][T][nf][dh], nf = number of set bits, a head's place
// = number of set bits below its own.
struct AttnSrc {
  const float* q; long long q_is; int q_ld; int form;     // form: 1 = the query-tile kernel also where the whole-sequence kernel applies (0: the launcher chooses)
  const float* k; long long k_is; int k_ld; int pad1_;
  const float* v; long long v_is; int v_ld; int pad2_;
  int n_heads, h0, head_cols, qbits;    // qbits: grid of the output codes (device_util.h, q_encode)
};
hipError_t launch_attention(const AttnSrc& src, uint8_t* zcodes, long long zc_is, float* zscale,
                            long long zs_is, float* zf32, long long zf_is, unsigned long long f32_mask, unsigned long long dead_mask, int n_inst, int B, int S,
                            int H, int dh, int ldz, int rope, const float* rope_tab, hipStream_t s);
// rope_tab: [n_pos][dh / 2] pairs (cos, sin), filled by launch_rope_table; read only when rope != 0, n_pos >= S
hipError_t launch_rope_table(float* tab, int n_pos, int dh, float theta, hipStream_t s);

hipError_t launch_combine(const CombineDesc* descs, int desc_index, const CombineSrc* srcs, int n_inst,
                          long long n_elem, int d, hipStream_t s);

// hidden rows [inst][T][m]: h = up (act 0), tanh-GELU(up) (act 1) or silu(gate) * up (act 2); row-quantise.
hipError_t launch_hidden_quant(const float* up, const float* gate, long long h_is, uint8_t* codes, long long c_is,
                               float* scale, long long s_is, int n_inst, int T, int m, int ldq, int act, int qbits,
                               hipStream_t s);

// logz[b] = log(sum_v exp(logits[b][v]))  (double)
hipError_t launch_logz(const float* logits, int rows, int V, int ldv, double* logz, hipStream_t s);
// kl[inst] = mean_b sum_v p_ref (log p_ref - log p_inst)
hipError_t launch_kl(const float* logits, long long l_is, const float* ref_logits, const double* ref_logz,
                     double* row_kl, double* kl, int n_inst, int B, int V, int ldv, hipStream_t s);

// fp32 hidden rows in place: up = silu(gate) * up (the all-fp32 mode's SwiGLU; GELU is the fp32 GEMM's epilogue)
hipError_t launch_swiglu_f32(float* up, const float* gate, long long n_elem, hipStream_t s);

// the gather / patch kernels' output quantiser on given rows (cols a multiple of 64, at most 4096; codes row stride cols)
hipError_t launch_emit_rows(const float* x, int rows, int cols, uint8_t* codes, float* scales, int qbits, hipStream_t s);
hipError_t launch_quant_rows_plain(const float* x, int rows, int cols, uint8_t* codes, float* scales, int qbits,
                                   hipStream_t s);

// Logit-difference task metric.  ld[inst * B + b] = logit[answer[b]] - logit[distractor[b]] of row (inst, b), from the
// row's e4m3 codes and scale and the unembedding's codes [vocab][ldw] (or, fp32 variant, from unquantised rows and
// the fp32 unembedding [d][ldw]); score[inst] = mean_b (ref_ld[b] - ld[inst * B + b]).
hipError_t launch_logit_pair(const uint8_t* codes, long long c_is, const float* scale, long long s_is, int ldq, int K,
                             const uint8_t* wcodes, int ldw, const float* wscale, const float* bias, const int* ans,
                             const int* dis, int n_inst, int B, double* ld, int b16, hipStream_t s);
hipError_t launch_logit_pair_f32(const float* x, long long x_is, int d, const float* W, int ldw, const float* bias,
                                 const int* ans, const int* dis, int n_inst, int B, double* ld, hipStream_t s);
hipError_t launch_metric_mean(const double* ld, const double* ref_ld, double* score, int n_inst, int B, hipStream_t s);

}  // namespace pahq
