// Host-side state of one model and the pass executor.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <vector>
#include "../../include/pahq.h"
#include "graph.h"
#include "controller.h"
#include "kernels.h"

namespace pahq {

enum PassKind { BASE_CLEAN = 0, BASE_CORRUPT, PI_CORRUPT, PI_REF, STATE, CAND, PREFIX, PI_REF_LAYER };

struct PassArgs {
  PassKind kind;
  int p0;              // first position recomputed
  int n;               // instances
  int pl, ph;          // fp32 head (layer, head) or -1
  int v;               // patched receiver (CAND) or -1
  int patch_mode;      // 1 independent, 2 cumulative
  int io_off = 0;      // first element of send_dev / kl_dev this pass reads / writes
  const unsigned long long* heads = nullptr;   // per layer: bit h set = head h in fp32 (a set of fp32 heads instead of (pl, ph))
  bool keep_logits = false;                    // a scored pass also stores its logits (M->logits)
  int chan_count[3] = {0, 0, 0};               // CAND into a head input with an fp32 head: when not all zero, the first
                                               // chan_count[0] instances patch the head's query input, the next its key
                                               // input, the rest its value input (their current inputs in M->xvc)
};

struct Arena {          // descriptor staging: pinned host mirror + device copy, a small ring
  static const int SLOTS = 4;
  char* host[SLOTS];
  char* dev[SLOTS];
  hipEvent_t ev[SLOTS];
  size_t slot_bytes;
  int next;
};

// fp32 head weights kept in pinned host memory (pahq_config.fp32_residency = PAHQ_FP32_ON_HOST): one block per head
// [W_Q | W_K | W_V | W_O | b_Q | b_K | b_V]; the device holds 2 H blocks (controller.h, HeadSlots) that a second stream
// fills.  ready[s] is recorded on the copy stream behind a slot's transfer, released[s] on the compute stream behind
// the last pass that read the slot; each stream waits for the other's event before it touches the slot.
struct W32Cache {
  bool on = false;
  float* host = nullptr;            // pinned, [L * H][head_floats]
  float* dev = nullptr;             // [2 H][head_floats], inside the workspace
  size_t head_floats = 0, off[7] = {0, 0, 0, 0, 0, 0, 0};    // offsets of W_Q, W_K, W_V, W_O, b_Q, b_K, b_V in a block
  HeadSlots slots;
  std::vector<hipEvent_t> ready, released;
  hipStream_t copy_stream = nullptr;
  long long bytes_moved = 0;
};

}  // namespace pahq

struct pahq_model {
  pahq_config cfg;
  pahq::GraphDims g;
  int B, S, T, L, H, dh, d, m, V;
  int Kd, Kh, Km;        // K extents padded to multiples of 128
  int Vp;                // row stride of logits buffers (vocab rounded up to 4 floats)
  int nmax, G;           // max instances; max groups per layer (3H + 1)
  long long tile;        // T * d
  hipStream_t stream;

  // device memory (all inside the caller's workspace)
  char* ws; size_t ws_bytes, ws_used;
  float *W_E, *W_pos, *W_Q, *W_K, *W_V, *W_O, *b_Q, *b_K, *b_V, *b_O;
  float *ln1_g, *ln1_b, *ln2_g, *ln2_b, *W_in, *b_in, *W_gate, *W_out, *b_out, *lnf_g, *lnf_b, *W_U, *b_U;
  float* zeros_d;                         // [max(d, 64)] zeros (norm offset for RMSNorm)
  float* rope_tab;                        // [32][dh / 2] (cos, sin) pairs of the rotary positions (null without them)
  float* bqkv;                            // [L][3][H][dh] fused projection bias
  uint8_t *qkv_codes, *o_codes, *in_codes, *gate_codes, *out_codes, *u_codes;
  float *qkv_scale, *o_scale, *in_scale, *gate_scale, *out_scale, *u_scale;
  unsigned* amax_tmp; int* flag_tmp;
  int *tok_clean, *tok_corrupt, *send_dev;
  float *clean, *corrupt, *delta;         // [Ns] tiles each (delta has one more, all zero)
  float *rc, *rx;                         // [2L+1] residual prefixes (entry 0 unused: it is sender 0's tile)
  float *logits_clean, *logits_corrupt;   // [B][V]
  double* logz_clean;                     // [B]
  float *cpi, *rxpi, *ref_logits; double* ref_logz;   // state of the current fp32 head (the ref_* point into the *_all arrays)
  float* ref_logits_all; double *ref_logz_all, *psum_ref_all, *ld_ref_all;   // [H] copies: the reference runs of all heads of layer ref_layer
  int ref_layer = -1;                     // layer whose H reference runs the *_all arrays hold (one H-instance pass), or -1
  long long plan_serial = 0;              // counts make_plan calls: the per-layer sums of dead heads' stand-ins are kept per plan
  std::vector<long long> deadsum_tag;     // per layer: 2 * plan_serial + (precision-set pass) the layer's tile was made for, or -1
  int qbits;                              // grid of the low-precision operands: 8 = E4M3, 4 = 4-bit round-to-nearest
  bool nb16;                              // the MLP matrices and the unembedding multiply bfloat16 operands instead
  int Kd_o, Km_o;                         // bytes of a d_model / d_mlp row of those operands (= Kd, Km unless nb16)
  int attn_form = 0;                      // 1: the query-tile attention kernel at every sequence length (AttnSrc.form)
  bool skip_dead;                         // passes over a pruned graph leave out nodes no kept path connects to the output
  bool all_f32;                           // PAHQ_ALL_FP32: every matrix product on the fp32 masters, no quantiser
  int f32_groups;                         // receiver-input groups of a layer that may need fp32 rows (per instance)
  int f32_heads_max;                      // heads whose attention output may be needed unquantised (per instance)
  float* xv;                              // current input of the receiver under evaluation
  float *qkv_sh, *oth, *deadsum, *sh_slots, *qv, *xvc;    // xvc: three tiles, the current inputs of a head's query / key / value receivers    // first-layer state shared by all candidates of a receiver
  float *run_a, *run_b;                   // [nmax] tiles each
  uint8_t* xcodes; float* xscale; float* xf32;
  float* qkv; uint8_t* zcodes; float* zscale; float* zf32;
  float *headout, *mlpout, *hid, *hid2; uint8_t* hcodes; float* hscale;
  uint8_t* lastcodes; float* lastscale; float* logits;
  float* slots; long long pool_tiles;
  double *row_kl, *kl_dev;
  double *psum_clean, *psum_ref;          // [B] sums of the reference rows' probabilities
  int metric;                             // PAHQ_METRIC_*
  int *ans_dev, *dis_dev;                 // [B] answer / distractor token of each sequence (logit-difference metric)
  double *ld_clean, *ld_ref;              // [B] logit difference of the cached clean run / of the current fp32 head's reference run
  float* kl_part; int kl_npart;           // [nmax * B][kl_npart][4]: what the unembedding leaves of a scored pass
  double* kl_host;                        // pinned
  int* send_host;                         // pinned
  int ncap;                               // candidates one host round trip can carry (size of the send / kl arrays)
  pahq::Arena arena;
  pahq::W32Cache w32;
  float* stage = nullptr;                 // fp32 masters pass through here on their way to the quantiser (host residency)

  // host state
  std::vector<uint8_t> removed;           // canonical edge order
  std::vector<int64_t> edge_off;          // [Nr + 1]
  bool has_cache;
  bool pi_corrupt = false;                // the corrupted run under that head's precision set (cpi, rxpi) is current too
  int pi_l, pi_h, pi_p0;                  // fp32 head whose state (cpi, rxpi, ref_*) is current; -2 = none
  pahq::RecvPlan plan;
  int64_t counters[3];

  // optional per-kernel-class timing with HIP events
  bool prof_on;
  std::vector<hipEvent_t> prof_ev;        // pairs (start, stop)
  std::vector<int> prof_cls;              // class of each recorded pair
  int prof_used;                          // pairs recorded since the last harvest
  unsigned prof_mask = 0xFFFFFFFFu;       // kernel classes that are recorded
  int prof_every = 1;                     // ... in every prof_every-th pass
  long long prof_pass = 0;                // passes seen while profiling
  pahq_kernel_stat prof[PAHQ_N_KERNEL_CLASSES];
};

namespace pahq {
// Residual-stream prefix tiles of the cached clean / corrupted run.  Position 0
// is the embedding's own tile; in attention-only models the position before
// layer l+1 is the position after the heads of layer l.
static inline int canon_pos(const pahq_model* M, int p) {
  return (M->g.mu == 0 && p > 0 && (p & 1) == 0) ? p - 1 : p;
}
static inline float* clean_prefix(pahq_model* M, int p) {
  return p == 0 ? M->clean : M->rc + (long long)canon_pos(M, p) * M->tile;
}
static inline float* corrupt_prefix(pahq_model* M, int p) {
  return p == 0 ? M->corrupt : M->rx + (long long)canon_pos(M, p) * M->tile;
}
int run_pass(pahq_model* M, const PassArgs& a, const RecvPlan* plan);
void make_plan(pahq_model* M, int p0, int v, RecvPlan& out);
// fp32 matrix (which = 0..3: W_Q, W_K, W_V, W_O) or projection bias (4..6: b_Q, b_K, b_V) of head (l, h): where a pass
// reads it.  With host residency that is the head's slot, valid between w32_acquire and w32_release.
static inline const float* w32_ptr(const pahq_model* M, int which, int l, int h) {
  const long long id = (long long)l * M->H + h;
  if (M->w32.on) return M->w32.dev + (size_t)M->w32.slots.slot_of((int)id) * M->w32.head_floats + M->w32.off[which];
  const float* base[7] = {M->W_Q, M->W_K, M->W_V, M->W_O, M->b_Q, M->b_K, M->b_V};
  return base[which] + id * (which < 3 ? (long long)M->d * M->dh : which == 3 ? (long long)M->dh * M->d : (long long)M->dh);
}
int w32_acquire(pahq_model* M, int l, unsigned long long mask);     // before the first launch that reads them
int w32_release(pahq_model* M, int l, unsigned long long mask);     // behind the last
int w32_prefetch(pahq_model* M, int l, unsigned long long mask);    // expected next: starts the transfers, waits for nothing
int prof_harvest(pahq_model* M);     // synchronises the stream and folds recorded event pairs into M->prof
}  // namespace pahq
