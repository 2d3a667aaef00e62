/*
 * pahq.h -- C ABI of libpahq: the ACDC edge-ablation loop under per-attention-head
 * mixed precision (PAHQ) on one AMD MI355X (gfx950).
 *
 * What the library computes (citations are to the PAHQ paper):
 *   - A transformer is a graph whose nodes are attention heads and MLP layers
 *     (plus the embedding and the unembedding); a node's input is the sum of
 *     the outputs of its predecessors (Appendix "Preliminaries", Circuit
 *     Discovery).  Head inputs are split into query, key and value inputs
 *     (split_qkv = 1, the default) or are one input per head (split_qkv = 0).
 *   - Removing an edge replaces the sender's activation at that receiver by the
 *     activation of a run on the corrupted prompt (activation patching, same
 *     appendix); ACDC removes an edge when the loss change stays below a
 *     threshold tau (Eq. C = G \ {e : Delta L(e) < tau}); the loss is the KL
 *     divergence to the clean model's output distribution (Appendix "Metrics").
 *   - While an edge is evaluated only the investigated head runs in fp32; all
 *     other heads, the MLPs and the unembedding run on FP8 E4M3 operands
 *     (Sec. "Selective Precision Allocation Strategy", Eq. P_t; Sec.
 *     "Mixed-Precision Computation Design"); the attention core, norms, residual
 *     sums and the loss stay in fp32 (Sec. "Scheduler Implementation", Phase 3).
 *   - Quantisation is round-to-nearest with the scale set by the absolute
 *     maximum (Appendix "Quantization", Eq. RTN-Q), applied to the E4M3 grid
 *     (bias 7, smallest normal 2^-6, largest 448):
 *         scale = amax / 448 (1 if amax = 0), inv = 1 / scale, code = rne_e4m3(x * inv),
 *     every step one IEEE binary32 operation, |x*inv| > 448 saturating.  Weights
 *     carry one scale per slice (each head's W_Q, W_K, W_V, W_O; each layer's
 *     W_in, W_gate, W_out; W_U), activations one scale per row of the GEMM's left
 *     operand (per head for the attention outputs).
 *
 * Ids.  mu = 1 if d_mlp > 0 else 0.
 *   senders    0 = EMBED; HEAD(l,h) = 1 + l*(H+mu) + h; MLP(l) = 1 + l*(H+mu) + H
 *   receivers  HEADIN(l,h,c) = l*(3H+mu) + 3h + c (c: 0 query, 1 key, 2 value);
 *              MLPIN(l) = l*(3H+mu) + 3H; OUT = L*(3H+mu)
 *              (split_qkv = 0: HEADIN(l,h) = l*(H+mu) + h; MLPIN(l) = l*(H+mu) + H; OUT = L*(H+mu))
 *   An edge (s -> r) exists iff s is strictly upstream of r; for every receiver
 *   these are the senders 0 .. pahq_n_upstream(r)-1.  Canonical edge order:
 *   receivers ascending, then senders ascending.
 *
 * Conventions.  Every function returns 0 or a negative PAHQ_E* code; nothing is
 * printed, nothing throws, and a failed call leaves the removed set unchanged.
 * Pointers are HOST pointers unless the comment says "device".  All device work
 * is enqueued on the stream given to pahq_init_model; calls that return host
 * values synchronise that stream.  The library performs no device allocation:
 * everything lives in the caller's workspace.  Not thread-safe per model.
 * There is no CPU fallback: without a usable HIP device every call that needs
 * one fails with PAHQ_EHIP.
 */
#ifndef PAHQ_H
#define PAHQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  PAHQ_OK = 0,
  PAHQ_EINVAL = -1,   /* bad argument (null pointer, id out of range, shape mismatch)   */
  PAHQ_ESTATE = -2,   /* call out of order (e.g. eval before clean_cache), or a removed  */
                      /* set with edges into receivers upstream of the one evaluated    */
  PAHQ_ENOMEM = -3,   /* workspace too small                                            */
  PAHQ_EHIP = -4,     /* a HIP runtime call failed / no device                          */
  PAHQ_ENAN = -5,     /* non-finite weight                                              */
  PAHQ_EUNSUPPORTED = -6, /* valid request that this build does not implement          */
  PAHQ_ETOOBIG = -7    /* input larger than the fixed capacity of an allocation-free call  */
};

enum { PAHQ_NORM_LAYER = 0, PAHQ_NORM_RMS = 1 };
enum { PAHQ_ACT_NONE = 0, PAHQ_ACT_GELU = 1, PAHQ_ACT_SWIGLU = 2 };
enum { PAHQ_POS_LEARNED = 0, PAHQ_POS_ROPE = 1 };
enum { PAHQ_ALL_FP32 = 0, PAHQ_ALL_FP8 = 1, PAHQ_PAHQ = 2 };
enum { PAHQ_LOGITS_CLEAN = 0, PAHQ_LOGITS_CORRUPT = 1, PAHQ_LOGITS_REF = 2 };
enum { PAHQ_MMA_FP8 = 0, PAHQ_MMA_F16_EXACT = 1 };
enum { PAHQ_W_Q = 0, PAHQ_W_K = 1, PAHQ_W_V = 2, PAHQ_W_O = 3, PAHQ_W_IN = 4, PAHQ_W_GATE = 5,
       PAHQ_W_OUT = 6, PAHQ_W_U = 7 };

typedef struct pahq_model pahq_model;   /* opaque, owned by the library (host memory) */

/* Plain data, caller-owned, copied by pahq_init_model. */
typedef struct {
  int32_t n_layers, n_heads, d_head, d_model;
  int32_t d_mlp;            /* 0 = attention-only model                                         */
  int32_t vocab, n_ctx;     /* n_ctx: rows of W_pos (learned positions); sequences must fit      */
  int32_t norm;             /* PAHQ_NORM_*: LayerNorm (biased variance) or RMSNorm (no offset)   */
  int32_t act;              /* PAHQ_ACT_*: GELU is the tanh form; SWIGLU = silu(x W_gate)*(x W_in) */
  int32_t pos;              /* PAHQ_POS_*: ROPE rotates pairs (i, i + d_head/2) of q and k        */
  float norm_eps, rope_theta;
  int32_t split_qkv;        /* 1: the query, key and value inputs of a head are separate receivers (the
                               graph the paper's edge counts fit: 32 491 edges for GPT-2 small);
                               0: a head has one receiver that all three projections read (11 611)  */
  int32_t precision;        /* PAHQ_PAHQ: fp32 investigated head (the head a candidate edge feeds);
                               PAHQ_ALL_FP8: no fp32 head (all-8-bit RTN baseline);
                               PAHQ_ALL_FP32: no quantiser anywhere, every matrix product on the fp32
                               masters (the unaccelerated ACDC of the paper's runtime table)        */
  int32_t max_batch_edges;  /* most candidates evaluated in one device batch (>= 1)               */
  int32_t mma;              /* how the E4M3 x E4M3 products are summed:
                               PAHQ_MMA_F16_EXACT (recommended): the codes are converted to fp16 in
                               registers (exact) and fed to the fp16 matrix cores: exact products,
                               fp32 accumulation.  This is the arithmetic the method defines.
                               PAHQ_MMA_FP8: the FP8 matrix-core instruction.  Its adder aligns the
                               products of one instruction to the largest one and drops what falls
                               below a window of about 14 bits (measured on gfx950: up to 2^-13 of
                               sum|a*w| per sum, truncating toward zero), which makes every KL come out
                               about 1.3 % low.  About 6 % faster end to end.
                               Codes and scales are identical in both modes.                        */
  int32_t low_bits;         /* grid of the low-precision operands (weights per slice, activation rows):
                               8 (or 0): FP8 E4M3, the paper's setting.
                               4: the 4-bit point of the paper's bit-width ablation (Sec. "Ablation
                               Studies", Different Quantization Precisions), Eq. RTN-Q with N = 4 as
                               printed: step = max|x| / 2^(N-1), values round to the nearest multiple
                               (ties to even), |multiple| <= 8.  The multiples are stored as the E4M3
                               codes of those integers (exact), so pahq_get_weight_q and the quantiser
                               hooks return, at 4 bits, E4M3 codes of integers and the step as scale;
                               the matrix products are the same exact kernels.
                               16: the 16-bit point of that table: every quantised operand, the
                               heads' included, is rounded to bfloat16 (nearest-even, no scale;
                               this implies nonattn_bf16).  d_head 32 or 64; needs
                               PAHQ_MMA_F16_EXACT.  Weights and rows are then two-byte patterns:
                               pahq_get_weight_bf16 / pahq_round_rows_bf16 instead of the E4M3
                               hooks.                                                             */
  int32_t nonattn_bf16;     /* 1: the components that are not attention heads -- the MLP matrices and the
                               unembedding -- multiply bfloat16 operands (activations and weights rounded
                               to bfloat16, nearest-even, no scale) instead of low_bits ones; the heads
                               keep low_bits (Sec. "Selective Precision Allocation Strategy": bfloat16 for
                               non-attention components).  Products are exact on the bf16 matrix cores,
                               sums fp32.  Needs PAHQ_MMA_F16_EXACT; ignored with PAHQ_ALL_FP32.
                               0 (default): every quantised product uses low_bits.                   */
  int32_t fp32_residency;   /* where the fp32 masters live after pahq_init_model (Sec. "Selective Precision
                               Allocation Strategy", Hierarchical Weight Scheduling; Sec. "Algorithm
                               Implementation in Practice", Scheduler Implementation):
                               PAHQ_FP32_IN_HBM (0, default): all of them in the workspace.
                               PAHQ_FP32_ON_HOST: the heads' W_Q / W_K / W_V / W_O and projection biases
                               stay in pinned host memory that the library allocates (hipHostMalloc, one
                               block per head); the device holds 2 * n_heads head slots, filled by a second
                               stream of the library's own: a pass waits for the heads it computes in fp32
                               (S_t), and the heads expected next (S_t+1: the following layer of the same
                               pass, the next head in the sweep's order) are transferred while it runs.
                               The fp32 masters of the MLPs and the unembedding only pass through a staging
                               buffer on their way to the quantiser.  The workspace shrinks by those
                               masters; every result is bit-identical to PAHQ_FP32_IN_HBM.
                               Not with PAHQ_ALL_FP32 (which multiplies the masters themselves).       */
} pahq_config;
enum { PAHQ_FP32_IN_HBM = 0, PAHQ_FP32_ON_HOST = 1 };

/* fp32 master weights, row-major.  All pointers host memory (on_device = 0) or
 * all device memory (on_device = 1); the library copies them into the workspace.
 *   W_E [vocab][d_model]   W_pos [n_ctx][d_model] (learned positions only, else NULL)
 *   W_Q, W_K, W_V [L][H][d_model][d_head]   b_Q, b_K, b_V [L][H][d_head]
 *   W_O [L][H][d_head][d_model]             b_O [L][d_model]
 *   ln1_g, ln1_b, ln2_g, ln2_b [L][d_model] lnf_g, lnf_b [d_model]  (the *_b are ignored for RMSNorm)
 *   W_in [L][d_model][d_mlp]  b_in [L][d_mlp]  W_gate [L][d_model][d_mlp] (SwiGLU only)
 *   W_out [L][d_mlp][d_model] b_out [L][d_model]   (all NULL when d_mlp = 0)
 *   W_U [d_model][vocab]      b_U [vocab]
 * b_O and b_out are constants of the residual stream, not part of any sender's output. */
typedef struct {
  const float *W_E, *W_pos, *W_Q, *W_K, *W_V, *W_O, *b_Q, *b_K, *b_V, *b_O;
  const float *ln1_g, *ln1_b, *ln2_g, *ln2_b, *W_in, *b_in, *W_gate, *W_out, *b_out;
  const float *lnf_g, *lnf_b, *W_U, *b_U;
  int32_t on_device;
} pahq_weights;

/* One evaluated candidate of a sweep, in evaluation order. */
typedef struct {
  int32_t receiver, sender;
  float kl_new;      /* KL with the candidate edge removed on top of the current removed set */
  float kl_cur;      /* KL of the current removed set before the decision                   */
  int32_t removed;   /* 1 if kl_new - kl_cur < tau (edge removed, kl_cur becomes kl_new)     */
} pahq_trace_rec;

/* ---- graph helpers (pure host arithmetic, no device needed) ---------------- */
int pahq_n_senders(const pahq_config*, int32_t* out);
int pahq_n_receivers(const pahq_config*, int32_t* out);
int pahq_n_upstream(const pahq_config*, int32_t receiver, int32_t* out);   /* senders 0..out-1 feed it */
int pahq_edge_count(const pahq_config*, int64_t* out);
int pahq_edge_id(const pahq_config*, int32_t sender, int32_t receiver, int64_t* out); /* canonical index */
int pahq_node_of_receiver(const pahq_config*, int32_t receiver, int32_t* sender_out); /* -1 for OUT */

/* Bytes of device workspace pahq_init_model needs for batches of B sequences
 * of S tokens (paper, Appendix "Integration with ACDC": all low-precision
 * weights resident on the device; here the fp32 masters and every activation
 * cache are resident too, unless fp32_residency says otherwise).  S <= 128, d_head one of
 * 16, 32, 64, 128, d_model a multiple of 64 up to 4096, at most 64 heads, d_mlp a
 * multiple of 4: PAHQ_EUNSUPPORTED otherwise. */
int pahq_workspace_bytes(const pahq_config*, int32_t B, int32_t S, size_t* out);

/* Copies the fp32 masters into `workspace` (DEVICE memory, 256-byte aligned,
 * caller-owned, must outlive the model) and quantises every weight slice to
 * E4M3 codes + scale (Appendix "Quantization", Eq. RTN-Q).  `hip_stream` is a
 * hipStream_t (NULL = default stream).  PAHQ_ENAN if a weight is not finite. */
int pahq_init_model(const pahq_config*, const pahq_weights*, int32_t B, int32_t S,
                    void* workspace, size_t workspace_bytes, void* hip_stream, pahq_model** out);

/* Runs the clean and the corrupted prompt batch through the model (no fp32
 * head) and caches every sender's output for both, their difference and the
 * residual stream (Appendix "Integration with ACDC": first and second
 * inference, done once instead of once per edge).  Tokens: host int32 [B][S],
 * 0 <= id < vocab.  Resets the removed set to empty. */
int pahq_clean_cache(pahq_model*, const int32_t* clean_tok, const int32_t* corrupt_tok);

/* Which loss every evaluation returns and the sweep decides on (Appendix "Metrics", "Task Metrics"):
 *   PAHQ_METRIC_KL          batch-mean KL(P_ref || P) at the last position (the default)
 *   PAHQ_METRIC_LOGIT_DIFF  the task metric: batch mean of how far logit[answer] - logit[distractor] at the
 *                           last position has dropped below its value in the reference run (0 for the unpruned
 *                           graph, like the KL; larger = worse); answer_ids, distractor_ids: host int32 [B],
 *                           0 <= id < vocab, different per sequence (ignored for PAHQ_METRIC_KL, may be NULL).
 *                           Only the two logits are computed for a candidate, not the unembedding.
 * Wherever this header says KL, the chosen loss is meant.  Call before pahq_clean_cache: the cache pass takes the
 * reference values of the loss, so a change of metric drops the caches (PAHQ_ESTATE until they are rebuilt). */
enum { PAHQ_METRIC_KL = 0, PAHQ_METRIC_LOGIT_DIFF = 1 };
int pahq_set_metric(pahq_model*, int32_t metric, const int32_t* answer_ids, const int32_t* distractor_ids);

/* Evaluates n candidate edges (sender_ids[i] -> receiver) INDEPENDENTLY: the
 * i-th result is the batch-mean KL(P_ref || P_i) at the last position, where
 * P_i is the clean run with the current removed set plus that one edge
 * removed, and P_ref the clean run with nothing removed, both under the
 * precision set of `receiver` (third inference of the paper's algorithm; Eq.
 * Delta L).  Does not modify the removed set.  kl_out: host, n floats.  Any n
 * >= 0; batches of max_batch_edges are formed internally.  Results do not
 * depend on n, on the other candidates or on earlier calls.
 * The removed set may only hold edges into receivers at or after `receiver`'s
 * position in the forward pass (its own layer's inputs and everything
 * downstream): what lies upstream is taken from the caches of the unmodified
 * runs.  Every state of the sweep (receivers in descending order) is of this
 * kind; any other removed set gives PAHQ_ESTATE, here and in
 * pahq_eval_current. */
int pahq_eval_edges(pahq_model*, int32_t receiver, const int32_t* sender_ids, int32_t n, float* kl_out);

/* The same evaluation for a list of candidate edges into any receivers: kl_out[i] is, bit for bit, what
 * pahq_eval_edges returns for the edge (sender_ids[i] -> receivers[i]) -- each candidate judged on its own, on top
 * of the current removed set, under the precision set of ITS receiver (Eq. Delta L; third inference of the
 * paper's algorithm) -- and the removed set is not modified.  receivers, sender_ids: host, n entries; kl_out: host,
 * n floats.  The list is taken in the order given: neighbouring entries with the same receiver form one run, and
 * with PAHQ_PAHQ up to three neighbouring runs that are the query, key and value inputs of one head, in that order,
 * share device batches (their candidates have the same fp32 head, the same reference and the same layer state and
 * differ in which of the head's three projections reads the patched input), which fills the batches of the early
 * layers, where a single receiver has few senders.  The condition on the removed set is that of pahq_eval_edges, for
 * every receiver of the list; a receiver that violates it gives PAHQ_ESTATE (results before it are written). */
int pahq_eval_edge_list(pahq_model*, int64_t n, const int32_t* receivers, const int32_t* sender_ids, float* kl_out);

/* KL of the current removed set itself under the precision set of `receiver`. */
int pahq_eval_current(pahq_model*, int32_t receiver, float* kl_out);

/* One reverse-topological ACDC pass from the empty removed set (Eq. C = G \
 * {e : Delta L(e) < tau}): receivers in descending id, senders in descending
 * id; an edge is removed iff kl_new - kl_cur < tau (then kl_cur = kl_new); a
 * receiver whose node has no kept outgoing edge is skipped and all its in-edges
 * are removed.  Candidates are evaluated in speculative device batches; the
 * decisions are exactly those of the one-by-one procedure.
 *   receivers/n_receivers  restrict the pass to these receiver ids (NULL/0 = all)
 *   kept      host, pahq_edge_count bytes, canonical order, 1 = edge kept (may be NULL)
 *   n_evals   number of candidates whose decision was taken (may be NULL)
 *   trace     host array of trace_cap records, first min(n_evals, trace_cap) filled (may be NULL)
 * The removed set of the model is left at the sweep's result. */
int pahq_acdc_sweep(pahq_model*, float tau, const int32_t* receivers, int32_t n_receivers,
                    uint8_t* kept, int64_t* n_evals, pahq_trace_rec* trace, int64_t trace_cap);

/* Continues an interrupted sweep: the same pass over `receivers` (NULL/0 = all), starting from the model's CURRENT
 * removed set instead of the empty one.  A sweep decides receiver by receiver, so its state after any receiver is
 * the removed set alone: rebuild it from the trace (or keep pahq_get_removed), hand it to pahq_set_removed -- on this
 * model or, after pahq_clean_cache with the same prompts, on a new one -- and name the receivers not yet decided.
 * The result is that of the uninterrupted sweep, decision for decision.  PAHQ_ESTATE if a named receiver already
 * has a removed edge, or if the removed set touches a receiver upstream of a named one. */
int pahq_acdc_sweep_resume(pahq_model*, float tau, const int32_t* receivers, int32_t n_receivers,
                           uint8_t* kept, int64_t* n_evals, pahq_trace_rec* trace, int64_t trace_cap);

/* The same pass for a grid of thresholds (the paper's Experiments section scans 21 log-spaced values of tau in
 * [0.001, 3.16] to trace a ROC curve): every sweep starts from the empty removed set and all of them share the
 * clean / corrupted caches of one pahq_clean_cache call, which is the only part of a sweep that does not depend
 * on tau.  taus: host, n_taus values; kept: host, n_taus x pahq_edge_count bytes (row i = result at taus[i]);
 * n_evals: host, n_taus counts (may be NULL).  The removed set is left at the last threshold's result. */
int pahq_acdc_sweep_grid(pahq_model*, const float* taus, int32_t n_taus, const int32_t* receivers, int32_t n_receivers,
                         uint8_t* kept, int64_t* n_evals);

/* The precision policy exactly as Eq. P_t prints it: FP32 for the SOURCE node of the evaluated edge (when it is a
 * head), FP8 for everything else.  Under it the precision set changes with every candidate, so nothing can be shared
 * between the candidates of a receiver: each one costs a corrupted run and a reference run under its set from the
 * sender's layer on, the current graph and the graph without the edge -- the three inferences per edge of the
 * appendix algorithm plus the current state.  kl_new_out[i] / kl_cur_out[i]: loss with / without the i-th edge
 * removed on top of the current removed set, both under the set of sender_ids[i]; the sweep decides on their
 * difference, in the same order and by the same rule as pahq_acdc_sweep.  Meant for comparing the two policies
 * (the default, receiver side, is what pahq_eval_edges and pahq_acdc_sweep implement); one candidate at a time. */
int pahq_eval_edges_sender_policy(pahq_model*, int32_t receiver, const int32_t* sender_ids, int32_t n, float* kl_new_out,
                                  float* kl_cur_out);
int pahq_acdc_sweep_sender_policy(pahq_model*, float tau, const int32_t* receivers, int32_t n_receivers, uint8_t* kept,
                                  int64_t* n_evals, pahq_trace_rec* trace, int64_t trace_cap);

/* Inference on a pruned graph with a SET of fp32 heads (Appendix "Integration with ACDC", last block of the
 * algorithm: forward on G_sparse with the heads H_high of every layer in high precision): the clean run in
 * which every edge that is not kept carries the corrupted run's activation, the flagged heads' query / key /
 * value and output projections on the fp32 masters and unquantised activations, everything else on E4M3
 * operands.  kl_out: batch-mean KL at the last position to the clean run with no edge removed under the
 * same set of fp32 heads (the corrupted activations come from a corrupted run under that set as well).
 *   kept        host, pahq_edge_count bytes, canonical order, 1 = kept; NULL = the model's current removed set
 *   f32_heads   host, [n_layers][n_heads] bytes, 1 = head in fp32; NULL = every head that still has a kept
 *               edge in and a kept edge out.  Ignored unless the model's precision is PAHQ_PAHQ (ALL_FP8: no
 *               fp32 head; ALL_FP32: everything is fp32 anyway)
 *   logits_out  host, [B][vocab] logits of the pruned run, or NULL
 * Any removed set is accepted (the pass starts at the embedding).  The model's removed set is not changed;
 * the state of the head investigated last is dropped (the next evaluation rebuilds it). */
int pahq_eval_circuit(pahq_model*, const uint8_t* kept, const uint8_t* f32_heads, float* kl_out, float* logits_out);

/* Dead nodes.  Once every edge out of a node is removed (or leads only to such nodes), each of its receivers reads
 * the corrupted run's cached activation from it whatever the node computes (Appendix "Preliminaries": a removed
 * edge carries the corrupted activation), and ACDC drops its incoming edges unevaluated (Appendix "Integration with
 * ACDC").  With on = 1 (the default) passes over a pruned graph -- current state, candidates, circuit evaluation,
 * sweeps -- do not compute such nodes: the stream takes their cached corrupted outputs in their place.  In exact
 * arithmetic nothing changes; in binary32 the order of a few additions does.  on = 0 computes every node (for
 * comparison and timing).  Takes effect from the next evaluation. */
int pahq_set_dead_node_skipping(pahq_model*, int32_t on);

/* Host-resident fp32 head weights (pahq_config.fp32_residency = PAHQ_FP32_ON_HOST; both calls return PAHQ_ESTATE
 * otherwise).
 * pahq_prefetch_heads: a caller that drives evaluations in an order of its own names the heads it will need next
 * (Eq. Prefetch(t): the weights of S_t+1 move while step t computes): their transfers are started on the library's
 * copy stream unless they are on the device or on their way already; nothing waits.  heads: bit h = head h of
 * `layer`.  The library's own loops (sweeps, edge lists, circuit evaluation) predict by themselves.
 * pahq_get_transfer_stats: since init, [0] head uses by passes, [1] of those, uses that had to start the transfer
 * themselves and wait for all of it (demand transfers), [2] transfers started ahead of use, [3] bytes moved from host
 * memory to the device, [4] bytes of pinned host memory held, [5] bytes of the device slots. */
int pahq_prefetch_heads(pahq_model*, int32_t layer, uint64_t heads);
int pahq_get_transfer_stats(pahq_model*, int64_t out[6]);

/* Removed set, canonical edge order, one byte per edge (1 = removed, 0 = kept).  Any set is stored; which
 * sets an evaluation accepts is said at pahq_eval_edges. */
int pahq_set_removed(pahq_model*, const uint8_t* removed);
int pahq_get_removed(pahq_model*, uint8_t* removed);

/* ---- test hooks --------------------------------------------------------------- */
/* E4M3 codes ([K][N] in the master's row-major layout) and scale of one weight
 * slice: which = PAHQ_W_*; head is ignored for W_IN/W_GATE/W_OUT, layer and head for W_U. */
int pahq_get_weight_q(pahq_model*, int32_t which, int32_t layer, int32_t head, uint8_t* codes, float* scale);
/* The activation quantiser as a function: host x [rows][cols] -> codes, one scale per row.
 * cols <= 16384. */
int pahq_quantize_rows(pahq_model*, const float* x, int32_t rows, int32_t cols, uint8_t* codes, float* scales);
/* Test hooks of the bfloat16 mode (nonattn_bf16 = 1; PAHQ_ESTATE otherwise for the first).
 * pahq_get_weight_bf16: the bfloat16 patterns of W_in / W_gate / W_out (which = PAHQ_W_*, layer; head ignored) or of
 * W_U, and with low_bits = 16 also of a head's W_Q / W_K / W_V / W_O (layer, head), as the model holds them, in the
 * master's layout [K][N]; out: host.  pahq_get_weight_q refuses whatever is held as patterns.
 * pahq_round_rows_bf16: host rows through the row kernel of site PAHQ_QSITE_HIDDEN, PAHQ_QSITE_NORM or
 * PAHQ_QSITE_ATTN (their column constraints as in pahq_quantize_rows_site) in its bfloat16 form; out: host
 * [rows][cols] patterns. */
int pahq_get_weight_bf16(pahq_model*, int32_t which, int32_t layer, int32_t head, uint16_t* out);
int pahq_round_rows_bf16(pahq_model*, int32_t site, const float* x, int32_t rows, int32_t cols, uint16_t* out);

/* The same function as the path's three quantisers implement it, each through the code of its own kernel:
 *   PAHQ_QSITE_HIDDEN  rows of hidden activations (what pahq_quantize_rows runs; cols <= 16384)
 *   PAHQ_QSITE_NORM    the quantiser at the end of the gather / patch / norm kernels (cols a multiple of 64, <= 4096)
 *   PAHQ_QSITE_ATTN    the per-head quantiser at the end of the attention kernel (cols = d_head: 16, 32, 64 or 128);
 *                      the rows are run through the kernel as the values of one-position sequences, whose
 *                      attention output is the value row itself
 * All three must give the codes and scales of the definition bit for bit. */
enum { PAHQ_QSITE_HIDDEN = 0, PAHQ_QSITE_NORM = 1, PAHQ_QSITE_ATTN = 2 };
int pahq_quantize_rows_site(pahq_model*, int32_t site, const float* x, int32_t rows, int32_t cols, uint8_t* codes,
                            float* scales);
/* The E4M3 x E4M3 matrix product of the path as a function (Eq. for A_{comp,8}: low-precision projection, sums in
 * fp32): out[i][j] = sum_k dec(a[i][k]) * dec(w[j][k]) with unit scales, through the GEMM kernels the model's `mma`
 * setting selects and the tile shapes its launcher picks for (m, n).  a: host codes [m][k], w: host codes [n][k]
 * (k contiguous, a multiple of 128), out: host [m][n].  PAHQ_ENOMEM when the model's batch buffers cannot stage
 * the problem, PAHQ_ESTATE in the all-fp32 mode. */
int pahq_gemm_codes(pahq_model*, const uint8_t* a, const uint8_t* w, int32_t m, int32_t n, int32_t k, float* out);
/* Attention has two kernels: one wavefront per sequence and head with the whole sequence in registers (S <= 64, S <= 32
 * for d_head = 128), and one wavefront per tile of 16 queries for longer sequences (S <= 128).  form = 1 takes the
 * second at every length (0, the default: only where the first does not apply).  Both add the same products in the
 * same order, so results do not depend on it (a test hook). */
int pahq_set_attention_form(pahq_model*, int32_t form);
/* The kernels take a value's E4M3 code from the hardware conversion; the code is defined by the round-to-nearest-even
 * encoder on the bit pattern (Appendix "Quantization", Eq. RTN-Q on the E4M3 grid), which the weights use.  Compares
 * the two on every finite binary32 pattern on the device: *mismatches must come back 0 (*example: one differing
 * pattern, may be NULL).  scratch: 16 bytes of device memory, 16-byte aligned.  Needs no model. */
int pahq_compare_encoders(void* hip_stream, void* scratch, uint64_t* mismatches, uint32_t* example);
/* Last-position logits [B][vocab]: PAHQ_LOGITS_CLEAN / PAHQ_LOGITS_CORRUPT of the cached runs;
 * PAHQ_LOGITS_REF of the clean run under the precision set of the head investigated last (the reference
 * distribution its candidates were scored against; PAHQ_ESTATE when no head's state is current). */
int pahq_get_logits(pahq_model*, int32_t which, float* out);
/* Cached output [B*S][d_model] of one sender in the clean (which=0) or corrupted (1) run. */
int pahq_get_sender_output(pahq_model*, int32_t which, int32_t sender, float* out);
/* Counters since init: [0] candidate evaluations, [1] device batches, [2] forward passes of any kind. */
int pahq_get_counters(pahq_model*, int64_t out[3]);

/* ---- measurement hooks --------------------------------------------------------
 * With profiling on, every kernel launch of the passes is bracketed by a pair of
 * HIP events on the model's stream; pahq_get_profile synchronises and returns,
 * per kernel class, the number of launches, the summed event time and the
 * algorithmic work (floating-point operations of the contraction for the
 * matrix-core kernels; bytes that must be read and written for the streaming
 * kernels).  Classes: 0 gather+norm+quantise, 1 edge patch, 2 fp8 GEMM (with
 * exact sums the unembedding's log-softmax / KL epilogue is part of it),
 * 3 fp32 GEMM, 4 attention, 5 stream update, 6 hidden quantise, 7 log-sum-exp
 * and reference probabilities, 8 KL (the reduction of the epilogue's parts, or
 * the whole log-softmax + KL over stored logits in the FP8 matrix-core mode),
 * 9 fused output projection + stream update (fp8 matrix cores).  Turning
 * profiling on resets the counters. */
typedef struct {
  int64_t launches;
  double ms;        /* sum of event-to-event times                                   */
  double flops;     /* algorithmic flops (classes 2, 3, 9), else 0                      */
  double bytes;     /* algorithmic bytes read + written (all classes but 4 and 9)     */
} pahq_kernel_stat;
enum { PAHQ_N_KERNEL_CLASSES = 10 };
int pahq_set_profiling(pahq_model*, int32_t on);
/* Restricts what pahq_set_profiling(model, 1) records: only kernel classes whose bit is set in
 * class_mask, and only in every every_nth_pass-th pass of the executor (1 = every pass).  Two event
 * records per launch cost a few microseconds each; a benchmark that wants its throughput
 * undisturbed samples the dominant class only.  Defaults: all classes, every pass.
 * PAHQ_EINVAL for a null model, an empty mask or every_nth_pass < 1. */
int pahq_set_profiling_sample(pahq_model*, uint32_t class_mask, int32_t every_nth_pass);
int pahq_get_profile(pahq_model*, pahq_kernel_stat out[PAHQ_N_KERNEL_CLASSES]);

/* Measured ceilings of the device, for reading the roofline fractions next to the published peaks (no model
 * needed): the rate of a pure issue loop of the fp16 matrix-core instruction the exact GEMM multiplies with, all
 * compute units busy for a few tens of milliseconds, and the rate (bytes read + written) of a streaming copy of
 * half of `scratch` to its other half.  hip_stream: a hipStream_t or NULL; scratch: device memory, 256-byte
 * aligned, at least 64 MiB (the caller's; its contents are overwritten).  Synchronises the stream. */
int pahq_measure_ceilings(void* hip_stream, void* scratch, size_t scratch_bytes, double* mfma_f16_tflops,
                          double* copy_gbs);

/* ---- for callers that cannot allocate -----------------------------------------
 * pahq_quantize_rows for code that may not allocate device or pinned memory and has no model
 * or workspace at hand: kernels recorded into a HIP graph, serving loops, harnesses that forbid
 * hipMalloc.  Same arithmetic, bit for bit (scale = amax / 448, 1 if amax = 0; inv = 1 / scale;
 * code = rne_e4m3(x * inv)), for rows of ANY length: a row is split over workgroups, and the per-row
 * maxima they combine live in a static device array of PAHQ_NOALLOC_MAX_ROWS words (128 KiB) that
 * every GPU the library runs on holds until the process ends.
 *   hip_stream  hipStream_t (NULL = default stream); the work is enqueued there, nothing is waited for
 *   x           DEVICE, rows x cols floats, row-major          (caller-owned, read)
 *   codes       DEVICE, rows x cols bytes                      (caller-owned, written)
 *   scales      DEVICE, rows floats                            (caller-owned, written)
 * The device that owns the pointers and the stream must be the current one.  rows = 0 does nothing;
 * rows > PAHQ_NOALLOC_MAX_ROWS gives PAHQ_ETOOBIG (split the call), rows < 0, cols < 1 or a null
 * pointer PAHQ_EINVAL.  No allocation, no memset node, no synchronisation.  All calls on one GPU
 * share that GPU's array: calls that overlap there (different streams or host threads) race. */
enum { PAHQ_NOALLOC_MAX_ROWS = 32768 };
int pahq_quantize_rows_noalloc(void* hip_stream, const float* x, int32_t rows, int32_t cols, uint8_t* codes,
                               float* scales);

const char* pahq_strerror(int code);
void pahq_free(pahq_model*);            /* frees host state only; the workspace stays the caller's */

#ifdef __cplusplus
}
#endif
#endif /* PAHQ_H */
