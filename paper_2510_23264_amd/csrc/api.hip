// C ABI of libpahq: model set-up, cache pass, edge evaluation, ACDC sweep.
#include "engine.h"
#include <algorithm>
#include <math.h>
#include <new>
#include <string.h>

using namespace pahq;

#define HIPCHK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) return PAHQ_EHIP; } while (0)
#define PCHK(x) do { int r_ = (x); if (r_ != PAHQ_OK) return r_; } while (0)

namespace {

int check_config(const pahq_config* c) {
  if (!c) return PAHQ_EINVAL;
  if (c->n_layers < 1 || c->n_heads < 1 || c->d_head < 1 || c->d_model < 1 || c->vocab < 2) return PAHQ_EINVAL;
  if (c->d_mlp < 0 || c->max_batch_edges < 1 || c->max_batch_edges > 4096) return PAHQ_EINVAL;
  if (c->norm != PAHQ_NORM_LAYER && c->norm != PAHQ_NORM_RMS) return PAHQ_EINVAL;
  if (c->pos != PAHQ_POS_LEARNED && c->pos != PAHQ_POS_ROPE) return PAHQ_EINVAL;
  if (c->act < PAHQ_ACT_NONE || c->act > PAHQ_ACT_SWIGLU) return PAHQ_EINVAL;
  if (c->precision < PAHQ_ALL_FP32 || c->precision > PAHQ_PAHQ) return PAHQ_EINVAL;
  if (!(c->norm_eps >= 0.f)) return PAHQ_EINVAL;
  if (c->mma != PAHQ_MMA_FP8 && c->mma != PAHQ_MMA_F16_EXACT) return PAHQ_EINVAL;
  if (c->split_qkv != 0 && c->split_qkv != 1) return PAHQ_EINVAL;
  if (c->low_bits != 0 && c->low_bits != 4 && c->low_bits != 8 && c->low_bits != 16) return PAHQ_EINVAL;
  if (c->nonattn_bf16 != 0 && c->nonattn_bf16 != 1) return PAHQ_EINVAL;
  if (c->fp32_residency != PAHQ_FP32_IN_HBM && c->fp32_residency != PAHQ_FP32_ON_HOST) return PAHQ_EINVAL;
  return PAHQ_OK;
}
// what this build of the kernels supports
int check_supported(const pahq_config* c, int B, int S) {
  if (c->n_heads > 64) return PAHQ_EUNSUPPORTED;                      // sets of heads are 64-bit masks
  if (c->fp32_residency == PAHQ_FP32_ON_HOST && c->precision == PAHQ_ALL_FP32) return PAHQ_EUNSUPPORTED;   // that mode multiplies the masters
  if ((c->nonattn_bf16 || c->low_bits == 16) && c->mma != PAHQ_MMA_F16_EXACT && c->precision != PAHQ_ALL_FP32) return PAHQ_EUNSUPPORTED;   // bfloat16 products have no FP8-instruction form
  if (c->low_bits == 16 && c->precision != PAHQ_ALL_FP32 && ((c->d_head != 32 && c->d_head != 64) || c->n_heads % (64 / c->d_head) != 0))
    return PAHQ_EUNSUPPORTED;                                         // the bfloat16 form of the fused output projection
  if (c->d_model % 64 != 0 || c->d_model > 4096) return PAHQ_EUNSUPPORTED;
  if (c->d_mlp % 4 != 0) return PAHQ_EUNSUPPORTED;                    // 16-byte rows of the hidden activations
  if (c->d_head != 16 && c->d_head != 32 && c->d_head != 64 && c->d_head != 128) return PAHQ_EUNSUPPORTED;
  if (c->pos == PAHQ_POS_ROPE && (c->d_head & 1)) return PAHQ_EUNSUPPORTED;
  if (c->d_mlp > 0 && c->act == PAHQ_ACT_NONE) return PAHQ_EUNSUPPORTED;
  if (B < 1 || S < 1 || S > 128) return PAHQ_EUNSUPPORTED;            // the attention kernels' tiles of positions
  if (c->pos == PAHQ_POS_LEARNED && S > c->n_ctx) return PAHQ_EINVAL;
  return PAHQ_OK;
}

inline int pad128(int x) { return (x + 127) / 128 * 128; }

struct Bump {
  char* base; size_t off;
  template <class Tp> Tp* take(size_t n) {
    off = (off + 255) / 256 * 256;
    Tp* p = base ? (Tp*)(base + off) : nullptr;
    off += n * sizeof(Tp);
    return p;
  }
};

void set_dims(pahq_model* M, const pahq_config* c, int B, int S) {
  M->cfg = *c;
  M->g = GraphDims(c->n_layers, c->n_heads, c->d_mlp > 0, c->split_qkv != 0);
  M->B = B; M->S = S; M->T = B * S; M->L = c->n_layers; M->H = c->n_heads; M->dh = c->d_head;
  M->d = c->d_model; M->m = c->d_mlp; M->V = c->vocab;
  M->Kd = pad128(M->d); M->Kh = pad128(M->dh); M->Km = pad128(M->m > 0 ? M->m : 1);
  M->Vp = (M->V + 31) / 32 * 32;      // logits rows start on 128-byte boundaries
  M->nmax = c->max_batch_edges; M->G = 3 * M->H + 1;
  M->all_f32 = c->precision == PAHQ_ALL_FP32;
  M->skip_dead = true;
  M->qbits = c->low_bits == 4 ? 4 : (c->low_bits == 16 ? 16 : 8);
  M->nb16 = (c->nonattn_bf16 != 0 || M->qbits == 16) && !M->all_f32;
  if (M->qbits == 16) {        // bfloat16 operands for the heads too: their rows take two bytes per element
    M->Kd = pad128(2 * M->d); M->Kh = pad128(2 * M->dh);
  }
  M->Kd_o = M->nb16 ? pad128(2 * M->d) : M->Kd;
  M->Km_o = M->nb16 ? pad128(2 * (M->m > 0 ? M->m : 1)) : M->Km;
  M->deadsum_tag.assign(M->L, -1);
  M->f32_groups = M->all_f32 ? 3 * M->H : 3;
  M->f32_heads_max = M->all_f32 ? M->H : 1;
  M->ncap = std::max(M->nmax, 1024);
  M->tile = (long long)M->T * M->d;
  M->w32.on = c->fp32_residency == PAHQ_FP32_ON_HOST;
  if (M->w32.on) {
    // one block per head: W_Q | W_K | W_V | W_O | b_Q | b_K | b_V, every part on a 256-byte boundary
    const size_t mat = (size_t)M->d * M->dh, vec = ((size_t)M->dh + 63) / 64 * 64;
    size_t o = 0;
    for (int i = 0; i < 7; i++) { M->w32.off[i] = o; o += i < 4 ? mat : vec; }
    M->w32.head_floats = o;
  }
}

size_t arena_slot_bytes(const pahq_model* M) {
  size_t Nr = M->g.Nr, Ns = M->g.Ns, L = M->L, H = M->H;
  size_t b = Nr * sizeof(GroupDesc) + Nr * (Ns / 2 + 2) * sizeof(Term) + L * (5 * H + 8) * sizeof(GemmProb) +
             4 * L * sizeof(CombineDesc) + L * (H + 3) * sizeof(CombineSrc) + (L + H) * sizeof(OprojDesc) +
             L * H * sizeof(HeadAux) + 65536;
  return (b + 4095) / 4096 * 4096;
}

// Carves the workspace; with base == nullptr only the total is computed.
size_t layout(pahq_model* M, char* base) {
  Bump b{base, 0};
  const size_t L = M->L, H = M->H, dh = M->dh, d = M->d, m = M->m, V = M->V, T = M->T, B = M->B;
  const size_t Kdo = M->Kd_o, Kmo = M->Km_o;
  const size_t Kd = M->Kd, Kh = M->Kh, Km = M->Km, n = M->nmax, G = M->G, Ns = M->g.Ns, tile = M->tile, Vp = M->Vp;
  const bool mlp = m > 0, swi = M->cfg.act == PAHQ_ACT_SWIGLU, learned = M->cfg.pos == PAHQ_POS_LEARNED;
  M->W_E = b.take<float>(V * d);
  M->W_pos = learned ? b.take<float>((size_t)M->cfg.n_ctx * d) : nullptr;
  const bool on_host = M->w32.on;          // then no fp32 matrix but the embeddings stays on the device
  M->W_Q = on_host ? nullptr : b.take<float>(L * H * d * dh); M->W_K = on_host ? nullptr : b.take<float>(L * H * d * dh);
  M->W_V = on_host ? nullptr : b.take<float>(L * H * d * dh);
  M->W_O = on_host ? nullptr : b.take<float>(L * H * dh * d);
  M->w32.dev = on_host ? b.take<float>(2 * H * M->w32.head_floats) : nullptr;
  M->stage = on_host ? b.take<float>(std::max(std::max(H * d * dh, d * m), d * V)) : nullptr;
  M->b_Q = b.take<float>(L * H * dh); M->b_K = b.take<float>(L * H * dh); M->b_V = b.take<float>(L * H * dh);
  M->b_O = b.take<float>(L * d);
  M->ln1_g = b.take<float>(L * d); M->ln1_b = b.take<float>(L * d);
  M->ln2_g = mlp ? b.take<float>(L * d) : nullptr; M->ln2_b = mlp ? b.take<float>(L * d) : nullptr;
  M->W_in = (mlp && !on_host) ? b.take<float>(L * d * m) : nullptr; M->b_in = mlp ? b.take<float>(L * m) : nullptr;
  M->W_gate = (mlp && swi && !on_host) ? b.take<float>(L * d * m) : nullptr;
  M->W_out = (mlp && !on_host) ? b.take<float>(L * m * d) : nullptr; M->b_out = mlp ? b.take<float>(L * d) : nullptr;
  M->lnf_g = b.take<float>(d); M->lnf_b = b.take<float>(d);
  M->W_U = on_host ? nullptr : b.take<float>(d * V); M->b_U = b.take<float>(V + 4);     // the GEMM epilogue reads bias in groups of four
  M->zeros_d = b.take<float>(d);
  M->rope_tab = M->cfg.pos == PAHQ_POS_ROPE ? b.take<float>((size_t)128 * dh) : nullptr;   // the attention kernels' (up to eight) 16-position tiles
  M->bqkv = b.take<float>(L * 3 * H * dh);
  M->qkv_codes = b.take<uint8_t>(L * 3 * H * dh * Kd); M->qkv_scale = b.take<float>(L * 3 * H);
  M->o_codes = b.take<uint8_t>(L * H * d * Kh); M->o_scale = b.take<float>(L * H);
  M->in_codes = mlp ? b.take<uint8_t>(L * m * Kdo) : nullptr; M->in_scale = mlp ? b.take<float>(L) : nullptr;
  M->gate_codes = (mlp && swi) ? b.take<uint8_t>(L * m * Kdo) : nullptr;
  M->gate_scale = (mlp && swi) ? b.take<float>(L) : nullptr;
  M->out_codes = mlp ? b.take<uint8_t>(L * d * Kmo) : nullptr; M->out_scale = mlp ? b.take<float>(L) : nullptr;
  M->u_codes = b.take<uint8_t>(V * Kdo); M->u_scale = b.take<float>(1);
  M->amax_tmp = b.take<unsigned>((L * H + 4 + 3) / 4 * 4); M->flag_tmp = b.take<int>(4);
  M->tok_clean = b.take<int>(T); M->tok_corrupt = b.take<int>(T); M->send_dev = b.take<int>(M->ncap);
  M->clean = b.take<float>(Ns * tile); M->corrupt = b.take<float>(Ns * tile); M->delta = b.take<float>((Ns + 1) * tile);   // tile Ns stays zero
  M->rc = b.take<float>((2 * L + 1) * tile); M->rx = b.take<float>((2 * L + 1) * tile);
  M->logits_clean = b.take<float>(B * Vp); M->logits_corrupt = b.take<float>(B * Vp); M->logz_clean = b.take<double>(B);
  M->cpi = b.take<float>(Ns * tile); M->rxpi = b.take<float>((2 * L + 1) * tile);
  M->ref_logits_all = b.take<float>(H * B * Vp); M->ref_logz_all = b.take<double>(H * B);
  M->ref_logits = M->ref_logits_all; M->ref_logz = M->ref_logz_all;
  M->xv = b.take<float>(tile);
  M->qkv_sh = b.take<float>(T * 3 * H * dh); M->oth = b.take<float>(tile); M->xvc = b.take<float>(3 * tile); M->deadsum = b.take<float>(L * tile); M->sh_slots = b.take<float>(H * tile);
  M->qv = b.take<float>(3 * n * T * dh);
  M->run_a = b.take<float>(n * tile); M->run_b = b.take<float>(n * tile);
  M->xcodes = b.take<uint8_t>(n * G * T * Kd); M->xscale = b.take<float>(n * G * T); M->xf32 = b.take<float>(std::max<size_t>(n * (size_t)M->f32_groups, 3 * H) * tile);
  M->qkv = b.take<float>(n * T * 3 * H * dh);
  M->zcodes = b.take<uint8_t>(n * T * H * Kh); M->zscale = b.take<float>(n * T * H); M->zf32 = b.take<float>(std::max<size_t>(n * (size_t)M->f32_heads_max, H) * T * dh);
  M->headout = b.take<float>(n * H * tile);
  M->mlpout = mlp ? b.take<float>(n * tile) : nullptr;
  M->hid = mlp ? b.take<float>(n * T * m) : nullptr; M->hid2 = (mlp && swi) ? b.take<float>(n * T * m) : nullptr;
  M->hcodes = mlp ? b.take<uint8_t>(n * T * Kmo) : nullptr; M->hscale = mlp ? b.take<float>(n * T) : nullptr;
  M->lastcodes = b.take<uint8_t>(n * B * Kdo); M->lastscale = b.take<float>(n * B); M->logits = b.take<float>(n * B * Vp);
  // Per-instance copies of recomputed sender outputs that some receiver reads individually: in the
  // worst case (most edges removed) every sender but the embedding needs one per candidate.  Room
  // for a full batch of those, capped at 64 GiB; a smaller pool only shrinks the batches.
  {
    const size_t want = n * (Ns - 1), cap = ((size_t)64 << 30) / (tile * sizeof(float));
    M->pool_tiles = (long long)std::max<size_t>(std::max<size_t>(2 * Ns, 4 * n), std::min(want, cap));
  }
  M->slots = b.take<float>((size_t)M->pool_tiles * tile);
  M->row_kl = b.take<double>(n * B); M->kl_dev = b.take<double>(M->ncap);
  M->psum_clean = b.take<double>(B); M->psum_ref_all = b.take<double>(H * B); M->psum_ref = M->psum_ref_all;
  M->ans_dev = b.take<int>(B); M->dis_dev = b.take<int>(B); M->ld_clean = b.take<double>(B); M->ld_ref_all = b.take<double>(H * B); M->ld_ref = M->ld_ref_all;
  M->kl_npart = kl_parts_per_row((int)V); M->kl_part = b.take<float>(n * B * (size_t)M->kl_npart * 4);
  M->arena.slot_bytes = arena_slot_bytes(M);
  for (int i = 0; i < Arena::SLOTS; i++) M->arena.dev[i] = b.take<char>(M->arena.slot_bytes);
  return (b.off + 255) / 256 * 256;
}

int copy_in(pahq_model* M, float* dst, const float* src, size_t n, int on_device) {
  if (!dst) return PAHQ_OK;
  if (!src) return PAHQ_EINVAL;
  HIPCHK(hipMemcpyAsync(dst, src, n * sizeof(float), on_device ? hipMemcpyDeviceToDevice : hipMemcpyHostToDevice, M->stream));
  return PAHQ_OK;
}

// quantise n_slices contiguous slices of shape [K][N]; slice i goes to codes0 + i*codes_stride, scale0 + i*scale_stride
int quantise_class(pahq_model* M, const float* w, int n_slices, int K, int N, uint8_t* codes0, long long codes_stride,
                   int ldq, float* scale0, int scale_stride, int qbits) {
  HIPCHK(launch_fill_zero(M->amax_tmp, ((size_t)n_slices * 4 + 15) / 16 * 16, M->stream));
  HIPCHK(launch_slice_absmax(w, (long long)K * N, n_slices, M->amax_tmp, M->flag_tmp, M->stream));
  for (int i = 0; i < n_slices; i++)
    HIPCHK(launch_quant_transpose(w + (long long)i * K * N, K, N, M->amax_tmp + i, scale0 + (long long)i * scale_stride,
                                  codes0 + i * codes_stride, ldq, qbits, M->stream));
  HIPCHK(hipStreamSynchronize(M->stream));       // amax_tmp is reused by the next class
  return PAHQ_OK;
}

inline int64_t edge_index(const pahq_model* M, int s, int r) { return M->edge_off[r] + s; }

bool node_is_live(const pahq_model* M, int v) { return node_is_live(M->g, M->removed.data(), M->edge_off.data(), v); }

// copies a small host table to the device through the descriptor ring
int upload_table(pahq_model* M, const void* src, size_t bytes, void** dev_out) {
  Arena& A = M->arena;
  if (bytes > A.slot_bytes) return PAHQ_ENOMEM;
  int slot = A.next;
  A.next = (A.next + 1) % Arena::SLOTS;
  HIPCHK(hipEventSynchronize(A.ev[slot]));
  memcpy(A.host[slot], src, bytes);
  HIPCHK(hipMemcpyAsync(A.dev[slot], A.host[slot], bytes, hipMemcpyHostToDevice, M->stream));
  HIPCHK(hipEventRecord(A.ev[slot], M->stream));
  *dev_out = A.dev[slot];
  return PAHQ_OK;
}

struct RecvCtx { int v, p0, pl, ph, n_eff; };

// dst = receiver w's input under the current removed set, from the cached streams and sender tiles (every sender
// upstream of w is cached); the plan must hold w's spec
int build_receiver_input(pahq_model* M, int w, int p0, float* dst) {
  const RecvSpec& sp = M->plan.spec[w];
  float* base = sp.form == 2 ? corrupt_prefix(M, p0) : clean_prefix(M, p0);
  std::vector<Term> terms;
  for (int s : sp.senders) {
    Term t; t.p = M->delta + (long long)s * M->tile; t.inst_stride = 0; t.sign = sp.form == 1 ? -1.f : 1.f; t.pad_ = 0;
    terms.push_back(t);
  }
  void* dterms = nullptr;
  if (!terms.empty()) PCHK(upload_table(M, terms.data(), terms.size() * sizeof(Term), &dterms));
  // the stream goes in after the removed senders' terms (form 1), a corrupted-run base before the kept ones
  // (form 2): the order in which the row kernels add the same sum when they build this input for the current state
  HIPCHK(launch_tile_lincomb(dst, base, (const Term*)dterms, (int)terms.size(), M->tile, sp.form == 1 ? 1 : 0, M->stream));
  return PAHQ_OK;
}

// Brings the model into the state needed to evaluate edges into receiver v:
// the state of v's fp32 head (corrupted run + reference distribution under that
// precision set), the receiver plan for the current removed set, and v's
// current input xv.
// What the caller will evaluate after v, for the prediction of the fp32 weights needed next (host residency): receiver
// ids in the order of their evaluation (repeats allowed); skip_dead: receivers whose node is dead are not evaluated.
struct Upcoming { const int32_t* ids; int64_t n; bool skip_dead; };

int setup_receiver(pahq_model* M, int v, RecvCtx& ctx, const Upcoming* up = nullptr) {
  const GraphDims& g = M->g;
  int kind, l, h, c;
  g.receiver_info(v, kind, l, h, c);
  ctx.v = v; ctx.p0 = g.pos_of_receiver(v);
  // Everything upstream of v comes from the caches, which hold the runs with no edge removed: the removed set may
  // only touch receivers at or after v's position (every state of the sweep is of this kind).
  for (int w = 0; w < g.Nr; w++) {
    if (g.pos_of_receiver(w) >= ctx.p0) continue;
    const uint8_t* row = M->removed.data() + M->edge_off[w];
    for (int s = 0, n_up = g.n_upstream(w); s < n_up; s++) if (row[s]) return PAHQ_ESTATE;
  }
  ctx.pl = ctx.ph = -1;
  if (M->cfg.precision == PAHQ_PAHQ && kind == 0) { ctx.pl = l; ctx.ph = h; }
  const bool layerwise = M->H > 1 && M->H <= M->nmax && M->cfg.mma == PAHQ_MMA_F16_EXACT;
  make_plan(M, ctx.p0, v, M->plan);
  if (ctx.pl >= 0) {
    PassArgs a; a.n = 1; a.p0 = ctx.p0; a.pl = ctx.pl; a.ph = ctx.ph; a.v = -1; a.patch_mode = 0;
    if (M->pi_l != ctx.pl || M->pi_h != ctx.ph) {
      M->pi_l = M->pi_h = -2; M->pi_corrupt = false;
      // The reference distribution under this head's precision set.  The reference runs of all H heads of a layer go
      // as one pass of H instances where the model has room for them (they differ only in which head of that layer is
      // in fp32); the state of head h is then copy h of the arrays that pass fills.
      const int copy = layerwise ? ctx.ph : 0;
      M->ref_logits = M->ref_logits_all + (long long)copy * M->B * M->Vp;
      M->ref_logz = M->ref_logz_all + (long long)copy * M->B;
      M->psum_ref = M->psum_ref_all + (long long)copy * M->B;
      M->ld_ref = M->ld_ref_all + (long long)copy * M->B;
      if (!layerwise) { M->ref_layer = -1; a.kind = PI_REF; PCHK(run_pass(M, a, nullptr)); }
      else if (M->ref_layer != ctx.pl) {
        M->ref_layer = -1;
        PassArgs r = a; r.kind = PI_REF_LAYER; r.n = M->H; r.ph = -1;
        PCHK(run_pass(M, r, nullptr));
        M->ref_layer = ctx.pl;
      }
      M->pi_l = ctx.pl; M->pi_h = ctx.ph;
    }
    // The corrupted run under the same precision set is read only where the plan has a receiver in kept form
    // downstream, a recomputed sender whose difference to it some receiver needs, or a dead node standing in with
    // it: not at all while nothing downstream is removed (every receiver then reads the running stream alone).
    bool need = M->plan.n_slots + M->plan.n_shared + M->plan.n_dead > 0;
    for (int w = 0; w < g.Nr && !need; w++) need = g.pos_of_receiver(w) > ctx.p0 && M->plan.spec[w].form == 2;
    if (need && !M->pi_corrupt) {
      a.kind = PI_CORRUPT; PCHK(run_pass(M, a, nullptr));
      M->pi_corrupt = true;
    }
  }
  ctx.n_eff = M->nmax;
  if (M->plan.n_slots > 0) ctx.n_eff = (int)std::min<long long>(M->nmax, M->pool_tiles / M->plan.n_slots);
  if (ctx.n_eff < 1) return PAHQ_ENOMEM;
  PCHK(build_receiver_input(M, v, ctx.p0, M->xv));
  if (M->plan.split_first) {
    // everything in v's layer that does not depend on the candidate: the other heads, and the
    // investigated head's two unpatched inputs
    PassArgs a; a.kind = PREFIX; a.p0 = ctx.p0; a.n = 1; a.pl = ctx.pl; a.ph = ctx.ph; a.v = v; a.patch_mode = 0;
    PCHK(run_pass(M, a, &M->plan));
  }
  if (M->w32.on && M->cfg.precision == PAHQ_PAHQ) {
    // Prefetch(t): the fp32 weights needed after this receiver's move while its candidates are evaluated -- those of
    // the next head the caller's list names (a whole layer where its heads' reference runs will be made together),
    // or, without a list, of the head that follows in the sweep's order
    int nl = -1;
    unsigned long long nm = 0;
    if (up) {
      const unsigned long long all = M->H >= 64 ? ~0ull : ((1ull << M->H) - 1ull);
      for (int64_t q = 0, lim = std::min<int64_t>(up->n, 1 << 16); q < lim; q++) {
        int k2, l2, h2, c2;
        g.receiver_info(up->ids[q], k2, l2, h2, c2);
        if (k2 != 0 || (l2 == ctx.pl && h2 == ctx.ph)) continue;
        if (up->skip_dead && !node_is_live(M, up->ids[q])) continue;
        nl = l2;
        nm = (layerwise && l2 != ctx.pl && M->ref_layer != l2) ? all : (1ull << h2);
        break;
      }
    } else if (ctx.pl >= 0) nl = next_heads_in_sweep_order(M->H, ctx.pl, ctx.ph, nm);
    PCHK(w32_prefetch(M, nl, nm));
  }
  return PAHQ_OK;
}

// evaluates one device batch of candidates (senders already in send_host[0..n)); results in kl_host[0..n)
int eval_batch(pahq_model* M, const RecvCtx& ctx, int n, int patch_mode) {
  HIPCHK(hipMemcpyAsync(M->send_dev, M->send_host, (size_t)n * sizeof(int), hipMemcpyHostToDevice, M->stream));
  PassArgs a; a.kind = CAND; a.p0 = ctx.p0; a.n = n; a.pl = ctx.pl; a.ph = ctx.ph; a.v = ctx.v; a.patch_mode = patch_mode;
  PCHK(run_pass(M, a, &M->plan));
  HIPCHK(hipMemcpyAsync(M->kl_host, M->kl_dev, (size_t)n * sizeof(double), hipMemcpyDeviceToHost, M->stream));
  HIPCHK(hipStreamSynchronize(M->stream));
  M->counters[0] += n; M->counters[1] += 1;
  return PAHQ_OK;
}

int eval_state(pahq_model* M, const RecvCtx& ctx, double* kl) {
  PassArgs a; a.kind = STATE; a.p0 = ctx.p0; a.n = 1; a.pl = ctx.pl; a.ph = ctx.ph; a.v = -1; a.patch_mode = 0;
  PCHK(run_pass(M, a, &M->plan));
  HIPCHK(hipMemcpyAsync(M->kl_host, M->kl_dev, sizeof(double), hipMemcpyDeviceToHost, M->stream));
  HIPCHK(hipStreamSynchronize(M->stream));
  *kl = M->kl_host[0];
  return PAHQ_OK;
}

}  // namespace

extern "C" {

int pahq_n_senders(const pahq_config* c, int32_t* out) {
  if (check_config(c) || !out) return PAHQ_EINVAL;
  *out = GraphDims(c->n_layers, c->n_heads, c->d_mlp > 0, c->split_qkv != 0).Ns; return PAHQ_OK;
}
int pahq_n_receivers(const pahq_config* c, int32_t* out) {
  if (check_config(c) || !out) return PAHQ_EINVAL;
  *out = GraphDims(c->n_layers, c->n_heads, c->d_mlp > 0, c->split_qkv != 0).Nr; return PAHQ_OK;
}
int pahq_n_upstream(const pahq_config* c, int32_t r, int32_t* out) {
  if (check_config(c) || !out) return PAHQ_EINVAL;
  GraphDims g(c->n_layers, c->n_heads, c->d_mlp > 0, c->split_qkv != 0);
  if (r < 0 || r >= g.Nr) return PAHQ_EINVAL;
  *out = g.n_upstream(r); return PAHQ_OK;
}
int pahq_edge_count(const pahq_config* c, int64_t* out) {
  if (check_config(c) || !out) return PAHQ_EINVAL;
  GraphDims g(c->n_layers, c->n_heads, c->d_mlp > 0, c->split_qkv != 0);
  int64_t n = 0;
  for (int r = 0; r < g.Nr; r++) n += g.n_upstream(r);
  *out = n; return PAHQ_OK;
}
int pahq_edge_id(const pahq_config* c, int32_t s, int32_t r, int64_t* out) {
  if (check_config(c) || !out) return PAHQ_EINVAL;
  GraphDims g(c->n_layers, c->n_heads, c->d_mlp > 0, c->split_qkv != 0);
  if (r < 0 || r >= g.Nr || s < 0 || s >= g.n_upstream(r)) return PAHQ_EINVAL;
  int64_t n = 0;
  for (int q = 0; q < r; q++) n += g.n_upstream(q);
  *out = n + s; return PAHQ_OK;
}
int pahq_node_of_receiver(const pahq_config* c, int32_t r, int32_t* out) {
  if (check_config(c) || !out) return PAHQ_EINVAL;
  GraphDims g(c->n_layers, c->n_heads, c->d_mlp > 0, c->split_qkv != 0);
  if (r < 0 || r >= g.Nr) return PAHQ_EINVAL;
  *out = g.node_of_receiver(r); return PAHQ_OK;
}

int pahq_workspace_bytes(const pahq_config* c, int32_t B, int32_t S, size_t* out) {
  PCHK(check_config(c));
  if (!out) return PAHQ_EINVAL;
  PCHK(check_supported(c, B, S));
  pahq_model* M = new (std::nothrow) pahq_model();
  if (!M) return PAHQ_ENOMEM;
  set_dims(M, c, B, S);
  *out = layout(M, nullptr);
  delete M;
  return PAHQ_OK;
}

int pahq_init_model(const pahq_config* c, const pahq_weights* w, int32_t B, int32_t S, void* workspace,
                    size_t workspace_bytes, void* hip_stream, pahq_model** out) {
  PCHK(check_config(c));
  if (!w || !workspace || !out) return PAHQ_EINVAL;
  PCHK(check_supported(c, B, S));
  if (((uintptr_t)workspace & 255) != 0) return PAHQ_EINVAL;
  const bool mlp = c->d_mlp > 0, swi = c->act == PAHQ_ACT_SWIGLU, learned = c->pos == PAHQ_POS_LEARNED;
  const float* req[] = {w->W_E, w->W_Q, w->W_K, w->W_V, w->W_O, w->b_Q, w->b_K, w->b_V, w->b_O, w->ln1_g, w->lnf_g, w->W_U, w->b_U};
  for (const float* p : req) if (!p) return PAHQ_EINVAL;
  if (learned && !w->W_pos) return PAHQ_EINVAL;
  if (mlp && (!w->ln2_g || !w->W_in || !w->b_in || !w->W_out || !w->b_out)) return PAHQ_EINVAL;
  if (mlp && swi && !w->W_gate) return PAHQ_EINVAL;
  if (c->norm == PAHQ_NORM_LAYER && (!w->ln1_b || !w->lnf_b || (mlp && !w->ln2_b))) return PAHQ_EINVAL;
  int ndev = 0;
  if (hipGetDeviceCount(&ndev) != hipSuccess || ndev < 1) return PAHQ_EHIP;

  pahq_model* M = new (std::nothrow) pahq_model();
  if (!M) return PAHQ_ENOMEM;
  set_dims(M, c, B, S);
  M->stream = (hipStream_t)hip_stream;
  size_t need = layout(M, (char*)workspace);
  if (need > workspace_bytes) { delete M; return PAHQ_ENOMEM; }
  M->ws = (char*)workspace; M->ws_bytes = workspace_bytes; M->ws_used = need;
  M->kl_host = nullptr; M->send_host = nullptr;
  for (int i = 0; i < Arena::SLOTS; i++) { M->arena.host[i] = nullptr; M->arena.ev[i] = nullptr; }
  M->arena.next = 0;
  int rc = PAHQ_OK;
  auto fail = [&](int code) { pahq_free(M); return code; };
  if (hipHostMalloc((void**)&M->kl_host, sizeof(double) * M->ncap, hipHostMallocDefault) != hipSuccess) return fail(PAHQ_EHIP);
  if (hipHostMalloc((void**)&M->send_host, sizeof(int) * M->ncap, hipHostMallocDefault) != hipSuccess) return fail(PAHQ_EHIP);
  for (int i = 0; i < Arena::SLOTS; i++) {
    if (hipHostMalloc((void**)&M->arena.host[i], M->arena.slot_bytes, hipHostMallocDefault) != hipSuccess) return fail(PAHQ_EHIP);
    if (hipEventCreateWithFlags(&M->arena.ev[i], hipEventDisableTiming) != hipSuccess) return fail(PAHQ_EHIP);
  }
  // zero everything (code buffers rely on zero padding), then bring the weights in
  if (launch_fill_zero(M->ws, need, M->stream) != hipSuccess) return fail(PAHQ_EHIP);
  const size_t L = M->L, H = M->H, dh = M->dh, d = M->d, m = M->m, V = M->V;
  const int od = w->on_device;
#define CP(dst, src, n) if ((rc = copy_in(M, dst, src, n, od)) != PAHQ_OK) return fail(rc)
  CP(M->W_E, w->W_E, V * d);
  if (learned) CP(M->W_pos, w->W_pos, (size_t)c->n_ctx * d);
  CP(M->W_Q, w->W_Q, L * H * d * dh); CP(M->W_K, w->W_K, L * H * d * dh); CP(M->W_V, w->W_V, L * H * d * dh);
  CP(M->W_O, w->W_O, L * H * dh * d);
  CP(M->b_Q, w->b_Q, L * H * dh); CP(M->b_K, w->b_K, L * H * dh); CP(M->b_V, w->b_V, L * H * dh); CP(M->b_O, w->b_O, L * d);
  CP(M->ln1_g, w->ln1_g, L * d);
  if (c->norm == PAHQ_NORM_LAYER) { CP(M->ln1_b, w->ln1_b, L * d); CP(M->lnf_b, w->lnf_b, d); }
  CP(M->lnf_g, w->lnf_g, d);
  if (mlp) {
    CP(M->ln2_g, w->ln2_g, L * d);
    if (c->norm == PAHQ_NORM_LAYER) CP(M->ln2_b, w->ln2_b, L * d);
    CP(M->W_in, w->W_in, L * d * m); CP(M->b_in, w->b_in, L * m);
    if (swi) CP(M->W_gate, w->W_gate, L * d * m);
    CP(M->W_out, w->W_out, L * m * d); CP(M->b_out, w->b_out, L * d);
  }
  CP(M->W_U, w->W_U, d * V); CP(M->b_U, w->b_U, V);
#undef CP
  // fused projection bias [L][3][H][dh]
  const float* bsrc[3] = {M->b_Q, M->b_K, M->b_V};
  for (size_t l = 0; l < L; l++)
    for (int cc = 0; cc < 3; cc++)
      if (hipMemcpyAsync(M->bqkv + (l * 3 + cc) * H * dh, bsrc[cc] + l * H * dh, H * dh * sizeof(float),
                         hipMemcpyDeviceToDevice, M->stream) != hipSuccess) return fail(PAHQ_EHIP);
  if (M->rope_tab && launch_rope_table(M->rope_tab, 128, (int)dh, c->rope_theta, M->stream) != hipSuccess) return fail(PAHQ_EHIP);
  // e4m3 codes + scales of every weight slice.  With the masters in the workspace a class is quantised where it lies;
  // with host residency it passes through the staging buffer a layer at a time (quantise_class ends with a
  // synchronisation, so the buffer is free again when it returns).
  const float* wc[3] = {M->W_Q, M->W_K, M->W_V};
  const float* wsrc[3] = {w->W_Q, w->W_K, w->W_V};
  const int qo = M->nb16 ? 16 : M->qbits;      // the grid of the components that are not attention heads
  const bool on_host = M->w32.on;
  auto staged = [&](const float* resident, const float* src, size_t count) -> const float* {
    if (!on_host) return resident;
    if (rc == PAHQ_OK) rc = copy_in(M, M->stage, src, count, od);
    return M->stage;
  };
  for (size_t l = 0; l < L && rc == PAHQ_OK; l++) {
    for (int cc = 0; cc < 3 && rc == PAHQ_OK; cc++) {
      const float* src = staged(on_host ? nullptr : wc[cc] + l * H * d * dh, wsrc[cc] + l * H * d * dh, H * d * dh);
      if (rc == PAHQ_OK)
        rc = quantise_class(M, src, (int)H, (int)d, (int)dh,
                            M->qkv_codes + (l * 3 * H * dh + (size_t)cc * H * dh) * M->Kd, (long long)dh * M->Kd, M->Kd,
                            M->qkv_scale + l * 3 * H + (size_t)cc * H, 1, M->qbits);
    }
    if (rc == PAHQ_OK) {
      const float* src = staged(on_host ? nullptr : M->W_O + l * H * dh * d, w->W_O + l * H * dh * d, H * dh * d);
      if (rc == PAHQ_OK)
        rc = quantise_class(M, src, (int)H, (int)dh, (int)d, M->o_codes + l * H * d * M->Kh, (long long)d * M->Kh, M->Kh, M->o_scale + l * H, 1, M->qbits);
    }
    if (mlp && rc == PAHQ_OK) {
      const float* src = staged(on_host ? nullptr : M->W_in + l * d * m, w->W_in + l * d * m, d * m);
      if (rc == PAHQ_OK) rc = quantise_class(M, src, 1, (int)d, (int)m, M->in_codes + l * m * M->Kd_o, 0, M->Kd_o, M->in_scale + l, 1, qo);
    }
    if (mlp && swi && rc == PAHQ_OK) {
      const float* src = staged(on_host ? nullptr : M->W_gate + l * d * m, w->W_gate + l * d * m, d * m);
      if (rc == PAHQ_OK) rc = quantise_class(M, src, 1, (int)d, (int)m, M->gate_codes + l * m * M->Kd_o, 0, M->Kd_o, M->gate_scale + l, 1, qo);
    }
    if (mlp && rc == PAHQ_OK) {
      const float* src = staged(on_host ? nullptr : M->W_out + l * m * d, w->W_out + l * m * d, m * d);
      if (rc == PAHQ_OK) rc = quantise_class(M, src, 1, (int)m, (int)d, M->out_codes + l * d * M->Km_o, 0, M->Km_o, M->out_scale + l, 1, qo);
    }
  }
  if (rc == PAHQ_OK) {
    const float* src = staged(M->W_U, w->W_U, d * V);
    if (rc == PAHQ_OK) rc = quantise_class(M, src, 1, (int)d, (int)V, M->u_codes, 0, M->Kd_o, M->u_scale, 1, qo);
  }
  if (rc != PAHQ_OK) return fail(rc);
  if (on_host) {
    // the heads' fp32 blocks: pinned host memory, one block per head in the layout of a device slot
    W32Cache& c32 = M->w32;
    const size_t hf = c32.head_floats, mat = d * dh;
    if (hipHostMalloc((void**)&c32.host, L * H * hf * sizeof(float), hipHostMallocDefault) != hipSuccess) return fail(PAHQ_EHIP);
    memset(c32.host, 0, L * H * hf * sizeof(float));
    const float* part[7] = {w->W_Q, w->W_K, w->W_V, w->W_O, w->b_Q, w->b_K, w->b_V};
    for (size_t id = 0; id < L * H; id++)
      for (int i = 0; i < 7; i++) {
        const size_t count = i < 4 ? mat : dh;
        float* dst = c32.host + id * hf + c32.off[i];
        if (od) { if (hipMemcpy(dst, part[i] + id * count, count * sizeof(float), hipMemcpyDeviceToHost) != hipSuccess) return fail(PAHQ_EHIP); }
        else memcpy(dst, part[i] + id * count, count * sizeof(float));
      }
    if (hipStreamCreateWithFlags(&c32.copy_stream, hipStreamNonBlocking) != hipSuccess) { c32.copy_stream = nullptr; return fail(PAHQ_EHIP); }
    c32.slots.init((int)(2 * H));
    c32.ready.assign(2 * H, nullptr); c32.released.assign(2 * H, nullptr);
    for (size_t i = 0; i < 2 * H; i++) {
      if (hipEventCreateWithFlags(&c32.ready[i], hipEventDisableTiming) != hipSuccess) return fail(PAHQ_EHIP);
      if (hipEventCreateWithFlags(&c32.released[i], hipEventDisableTiming) != hipSuccess) return fail(PAHQ_EHIP);
      // recorded once so that the first wait on either finds a completed event
      if (hipEventRecord(c32.ready[i], M->stream) != hipSuccess || hipEventRecord(c32.released[i], M->stream) != hipSuccess) return fail(PAHQ_EHIP);
    }
  }
  // embeddings, biases and norm parameters are used unquantised: check them too
  {
    struct { const float* p; size_t n; } extra[] = {{M->W_E, V * d}, {M->W_pos, learned ? (size_t)c->n_ctx * d : 0},
      {M->bqkv, L * 3 * H * dh}, {M->b_O, L * d}, {M->ln1_g, L * d}, {M->ln1_b, L * d}, {M->ln2_g, mlp ? L * d : 0},
      {M->ln2_b, mlp ? L * d : 0}, {M->b_in, mlp ? L * m : 0}, {M->b_out, mlp ? L * d : 0}, {M->lnf_g, d}, {M->lnf_b, d}, {M->b_U, V}};
    for (auto& e : extra)
      if (e.p && e.n)
        if (launch_slice_absmax(e.p, (long long)e.n, 1, M->amax_tmp, M->flag_tmp, M->stream) != hipSuccess) return fail(PAHQ_EHIP);
  }
  int flag = 0;
  if (hipMemcpyAsync(&flag, M->flag_tmp, sizeof(int), hipMemcpyDeviceToHost, M->stream) != hipSuccess) return fail(PAHQ_EHIP);
  if (hipStreamSynchronize(M->stream) != hipSuccess) return fail(PAHQ_EHIP);
  if (flag) return fail(PAHQ_ENAN);

  M->edge_off.assign(M->g.Nr + 1, 0);
  for (int r = 0; r < M->g.Nr; r++) M->edge_off[r + 1] = M->edge_off[r] + M->g.n_upstream(r);
  M->removed.assign((size_t)M->edge_off[M->g.Nr], 0);
  M->has_cache = false; M->pi_l = M->pi_h = -2; M->pi_p0 = -1; M->ref_layer = -1;
  M->metric = PAHQ_METRIC_KL;
  M->counters[0] = M->counters[1] = M->counters[2] = 0;
  M->prof_on = false; M->prof_used = 0; memset(M->prof, 0, sizeof(M->prof));
  *out = M;
  return PAHQ_OK;
}

void pahq_free(pahq_model* M) {
  if (!M) return;
  if (M->w32.copy_stream) { (void)hipStreamSynchronize(M->w32.copy_stream); (void)hipStreamDestroy(M->w32.copy_stream); }
  for (hipEvent_t e : M->w32.ready) if (e) (void)hipEventDestroy(e);
  for (hipEvent_t e : M->w32.released) if (e) (void)hipEventDestroy(e);
  if (M->w32.host) (void)hipHostFree(M->w32.host);
  if (M->kl_host) (void)hipHostFree(M->kl_host);
  if (M->send_host) (void)hipHostFree(M->send_host);
  for (hipEvent_t e : M->prof_ev) (void)hipEventDestroy(e);
  for (int i = 0; i < Arena::SLOTS; i++) {
    if (M->arena.host[i]) (void)hipHostFree(M->arena.host[i]);
    if (M->arena.ev[i]) (void)hipEventDestroy(M->arena.ev[i]);
  }
  delete M;
}

int pahq_clean_cache(pahq_model* M, const int32_t* clean_tok, const int32_t* corrupt_tok) {
  if (!M || !clean_tok || !corrupt_tok) return PAHQ_EINVAL;
  for (int i = 0; i < M->T; i++)
    if (clean_tok[i] < 0 || clean_tok[i] >= M->V || corrupt_tok[i] < 0 || corrupt_tok[i] >= M->V) return PAHQ_EINVAL;
  HIPCHK(hipMemcpyAsync(M->tok_clean, clean_tok, M->T * sizeof(int), hipMemcpyHostToDevice, M->stream));
  HIPCHK(hipMemcpyAsync(M->tok_corrupt, corrupt_tok, M->T * sizeof(int), hipMemcpyHostToDevice, M->stream));
  HIPCHK(launch_embed(M->tok_clean, M->W_E, M->W_pos, M->clean, M->T, M->S, M->d, M->stream));
  HIPCHK(launch_embed(M->tok_corrupt, M->W_E, M->W_pos, M->corrupt, M->T, M->S, M->d, M->stream));
  PassArgs a; a.p0 = 0; a.n = 1; a.pl = a.ph = -1; a.v = -1; a.patch_mode = 0;
  a.kind = BASE_CLEAN; PCHK(run_pass(M, a, nullptr));
  a.kind = BASE_CORRUPT; PCHK(run_pass(M, a, nullptr));
  HIPCHK(launch_tile_sub(M->delta, M->clean, M->corrupt, (long long)M->g.Ns * M->tile, M->stream));
  HIPCHK(hipStreamSynchronize(M->stream));
  std::fill(M->removed.begin(), M->removed.end(), 0);
  M->has_cache = true; M->pi_l = M->pi_h = -2; M->ref_layer = -1;
  return PAHQ_OK;
}

int pahq_set_metric(pahq_model* M, int32_t metric, const int32_t* answer_ids, const int32_t* distractor_ids) {
  if (!M || (metric != PAHQ_METRIC_KL && metric != PAHQ_METRIC_LOGIT_DIFF)) return PAHQ_EINVAL;
  if (metric == PAHQ_METRIC_LOGIT_DIFF) {
    if (!answer_ids || !distractor_ids) return PAHQ_EINVAL;
    for (int b = 0; b < M->B; b++)
      if (answer_ids[b] < 0 || answer_ids[b] >= M->V || distractor_ids[b] < 0 || distractor_ids[b] >= M->V ||
          answer_ids[b] == distractor_ids[b]) return PAHQ_EINVAL;
    HIPCHK(hipMemcpyAsync(M->ans_dev, answer_ids, M->B * sizeof(int), hipMemcpyHostToDevice, M->stream));
    HIPCHK(hipMemcpyAsync(M->dis_dev, distractor_ids, M->B * sizeof(int), hipMemcpyHostToDevice, M->stream));
    HIPCHK(hipStreamSynchronize(M->stream));
  }
  M->metric = metric;
  M->has_cache = false;          // the reference values of the metric are taken by the cache pass
  M->pi_l = M->pi_h = -2; M->ref_layer = -1;
  return PAHQ_OK;
}

// Independent candidates (sender_ids[i] -> receiver) for one receiver, or -- recv3 -- for the query, key and value
// inputs of one head side by side: cnt[c] candidates of channel c, senders and results in channel order.  The device
// batches of a call are queued back to back and the host waits once per ncap candidates: batch b reads its senders
// from send_dev + off and writes its results to kl_dev + off.
static int eval_candidates(pahq_model* M, const RecvCtx& ctx, const int* recv3, const int* cnt3, const int32_t* sender_ids, int n,
                           float* kl_out) {
  // receiver of candidate i
  auto recv_of = [&](int i) { if (!recv3) return ctx.v; int c = 0; while (i >= cnt3[c]) { i -= cnt3[c]; c++; } return recv3[c]; };
  for (int pos = 0; pos < n;) {
    const int chunk = std::min(M->ncap, n - pos);
    for (int off = 0; off < chunk;) {
      // batches of equal size: 131 candidates run as 66 + 65, not as 128 + 3 (a batch of three pays a full
      // batch's launches and leaves most compute units idle)
      const int left = chunk - off, parts = (left + ctx.n_eff - 1) / ctx.n_eff;
      int nb = (left + parts - 1) / parts;
      PassArgs a; a.kind = CAND; a.p0 = ctx.p0; a.n = nb; a.pl = ctx.pl; a.ph = ctx.ph; a.v = ctx.v; a.patch_mode = 1;
      a.io_off = off;
      // an edge that is already removed adds nothing: such a candidate patches with the all-zero tile
      for (int i = 0; i < nb; i++) {
        const int u = sender_ids[pos + off + i], w = recv_of(pos + off + i);
        M->send_host[off + i] = M->removed[edge_index(M, u, w)] ? M->g.Ns : u;
        if (recv3) { int k, l, h, c; M->g.receiver_info(w, k, l, h, c); a.chan_count[c]++; }
      }
      HIPCHK(hipMemcpyAsync(M->send_dev + off, M->send_host + off, (size_t)nb * sizeof(int), hipMemcpyHostToDevice, M->stream));
      PCHK(run_pass(M, a, &M->plan));
      M->counters[0] += nb; M->counters[1] += 1;
      off += nb;
    }
    HIPCHK(hipMemcpyAsync(M->kl_host, M->kl_dev, (size_t)chunk * sizeof(double), hipMemcpyDeviceToHost, M->stream));
    HIPCHK(hipStreamSynchronize(M->stream));
    for (int i = 0; i < chunk; i++) kl_out[pos + i] = (float)M->kl_host[i];
    pos += chunk;
  }
  return PAHQ_OK;
}

int pahq_eval_edges(pahq_model* M, int32_t receiver, const int32_t* sender_ids, int32_t n, float* kl_out) {
  if (!M || n < 0 || (n > 0 && (!sender_ids || !kl_out))) return PAHQ_EINVAL;
  if (receiver < 0 || receiver >= M->g.Nr) return PAHQ_EINVAL;
  if (!M->has_cache) return PAHQ_ESTATE;
  const int n_up = M->g.n_upstream(receiver);
  for (int i = 0; i < n; i++) if (sender_ids[i] < 0 || sender_ids[i] >= n_up) return PAHQ_EINVAL;
  if (n == 0) return PAHQ_OK;
  RecvCtx ctx;
  PCHK(setup_receiver(M, receiver, ctx));
  return eval_candidates(M, ctx, nullptr, nullptr, sender_ids, n, kl_out);
}

int pahq_eval_edge_list(pahq_model* M, int64_t n, const int32_t* receivers, const int32_t* sender_ids, float* kl_out) {
  if (!M || n < 0 || (n > 0 && (!receivers || !sender_ids || !kl_out))) return PAHQ_EINVAL;
  if (!M->has_cache) return PAHQ_ESTATE;
  const GraphDims& g = M->g;
  for (int64_t i = 0; i < n; i++) {
    if (receivers[i] < 0 || receivers[i] >= g.Nr) return PAHQ_EINVAL;
    if (sender_ids[i] < 0 || sender_ids[i] >= g.n_upstream(receivers[i])) return PAHQ_EINVAL;
  }
  // runs of one receiver; up to three neighbouring runs that are the query, key and value inputs of one head
  // (each at most once, in channel order) go to the device side by side when that head is the fp32 head of all three
  for (int64_t i = 0; i < n;) {
    int recv3[3] = {-1, -1, -1}, cnt3[3] = {0, 0, 0};
    int k0, l0, h0, c0;
    g.receiver_info(receivers[i], k0, l0, h0, c0);
    int runs = 0, last_c = -1;
    int64_t j = i;
    while (j < n && runs < 3) {
      int k, l, h, c;
      g.receiver_info(receivers[j], k, l, h, c);
      const bool joins = runs == 0 || (M->cfg.precision == PAHQ_PAHQ && g.C == 3 && k0 == 0 && k == 0 && l == l0 && h == h0 && c > last_c);
      if (!joins) break;
      int64_t r = j;
      while (r < n && receivers[r] == receivers[j]) r++;
      if (r - i > 0x7fffffff) return PAHQ_ETOOBIG;
      if (k == 0 && c >= 0) { recv3[c] = receivers[j]; cnt3[c] = (int)(r - j); }
      last_c = (k == 0 && c >= 0) ? c : 3;
      runs++;
      j = r;
      if (k != 0) break;
    }
    RecvCtx ctx;
    const Upcoming up = {receivers + j, n - j, false};
    PCHK(setup_receiver(M, receivers[i], ctx, &up));
    if (runs == 1) {
      PCHK(eval_candidates(M, ctx, nullptr, nullptr, sender_ids + i, (int)(j - i), kl_out + i));
    } else {
      // the three inputs share the head's state, the plan and the layer's shared part; each has its own current input
      for (int c = 0; c < 3; c++)
        if (recv3[c] >= 0) PCHK(build_receiver_input(M, recv3[c], ctx.p0, M->xvc + (long long)c * M->tile));
      PCHK(eval_candidates(M, ctx, recv3, cnt3, sender_ids + i, (int)(j - i), kl_out + i));
    }
    i = j;
  }
  return PAHQ_OK;
}

int pahq_eval_current(pahq_model* M, int32_t receiver, float* kl_out) {
  if (!M || !kl_out || receiver < 0 || receiver >= M->g.Nr) return PAHQ_EINVAL;
  if (!M->has_cache) return PAHQ_ESTATE;
  RecvCtx ctx;
  PCHK(setup_receiver(M, receiver, ctx));
  double kl;
  PCHK(eval_state(M, ctx, &kl));
  *kl_out = (float)kl;
  return PAHQ_OK;
}

static int sweep_impl(pahq_model* M, float tau, const int32_t* receivers, int32_t n_receivers, uint8_t* kept,
                      int64_t* n_evals, pahq_trace_rec* trace, int64_t trace_cap, bool from_current = false);

int pahq_acdc_sweep(pahq_model* M, float tau, const int32_t* receivers, int32_t n_receivers, uint8_t* kept,
                    int64_t* n_evals, pahq_trace_rec* trace, int64_t trace_cap) {
  if (!M) return PAHQ_EINVAL;
  const std::vector<uint8_t> before = M->removed;       // a failed sweep leaves the removed set as it found it
  int rc = sweep_impl(M, tau, receivers, n_receivers, kept, n_evals, trace, trace_cap);
  if (rc != PAHQ_OK) M->removed = before;
  return rc;
}

int pahq_acdc_sweep_resume(pahq_model* M, float tau, const int32_t* receivers, int32_t n_receivers, uint8_t* kept,
                           int64_t* n_evals, pahq_trace_rec* trace, int64_t trace_cap) {
  if (!M) return PAHQ_EINVAL;
  const std::vector<uint8_t> before = M->removed;
  int rc = sweep_impl(M, tau, receivers, n_receivers, kept, n_evals, trace, trace_cap, true);
  if (rc != PAHQ_OK) M->removed = before;
  return rc;
}

int pahq_acdc_sweep_grid(pahq_model* M, const float* taus, int32_t n_taus, const int32_t* receivers, int32_t n_receivers,
                         uint8_t* kept, int64_t* n_evals) {
  if (!M || !taus || n_taus < 1 || !kept) return PAHQ_EINVAL;
  for (int i = 0; i < n_taus; i++) if (taus[i] != taus[i]) return PAHQ_EINVAL;
  const std::vector<uint8_t> before = M->removed;
  const size_t ne = M->removed.size();
  for (int i = 0; i < n_taus; i++) {
    int64_t evals = 0;
    int rc = sweep_impl(M, taus[i], receivers, n_receivers, kept + (size_t)i * ne, &evals, nullptr, 0);
    if (rc != PAHQ_OK) { M->removed = before; return rc; }
    if (n_evals) n_evals[i] = evals;
  }
  return PAHQ_OK;
}

static int sweep_impl(pahq_model* M, float tau, const int32_t* receivers, int32_t n_receivers, uint8_t* kept,
                      int64_t* n_evals, pahq_trace_rec* trace, int64_t trace_cap, bool from_current) {
  if (!M || n_receivers < 0 || (n_receivers > 0 && !receivers) || trace_cap < 0 || (trace_cap > 0 && !trace)) return PAHQ_EINVAL;
  if (tau != tau) return PAHQ_EINVAL;
  if (!M->has_cache) return PAHQ_ESTATE;
  const GraphDims& g = M->g;
  std::vector<int> order;
  if (!sweep_order(g, receivers, n_receivers, order)) return PAHQ_EINVAL;
  if (!from_current) std::fill(M->removed.begin(), M->removed.end(), 0);
  else {
    // a resumed sweep decides receivers whose edges are all still kept
    for (int v : order) {
      const uint8_t* row = M->removed.data() + M->edge_off[v];
      for (int s = 0, n_up = g.n_upstream(v); s < n_up; s++) if (row[s]) return PAHQ_ESTATE;
    }
  }
  int64_t evals = 0;
  for (size_t oi = 0; oi < order.size(); oi++) {
    const int v = order[oi];
    const int n_up = g.n_upstream(v);
    uint8_t* row = M->removed.data() + M->edge_off[v];
    if (!node_is_live(M, v)) { memset(row, 1, n_up); continue; }
    RecvCtx ctx;
    const Upcoming up = {order.data() + oi + 1, (int64_t)(order.size() - oi - 1), true};
    PCHK(setup_receiver(M, v, ctx, &up));
    double kl_cur;
    PCHK(eval_state(M, ctx, &kl_cur));
    // the accept scan (controller.h) drives the device batches; send_host / kl_host are its work arrays
    PCHK(scan_receiver(
        n_up, ctx.n_eff, (double)tau, kl_cur, row, M->send_host, M->kl_host,
        [&](const int*, int nb, int mode, double*) -> int { return eval_batch(M, ctx, nb, mode); },
        [&](int first, int count) -> int {
          // same subtraction order as the patch kernel used for these candidates
          HIPCHK(launch_xv_advance(M->xv, M->delta, M->tile, M->send_dev + first, count, M->tile, M->stream));
          return PAHQ_OK;
        },
        [&](int u, double kn, double kc, bool rm) {
          if (evals < trace_cap) {
            pahq_trace_rec& t = trace[evals];
            t.receiver = v; t.sender = u; t.kl_new = (float)kn; t.kl_cur = (float)kc; t.removed = rm ? 1 : 0;
          }
          evals++;
        }));
  }
  if (kept) for (size_t i = 0; i < M->removed.size(); i++) kept[i] = M->removed[i] ? 0 : 1;
  if (n_evals) *n_evals = evals;
  HIPCHK(hipStreamSynchronize(M->stream));
  return PAHQ_OK;
}

int pahq_eval_circuit(pahq_model* M, const uint8_t* kept, const uint8_t* f32_heads, float* kl_out, float* logits_out) {
  if (!M || !kl_out) return PAHQ_EINVAL;
  if (!M->has_cache) return PAHQ_ESTATE;
  const GraphDims& g = M->g;
  const int L = M->L, H = M->H;
  if (kept) for (size_t i = 0; i < M->removed.size(); i++) if (kept[i] > 1) return PAHQ_EINVAL;
  if (f32_heads) for (int i = 0; i < L * H; i++) if (f32_heads[i] > 1) return PAHQ_EINVAL;
  std::vector<uint8_t> saved;
  if (kept) {
    saved = M->removed;
    for (size_t i = 0; i < M->removed.size(); i++) M->removed[i] = kept[i] ? 0 : 1;
  }
  // fp32 heads: the caller's, or every head that is still part of the graph (a kept edge in and a kept edge out)
  std::vector<unsigned long long> masks(L, 0ull);
  bool any = false;
  if (M->cfg.precision == PAHQ_PAHQ) {
    for (int l = 0; l < L; l++)
      for (int h = 0; h < H; h++) {
        bool on;
        if (f32_heads) on = f32_heads[l * H + h] != 0;
        else {
          bool in_kept = false;
          for (int c = 0; c < 3 && !in_kept; c++) {
            const int r = g.headin(l, h, c);
            const uint8_t* row = M->removed.data() + M->edge_off[r];
            for (int s = 0, n_up = g.n_upstream(r); s < n_up; s++) if (!row[s]) { in_kept = true; break; }
          }
          on = in_kept && node_is_live(M, g.headin(l, h, 0));
        }
        if (on) { masks[l] |= 1ull << h; any = true; }
      }
  }
  int rc = PAHQ_OK;
  double kl = 0.0;
  do {
    PassArgs a; a.n = 1; a.p0 = 0; a.pl = a.ph = -1; a.v = -1; a.patch_mode = 0;
    a.heads = any ? masks.data() : nullptr;
    if (any) {
      // corrupted run and reference distribution under this precision set (they replace the state of the
      // last investigated head)
      M->pi_l = M->pi_h = -2; M->ref_layer = -1;
      a.kind = PI_CORRUPT; if ((rc = run_pass(M, a, nullptr)) != PAHQ_OK) break;
      a.kind = PI_REF; if ((rc = run_pass(M, a, nullptr)) != PAHQ_OK) break;
    }
    make_plan(M, 0, g.out(), M->plan);
    if (M->plan.n_slots > M->pool_tiles) { rc = PAHQ_ENOMEM; break; }
    a.kind = STATE; a.keep_logits = logits_out != nullptr;
    if ((rc = run_pass(M, a, &M->plan)) != PAHQ_OK) break;
    if (hipMemcpyAsync(M->kl_host, M->kl_dev, sizeof(double), hipMemcpyDeviceToHost, M->stream) != hipSuccess) { rc = PAHQ_EHIP; break; }
    if (logits_out && hipMemcpy2DAsync(logits_out, (size_t)M->V * sizeof(float), M->logits, (size_t)M->Vp * sizeof(float),
                                       (size_t)M->V * sizeof(float), M->B, hipMemcpyDeviceToHost, M->stream) != hipSuccess) { rc = PAHQ_EHIP; break; }
    if (hipStreamSynchronize(M->stream) != hipSuccess) { rc = PAHQ_EHIP; break; }
    kl = M->kl_host[0];
  } while (0);
  if (kept) M->removed.swap(saved);
  if (rc != PAHQ_OK) return rc;
  *kl_out = (float)kl;
  return PAHQ_OK;
}

namespace {
// One candidate under the precision set of its SENDER (Eq. P_t as printed): corrupted run and reference under that
// set from the sender's layer on, then the current graph and the graph without the edge.  Four passes of one
// instance each: the cost of a policy under which nothing can be shared between the candidates of a receiver.
int eval_pair_sender(pahq_model* M, int v, int u, double* kl_cur, double* kl_new) {
  const GraphDims& g = M->g;
  const int L = M->L, H = M->H;
  int p0 = g.pos_of_receiver(v);
  std::vector<unsigned long long> masks(L, 0ull);
  bool any = false;
  if (M->cfg.precision == PAHQ_PAHQ && u > 0) {
    const int l = (u - 1) / (H + g.mu), r = (u - 1) % (H + g.mu);
    if (r < H) { masks[l] = 1ull << r; any = true; p0 = std::min(p0, 2 * l); }
  }
  for (int w = 0; w < g.Nr; w++) {                 // what lies upstream of the first recomputed position comes from the caches
    if (g.pos_of_receiver(w) >= p0) continue;
    const uint8_t* row = M->removed.data() + M->edge_off[w];
    for (int s = 0, n_up = g.n_upstream(w); s < n_up; s++) if (row[s]) return PAHQ_ESTATE;
  }
  PassArgs a; a.n = 1; a.p0 = p0; a.pl = a.ph = -1; a.v = -1; a.patch_mode = 0;
  a.heads = any ? masks.data() : nullptr;
  if (any) {
    M->pi_l = M->pi_h = -2; M->ref_layer = -1;
    a.kind = PI_CORRUPT; PCHK(run_pass(M, a, nullptr));
    a.kind = PI_REF; PCHK(run_pass(M, a, nullptr));
  }
  uint8_t& flag = M->removed[edge_index(M, u, v)];
  const uint8_t was = flag;
  int rc = PAHQ_OK;
  a.kind = STATE;
  for (int step = 0; step < 2 && rc == PAHQ_OK; step++) {
    if (step == 1) flag = 1;
    make_plan(M, p0, g.out(), M->plan);
    if (M->plan.n_slots > M->pool_tiles) { rc = PAHQ_ENOMEM; break; }
    rc = run_pass(M, a, &M->plan);
    if (rc == PAHQ_OK && hipMemcpyAsync(M->kl_host + step, M->kl_dev, sizeof(double), hipMemcpyDeviceToHost, M->stream) != hipSuccess) rc = PAHQ_EHIP;
    if (rc == PAHQ_OK && hipStreamSynchronize(M->stream) != hipSuccess) rc = PAHQ_EHIP;
  }
  flag = was;
  if (rc != PAHQ_OK) return rc;
  *kl_cur = M->kl_host[0]; *kl_new = M->kl_host[1];
  M->counters[0] += 1; M->counters[1] += 1;
  return PAHQ_OK;
}
}  // namespace

int pahq_eval_edges_sender_policy(pahq_model* M, int32_t receiver, const int32_t* sender_ids, int32_t n, float* kl_new_out,
                                  float* kl_cur_out) {
  if (!M || n < 0 || (n > 0 && (!sender_ids || !kl_new_out || !kl_cur_out))) return PAHQ_EINVAL;
  if (receiver < 0 || receiver >= M->g.Nr) return PAHQ_EINVAL;
  if (!M->has_cache) return PAHQ_ESTATE;
  const int n_up = M->g.n_upstream(receiver);
  for (int i = 0; i < n; i++) if (sender_ids[i] < 0 || sender_ids[i] >= n_up) return PAHQ_EINVAL;
  for (int i = 0; i < n; i++) {
    double c, k;
    PCHK(eval_pair_sender(M, receiver, sender_ids[i], &c, &k));
    kl_cur_out[i] = (float)c; kl_new_out[i] = (float)k;
  }
  return PAHQ_OK;
}

int pahq_acdc_sweep_sender_policy(pahq_model* M, float tau, const int32_t* receivers, int32_t n_receivers, uint8_t* kept,
                                  int64_t* n_evals, pahq_trace_rec* trace, int64_t trace_cap) {
  if (!M || n_receivers < 0 || (n_receivers > 0 && !receivers) || trace_cap < 0 || (trace_cap > 0 && !trace) || tau != tau) return PAHQ_EINVAL;
  if (!M->has_cache) return PAHQ_ESTATE;
  const GraphDims& g = M->g;
  std::vector<int> order;
  if (!sweep_order(g, receivers, n_receivers, order)) return PAHQ_EINVAL;
  const std::vector<uint8_t> before = M->removed;
  std::fill(M->removed.begin(), M->removed.end(), 0);
  int64_t evals = 0;
  for (int v : order) {
    const int n_up = g.n_upstream(v);
    uint8_t* row = M->removed.data() + M->edge_off[v];
    if (!node_is_live(M, v)) { memset(row, 1, n_up); continue; }
    for (int u = n_up - 1; u >= 0; u--) {
      double kc, kn;
      int rc = eval_pair_sender(M, v, u, &kc, &kn);
      if (rc != PAHQ_OK) { M->removed = before; return rc; }
      const bool rm = (kn - kc) < (double)tau;
      if (evals < trace_cap) {
        pahq_trace_rec& t = trace[evals];
        t.receiver = v; t.sender = u; t.kl_new = (float)kn; t.kl_cur = (float)kc; t.removed = rm ? 1 : 0;
      }
      evals++;
      if (rm) row[u] = 1;
    }
  }
  if (kept) for (size_t i = 0; i < M->removed.size(); i++) kept[i] = M->removed[i] ? 0 : 1;
  if (n_evals) *n_evals = evals;
  return PAHQ_OK;
}

int pahq_set_dead_node_skipping(pahq_model* M, int32_t on) {
  if (!M || (on != 0 && on != 1)) return PAHQ_EINVAL;
  M->skip_dead = on != 0;
  return PAHQ_OK;
}

int pahq_set_removed(pahq_model* M, const uint8_t* removed) {
  if (!M || !removed) return PAHQ_EINVAL;
  for (size_t i = 0; i < M->removed.size(); i++) if (removed[i] > 1) return PAHQ_EINVAL;
  memcpy(M->removed.data(), removed, M->removed.size());
  return PAHQ_OK;
}
int pahq_get_removed(pahq_model* M, uint8_t* removed) {
  if (!M || !removed) return PAHQ_EINVAL;
  memcpy(removed, M->removed.data(), M->removed.size());
  return PAHQ_OK;
}

int pahq_get_weight_q(pahq_model* M, int32_t which, int32_t layer, int32_t head, uint8_t* codes, float* scale) {
  if (!M || !codes || !scale) return PAHQ_EINVAL;
  const uint8_t* src; const float* ssrc; int K, N, ldq;
  const int L = M->L, H = M->H, dh = M->dh, d = M->d, m = M->m, V = M->V;
  if (which >= PAHQ_W_Q && which <= PAHQ_W_O) { if (layer < 0 || layer >= L || head < 0 || head >= H) return PAHQ_EINVAL; }
  else if (which >= PAHQ_W_IN && which <= PAHQ_W_OUT) { if (layer < 0 || layer >= L || m == 0) return PAHQ_EINVAL; }
  if ((M->nb16 && which >= PAHQ_W_IN) || M->qbits == 16) return PAHQ_EUNSUPPORTED;      // those are bfloat16 patterns: pahq_get_weight_bf16
  switch (which) {
    case PAHQ_W_Q: case PAHQ_W_K: case PAHQ_W_V: {
      int cc = which - PAHQ_W_Q;
      K = d; N = dh; ldq = M->Kd;
      src = M->qkv_codes + ((long long)layer * 3 * H * dh + ((long long)cc * H + head) * dh) * M->Kd;
      ssrc = M->qkv_scale + (long long)layer * 3 * H + cc * H + head; break; }
    case PAHQ_W_O: K = dh; N = d; ldq = M->Kh; src = M->o_codes + ((long long)layer * H + head) * d * M->Kh; ssrc = M->o_scale + layer * H + head; break;
    case PAHQ_W_IN: K = d; N = m; ldq = M->Kd; src = M->in_codes + (long long)layer * m * M->Kd; ssrc = M->in_scale + layer; break;
    case PAHQ_W_GATE: if (!M->gate_codes) return PAHQ_EINVAL;
      K = d; N = m; ldq = M->Kd; src = M->gate_codes + (long long)layer * m * M->Kd; ssrc = M->gate_scale + layer; break;
    case PAHQ_W_OUT: K = m; N = d; ldq = M->Km; src = M->out_codes + (long long)layer * d * M->Km; ssrc = M->out_scale + layer; break;
    case PAHQ_W_U: K = d; N = V; ldq = M->Kd; src = M->u_codes; ssrc = M->u_scale; break;
    default: return PAHQ_EINVAL;
  }
  std::vector<uint8_t> tmp((size_t)N * ldq);
  HIPCHK(hipMemcpyAsync(tmp.data(), src, tmp.size(), hipMemcpyDeviceToHost, M->stream));
  HIPCHK(hipMemcpyAsync(scale, ssrc, sizeof(float), hipMemcpyDeviceToHost, M->stream));
  HIPCHK(hipStreamSynchronize(M->stream));
  for (int k = 0; k < K; k++)
    for (int n = 0; n < N; n++) codes[(size_t)k * N + n] = tmp[(size_t)n * ldq + k];
  return PAHQ_OK;
}

int pahq_get_weight_bf16(pahq_model* M, int32_t which, int32_t layer, int32_t head, uint16_t* out) {
  if (!M || !out) return PAHQ_EINVAL;
  if (!M->nb16) return PAHQ_ESTATE;
  const int L = M->L, H = M->H, dh = M->dh, d = M->d, m = M->m, V = M->V;
  const uint8_t* src; int K, N, ldq;
  if (which >= PAHQ_W_IN && which <= PAHQ_W_OUT) { if (layer < 0 || layer >= L || m == 0) return PAHQ_EINVAL; }
  if (which >= PAHQ_W_Q && which <= PAHQ_W_O) {
    if (M->qbits != 16) return PAHQ_ESTATE;              // the heads' weights are patterns only at 16 bits
    if (layer < 0 || layer >= L || head < 0 || head >= H) return PAHQ_EINVAL;
  }
  switch (which) {
    case PAHQ_W_Q: case PAHQ_W_K: case PAHQ_W_V: {
      const int cc = which - PAHQ_W_Q;
      K = d; N = dh; ldq = M->Kd;
      src = M->qkv_codes + ((long long)layer * 3 * H * dh + ((long long)cc * H + head) * dh) * M->Kd; break; }
    case PAHQ_W_O: K = dh; N = d; ldq = M->Kh; src = M->o_codes + ((long long)layer * H + head) * d * M->Kh; break;
    case PAHQ_W_IN: K = d; N = m; ldq = M->Kd_o; src = M->in_codes + (long long)layer * m * ldq; break;
    case PAHQ_W_GATE: if (!M->gate_codes) return PAHQ_EINVAL;
      K = d; N = m; ldq = M->Kd_o; src = M->gate_codes + (long long)layer * m * ldq; break;
    case PAHQ_W_OUT: K = m; N = d; ldq = M->Km_o; src = M->out_codes + (long long)layer * d * ldq; break;
    case PAHQ_W_U: K = d; N = V; ldq = M->Kd_o; src = M->u_codes; break;
    default: return PAHQ_EINVAL;
  }
  std::vector<uint8_t> tmp((size_t)N * ldq);
  HIPCHK(hipMemcpyAsync(tmp.data(), src, tmp.size(), hipMemcpyDeviceToHost, M->stream));
  HIPCHK(hipStreamSynchronize(M->stream));
  for (int k = 0; k < K; k++)
    for (int n = 0; n < N; n++) out[(size_t)k * N + n] = *(const uint16_t*)(tmp.data() + (size_t)n * ldq + 2 * (size_t)k);
  return PAHQ_OK;
}

int pahq_round_rows_bf16(pahq_model* M, int32_t site, const float* x, int32_t rows, int32_t cols, uint16_t* out) {
  if (!M || rows < 0 || cols < 1 || (rows > 0 && (!x || !out))) return PAHQ_EINVAL;
  if (site < PAHQ_QSITE_HIDDEN || site > PAHQ_QSITE_ATTN) return PAHQ_EINVAL;
  if (site == PAHQ_QSITE_ATTN && cols != 16 && cols != 32 && cols != 64 && cols != 128) return PAHQ_EINVAL;
  if (site == PAHQ_QSITE_NORM && (cols % 64 != 0 || cols > 4096)) return PAHQ_EINVAL;
  if (site == PAHQ_QSITE_HIDDEN && cols % 4 != 0) return PAHQ_EINVAL;
  if (rows == 0) return PAHQ_OK;
  // staged through the candidate buffers: fp32 rows in `logits`, patterns in `xcodes`, the (unit) scales in `xscale`
  size_t cap_f = (size_t)M->nmax * M->B * M->Vp, cap_c = (size_t)M->nmax * M->G * M->T * M->Kd, cap_s = (size_t)M->nmax * M->G * M->T;
  size_t chunk = std::min(std::min(cap_f / cols, cap_c / (2 * (size_t)cols)), cap_s);
  if (chunk < 1) return PAHQ_ENOMEM;
  for (size_t r0 = 0; r0 < (size_t)rows; r0 += chunk) {
    size_t nr = std::min(chunk, (size_t)rows - r0);
    HIPCHK(hipMemcpyAsync(M->logits, x + r0 * cols, nr * cols * sizeof(float), hipMemcpyHostToDevice, M->stream));
    if (site == PAHQ_QSITE_HIDDEN)
      HIPCHK(launch_hidden_quant(M->logits, nullptr, 0LL, M->xcodes, 0LL, M->xscale, 0LL, 1, (int)nr, cols, 2 * cols, 0, 16, M->stream));
    else if (site == PAHQ_QSITE_NORM) HIPCHK(launch_emit_rows(M->logits, (int)nr, cols, M->xcodes, M->xscale, 16, M->stream));
    else {
      // one position, one head whose value row is the given row: the attention output is that row (see pahq_quantize_rows_site)
      AttnSrc src; memset(&src, 0, sizeof(src));
      src.q = src.k = src.v = M->logits; src.q_ld = src.k_ld = src.v_ld = cols;
      src.n_heads = 1; src.h0 = 0; src.head_cols = 0; src.qbits = 16;
      HIPCHK(launch_attention(src, M->xcodes, 0, M->xscale, 0, nullptr, 0, 0ull, 0ull, 1, (int)nr, 1, 1, cols, 2 * cols, 0, nullptr, M->stream));
    }
    HIPCHK(hipMemcpyAsync(out + r0 * cols, M->xcodes, nr * cols * 2, hipMemcpyDeviceToHost, M->stream));
    HIPCHK(hipStreamSynchronize(M->stream));
  }
  return PAHQ_OK;
}

int pahq_quantize_rows_site(pahq_model* M, int32_t site, const float* x, int32_t rows, int32_t cols, uint8_t* codes,
                            float* scales) {
  if (!M || !x || !codes || !scales || rows < 0 || cols < 1 || cols > 16384) return PAHQ_EINVAL;
  if (M->qbits == 16) return PAHQ_EUNSUPPORTED;          // two-byte patterns: pahq_round_rows_bf16
  if (site == PAHQ_QSITE_NORM && (cols % 64 != 0 || cols > 4096)) return PAHQ_EINVAL;
  if (site == PAHQ_QSITE_ATTN && cols != 16 && cols != 32 && cols != 64 && cols != 128) return PAHQ_EINVAL;
  if (site < PAHQ_QSITE_HIDDEN || site > PAHQ_QSITE_ATTN) return PAHQ_EINVAL;
  if (rows == 0) return PAHQ_OK;
  // staged through the candidate buffers: fp32 rows in `logits`, codes in `xcodes`, scales in `xscale`
  const size_t ldc = site == PAHQ_QSITE_ATTN ? 128 : (size_t)cols;        // the attention kernel writes rows padded to 128 codes
  size_t cap_f = (size_t)M->nmax * M->B * M->Vp, cap_c = (size_t)M->nmax * M->G * M->T * M->Kd, cap_s = (size_t)M->nmax * M->G * M->T;
  size_t chunk = std::min(std::min(cap_f / cols, cap_c / ldc), cap_s);
  if (chunk < 1) return PAHQ_ENOMEM;
  for (size_t r0 = 0; r0 < (size_t)rows; r0 += chunk) {
    size_t nr = std::min(chunk, (size_t)rows - r0);
    HIPCHK(hipMemcpyAsync(M->logits, x + r0 * cols, nr * cols * sizeof(float), hipMemcpyHostToDevice, M->stream));
    if (site == PAHQ_QSITE_HIDDEN) HIPCHK(launch_quant_rows_plain(M->logits, (int)nr, cols, M->xcodes, M->xscale, M->qbits, M->stream));
    else if (site == PAHQ_QSITE_NORM) HIPCHK(launch_emit_rows(M->logits, (int)nr, cols, M->xcodes, M->xscale, M->qbits, M->stream));
    else {
      // nr sequences of one position and one head whose value row is the given row: the softmax over a single
      // key is 1, so the attention output IS the value row, and what leaves the kernel is its quantisation
      AttnSrc src; memset(&src, 0, sizeof(src));
      src.q = src.k = src.v = M->logits; src.q_ld = src.k_ld = src.v_ld = cols;
      src.n_heads = 1; src.h0 = 0; src.head_cols = 0; src.qbits = M->qbits;
      HIPCHK(launch_attention(src, M->xcodes, 0, M->xscale, 0, nullptr, 0, 0ull, 0ull, 1, (int)nr, 1, 1, cols, (int)ldc, 0, nullptr, M->stream));
    }
    HIPCHK(hipMemcpy2DAsync(codes + r0 * cols, (size_t)cols, M->xcodes, ldc, (size_t)cols, nr, hipMemcpyDeviceToHost, M->stream));
    HIPCHK(hipMemcpyAsync(scales + r0, M->xscale, nr * sizeof(float), hipMemcpyDeviceToHost, M->stream));
    HIPCHK(hipStreamSynchronize(M->stream));
  }
  // the staging area doubles as zero-padded code storage: restore the zeros
  size_t used = std::min((size_t)rows, chunk) * ldc;
  HIPCHK(launch_fill_zero(M->xcodes, std::min(cap_c, (used + 15) / 16 * 16), M->stream));
  HIPCHK(hipStreamSynchronize(M->stream));
  return PAHQ_OK;
}

int pahq_quantize_rows(pahq_model* M, const float* x, int32_t rows, int32_t cols, uint8_t* codes, float* scales) {
  return pahq_quantize_rows_site(M, PAHQ_QSITE_HIDDEN, x, rows, cols, codes, scales);
}

int pahq_gemm_codes(pahq_model* M, const uint8_t* a, const uint8_t* w, int32_t m, int32_t n, int32_t k, float* out) {
  if (!M || !a || !w || !out || m < 1 || n < 1 || k < 128 || k % 128 != 0) return PAHQ_EINVAL;
  if (M->all_f32) return PAHQ_ESTATE;                     // no E4M3 product in that mode
  const size_t ldc = ((size_t)n + 3) / 4 * 4;
  const size_t cap_f = (size_t)M->nmax * M->B * M->Vp, cap_c = (size_t)M->nmax * M->G * M->T * M->Kd, cap_s = (size_t)M->nmax * M->G * M->T;
  const size_t a_bytes = ((size_t)m * k + 255) / 256 * 256;
  if ((size_t)m * ldc > cap_f || a_bytes + (size_t)n * k > cap_c || (size_t)m + 16 > cap_s) return PAHQ_ENOMEM;
  uint8_t* da = M->xcodes;
  uint8_t* dw = M->xcodes + a_bytes;
  HIPCHK(hipMemcpyAsync(da, a, (size_t)m * k, hipMemcpyHostToDevice, M->stream));
  HIPCHK(hipMemcpyAsync(dw, w, (size_t)n * k, hipMemcpyHostToDevice, M->stream));
  std::vector<float> ones((size_t)m + 16, 1.0f);
  HIPCHK(hipMemcpyAsync(M->xscale, ones.data(), ones.size() * sizeof(float), hipMemcpyHostToDevice, M->stream));
  GemmProb p; memset(&p, 0, sizeof(p));
  p.A = da; p.a_is = 0; p.lda = k; p.rpi = m; p.ascale = M->xscale; p.as_is = 0; p.as_stride = 1; p.k_real = k;
  p.W = dw; p.ldw = k; p.wscale_block = n; p.ws_shift = -1;
  p.wscale = M->xscale + m;                                // one more 1.0: the whole matrix is one weight slice
  p.C = M->logits; p.c_is = 0; p.ldc = (int)ldc; p.M = m; p.N = n; p.K = k;
  if (!gemm8_prob_ok(p)) return PAHQ_EINVAL;
  void* dp = nullptr;
  PCHK(upload_table(M, &p, sizeof(p), &dp));
  HIPCHK(launch_gemm_fp8((const GemmProb*)dp, 1, m, n, M->cfg.mma == PAHQ_MMA_F16_EXACT, 0, M->stream));
  HIPCHK(hipMemcpy2DAsync(out, (size_t)n * sizeof(float), M->logits, ldc * sizeof(float), (size_t)n * sizeof(float), m,
                          hipMemcpyDeviceToHost, M->stream));
  HIPCHK(hipStreamSynchronize(M->stream));
  HIPCHK(launch_fill_zero(M->xcodes, std::min(cap_c, (a_bytes + (size_t)n * k + 15) / 16 * 16), M->stream));
  HIPCHK(hipStreamSynchronize(M->stream));
  return PAHQ_OK;
}

int pahq_get_logits(pahq_model* M, int32_t which, float* out) {
  if (!M || !out || (which != PAHQ_LOGITS_CLEAN && which != PAHQ_LOGITS_CORRUPT && which != PAHQ_LOGITS_REF)) return PAHQ_EINVAL;
  if (!M->has_cache) return PAHQ_ESTATE;
  if (which == PAHQ_LOGITS_REF && M->pi_l < 0) return PAHQ_ESTATE;      // no fp32 head's state is current
  const float* src = which == PAHQ_LOGITS_CLEAN ? M->logits_clean : (which == PAHQ_LOGITS_CORRUPT ? M->logits_corrupt : M->ref_logits);
  HIPCHK(hipMemcpy2DAsync(out, (size_t)M->V * sizeof(float), src, (size_t)M->Vp * sizeof(float), (size_t)M->V * sizeof(float),
                          M->B, hipMemcpyDeviceToHost, M->stream));
  HIPCHK(hipStreamSynchronize(M->stream));
  return PAHQ_OK;
}

int pahq_get_sender_output(pahq_model* M, int32_t which, int32_t sender, float* out) {
  if (!M || !out || (which != 0 && which != 1) || sender < 0 || sender >= M->g.Ns) return PAHQ_EINVAL;
  if (!M->has_cache) return PAHQ_ESTATE;
  const float* src = (which == 0 ? M->clean : M->corrupt) + (long long)sender * M->tile;
  HIPCHK(hipMemcpyAsync(out, src, (size_t)M->tile * sizeof(float), hipMemcpyDeviceToHost, M->stream));
  HIPCHK(hipStreamSynchronize(M->stream));
  return PAHQ_OK;
}

int pahq_get_counters(pahq_model* M, int64_t out[3]) {
  if (!M || !out) return PAHQ_EINVAL;
  out[0] = M->counters[0]; out[1] = M->counters[1]; out[2] = M->counters[2];
  return PAHQ_OK;
}

int pahq_set_attention_form(pahq_model* M, int32_t form) {
  if (!M || (form != 0 && form != 1)) return PAHQ_EINVAL;
  M->attn_form = form;
  return PAHQ_OK;
}

int pahq_prefetch_heads(pahq_model* M, int32_t layer, uint64_t heads) {
  if (!M) return PAHQ_EINVAL;
  if (!M->w32.on) return PAHQ_ESTATE;
  if (layer < 0 || layer >= M->L || (M->H < 64 && (heads >> M->H) != 0)) return PAHQ_EINVAL;
  return w32_prefetch(M, layer, heads);
}

int pahq_get_transfer_stats(pahq_model* M, int64_t out[6]) {
  if (!M || !out) return PAHQ_EINVAL;
  if (!M->w32.on) return PAHQ_ESTATE;
  const W32Cache& c = M->w32;
  out[0] = c.slots.n_acquire; out[1] = c.slots.n_demand; out[2] = c.slots.n_prefetch; out[3] = c.bytes_moved;
  out[4] = (int64_t)((size_t)M->L * M->H * c.head_floats * sizeof(float));
  out[5] = (int64_t)((size_t)c.slots.n_slots * c.head_floats * sizeof(float));
  return PAHQ_OK;
}

int pahq_set_profiling(pahq_model* M, int32_t on) {
  if (!M) return PAHQ_EINVAL;
  if (on && M->prof_ev.empty()) {
    const int pairs = 4096;
    M->prof_ev.resize(2 * pairs); M->prof_cls.assign(pairs, 0);
    for (auto& e : M->prof_ev)
      if (hipEventCreate(&e) != hipSuccess) { M->prof_ev.clear(); return PAHQ_EHIP; }
  }
  if (M->prof_on) PCHK(prof_harvest(M));
  if (on) memset(M->prof, 0, sizeof(M->prof));
  M->prof_on = on != 0;
  return PAHQ_OK;
}
int pahq_set_profiling_sample(pahq_model* M, uint32_t class_mask, int32_t every_nth_pass) {
  if (!M || every_nth_pass < 1 || (class_mask & ((1u << PAHQ_N_KERNEL_CLASSES) - 1)) == 0) return PAHQ_EINVAL;
  if (M->prof_on) PCHK(prof_harvest(M));
  M->prof_mask = class_mask; M->prof_every = every_nth_pass; M->prof_pass = 0;
  return PAHQ_OK;
}
int pahq_get_profile(pahq_model* M, pahq_kernel_stat out[PAHQ_N_KERNEL_CLASSES]) {
  if (!M || !out) return PAHQ_EINVAL;
  if (M->prof_on) PCHK(prof_harvest(M));
  memcpy(out, M->prof, sizeof(M->prof));
  return PAHQ_OK;
}

const char* pahq_strerror(int code) {
  switch (code) {
    case PAHQ_OK: return "ok";
    case PAHQ_EINVAL: return "invalid argument";
    case PAHQ_ESTATE: return "call out of order (run pahq_clean_cache first), or removed edges into receivers upstream of the one evaluated";
    case PAHQ_ENOMEM: return "workspace too small";
    case PAHQ_EHIP: return "HIP runtime error or no device";
    case PAHQ_ENAN: return "non-finite weight";
    case PAHQ_EUNSUPPORTED: return "not supported by this build";
    case PAHQ_ETOOBIG: return "input exceeds the fixed capacity of the allocation-free call";
    default: return "unknown error";
  }
}

}  // extern "C"
