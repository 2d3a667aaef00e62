// The pass executor: one function runs every kind of forward pass the method
// needs (cache passes, passes under a precision set, the state pass and the
// edge-batched candidate pass) from a residual-stream position onwards, for n
// instances at once.  The host only builds descriptor tables; every step of the
// computation runs in the kernels.
//
// Receiver inputs.  Paper, Appendix "Preliminaries": a receiver reads the sum
// of its upstream senders' outputs, a removed edge carrying the corrupted
// run's output instead.  With r the running clean stream, c the corrupted
// run's stream at the same position and D_s = out_s - corrupt_s this sum is
//     removed form  x = r - sum_{s removed} D_s      (few removed edges)
//     kept form     x = c + sum_{s kept}    D_s      (few kept edges)
// and the cheaper form is chosen per receiver.  D_s of senders below the start
// position comes from the cache (clean - corrupt); for recomputed senders it is
// written by the kernel that adds the sender's output to the stream.
#include "engine.h"
#include <map>
#include <string.h>

namespace pahq {

#define HIPCHK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) return PAHQ_EHIP; } while (0)

static inline int canon(const pahq_model* M, int p) { return canon_pos(M, p); }

void make_plan(pahq_model* M, int p0, int v, RecvPlan& out) {
  M->plan_serial++;
  plan_receivers(M->g, M->removed.data(), M->edge_off.data(), M->cfg.precision == PAHQ_PAHQ, p0, v, out, M->skip_dead);
}

// ---- fp32 head weights resident in host memory: transfers into the heads' device slots
static int w32_fetch(pahq_model* M, int id) {
  W32Cache& c = M->w32;
  const int s = c.slots.slot_of(id);
  const size_t bytes = c.head_floats * sizeof(float);
  HIPCHK(hipStreamWaitEvent(c.copy_stream, c.released[s], 0));        // the slot's last readers are done
  HIPCHK(hipMemcpyAsync(c.dev + (size_t)s * c.head_floats, c.host + (size_t)id * c.head_floats, bytes, hipMemcpyHostToDevice, c.copy_stream));
  HIPCHK(hipEventRecord(c.ready[s], c.copy_stream));
  c.bytes_moved += (long long)bytes;
  return PAHQ_OK;
}
int w32_acquire(pahq_model* M, int l, unsigned long long mask) {
  W32Cache& c = M->w32;
  if (!c.on) return PAHQ_OK;
  for (int h = 0; h < M->H; h++) {
    if (!((mask >> h) & 1ull)) continue;
    const int id = l * M->H + h, r = c.slots.acquire(id);
    if (r < 0) return PAHQ_ESTATE;                                     // two heads of one pass in one slot
    if (r == 1) { int rc = w32_fetch(M, id); if (rc != PAHQ_OK) return rc; }
    HIPCHK(hipStreamWaitEvent(M->stream, c.ready[c.slots.slot_of(id)], 0));
  }
  return PAHQ_OK;
}
int w32_release(pahq_model* M, int l, unsigned long long mask) {
  W32Cache& c = M->w32;
  if (!c.on) return PAHQ_OK;
  for (int h = 0; h < M->H; h++) {
    if (!((mask >> h) & 1ull)) continue;
    const int id = l * M->H + h;
    HIPCHK(hipEventRecord(c.released[c.slots.slot_of(id)], M->stream));
    c.slots.release(id);
  }
  return PAHQ_OK;
}
int w32_prefetch(pahq_model* M, int l, unsigned long long mask) {
  W32Cache& c = M->w32;
  if (!c.on || l < 0 || l >= M->L) return PAHQ_OK;
  for (int h = 0; h < M->H; h++) {
    if (!((mask >> h) & 1ull)) continue;
    const int id = l * M->H + h;
    if (c.slots.prefetch(id)) { int rc = w32_fetch(M, id); if (rc != PAHQ_OK) return rc; }
  }
  return PAHQ_OK;
}

namespace {

enum OpType { OP_BUILD, OP_GEMM8, OP_GEMM32, OP_ATTN, OP_COMBINE, OP_HIDQ, OP_LOGZ, OP_KL, OP_PATCH, OP_OPROJ, OP_KLRED, OP_PREF, OP_SWIGLU32, OP_LD, OP_W32ACQ, OP_W32REL };
struct Op { OpType t; int i0, i1, i2, i3; void* p0; void* p1; double flops, bytes; unsigned long long u64, u64b; };

struct Stream { float* p; long long is; };

struct Builder {
  pahq_model* M;
  const PassArgs& a;
  const RecvPlan* plan;
  std::vector<GroupDesc> groups;
  std::vector<Term> terms;
  std::vector<GemmProb> probs;
  std::vector<CombineDesc> cdescs;
  std::vector<CombineSrc> csrcs;
  std::vector<OprojDesc> odescs;
  std::vector<HeadAux> haux;
  std::vector<AttnSrc> asrcs;
  std::vector<Op> ops;
  bool general, has_pi, f32_rest;
  int nstat;
  // stand-ins of dead blocks the stream has not taken yet: cached corrupted outputs (tiles) and block biases (rows)
  std::vector<const float*> pend_tiles, pend_rows;
  std::vector<std::pair<int, long long>> new_tags;     // (layer, tag) of the dead-head sums this pass makes

  Builder(pahq_model* M_, const PassArgs& a_, const RecvPlan* p_) : M(M_), a(a_), plan(p_) {
    general = (a.kind == STATE || a.kind == CAND || a.kind == PREFIX);
    f32_rest = M->all_f32;
    has_pi = false;
    if (!M->all_f32) {
      if (a.heads) { for (int l = 0; l < M->L; l++) if (a.heads[l]) has_pi = true; }
      else has_pi = a.pl >= 0;
    }
    nstat = M->g.n_static(a.p0);
  }

  // heads of layer l whose projections run on the fp32 masters
  unsigned long long mask_of(int l) const {
    if (M->all_f32) return M->H >= 64 ? ~0ull : ((1ull << M->H) - 1ull);
    if (a.heads) return a.heads[l];
    return (a.pl == l && a.ph >= 0) ? (1ull << a.ph) : 0ull;
  }
  float* corrupt_prefix_pi(int p) {
    if (has_pi && p > a.p0) return M->rxpi + (long long)canon(M, p) * M->tile;
    return corrupt_prefix(M, p);
  }
  // slot of a recomputed sender that some receiver reads: per instance, or one for all instances
  float* slot_ptr(int s) {
    return plan->shared[s] ? M->sh_slots + (long long)plan->slot_of[s] * M->tile
                           : M->slots + (long long)plan->slot_of[s] * M->tile;
  }
  long long slot_is(int s) { return plan->shared[s] ? 0 : (long long)plan->n_slots * M->tile; }
  float* corrupt_ref_tile(int s) {      // corrupted-run output of a recomputed sender under the current precision set
    return (has_pi ? M->cpi : M->corrupt) + (long long)s * M->tile;
  }

  // fills base / run / terms of a group from a receiver spec
  void fill_input(GroupDesc& gd, const RecvSpec* sp, int pw, Stream run) {
    gd.base = nullptr; gd.base_is = 0; gd.run = nullptr; gd.run_is = 0;
    gd.term_begin = (int)terms.size(); gd.term_count = 0;
    int form = sp ? sp->form : 0;
    if (form == 2) { gd.base = corrupt_prefix_pi(pw); }
    else { gd.run = run.p; gd.run_is = run.is; }
    if (form != 0) {
      float sign = form == 1 ? -1.f : 1.f;
      for (int s : sp->senders) {
        Term t;
        if (s < nstat) { t.p = M->delta + (long long)s * M->tile; t.inst_stride = 0; }
        else { t.p = slot_ptr(s); t.inst_stride = slot_is(s); }
        t.sign = sign; t.pad_ = 0;
        terms.push_back(t);
      }
      gd.term_count = (int)sp->senders.size();
    }
  }

  // Mr rows per instance; the problem covers all a.n instances (rows numbered across instances)
  GemmProb prob8(const void* A, long long a_is, int lda, const float* as, long long as_is, int as_stride,
                 const void* W, int ldw, const float* ws, int ws_block, const float* bias, float* C, long long c_is,
                 int ldc, int act, int Mr, int N, int K, int k_real) {
    GemmProb p; memset(&p, 0, sizeof(p));
    p.A = A; p.a_is = a_is; p.lda = lda; p.ascale = as; p.as_is = as_is; p.as_stride = as_stride;
    p.W = W; p.ldw = ldw; p.wscale = ws; p.wscale_block = ws_block; p.bias = bias;
    p.C = C; p.c_is = c_is; p.ldc = ldc; p.act = act; p.rpi = Mr; p.M = Mr * a.n; p.N = N; p.K = K; p.k_real = k_real;
    p.ws_shift = -1;
    if (ws_block > 0 && (ws_block & (ws_block - 1)) == 0) { p.ws_shift = 0; while ((1 << p.ws_shift) < ws_block) p.ws_shift++; }
    return p;
  }

  void add_op(OpType t, int i0 = 0, int i1 = 0, int i2 = 0, int i3 = 0, void* p0 = nullptr, void* p1 = nullptr) {
    Op o; o.t = t; o.i0 = i0; o.i1 = i1; o.i2 = i2; o.i3 = i3; o.p0 = p0; o.p1 = p1; o.flops = 0; o.bytes = 0; o.u64 = 0; o.u64b = 0;
    ops.push_back(o);
  }
  // fp32 head weights of layer l that the launches between the two calls read (host residency: the heads' slots are
  // filled and held in between; nothing otherwise)
  void w32_begin(int l, unsigned long long mask) { if (M->w32.on && mask) { add_op(OP_W32ACQ, l, -1); ops.back().u64 = mask; } }
  void w32_end(int l, unsigned long long mask) { if (M->w32.on && mask) { add_op(OP_W32REL, l); ops.back().u64 = mask; } }
  // algorithmic work of the op just added (all instances)
  void work_gemm(int pb) {
    // flops of the contraction; bytes that must move: operand codes once (A: M x K, W: N x K; for
    // the fp32 GEMM four bytes per element), row scales, the fp32 result, and the residual /
    // second-output tiles when the problem has them
    double f = 0, by = 0;
    for (size_t i = pb; i < probs.size(); i++) {
      const GemmProb& q = probs[i];
      const double M_ = q.M, N_ = q.N, K_ = q.k_real, eb = q.ascale ? (q.b16 ? 2.0 : 1.0) : 4.0;
      f += 2.0 * M_ * N_ * K_;
      by += eb * (M_ * K_ + N_ * K_) + (q.C ? 4.0 * M_ * N_ : 0.0) + (q.kl_ref ? 4.0 * (double)q.rpi * N_ : 0.0) +
            (q.ascale ? 4.0 * M_ : 0.0) + (q.add ? 4.0 * M_ * N_ : 0.0) +
            (q.aux ? 4.0 * M_ * N_ : 0.0) + (q.aux_sub ? 4.0 * (double)q.rpi * N_ : 0.0);
    }
    ops.back().flops = f;
    ops.back().bytes = by;
  }
  void work_build(int g0, int n_groups, int skip = -1) {
    double by = 0;
    for (int i = g0; i < g0 + n_groups; i++) {
      if (i == skip) continue;
      const GroupDesc& gd = groups[i];
      double rows = gd.last_only ? M->B : M->T, d = M->d;
      double reads = (gd.base ? 1 : 0) + (gd.run ? 1 : 0) + gd.term_count;
      by += rows * d * 4.0 * reads + (gd.out_f32 ? rows * d * 4.0 : 0) + (gd.out_codes ? rows * (d + 4.0) : 0);
    }
    ops.back().bytes = by * a.n;
  }
  // the edge-batched patch of group gi: per instance one delta tile (+ the shared current input once)
  void add_patch(int gi, int inst0 = 0, int count = 0, float* xv = nullptr) {
    const int n = count ? count : a.n;        // instances inst0 .. inst0 + n - 1 (the group's outputs start at inst0)
    add_op(OP_PATCH, gi, inst0, n, 0, xv ? xv : M->xv);
    const GroupDesc& gd = groups[gi];
    double rows = gd.last_only ? M->B : M->T, d = M->d;
    ops.back().bytes = n * (rows * d * 4.0 * (1.0 + 1.0 / n) + (gd.out_f32 ? rows * d * 4.0 : 0) +
                            (gd.out_codes ? rows * (d + 4.0) : 0));
  }
  void add_build(int g0, int n_groups, int patch_group) {
    if (n_groups - (patch_group >= 0 ? 1 : 0) > 0) {
      int shared_terms = 0;      // terms every instance reads from the same tile
      for (int i = g0; i < g0 + n_groups; i++) {
        if (i == patch_group) continue;
        int c = 0;
        for (int t = 0; t < groups[i].term_count; t++) c += terms[groups[i].term_begin + t].inst_stride == 0;
        shared_terms = std::max(shared_terms, c);
      }
      add_op(OP_BUILD, g0, n_groups, patch_group, shared_terms);
      work_build(g0, n_groups, patch_group);
    }
    if (patch_group >= 0) add_patch(patch_group);
  }

  // where a recomputed sender's raw output goes
  Stream sender_dest(int s, float* scratch, long long scratch_is) {
    Stream d;
    switch (a.kind) {
      case BASE_CLEAN: d.p = M->clean + (long long)s * M->tile; d.is = 0; break;
      case BASE_CORRUPT: d.p = M->corrupt + (long long)s * M->tile; d.is = 0; break;
      case PI_CORRUPT: d.p = M->cpi + (long long)s * M->tile; d.is = 0; break;
      default: d.p = scratch; d.is = scratch_is; break;
    }
    return d;
  }
  // where the stream after a block is written
  Stream next_run(int p_after, float* scratch) {
    Stream r;
    switch (a.kind) {
      case BASE_CLEAN: r.p = M->rc + (long long)canon(M, p_after) * M->tile; r.is = 0; break;
      case BASE_CORRUPT: r.p = M->rx + (long long)canon(M, p_after) * M->tile; r.is = 0; break;
      case PI_CORRUPT: r.p = M->rxpi + (long long)canon(M, p_after) * M->tile; r.is = 0; break;
      default: r.p = scratch; r.is = M->tile; break;
    }
    return r;
  }

  void norm_params(GroupDesc& gd, const float* gain, const float* offset) {
    gd.gain = gain;
    gd.offset = (M->cfg.norm == PAHQ_NORM_RMS || !offset) ? M->zeros_d : offset;
  }

  void add_attention(const AttnSrc& src, unsigned long long f32_mask, unsigned long long dead_mask = 0) {
    asrcs.push_back(src);
    add_op(OP_ATTN, (int)asrcs.size() - 1);
    ops.back().u64 = f32_mask;
    ops.back().u64b = dead_mask;
  }

  // heads of layer l that are not computed: no kept path carries their output to the output node
  unsigned long long dead_heads(int l) const {
    unsigned long long m = 0;
    if (general && plan)
      for (int h = 0; h < M->H; h++) if (!plan->live[M->g.head(l, h)]) m |= 1ull << h;
    return m;
  }
  // A dead block leaves its stand-ins here; the stream takes all that have gathered in one pass over its tiles
  // when the next live block (or the final norm) reads it.
  void defer_standins(const float* bias, const std::vector<int>& senders) {
    for (int s : senders) pend_tiles.push_back(corrupt_ref_tile(s));
    if (bias) pend_rows.push_back(bias);
  }
  void take_standins(Stream& run) {
    if (pend_tiles.empty() && pend_rows.empty()) return;
    Stream nx; nx.p = run.p == M->run_a ? M->run_b : M->run_a; nx.is = M->tile;
    CombineDesc cd; memset(&cd, 0, sizeof(cd));
    cd.run_in = run.p; cd.run_in_is = run.is; cd.run_out = nx.p; cd.run_out_is = nx.is;
    cd.bias = nullptr; cd.src_begin = (int)csrcs.size(); cd.n_src = (int)(pend_tiles.size() + pend_rows.size());
    for (const float* t : pend_tiles) { CombineSrc cs; memset(&cs, 0, sizeof(cs)); cs.src = t; csrcs.push_back(cs); }
    for (const float* r : pend_rows) { CombineSrc cs; memset(&cs, 0, sizeof(cs)); cs.src = r; cs.bcast = 1; csrcs.push_back(cs); }
    cdescs.push_back(cd);
    add_op(OP_COMBINE, (int)cdescs.size() - 1, 0);
    ops.back().bytes = (double)a.n * M->tile * 8.0 + (double)pend_tiles.size() * M->tile * 4.0;
    pend_tiles.clear(); pend_rows.clear();
    run = nx;
  }
  // out = in + bias + the corrupted-run outputs of the given senders (what dead senders contribute to every
  // receiver); one_inst: a single instance-independent tile instead of one per instance
  void add_standins(const float* in, long long in_is, float* out, long long out_is, const float* bias,
                    const std::vector<int>& senders, bool one_inst) {
    CombineDesc cd; memset(&cd, 0, sizeof(cd));
    cd.run_in = in; cd.run_in_is = in_is; cd.run_out = out; cd.run_out_is = out_is;
    cd.bias = bias; cd.src_begin = (int)csrcs.size(); cd.n_src = (int)senders.size();
    for (int s : senders) {
      CombineSrc cs; memset(&cs, 0, sizeof(cs));
      cs.src = corrupt_ref_tile(s); cs.src_is = 0;
      csrcs.push_back(cs);
    }
    cdescs.push_back(cd);
    add_op(OP_COMBINE, (int)cdescs.size() - 1, one_inst ? 1 : 0);
    ops.back().bytes = (one_inst ? 1.0 : (double)a.n) * (double)M->tile * 4.0 * 2.0 + (double)senders.size() * M->tile * 4.0;
  }

  // First layer of a candidate pass into a head input (fp32 investigated head): the PREFIX pass
  // has left the layer's q/k/v (qkv_sh) and the stream plus all other heads (oth); only the
  // patched input's projection, the investigated head's attention and its output projection
  // are per candidate.
  void first_block_split(int l, Stream& run) {
    const GraphDims& g = M->g;
    const int H = M->H, dh = M->dh, d = M->d, T = M->T;
    int vk, vl, hv, cv;
    g.receiver_info(a.v, vk, vl, hv, cv);
    // instances [off, off + cnt[c]) patch input c (query, key, value) of the investigated head: one receiver's
    // candidates, or the candidates of all three inputs of the head side by side (they share everything else)
    int cnt[3] = {0, 0, 0};
    const bool multi = a.chan_count[0] + a.chan_count[1] + a.chan_count[2] > 0;
    const float* Wc[3] = {w32_ptr(M, 0, l, hv), w32_ptr(M, 1, l, hv), w32_ptr(M, 2, l, hv)};
    const float* bc[3] = {w32_ptr(M, 4, l, hv), w32_ptr(M, 5, l, hv), w32_ptr(M, 6, l, hv)};
    const float* shared0 = M->qkv_sh + (long long)hv * dh;
    w32_begin(l, 1ull << hv);
    const int ld_sh = 3 * H * dh;
    if (cv < 0) {
      // a head with a single input: every instance patches it, and all three projections read the patched rows
      GroupDesc gd; memset(&gd, 0, sizeof(gd));
      norm_params(gd, M->ln1_g + (long long)l * d, M->ln1_b + (long long)l * d);
      gd.out_f32 = M->xf32; gd.out_f32_is = M->tile;
      int g1 = (int)groups.size();
      groups.push_back(gd);
      add_patch(g1);
      const long long blk = (long long)a.n * T * dh;              // q, k, v of all instances one after the other
      int pq = (int)probs.size();
      for (int c = 0; c < 3; c++)
        probs.push_back(prob8(M->xf32, M->tile, d, nullptr, 0, 0, Wc[c], dh, nullptr, 1, bc[c],
                              M->qv + c * blk, (long long)T * dh, dh, 0, T, dh, d, d));
      add_op(OP_GEMM32, pq, 3, T * a.n, dh); work_gemm(pq);
      AttnSrc src; memset(&src, 0, sizeof(src));
      src.q = M->qv; src.k = M->qv + blk; src.v = M->qv + 2 * blk;
      src.q_is = src.k_is = src.v_is = (long long)T * dh;
      src.q_ld = src.k_ld = src.v_ld = dh;
      src.n_heads = 1; src.h0 = hv; src.head_cols = 0;
      add_attention(src, 1ull << hv);
    } else {
    if (multi) { for (int c = 0; c < 3; c++) cnt[c] = a.chan_count[c]; } else cnt[cv] = a.n;
    // patched rows of every range, then their projections in one launch, then the head's attention per range
    int gi[3] = {-1, -1, -1};
    for (int c = 0, off = 0; c < 3; off += cnt[c], c++) {
      if (!cnt[c]) continue;
      GroupDesc gd; memset(&gd, 0, sizeof(gd));
      norm_params(gd, M->ln1_g + (long long)l * d, M->ln1_b + (long long)l * d);
      gd.out_f32 = M->xf32 + (long long)off * M->tile; gd.out_f32_is = M->tile;
      gi[c] = (int)groups.size();
      groups.push_back(gd);
      add_patch(gi[c], off, cnt[c], multi ? M->xvc + (long long)c * M->tile : M->xv);
    }
    int pq0 = (int)probs.size(), np = 0;
    for (int c = 0, off = 0; c < 3; off += cnt[c], c++) {
      if (!cnt[c]) continue;
      GemmProb pq = prob8(M->xf32 + (long long)off * M->tile, M->tile, d, nullptr, 0, 0, Wc[c], dh, nullptr, 1,
                          bc[c], M->qv + (long long)off * T * dh, (long long)T * dh, dh, 0, T, dh, d, d);
      pq.M = T * cnt[c];
      probs.push_back(pq); np++;
    }
    add_op(OP_GEMM32, pq0, np, T * a.n, dh); work_gemm(pq0);
    for (int c = 0, off = 0; c < 3; off += cnt[c], c++) {
      if (!cnt[c]) continue;
      const float* own = M->qv + (long long)off * T * dh;
      AttnSrc src; memset(&src, 0, sizeof(src));
      src.q = c == 0 ? own : shared0;               src.q_is = c == 0 ? (long long)T * dh : 0; src.q_ld = c == 0 ? dh : ld_sh;
      src.k = c == 1 ? own : shared0 + H * dh;      src.k_is = c == 1 ? (long long)T * dh : 0; src.k_ld = c == 1 ? dh : ld_sh;
      src.v = c == 2 ? own : shared0 + 2 * H * dh;  src.v_is = c == 2 ? (long long)T * dh : 0; src.v_ld = c == 2 ? dh : ld_sh;
      src.n_heads = 1; src.h0 = hv; src.head_cols = 0;
      add_attention(src, 1ull << hv);
      ops.back().i1 = off; ops.back().i2 = cnt[c];
    }
    }
    Stream nxt = next_run(2 * l + 1, run.p == M->run_a ? M->run_b : M->run_a);
    int s = g.head(l, hv);
    const int pf = (int)probs.size();
    GemmProb pp = prob8(M->zf32, (long long)T * dh, dh, nullptr, 0, 0, w32_ptr(M, 3, l, hv), d, nullptr, 1, nullptr,
                        nxt.p, nxt.is, d, 0, T, d, dh, dh);
    pp.add = M->oth; pp.add_is = 0;
    if (plan->slot_of[s] >= 0) { pp.aux = slot_ptr(s); pp.aux_is = slot_is(s); pp.aux_sub = corrupt_ref_tile(s); }
    probs.push_back(pp);
    add_op(OP_GEMM32, pf, 1, T * a.n, d); work_gemm(pf);
    w32_end(l, 1ull << hv);
    run = nxt;
  }

  // First layer of the reference runs of all H heads of layer l as one pass of H instances (PI_REF_LAYER): instance i is
  // the run with head (l, i) in fp32 and nothing removed.  The instances share the layer's input, so everything is
  // computed once -- the quantised projections and attention of every head, the fp32 projections and attention of every
  // head -- and instance i's stream is the fused output projection with head i left out plus head i's fp32 output:
  // launch for launch what the single-head reference pass (attention_block with that one head in fp32) does, with the
  // same kernels on the same operands, so the two give the same bits.
  void ref_layer_block(int l, Stream& run) {
    const int H = M->H, dh = M->dh, d = M->d, T = M->T, Kd = M->Kd, Kh = M->Kh;
    const unsigned long long all_heads = H >= 64 ? ~0ull : ((1ull << H) - 1ull);
    const long long qkv_ld = 3LL * H * dh;
    GroupDesc gd; memset(&gd, 0, sizeof(gd));
    fill_input(gd, nullptr, 2 * l, run);
    norm_params(gd, M->ln1_g + (long long)l * d, M->ln1_b + (long long)l * d);
    gd.out_f32 = M->xf32; gd.out_f32_is = M->tile;
    gd.out_codes = M->xcodes; gd.out_codes_is = (long long)T * Kd;
    gd.out_scale = M->xscale; gd.out_scale_is = T;
    int gi = (int)groups.size();
    groups.push_back(gd);
    add_op(OP_BUILD, gi, 1, -1, 0); ops.back().u64 = 1;            // one instance
    work_build(gi, 1); ops.back().bytes /= a.n;
    // quantised projections of all heads -> qkv_sh; fp32 projections of all heads -> qkv
    int pb = (int)probs.size();
    GemmProb p8 = prob8(gd.out_codes, gd.out_codes_is, Kd, gd.out_scale, gd.out_scale_is, 1,
                        M->qkv_codes + (long long)l * 3 * H * dh * Kd, Kd, M->qkv_scale + (long long)l * 3 * H, dh,
                        M->bqkv + (long long)l * 3 * H * dh, M->qkv_sh, (long long)T * qkv_ld, (int)qkv_ld, 0, T, 3 * H * dh, Kd, d);
    p8.M = T; p8.b16 = M->qbits == 16;
    probs.push_back(p8);
    add_op(OP_GEMM8, pb, 1, T, 3 * H * dh); work_gemm(pb);
    int pf = (int)probs.size();
    w32_begin(l, all_heads);
    for (int h = 0; h < H; h++)
      for (int c = 0; c < 3; c++) {
        GemmProb pq = prob8(gd.out_f32, gd.out_f32_is, d, nullptr, 0, 0, w32_ptr(M, c, l, h), dh, nullptr, 1, w32_ptr(M, 4 + c, l, h),
                            M->qkv + ((long long)c * H + h) * dh, (long long)T * qkv_ld, (int)qkv_ld, 0, T, dh, d, d);
        pq.M = T;
        probs.push_back(pq);
      }
    add_op(OP_GEMM32, pf, 3 * H, T, dh); work_gemm(pf);
    for (int f32 = 0; f32 < 2; f32++) {
      const float* buf = f32 ? M->qkv : M->qkv_sh;
      AttnSrc src; memset(&src, 0, sizeof(src));
      src.q = buf; src.k = buf + H * dh; src.v = buf + 2 * H * dh;
      src.q_ld = src.k_ld = src.v_ld = (int)qkv_ld;
      src.n_heads = H; src.h0 = 0; src.head_cols = dh;
      add_attention(src, f32 ? all_heads : 0ull);
      ops.back().i1 = 0; ops.back().i2 = 1;                          // one instance
    }
    // every head's fp32 output (H problems, one launch), then per instance the fused projection of the other heads
    pf = (int)probs.size();
    for (int h = 0; h < H; h++) {
      GemmProb pp = prob8(M->zf32 + (long long)h * dh, (long long)T * H * dh, H * dh, nullptr, 0, 0,
                          w32_ptr(M, 3, l, h), d, nullptr, 1, nullptr, M->headout + (long long)h * M->tile, M->tile, d, 0, T, d, dh, dh);
      pp.M = T;
      probs.push_back(pp);
    }
    add_op(OP_GEMM32, pf, H, T, d); work_gemm(pf);
    w32_end(l, all_heads);
    Stream nxt = next_run(2 * l + 1, run.p == M->run_a ? M->run_b : M->run_a);
    for (int h = 0; h < H; h++) {
      OprojDesc od; memset(&od, 0, sizeof(od));
      od.zc = M->zcodes; od.zc_is = (long long)T * H * Kh; od.zs = M->zscale; od.zs_is = (long long)T * H;
      od.W = M->o_codes + (long long)l * H * d * Kh; od.ws = M->o_scale + (long long)l * H;
      od.run_in = run.p; od.run_in_is = run.is; od.run_out = nxt.p + (long long)h * nxt.is; od.run_out_is = nxt.is;
      od.bias = M->b_O + (long long)l * d;
      od.H = H; od.Kh = Kh; od.skip_mask = 1ull << h; od.rpi = T; od.M = T; od.N = d;
      od.aux_begin = -1; od.dh = M->dh;
      od.extra = M->headout + (long long)h * M->tile; od.extra_is = M->tile;
      odescs.push_back(od);
      add_op(OP_OPROJ, (int)odescs.size() - 1, T, d);
      ops.back().flops = 2.0 * T * d * dh * (H - 1);
    }
    run = nxt;
  }

  void attention_block(int l, Stream& run) {
    const GraphDims& g = M->g;
    const int H = M->H, dh = M->dh, d = M->d, T = M->T, Kd = M->Kd, Kh = M->Kh;
    const unsigned long long all_heads = H >= 64 ? ~0ull : ((1ull << H) - 1ull);
    const unsigned long long dead = dead_heads(l);             // heads of this layer that are not computed at all
    const unsigned long long fmask = mask_of(l) & ~dead;       // live heads of this layer computed in fp32
    const unsigned long long off8 = fmask | dead;              // heads that take no part in the quantised kernels
    const int nf = __builtin_popcountll(fmask);
    const bool prefix = a.kind == PREFIX;
    float* const qkv_buf = prefix ? M->qkv_sh : M->qkv;
    std::vector<int> dead_list;
    for (int h = 0; h < H; h++) if ((dead >> h) & 1ull) dead_list.push_back(g.head(l, h));
    if (dead == all_heads) {
      // nothing of this layer reaches the output: the stream moves on with the corrupted run's head outputs
      defer_standins(M->b_O + (long long)l * d, dead_list);
      return;
    }
    take_standins(run);
    // sum of the dead heads' stand-ins: the same for every instance and for every pass under this plan (the state
    // pass and all candidate batches of a receiver), so it is made by the first pass that needs it
    const float* deadsum = nullptr;
    if (!dead_list.empty()) {
      float* ds = M->deadsum + (long long)l * M->tile;
      const long long tag = 2 * M->plan_serial + (has_pi ? 1 : 0);
      if (M->deadsum_tag[l] != tag) {
        std::vector<int> rest(dead_list.begin() + 1, dead_list.end());
        add_standins(corrupt_ref_tile(dead_list[0]), 0, ds, 0, nullptr, rest, true);
        new_tags.push_back(std::make_pair(l, tag));
      }
      deadsum = ds;
    }
    // ---- groups
    std::map<std::pair<int, std::vector<int>>, int> seen;
    std::vector<int> grp_of(3 * H, -1);          // index into `groups` per (h, c) block
    int g_begin = (int)groups.size(), n_f32 = 0, patch_group = -1;
    for (int h = 0; h < H; h++)
      for (int c = 0; c < 3; c++) {
        if ((dead >> h) & 1ull) continue;
        int w = g.headin(l, h, c);
        const bool is_pi = (fmask >> h) & 1ull;
        int gi;
        if (a.kind == CAND && w == a.v) {
          if (patch_group < 0) {           // (a head with a single input meets it three times: one group)
            GroupDesc gd; memset(&gd, 0, sizeof(gd));
            norm_params(gd, M->ln1_g + (long long)l * d, M->ln1_b + (long long)l * d);
            patch_group = (int)groups.size(); groups.push_back(gd);
          }
          gi = patch_group;
        } else {
          const RecvSpec* sp = general ? &plan->spec[w] : nullptr;
          std::pair<int, std::vector<int>> key(sp ? sp->form : 0, sp ? sp->senders : std::vector<int>());
          auto it = seen.find(key);
          if (it == seen.end()) {
            GroupDesc gd; memset(&gd, 0, sizeof(gd));
            fill_input(gd, sp, 2 * l, run);
            norm_params(gd, M->ln1_g + (long long)l * d, M->ln1_b + (long long)l * d);
            gi = (int)groups.size(); groups.push_back(gd); seen[key] = gi;
          } else gi = it->second;
        }
        grp_of[c * H + h] = gi;
        GroupDesc& gd = groups[gi];
        int local = gi - g_begin;
        if (is_pi) {
          // fp32 rows of a group: a.n instances back to back, one block per group that needs them
          if (!gd.out_f32) { gd.out_f32 = M->xf32 + (long long)n_f32 * a.n * M->tile; gd.out_f32_is = M->tile; n_f32++; }
        } else if (!gd.out_codes) {
          gd.out_codes = M->xcodes + (long long)local * M->nmax * T * Kd; gd.out_codes_is = (long long)T * Kd;
          gd.out_scale = M->xscale + (long long)local * M->nmax * T; gd.out_scale_is = T;
        }
      }
    int n_groups = (int)groups.size() - g_begin;
    add_build(g_begin, n_groups, patch_group);
    // ---- fp8 projections: runs of consecutive column blocks of quantised heads that read the same group
    int pb = (int)probs.size(), maxN = 0;
    const long long qkv_ld = 3LL * H * dh;
    for (int nb = 0; nb < 3 * H;) {
      int gi = grp_of[nb];
      if ((off8 >> (nb % H)) & 1ull) { nb++; continue; }
      int e = nb + 1;
      while (e < 3 * H && grp_of[e] == gi && !((off8 >> (e % H)) & 1ull)) e++;
      const GroupDesc& gd = groups[gi];
      probs.push_back(prob8(gd.out_codes, gd.out_codes_is, Kd, gd.out_scale, gd.out_scale_is, 1,
                            M->qkv_codes + ((long long)l * 3 * H * dh + (long long)nb * dh) * Kd, Kd,
                            M->qkv_scale + (long long)l * 3 * H + nb, dh, M->bqkv + (long long)l * 3 * H * dh + (long long)nb * dh,
                            qkv_buf + (long long)nb * dh, (long long)T * qkv_ld, (int)qkv_ld, 0, T, (e - nb) * dh, Kd, d));
      probs.back().b16 = M->qbits == 16;
      if ((e - nb) * dh > maxN) maxN = (e - nb) * dh;
      nb = e;
    }
    if ((int)probs.size() > pb) { add_op(OP_GEMM8, pb, (int)probs.size() - pb, T * a.n, maxN); work_gemm(pb); }
    // ---- fp32 projections of the heads in the precision set
    if (nf) {
      int pf = (int)probs.size();
      w32_begin(l, fmask);
      for (int h = 0; h < H; h++) {
        if (!((fmask >> h) & 1ull)) continue;
        for (int c = 0; c < 3; c++) {
          const GroupDesc& gd = groups[grp_of[c * H + h]];
          probs.push_back(prob8(gd.out_f32, gd.out_f32_is, d, nullptr, 0, 0, w32_ptr(M, c, l, h), dh, nullptr, 1,
                                w32_ptr(M, 4 + c, l, h), qkv_buf + ((long long)c * H + h) * dh, (long long)T * qkv_ld,
                                (int)qkv_ld, 0, T, dh, d, d));
        }
      }
      add_op(OP_GEMM32, pf, 3 * nf, T * a.n, dh); work_gemm(pf);
      if (prefix) w32_end(l, fmask);                    // a prefix pass stops before the output projection
    }
    if (prefix && off8 == all_heads) {
      // only the investigated head of this layer is live: what every candidate shares is the stream, the bias and
      // the dead heads' stand-ins
      add_standins(run.p, run.is, M->oth, 0, M->b_O + (long long)l * d, dead_list, false);
      run.p = M->oth; run.is = 0;
      return;
    }
    {
      AttnSrc src; memset(&src, 0, sizeof(src));
      src.q = qkv_buf; src.k = qkv_buf + H * dh; src.v = qkv_buf + 2 * H * dh;
      src.q_is = src.k_is = src.v_is = (long long)T * qkv_ld;
      src.q_ld = src.k_ld = src.v_ld = (int)qkv_ld;
      src.n_heads = H; src.h0 = 0; src.head_cols = dh;
      add_attention(src, fmask, dead);
    }
    // ---- output projections of all heads fused with the stream update.  Only heads whose
    // individual output is needed (cache passes; a downstream receiver that treats the head's
    // edge differently from the stream) are written out.
    Stream nxt = next_run(2 * l + 1, run.p == M->run_a ? M->run_b : M->run_a);
    if (prefix) { nxt.p = M->oth; nxt.is = 0; }       // stream + bias + every head but the investigated one
    const bool store_raw = (a.kind == BASE_CLEAN || a.kind == BASE_CORRUPT || a.kind == PI_CORRUPT);
    OprojDesc od; memset(&od, 0, sizeof(od));
    od.zc = M->zcodes; od.zc_is = (long long)T * H * Kh; od.zs = M->zscale; od.zs_is = (long long)T * H;
    od.W = M->o_codes + (long long)l * H * d * Kh; od.ws = M->o_scale + (long long)l * H;
    od.run_in = run.p; od.run_in_is = run.is; od.run_out = nxt.p; od.run_out_is = nxt.is;
    od.bias = M->b_O + (long long)l * d;
    od.H = H; od.Kh = Kh; od.skip_mask = off8; od.rpi = T; od.M = T * a.n; od.N = d;
    od.aux_begin = -1; od.dh = M->dh;
    od.extra = deadsum; od.extra_is = 0;              // replaced below when fp32 heads are chained in front of it
    bool any_aux = false;
    std::vector<HeadAux> hx(H);
    for (int h = 0; h < H; h++) {
      int s = g.head(l, h);
      hx[h].dst = nullptr; hx[h].dst_is = 0; hx[h].sub = nullptr;
      if (store_raw) { Stream dst = sender_dest(s, nullptr, 0); hx[h].dst = dst.p; hx[h].dst_is = dst.is; }
      else if (general && plan->slot_of[s] >= 0) {
        hx[h].dst = slot_ptr(s); hx[h].dst_is = slot_is(s);
        hx[h].sub = corrupt_ref_tile(s);
      }
      if (hx[h].dst && !((fmask >> h) & 1ull)) any_aux = true;
    }
    if (nf && !prefix) {
      // the fp32 heads' projections, one fp32 GEMM each, summed in ascending head order into one tile (the
      // fused kernel, or the plain stream update when every head is fp32, adds it); a head's own output goes,
      // where needed, to its cache tile / slot through the second output
      int k = 0;
      for (int h = 0; h < H; h++) {
        if (!((fmask >> h) & 1ull)) continue;
        int pf = (int)probs.size();
        GemmProb pp = prob8(M->zf32 + (long long)k * dh, (long long)T * nf * dh, nf * dh, nullptr, 0, 0,
                            w32_ptr(M, 3, l, h), d, nullptr, 1, nullptr, M->headout, M->tile, d, 0, T, d, dh, dh);
        if (k > 0) { pp.add = M->headout; pp.add_is = M->tile; }
        else if (deadsum) { pp.add = deadsum; pp.add_is = 0; }          // the chain starts from the dead heads' stand-ins
        pp.aux = hx[h].dst; pp.aux_is = hx[h].dst_is; pp.aux_sub = hx[h].sub;
        probs.push_back(pp);
        add_op(OP_GEMM32, pf, 1, T * a.n, d); work_gemm(pf);
        k++;
      }
      w32_end(l, fmask);
      od.extra = M->headout; od.extra_is = M->tile;
    }
    if (off8 == all_heads && nf && !prefix) {
      // nothing is quantised in this layer: next = run + b_O + (sum of the fp32 heads)
      CombineDesc cd; memset(&cd, 0, sizeof(cd));
      cd.run_in = run.p; cd.run_in_is = run.is; cd.run_out = nxt.p; cd.run_out_is = nxt.is;
      cd.bias = M->b_O + (long long)l * d; cd.src_begin = (int)csrcs.size(); cd.n_src = 1;
      CombineSrc cs; memset(&cs, 0, sizeof(cs));
      cs.src = M->headout; cs.src_is = M->tile;
      csrcs.push_back(cs);
      cdescs.push_back(cd);
      add_op(OP_COMBINE, (int)cdescs.size() - 1);
      ops.back().bytes = 3.0 * a.n * (double)M->tile * 4.0;
    } else {
      if (any_aux) { od.aux_begin = (int)haux.size(); haux.insert(haux.end(), hx.begin(), hx.end()); }
      odescs.push_back(od);
      add_op(OP_OPROJ, (int)odescs.size() - 1, T * a.n, d);
      ops.back().flops = 2.0 * T * a.n * d * dh * (H - __builtin_popcountll(off8));
    }
    run = nxt;
  }

  void mlp_block(int l, Stream& run) {
    const GraphDims& g = M->g;
    const int d = M->d, T = M->T, Kd = M->Kd, Km = M->Km, m = M->m;
    int w = g.mlpin(l), s = g.mlp(l);
    if (general && plan && !plan->live[s]) {
      // a dead MLP: the stream moves on with the corrupted run's output in its place
      defer_standins(M->b_out + (long long)l * d, std::vector<int>(1, s));
      return;
    }
    take_standins(run);
    GroupDesc gd; memset(&gd, 0, sizeof(gd));
    int patch_group = -1, gi = (int)groups.size();
    if (a.kind == CAND && w == a.v) patch_group = gi;
    else fill_input(gd, general ? &plan->spec[w] : nullptr, 2 * l + 1, run);
    norm_params(gd, M->ln2_g + (long long)l * d, M->ln2_b + (long long)l * d);
    const int Ko = M->Kd_o, Kmo = M->Km_o, b16 = M->nb16 ? 1 : 0;      // row bytes of this block's operands (bfloat16: two per element)
    if (f32_rest) { gd.out_f32 = M->xf32; gd.out_f32_is = M->tile; }
    else {
      gd.out_codes = M->xcodes; gd.out_codes_is = (long long)T * Ko;
      gd.out_scale = M->xscale; gd.out_scale_is = T;
      if (b16) gd.qbits = 16;
    }
    groups.push_back(gd);
    add_build(gi, 1, patch_group);
    const bool swiglu = M->cfg.act == PAHQ_ACT_SWIGLU;
    Stream nxt = next_run(2 * l + 2, run.p == M->run_a ? M->run_b : M->run_a);
    const bool store_raw = a.kind == BASE_CLEAN || a.kind == BASE_CORRUPT || a.kind == PI_CORRUPT;
    auto second_output = [&](GemmProb& po) {
      // the sender's own output (cache passes) or its difference to the corrupted run (a slot some receiver
      // reads) leaves through the second output
      if (store_raw) { Stream dest = sender_dest(s, nullptr, 0); po.aux = dest.p; po.aux_is = dest.is; }
      else if (general && plan->slot_of[s] >= 0) { po.aux = slot_ptr(s); po.aux_is = slot_is(s); po.aux_sub = corrupt_ref_tile(s); }
    };
    if (f32_rest) {
      // all-fp32 mode: both matrix products on the fp32 masters; GELU in the first one's epilogue, SwiGLU by an
      // elementwise kernel over the two results
      int pb = (int)probs.size();
      probs.push_back(prob8(gd.out_f32, gd.out_f32_is, d, nullptr, 0, 0, M->W_in + (long long)l * d * m, m, nullptr, 1,
                            M->b_in + (long long)l * m, M->hid, (long long)T * m, m, M->cfg.act == PAHQ_ACT_GELU ? 1 : 0, T, m, d, d));
      if (swiglu)
        probs.push_back(prob8(gd.out_f32, gd.out_f32_is, d, nullptr, 0, 0, M->W_gate + (long long)l * d * m, m, nullptr, 1,
                              nullptr, M->hid2, (long long)T * m, m, 0, T, m, d, d));
      add_op(OP_GEMM32, pb, swiglu ? 2 : 1, T * a.n, m); work_gemm(pb);
      if (swiglu) { add_op(OP_SWIGLU32); ops.back().bytes = 3.0 * a.n * T * (double)m * 4.0; }
      pb = (int)probs.size();
      GemmProb po = prob8(M->hid, (long long)T * m, m, nullptr, 0, 0, M->W_out + (long long)l * m * d, d, nullptr, 1,
                          M->b_out + (long long)l * d, nxt.p, nxt.is, d, 0, T, d, m, m);
      po.add = run.p; po.add_is = run.is;
      second_output(po);
      probs.push_back(po);
      add_op(OP_GEMM32, pb, 1, T * a.n, d); work_gemm(pb);
      run = nxt;
      return;
    }
    int pb = (int)probs.size();
    probs.push_back(prob8(gd.out_codes, gd.out_codes_is, Ko, gd.out_scale, gd.out_scale_is, 1,
                          M->in_codes + (long long)l * m * Ko, Ko, M->in_scale + l, m, M->b_in + (long long)l * m, M->hid,
                          (long long)T * m, m, 0, T, m, Ko, d));       // the activation is applied by the hidden quantiser
    probs.back().b16 = b16;
    if (swiglu) {
      probs.push_back(prob8(gd.out_codes, gd.out_codes_is, Ko, gd.out_scale, gd.out_scale_is, 1,
                            M->gate_codes + (long long)l * m * Ko, Ko, M->gate_scale + l, m, nullptr, M->hid2,
                            (long long)T * m, m, 0, T, m, Ko, d));
      probs.back().b16 = b16;
    }
    add_op(OP_GEMM8, pb, swiglu ? 2 : 1, T * a.n, m); work_gemm(pb);
    add_op(OP_HIDQ, swiglu ? 2 : (M->cfg.act == PAHQ_ACT_GELU ? 1 : 0));
    ops.back().bytes = (double)a.n * T * m * ((swiglu ? 8.0 : 4.0) + (b16 ? 2.0 : 1.0));
    // output projection fused with the stream update: next = run + b_out + out
    pb = (int)probs.size();
    GemmProb po = prob8(M->hcodes, (long long)T * Kmo, Kmo, M->hscale, T, 1, M->out_codes + (long long)l * d * Kmo, Kmo,
                        M->out_scale + l, d, M->b_out + (long long)l * d, nxt.p, nxt.is, d, 0, T, d, Kmo, m);
    po.b16 = b16;
    po.add = run.p; po.add_is = run.is;
    second_output(po);
    probs.push_back(po);
    add_op(OP_GEMM8, pb, 1, T * a.n, d); work_gemm(pb);
    run = nxt;
  }

  // The logit-difference metric of the rows the final group just produced: for a reference pass into that
  // run's reference values, for a scored pass into one score per instance.
  void add_logit_diff() {
    const bool ref_pass = a.kind == BASE_CLEAN || a.kind == PI_REF || a.kind == PI_REF_LAYER;
    if (ref_pass) add_op(OP_LD, 0, 0, 0, 0, a.kind == BASE_CLEAN ? M->ld_clean : (a.kind == PI_REF_LAYER ? M->ld_ref_all : M->ld_ref));
    else if (general) add_op(OP_LD, 1, 0, 0, 0, has_pi ? M->ld_ref : M->ld_clean);
    else return;
    ops.back().bytes = (double)a.n * M->B * (3.0 * M->d + 16.0);
  }

  void final_block(Stream run) {
    take_standins(run);
    const bool ld = M->metric == PAHQ_METRIC_LOGIT_DIFF;
    // with that metric a scored pass needs two logits per sequence, not the unembedding (unless its logits are asked for)
    final_block_kl(run, ld && general && !a.keep_logits);
    if (ld && a.kind != PI_CORRUPT && a.kind != BASE_CORRUPT) add_logit_diff();
  }

  void final_block_kl(Stream run, bool group_only) {
    const GraphDims& g = M->g;
    const int d = M->d, B = M->B, Kd = M->Kd, V = M->V, Vp = M->Vp;
    if (a.kind == PI_CORRUPT) return;           // only the sender outputs are needed
    int w = g.out();
    GroupDesc gd; memset(&gd, 0, sizeof(gd));
    int patch_group = -1, gi = (int)groups.size();
    if (a.kind == CAND && w == a.v) patch_group = gi;
    else fill_input(gd, general ? &plan->spec[w] : nullptr, 2 * M->L, run);
    norm_params(gd, M->lnf_g, M->lnf_b);
    gd.last_only = 1;
    if (f32_rest) { gd.out_f32 = M->xf32; gd.out_f32_is = (long long)B * d; }
    else {
      gd.out_codes = M->lastcodes; gd.out_codes_is = (long long)B * M->Kd_o;
      gd.out_scale = M->lastscale; gd.out_scale_is = B;
      if (M->nb16) gd.qbits = 16;
    }
    groups.push_back(gd);
    add_build(gi, 1, patch_group);
    if (group_only) return;
    float* lg; long long lg_is = 0;
    switch (a.kind) {
      case BASE_CLEAN: lg = M->logits_clean; break;
      case BASE_CORRUPT: lg = M->logits_corrupt; break;
      case PI_REF: lg = M->ref_logits; break;
      case PI_REF_LAYER: lg = M->ref_logits_all; lg_is = (long long)B * Vp; break;
      default: lg = M->logits; lg_is = (long long)B * Vp; break;
    }
    int pb = (int)probs.size();
    if (f32_rest) {
      // all-fp32 mode: the unembedding on the fp32 master, logits in memory, log-softmax + KL over them
      probs.push_back(prob8(gd.out_f32, gd.out_f32_is, d, nullptr, 0, 0, M->W_U, V, nullptr, 1, M->b_U, lg, lg_is, Vp, 0,
                            B, V, d, d));
      add_op(OP_GEMM32, pb, 1, B * a.n, V); work_gemm(pb);
      if (a.kind == BASE_CLEAN) { add_op(OP_LOGZ, 0, 0, 0, 0, M->logits_clean, M->logz_clean); ops.back().bytes = (double)B * V * 4.0; }
      else if (general) {
        add_op(OP_KL, 0, 0, 0, 0, (void*)M->logits_clean, (void*)M->logz_clean);
        ops.back().bytes = (double)a.n * B * V * 4.0 * (1.0 + 1.0 / a.n);
      }
      return;
    }
    probs.push_back(prob8(gd.out_codes, gd.out_codes_is, M->Kd_o, gd.out_scale, gd.out_scale_is, 1, M->u_codes, M->Kd_o,
                          M->u_scale, V, M->b_U, lg, lg_is, Vp, 0, B, V, M->Kd_o, d));
    probs.back().b16 = M->nb16 ? 1 : 0;
    // With exact sums the unembedding itself reduces its rows to the parts of a log-sum-exp and of the KL
    // against the reference (one row of parts instead of one row of logits per candidate and sequence); the
    // reference passes also keep their logits and get their log-sum-exp from the same parts, so that a candidate
    // with the reference's logits scores exactly 0.  The FP8 matrix-core mode keeps the two-kernel path.
    const bool fused = M->cfg.mma == PAHQ_MMA_F16_EXACT;
    const bool ref_pass = a.kind == BASE_CLEAN || a.kind == PI_REF || a.kind == PI_REF_LAYER;
    if (fused && (ref_pass || general)) {
      GemmProb& q = probs.back();
      q.kl_part = M->kl_part; q.kl_npart = M->kl_npart;
      if (general) {
        if (!a.keep_logits) q.C = nullptr;
        q.kl_ref = has_pi ? M->ref_logits : M->logits_clean;
        q.kl_ref_logz = has_pi ? M->ref_logz : M->logz_clean;
      }
      add_op(OP_GEMM8, pb, 1, B * a.n, V, (void*)1); work_gemm(pb);
      const double part_bytes = (double)a.n * B * M->kl_npart * 16.0;
      ops.back().bytes += part_bytes;
      if (ref_pass) {
        const bool cl = a.kind == BASE_CLEAN, lay = a.kind == PI_REF_LAYER;      // lay: a.n reference runs side by side
        add_op(OP_KLRED, 0, 0, 0, 0, cl ? M->logz_clean : (lay ? M->ref_logz_all : M->ref_logz), nullptr);
        ops.back().bytes = part_bytes;
        add_op(OP_PREF, 0, 0, 0, 0, cl ? (void*)M->logits_clean : (lay ? (void*)M->ref_logits_all : (void*)M->ref_logits),
               cl ? (void*)M->psum_clean : (lay ? (void*)M->psum_ref_all : (void*)M->psum_ref));
        ops.back().u64 = (unsigned long long)(uintptr_t)(cl ? M->logz_clean : (lay ? M->ref_logz_all : M->ref_logz));
        ops.back().bytes = (double)a.n * B * V * 4.0;
      } else {
        add_op(OP_KLRED, 1, 0, 0, 0, has_pi ? M->ref_logz : M->logz_clean, has_pi ? M->psum_ref : M->psum_clean);
        ops.back().bytes = part_bytes;
      }
      return;
    }
    add_op(OP_GEMM8, pb, 1, B * a.n, V); work_gemm(pb);
    if (a.kind == BASE_CLEAN) add_op(OP_LOGZ, 0, 0, 0, 0, M->logits_clean, M->logz_clean);
    else if (a.kind == PI_REF) add_op(OP_LOGZ, 0, 0, 0, 0, M->ref_logits, M->ref_logz);
    else if (general) {
      add_op(OP_KL, 0, 0, 0, 0, has_pi ? (void*)M->ref_logits : (void*)M->logits_clean,
             has_pi ? (void*)M->ref_logz : (void*)M->logz_clean);
      ops.back().bytes = (double)a.n * B * V * 4.0 * (1.0 + 1.0 / a.n);   // candidate logits + the shared reference
    }
    if (ops.back().t == OP_LOGZ) ops.back().bytes = (double)B * V * 4.0;
  }
};

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

}  // namespace

int run_pass(pahq_model* M, const PassArgs& a, const RecvPlan* plan) {
  if (a.n < 1 || a.n > M->nmax) return PAHQ_EINVAL;
  Builder b(M, a, plan);
  const int L = M->L;
  Stream run;
  const bool corrupt_tokens = (a.kind == BASE_CORRUPT || a.kind == PI_CORRUPT);
  run.p = corrupt_tokens ? corrupt_prefix(M, a.p0) : clean_prefix(M, a.p0);
  run.is = 0;
  if (a.kind == PREFIX) {
    b.attention_block(a.p0 / 2, run);
  } else {
    for (int l = a.p0 / 2; l < L; l++) {
      if (a.p0 <= 2 * l) {
        if (a.kind == CAND && plan->split_first && 2 * l == a.p0) b.first_block_split(l, run);
        else if (a.kind == PI_REF_LAYER && 2 * l == a.p0) b.ref_layer_block(l, run);
        else b.attention_block(l, run);
      }
      if (M->g.mu && a.p0 <= 2 * l + 1) b.mlp_block(l, run);
    }
    b.final_block(run);
  }

  if (M->w32.on) {
    // a pass that failed half way may have left slots held: nothing of it may still be running when they are reused
    bool held = false;
    for (char c : M->w32.slots.busy) held = held || c;
    if (held) { HIPCHK(hipStreamSynchronize(M->stream)); M->w32.slots.release_all(); }
    // each acquisition also names the next one of this pass, whose transfers start while this layer computes
    int nxt = -1;
    for (int i = (int)b.ops.size() - 1; i >= 0; i--)
      if (b.ops[i].t == OP_W32ACQ) {
        if (nxt >= 0) { b.ops[i].i1 = b.ops[nxt].i0; b.ops[i].u64b = b.ops[nxt].u64; }
        nxt = i;
      }
  }
  for (GroupDesc& gd : b.groups) if (!gd.qbits) gd.qbits = M->qbits;      // groups of bfloat16 blocks have said 16
  for (AttnSrc& as : b.asrcs) { as.qbits = M->qbits; as.form = M->attn_form; }
  // ---- upload the descriptor tables
  Arena& A = M->arena;
  int slot = A.next;
  A.next = (A.next + 1) % Arena::SLOTS;
  HIPCHK(hipEventSynchronize(A.ev[slot]));
  size_t o_groups = 0;
  size_t o_terms = align_up(o_groups + b.groups.size() * sizeof(GroupDesc), 256);
  size_t o_probs = align_up(o_terms + b.terms.size() * sizeof(Term), 256);
  size_t o_cdesc = align_up(o_probs + b.probs.size() * sizeof(GemmProb), 256);
  size_t o_csrc = align_up(o_cdesc + b.cdescs.size() * sizeof(CombineDesc), 256);
  size_t o_odesc = align_up(o_csrc + b.csrcs.size() * sizeof(CombineSrc), 256);
  size_t o_haux = align_up(o_odesc + b.odescs.size() * sizeof(OprojDesc), 256);
  size_t total = align_up(o_haux + b.haux.size() * sizeof(HeadAux), 256);
  if (total > A.slot_bytes) return PAHQ_ENOMEM;
  char* h = A.host[slot];
  if (!b.groups.empty()) memcpy(h + o_groups, b.groups.data(), b.groups.size() * sizeof(GroupDesc));
  if (!b.terms.empty()) memcpy(h + o_terms, b.terms.data(), b.terms.size() * sizeof(Term));
  if (!b.probs.empty()) memcpy(h + o_probs, b.probs.data(), b.probs.size() * sizeof(GemmProb));
  if (!b.cdescs.empty()) memcpy(h + o_cdesc, b.cdescs.data(), b.cdescs.size() * sizeof(CombineDesc));
  if (!b.csrcs.empty()) memcpy(h + o_csrc, b.csrcs.data(), b.csrcs.size() * sizeof(CombineSrc));
  if (!b.odescs.empty()) memcpy(h + o_odesc, b.odescs.data(), b.odescs.size() * sizeof(OprojDesc));
  if (!b.haux.empty()) memcpy(h + o_haux, b.haux.data(), b.haux.size() * sizeof(HeadAux));
  HIPCHK(hipMemcpyAsync(A.dev[slot], h, total, hipMemcpyHostToDevice, M->stream));
  HIPCHK(hipEventRecord(A.ev[slot], M->stream));
  const GroupDesc* d_groups = (const GroupDesc*)(A.dev[slot] + o_groups);
  const Term* d_terms = (const Term*)(A.dev[slot] + o_terms);
  const GemmProb* d_probs = (const GemmProb*)(A.dev[slot] + o_probs);
  const CombineDesc* d_cdesc = (const CombineDesc*)(A.dev[slot] + o_cdesc);
  const CombineSrc* d_csrc = (const CombineSrc*)(A.dev[slot] + o_csrc);
  const OprojDesc* d_odesc = (const OprojDesc*)(A.dev[slot] + o_odesc);
  const HeadAux* d_haux = (const HeadAux*)(A.dev[slot] + o_haux);

  // ---- launch
  const int n = a.n, T = M->T, B = M->B, S = M->S, d = M->d;
  hipStream_t st = M->stream;
  static const int cls_of[] = {0, 2, 3, 4, 5, 6, 7, 8, 1, 9, 8, 7, 6, 8};   // OpType -> kernel class
  const bool prof_pass = M->prof_on && (M->prof_pass++ % M->prof_every) == 0;
  for (const Op& o : b.ops) {
    int pair = -1;
    if (o.t == OP_W32ACQ) {
      int rc = w32_acquire(M, o.i0, o.u64);
      if (rc == PAHQ_OK && o.i1 >= 0 && o.i1 != o.i0) rc = w32_prefetch(M, o.i1, o.u64b);
      if (rc != PAHQ_OK) return rc;
      continue;
    }
    if (o.t == OP_W32REL) { int rc = w32_release(M, o.i0, o.u64); if (rc != PAHQ_OK) return rc; continue; }
    if (prof_pass && ((M->prof_mask >> cls_of[o.t]) & 1u)) {
      if (M->prof_used * 2 + 2 > (int)M->prof_ev.size()) { int r = prof_harvest(M); if (r != PAHQ_OK) return r; }
      pair = M->prof_used++;
      int cls = cls_of[o.t];
      M->prof_cls[pair] = cls;
      M->prof[cls].launches += 1;
      M->prof[cls].flops += o.flops;
      M->prof[cls].bytes += o.bytes;
      HIPCHK(hipEventRecord(M->prof_ev[2 * pair], st));
    }
    switch (o.t) {
      case OP_BUILD: {
        // the patched receiver's group (if any) is built by the edge-batched patch kernel
        int pg = o.i2;
        if (pg < 0) {
          HIPCHK(launch_build_inputs(d_groups + o.i0, o.i1, d_terms, o.u64 ? 1 : n, T, B, S, d, M->Kd, M->cfg.norm, M->cfg.norm_eps, o.i3, st));
        } else {
          if (pg > o.i0)
            HIPCHK(launch_build_inputs(d_groups + o.i0, pg - o.i0, d_terms, n, T, B, S, d, M->Kd, M->cfg.norm, M->cfg.norm_eps, o.i3, st));
          if (o.i0 + o.i1 > pg + 1)
            HIPCHK(launch_build_inputs(d_groups + pg + 1, o.i0 + o.i1 - pg - 1, d_terms, n, T, B, S, d, M->Kd, M->cfg.norm, M->cfg.norm_eps, o.i3, st));
        }
        break;
      }
      case OP_PATCH:
        HIPCHK(launch_patch_build(d_groups + o.i0, (const float*)o.p0, M->delta, M->tile, M->send_dev + a.io_off + o.i1, o.i2, a.patch_mode,
                                  T, B, S, d, M->Kd, M->cfg.norm, M->cfg.norm_eps, st));
        break;
      case OP_GEMM8:
        for (int q = 0; q < o.i1; q++)
          if (!gemm8_prob_ok(b.probs[o.i0 + q]))      // the problem does not meet what the kernels assume
            return PAHQ_EINVAL;
        if (o.p0) HIPCHK(launch_gemm_fp8_kl(d_probs + o.i0, o.i1, o.i2, o.i3, b.probs[o.i0].b16, st));      // log-softmax / KL epilogue
        else {
          for (int q = 0; q < o.i1; q++) if (b.probs[o.i0 + q].kl_part || !b.probs[o.i0 + q].C) return PAHQ_EINVAL;
          HIPCHK(launch_gemm_fp8(d_probs + o.i0, o.i1, o.i2, o.i3, M->cfg.mma == PAHQ_MMA_F16_EXACT, b.probs[o.i0].b16, st));
        }
        break;
      case OP_KLRED:
        if (o.i0 == 0) HIPCHK(launch_kl_reduce(M->kl_part, M->kl_npart, n * B, B, nullptr, nullptr, (double*)o.p0, nullptr, nullptr, st));
        else HIPCHK(launch_kl_reduce(M->kl_part, M->kl_npart, n * B, B, (const double*)o.p0, (const double*)o.p1, nullptr,
                                     M->row_kl, M->kl_dev + a.io_off, st));
        break;
      case OP_PREF: {
        // n reference runs side by side (their logits, log-sum-exps and sums are contiguous copies)
        HIPCHK(launch_ref_probs((const float*)o.p0, (const double*)(uintptr_t)o.u64, (double*)o.p1, n * B, M->V, M->Vp, st));
        break;
      }
      case OP_GEMM32: HIPCHK(launch_gemm_f32(d_probs + o.i0, o.i1, o.i2, o.i3, st)); break;
      case OP_ATTN: {
        // o.i2 instances starting at o.i1 (0: all of the pass); the sources of such a range are already offset
        const long long zc_is = (long long)T * M->H * M->Kh, zs_is = (long long)T * M->H,
                        zf_is = (long long)T * M->dh * __builtin_popcountll(o.u64);
        HIPCHK(launch_attention(b.asrcs[o.i0], M->zcodes + o.i1 * zc_is, zc_is, M->zscale + o.i1 * zs_is, zs_is,
                                M->zf32 + o.i1 * zf_is, zf_is, o.u64, o.u64b, o.i2 ? o.i2 : n, B, S, M->H,
                                M->dh, M->Kh, M->cfg.pos == PAHQ_POS_ROPE, M->rope_tab, st));
        break;
      }
      case OP_COMBINE: HIPCHK(launch_combine(d_cdesc, o.i0, d_csrc, o.i1 ? 1 : n, M->tile, d, st)); break;
      case OP_OPROJ:
        HIPCHK(launch_oproj_fused(d_odesc, o.i0, d_haux, o.i1, o.i2, M->H, M->dh, M->cfg.mma == PAHQ_MMA_F16_EXACT, M->qbits == 16, st));
        break;
      case OP_HIDQ:
        HIPCHK(launch_hidden_quant(M->hid, o.i0 == 2 ? M->hid2 : nullptr, (long long)T * M->m, M->hcodes, (long long)T * M->Km_o,
                                   M->hscale, T, n, T, M->m, M->Km_o, o.i0, M->nb16 ? 16 : M->qbits, st));
        break;
      case OP_SWIGLU32: HIPCHK(launch_swiglu_f32(M->hid, M->hid2, (long long)n * T * M->m, st)); break;
      case OP_LD: {
        double* ld = o.i0 ? M->row_kl : (double*)o.p0;
        if (M->all_f32) HIPCHK(launch_logit_pair_f32(M->xf32, (long long)B * d, d, M->W_U, M->V, M->b_U, M->ans_dev, M->dis_dev, n, B, ld, st));
        else HIPCHK(launch_logit_pair(M->lastcodes, (long long)B * M->Kd_o, M->lastscale, B, M->Kd_o, M->Kd_o, M->u_codes, M->Kd_o, M->u_scale,
                                      M->b_U, M->ans_dev, M->dis_dev, n, B, ld, M->nb16 ? 1 : 0, st));
        if (o.i0) HIPCHK(launch_metric_mean(M->row_kl, (const double*)o.p0, M->kl_dev + a.io_off, n, B, st));
        break;
      }
      case OP_LOGZ: HIPCHK(launch_logz((const float*)o.p0, B, M->V, M->Vp, (double*)o.p1, st)); break;
      case OP_W32ACQ: case OP_W32REL: break;             // handled above
      case OP_KL:
        HIPCHK(launch_kl(M->logits, (long long)B * M->Vp, (const float*)o.p0, (const double*)o.p1, M->row_kl, M->kl_dev + a.io_off,
                         n, B, M->V, M->Vp, st));
        break;
    }
    if (pair >= 0) HIPCHK(hipEventRecord(M->prof_ev[2 * pair + 1], st));
  }
  for (const auto& t : b.new_tags) M->deadsum_tag[t.first] = t.second;      // every launch of the pass is queued
  M->counters[2]++;
  return PAHQ_OK;
}


int prof_harvest(pahq_model* M) {
  HIPCHK(hipStreamSynchronize(M->stream));
  for (int i = 0; i < M->prof_used; i++) {
    float ms = 0.f;
    HIPCHK(hipEventElapsedTime(&ms, M->prof_ev[2 * i], M->prof_ev[2 * i + 1]));
    M->prof[M->prof_cls[i]].ms += ms;
  }
  M->prof_used = 0;
  return PAHQ_OK;
}

}  // namespace pahq
