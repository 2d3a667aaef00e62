// CPU check of the sweep's host logic (csrc/controller.h, csrc/graph.h), built with the address and
// undefined-behaviour sanitizers by tests/test_host_controller.py.  No GPU code is involved: the device
// batches are played by a synthetic metric that is a fixed function of the removed set, so the decisions
// the accept scan reaches through speculative batches can be compared, one by one, with the sequential
// procedure of the paper's Appendix "Preliminaries" (remove an edge iff it raises the metric by less
// than tau, edges in descending order, each judged with all earlier decisions applied).
#include <stdio.h>
#include <stdlib.h>
#include <stdint.h>
#include <vector>
#include <set>
#include "controller.h"

using namespace pahq;

static int failures = 0;
static long plans_with_dead = 0, dead_total = 0;
#define CHECK(cond, ...) do { if (!(cond)) { failures++; printf("FAIL %s:%d: ", __FILE__, __LINE__); printf(__VA_ARGS__); printf("\n"); if (failures > 20) exit(1); } } while (0)

static uint64_t mix(uint64_t x) { x += 0x9E3779B97F4A7C15ull; x = (x ^ (x >> 30)) * 0xBF58476D1CE4E5B9ull; x = (x ^ (x >> 27)) * 0x94D049BB133111EBull; return x ^ (x >> 31); }
static double unit(uint64_t x) { return (double)(mix(x) >> 11) * (1.0 / 9007199254740992.0); }

// A metric that depends on the whole removed set (not a sum over edges): every edge has a weight, most of
// them tiny, and a set-dependent term couples them, so that cumulative and independent candidates differ.
struct Metric {
  uint64_t seed; int n;
  double weight(int s) const { double u = unit(seed * 1315423911ull + s); return u < 0.6 ? 1e-6 * u : 1e-3 * u; }
  double operator()(const std::vector<uint8_t>& R) const {
    double f = 0.01; uint64_t h = seed;
    for (int s = 0; s < n; s++) if (R[s]) { f += weight(s); h = mix(h ^ (uint64_t)(s + 1)); }
    return f + 2e-4 * unit(h);
  }
};

struct Decision { int u; double kn, kc; bool rm; };
static bool same(const Decision& a, const Decision& b) { return a.u == b.u && a.kn == b.kn && a.kc == b.kc && a.rm == b.rm; }

static void sequential(const Metric& F, double tau, std::vector<uint8_t>& R, std::vector<Decision>& out) {
  double cur = F(R);
  for (int u = F.n - 1; u >= 0; u--) {
    R[u] = 1; double kn = F(R);
    bool rm = (kn - cur) < tau;
    out.push_back({u, kn, cur, rm});
    if (rm) cur = kn; else R[u] = 0;
  }
}

static void check_scan(uint64_t seed, int n_up, int max_batch, double tau, int fail_at) {
  Metric F{seed, n_up};
  std::vector<uint8_t> Rseq(n_up, 0), row(n_up, 0), Rdev(n_up, 0);
  std::vector<Decision> want, got;
  sequential(F, tau, Rseq, want);
  std::vector<int> senders(std::max(max_batch, 1));
  std::vector<double> kl(std::max(max_batch, 1));
  std::vector<int> last; int calls = 0, max_nb = 0;
  double kl_cur = F(Rdev);
  int rc = scan_receiver(
      n_up, max_batch, tau, kl_cur, row.data(), senders.data(), kl.data(),
      [&](const int* s, int nb, int mode, double* out) -> int {
        if (calls++ == fail_at) return -4;
        CHECK(nb >= 1 && nb <= max_batch, "batch of %d with a limit of %d", nb, max_batch);
        CHECK(Rdev == row, "the evaluator's input lags behind the decisions (seed %llu)", (unsigned long long)seed);
        max_nb = std::max(max_nb, nb);
        last.assign(s, s + nb);
        std::vector<uint8_t> R = Rdev;
        for (int i = 0; i < nb; i++) {
          CHECK(s[i] >= 0 && s[i] < n_up && !Rdev[s[i]], "candidate %d out of range or already removed", s[i]);
          if (mode == 2) { R[s[i]] = 1; out[i] = F(R); }
          else { std::vector<uint8_t> Q = Rdev; Q[s[i]] = 1; out[i] = F(Q); }
        }
        return 0;
      },
      [&](int first, int count) -> int {
        CHECK(first >= 0 && count >= 1 && first + count <= (int)last.size(), "advance(%d, %d) outside the last batch of %zu", first, count, last.size());
        for (int i = first; i < first + count && i < (int)last.size(); i++) Rdev[last[i]] = 1;
        return 0;
      },
      [&](int u, double kn, double kc, bool rm) { got.push_back({u, kn, kc, rm}); });
  if (fail_at >= 0 && fail_at < calls) {
    CHECK(rc == -4, "an evaluator error must come back (got %d)", rc);
    CHECK(got.size() <= want.size(), "more decisions than edges");
    for (size_t i = 0; i < got.size(); i++) CHECK(same(got[i], want[i]), "decision %zu before the error differs", i);
    return;
  }
  CHECK(rc == 0, "scan returned %d", rc);
  CHECK(got.size() == want.size(), "seed %llu n_up %d batch %d: %zu decisions, want %zu", (unsigned long long)seed, n_up, max_batch, got.size(), want.size());
  for (size_t i = 0; i < got.size() && i < want.size(); i++)
    if (!same(got[i], want[i])) { CHECK(false, "seed %llu n_up %d batch %d tau %g: decision %zu differs (sender %d/%d removed %d/%d)", (unsigned long long)seed, n_up, max_batch, tau, i, got[i].u, want[i].u, got[i].rm, want[i].rm); break; }
  CHECK(row == Rseq, "removed row differs from the sequential procedure's");
  CHECK(Rdev == row, "the evaluator's input does not hold the final decisions");
  CHECK(kl_cur == F(Rseq), "kl_cur is not the metric of the final state");
  if (n_up > 0) CHECK(calls <= n_up, "%d device batches for %d edges", calls, n_up);
}

static void check_graph_and_plan(uint64_t seed, int L, int H, bool mlp, bool split) {
  GraphDims g(L, H, mlp, split);
  CHECK(g.Nr == L * ((split ? 3 : 1) * H + (mlp ? 1 : 0)) + 1, "receiver count");
  // ids: receivers enumerate (layer, head, channel) / MLP inputs / the output once each, in stream order
  std::set<int> seen; int prev_pos = -1;
  for (int r = 0; r < g.Nr; r++) {
    int k, l, h, c; g.receiver_info(r, k, l, h, c);
    int id = k == 0 ? g.headin(l, h, split ? c : 2) : (k == 1 ? g.mlpin(l) : g.out());
    CHECK(k != 0 || (split ? (c >= 0 && c < 3) : c == -1), "channel of receiver %d", r);
    CHECK(id == r, "receiver %d does not map back to itself", r);
    CHECK(g.pos_of_receiver(r) >= prev_pos, "receiver ids do not follow the stream"); prev_pos = g.pos_of_receiver(r);
    int n = 0; for (int s = 0; s < g.Ns; s++) n += g.pos_after_sender(s) <= g.pos_of_receiver(r);
    CHECK(n == g.n_upstream(r), "receiver %d: %d senders upstream by position, n_upstream says %d", r, n, g.n_upstream(r));
    seen.insert(id);
  }
  CHECK((int)seen.size() == g.Nr, "receiver ids not unique");
  std::vector<int64_t> off(g.Nr + 1, 0);
  for (int r = 0; r < g.Nr; r++) off[r + 1] = off[r] + g.n_upstream(r);
  // random removed sets restricted to receivers at or after a random position; plans must describe them exactly
  for (int rep = 0; rep < 8; rep++) {
    std::vector<uint8_t> removed(off[g.Nr], 0);
    const int v = (int)(mix(seed + rep) % g.Nr), p0 = g.pos_of_receiver(v);
    const double dens = unit(seed * 7 + rep);
    for (int r = 0; r < g.Nr; r++) if (g.pos_of_receiver(r) >= p0)
      for (int s = 0; s < g.n_upstream(r); s++) {
        const bool sender_off = unit(seed * 131 + rep * 7919ull + s) < 0.4;       // all edges out of some senders go
        removed[off[r] + s] = sender_off || unit(seed * 31 + rep * 1000003ull + off[r] + s) < dens;
      }
    for (int variant = 0; variant < 4; variant++) {
      const int pahq = variant & 1; const bool skip = (variant & 2) != 0;
      RecvPlan plan; plan_receivers(g, removed.data(), off.data(), pahq, p0, v, plan, skip);
      const int nstat = g.n_static(p0);
      int vk, vl, vh, vc; g.receiver_info(v, vk, vl, vh, vc);
      // liveness by its definition, as a fixed point over all (sender, receiver) pairs in no particular order:
      // a recomputed sender is live if it is the candidates' own node or a kept edge leads to the output or to a live node
      std::vector<char> live(g.Ns, 1);
      if (skip) {
        for (int s = nstat; s < g.Ns; s++) live[s] = (s == g.node_of_receiver(v));
        for (bool changed = true; changed;) {
          changed = false;
          for (int s = nstat; s < g.Ns; s++) for (int w = 0; w < g.Nr && !live[s]; w++) {
            if (g.pos_after_sender(s) > g.pos_of_receiver(w) || removed[off[w] + s]) continue;
            const int nw = g.node_of_receiver(w);
            if (nw < 0 || live[nw]) { live[s] = 1; changed = true; }
          }
        }
      }
      int n_dead = 0;
      for (int s = 0; s < g.Ns; s++) { CHECK(plan.live[s] == live[s], "liveness of sender %d: plan %d, definition %d", s, (int)plan.live[s], (int)live[s]); n_dead += !live[s]; }
      CHECK(plan.n_dead == n_dead, "n_dead %d, counted %d", plan.n_dead, n_dead);
      plans_with_dead += n_dead > 0; dead_total += n_dead;
      std::vector<char> needed(g.Ns, 0);
      for (int r = 0; r < g.Nr; r++) {
        if (g.pos_of_receiver(r) < p0) continue;
        const RecvSpec& sp = plan.spec[r];
        const int nr = g.node_of_receiver(r);
        if (nr >= 0 && !live[nr]) { CHECK(sp.form == -1 && sp.senders.empty(), "receiver %d of a dead node has form %d", r, sp.form); continue; }
        CHECK(sp.form >= 0 && sp.form <= 2, "receiver %d: form %d", r, sp.form);
        // the edges the plan describes: form 2 lists the kept ones; forms 0 and 1 list the removed ones from live
        // senders, and every edge from a dead sender is removed without being listed
        std::vector<uint8_t> row(g.n_upstream(r), sp.form == 2 ? 1 : 0);
        if (sp.form != 2) for (int s = 0; s < g.n_upstream(r); s++) if (!live[s]) row[s] = 1;
        for (int s : sp.senders) {
          CHECK(s >= 0 && s < g.n_upstream(r), "sender %d not upstream of %d", s, r);
          if (s < 0 || s >= g.n_upstream(r)) continue;
          CHECK(live[s], "dead sender %d listed for receiver %d", s, r);
          row[s] = sp.form == 2 ? 0 : 1;
          if (s >= nstat) needed[s] = 1;
        }
        if (sp.form == 0) CHECK(sp.senders.empty(), "dense form with terms");
        for (int s = 0; s < g.n_upstream(r); s++) CHECK(row[s] == removed[off[r] + s], "plan of receiver %d misdescribes edge from %d", r, s);
        int n_rem = 0, n_kept = 0; for (int s = 0; s < g.n_upstream(r); s++) { n_rem += removed[off[r] + s] && live[s]; n_kept += !removed[off[r] + s]; }
        CHECK((int)sp.senders.size() == std::min(n_rem, n_kept), "receiver %d does not take the cheaper form", r);
      }
      std::set<int> own, shared;
      for (int s = 0; s < g.Ns; s++) {
        CHECK((plan.slot_of[s] >= 0) == (bool)needed[s], "sender %d: slot %d, needed %d", s, plan.slot_of[s], (int)needed[s]);
        if (plan.slot_of[s] < 0) continue;
        if (plan.shared[s]) {
          CHECK(pahq && vk == 0 && s != g.node_of_receiver(v) && s >= g.head(vl, 0) && s < g.head(vl, 0) + H, "sender %d shared without being another head of the receiver's layer", s);
          shared.insert(plan.slot_of[s]);
        } else {
          CHECK(!(pahq && vk == 0 && s != g.node_of_receiver(v) && s >= g.head(vl, 0) && s < g.head(vl, 0) + H), "another head of the receiver's layer has a per-candidate slot");
          own.insert(plan.slot_of[s]);
        }
      }
      CHECK((int)own.size() == plan.n_slots && (int)shared.size() == plan.n_shared, "slot numbers not a bijection");
      if (!own.empty()) CHECK(*own.rbegin() == plan.n_slots - 1, "slot numbers not dense");
    }
    // liveness: a node is live iff one of its outgoing edges is kept
    for (int r = 0; r < g.Nr; r++) {
      const int s = g.node_of_receiver(r);
      bool live = s < 0;
      for (int w = 0; w < g.Nr && !live; w++) if (g.pos_after_sender(s) <= g.pos_of_receiver(w) && !removed[off[w] + s]) live = true;
      CHECK(live == node_is_live(g, removed.data(), off.data(), r), "liveness of receiver %d", r);
    }
  }
  // order of the sweep
  std::vector<int> order;
  CHECK(sweep_order(g, nullptr, 0, order) && (int)order.size() == g.Nr && order.front() == g.Nr - 1 && order.back() == 0, "full order");
  int32_t some[5] = {0, g.Nr - 1, 0, g.Nr / 2, g.Nr - 1};
  CHECK(sweep_order(g, some, 5, order), "subset order");
  for (size_t i = 1; i < order.size(); i++) CHECK(order[i] < order[i - 1], "subset order not strictly descending");
  int32_t bad[2] = {0, g.Nr};
  CHECK(!sweep_order(g, bad, 2, order), "an id out of range must be refused");
  int32_t neg[1] = {-1};
  CHECK(!sweep_order(g, neg, 1, order), "a negative id must be refused");
}

// Slots of host-resident fp32 head weights: a model of the device (what each slot really contains, which slots a
// running pass reads) follows the bookkeeping's answers.  A pass must always find its heads in their slots, no
// transfer may land in a slot a running pass reads, and with the sweep-order prediction only the very first head
// is fetched on demand.
static void check_head_slots(int L, int H, uint64_t seed) {
  HeadSlots hs; hs.init(2 * H);
  std::vector<int> content(2 * H, -1);      // the model: head id whose weights the slot contains
  std::vector<char> in_use(2 * H, 0);
  long demand = 0;
  auto transfer = [&](int id) { int s = hs.slot_of(id); CHECK(!in_use[s], "transfer into a slot in use (head %d)", id); content[s] = id; };
  auto use = [&](int l, unsigned long long mask) {
    for (int h = 0; h < H; h++) if ((mask >> h) & 1ull) {
      int id = l * H + h, r = hs.acquire(id);
      CHECK(r >= 0, "two heads of one pass in one slot");
      if (r == 1) { transfer(id); demand++; }
      in_use[hs.slot_of(id)] = 1;
      CHECK(content[hs.slot_of(id)] == id, "head %d not in its slot", id);
    }
  };
  auto done = [&](int l, unsigned long long mask) {
    for (int h = 0; h < H; h++) if ((mask >> h) & 1ull) { hs.release(l * H + h); in_use[hs.slot_of(l * H + h)] = 0; }
  };
  const unsigned long long all = H >= 64 ? ~0ull : ((1ull << H) - 1ull);
  // the sweep: per layer from the top the reference runs of all heads together, then head by head downwards,
  // each predicting its successor
  for (int l = L - 1; l >= 0; l--) {
    for (int h = H - 1; h >= 0; h--) {
      if (h == H - 1) { use(l, all); done(l, all); }
      for (int pass = 0; pass < 3; pass++) {
        use(l, 1ull << h);
        unsigned long long nm; int nl = next_heads_in_sweep_order(H, l, h, nm);
        if (nl >= 0) for (int q = 0; q < H; q++) if ((nm >> q) & 1ull) if (hs.prefetch(nl * H + q)) transfer(nl * H + q);
        done(l, 1ull << h);
      }
    }
  }
  CHECK(demand == H, "sweep order: %ld demand transfers, expected the %d of the first layer's joint pass", demand, H);
  // a forward pass over every layer with a random set of fp32 heads, the next layer's set predicted at each layer
  std::vector<unsigned long long> masks(L);
  for (int l = 0; l < L; l++) masks[l] = mix(seed * 131 + l) & all;
  for (int l = 0; l < L; l++) {
    use(l, masks[l]);
    if (l + 1 < L) for (int q = 0; q < H; q++) if ((masks[l + 1] >> q) & 1ull) if (hs.prefetch((l + 1) * H + q)) transfer((l + 1) * H + q);
    done(l, masks[l]);
  }
  // random order, random predictions (some wrong, some into busy slots)
  for (int it = 0; it < 2000; it++) {
    int l = (int)(mix(seed + it) % L), h = (int)(mix(seed * 7 + it) % H);
    use(l, 1ull << h);
    int pl = (int)(mix(seed * 13 + it) % L), ph = (int)(mix(seed * 17 + it) % H);
    if (hs.prefetch(pl * H + ph)) transfer(pl * H + ph);
    done(l, 1ull << h);
  }
  CHECK(hs.n_acquire > 0 && hs.n_demand <= hs.n_acquire, "counters");
  // a failed pass leaves slots busy: release_all frees them
  use(0, 1ull); hs.release_all(); std::fill(in_use.begin(), in_use.end(), 0);
  CHECK(hs.prefetch(2 * H) == (2 * H < L * H) || L * H <= 2 * H, "a slot freed by release_all takes a transfer again");
}

int main() {
  int cases = 0;
  { const int hs_shapes[][2] = {{1, 1}, {2, 1}, {3, 2}, {4, 4}, {12, 12}, {5, 64}};
    for (auto& sh : hs_shapes) for (uint64_t seed = 1; seed <= 3; seed++) { check_head_slots(sh[0], sh[1], seed); cases++; } }
  const double taus[] = {-1.0, 0.0, 5e-7, 2e-5, 1.5e-4, 6e-4, 1.0};
  const int sizes[] = {0, 1, 2, 3, 7, 16, 33, 100, 157, 301};
  const int batches[] = {1, 2, 3, 8, 64, 128, 512};
  for (int n_up : sizes) for (int mb : batches) for (double tau : taus)
    for (uint64_t seed = 1; seed <= 6; seed++) { check_scan(seed * 1000 + n_up, n_up, mb, tau, -1); cases++; }
  for (int fail_at = 0; fail_at < 6; fail_at++) for (uint64_t seed = 1; seed <= 4; seed++) { check_scan(seed, 100, 8, 2e-5, fail_at); cases++; }
  const int shapes[][3] = {{1, 1, 0}, {1, 1, 1}, {2, 2, 0}, {2, 3, 1}, {3, 4, 1}, {4, 2, 1}, {12, 12, 1}};
  for (auto& sh : shapes) for (int split = 0; split < 2; split++) for (uint64_t seed = 1; seed <= 3; seed++) { check_graph_and_plan(seed * 77 + sh[0], sh[0], sh[1], sh[2], split); cases++; }
  CHECK(plans_with_dead > 50, "the removed sets of this check hardly ever leave a node dead (%ld plans)", plans_with_dead);
  printf("%d cases (%ld plans with dead nodes, %ld dead nodes), %d failures\n", cases, plans_with_dead, dead_total, failures);
  return failures ? 1 : 0;
}
