// Host-side control logic of the sweep, free of any GPU type so that it also builds as plain C++
// (the CPU check under tests/host compiles this header with the address and undefined-behaviour
// sanitizers): the order of receivers, the liveness rule, the plan of how each recomputed receiver
// forms its input, and the accept scan that turns device batches of speculative candidates into
// the decisions of the one-by-one procedure.
//
// Paper, Appendix "Preliminaries" (pruning rule: an edge goes iff removing it raises the metric
// by less than tau, nodes visited from the output backwards) and Appendix "Integration with
// ACDC" (the loop over receivers and their incoming edges).
#pragma once
#include <stdint.h>
#include <string.h>
#include <algorithm>
#include <vector>
#include "graph.h"

namespace pahq {

// How one recomputed receiver forms its input from the residual streams.
struct RecvSpec {
  int form;                    // 0 dense (running stream only), 1 removed form, 2 kept form, -1 not computed (dead node)
  std::vector<int> senders;    // removed senders (form 1) or kept senders (form 2), ascending
};

struct RecvPlan {
  int p0 = -1;
  std::vector<RecvSpec> spec;  // indexed by receiver id (only receivers at positions >= p0 are filled)
  std::vector<int> slot_of;    // per sender: slot index or -1
  std::vector<char> shared;    // per sender: its slot is the same for every instance (see split_first)
  std::vector<char> live;      // per sender: 0 = recomputed sender whose output no kept path carries to the output
  int n_slots = 0;             // per-instance slots
  int n_shared = 0;            // instance-independent slots
  int n_dead = 0;              // recomputed senders with live == 0
  bool split_first = false;    // candidates recompute only the investigated head in their first layer
};

// Receivers in the order the sweep visits them: all of them, or the given subset, descending, each once.
// Returns false if an id is out of range.
inline bool sweep_order(const GraphDims& g, const int32_t* receivers, int n_receivers, std::vector<int>& order) {
  order.clear();
  if (n_receivers == 0) { for (int r = g.Nr - 1; r >= 0; r--) order.push_back(r); return true; }
  for (int i = 0; i < n_receivers; i++) {
    if (receivers[i] < 0 || receivers[i] >= g.Nr) return false;
    order.push_back(receivers[i]);
  }
  std::sort(order.begin(), order.end(), [](int x, int y) { return x > y; });
  order.erase(std::unique(order.begin(), order.end()), order.end());
  return true;
}

// A receiver whose node has no outgoing edge left cannot influence the output: all its incoming
// edges go without being evaluated.  removed holds one byte per edge, the row of receiver r at edge_off[r].
inline bool node_is_live(const GraphDims& g, const uint8_t* removed, const int64_t* edge_off, int v) {
  const int s = g.node_of_receiver(v);
  if (s < 0) return true;
  for (int r = 0; r < g.Nr; r++)
    if (s < g.n_upstream(r) && !removed[edge_off[r] + s]) return true;
  return false;
}

// Plan of a pass that recomputes everything from position p0 on, for candidates into receiver v
// (v < 0: no candidates).
//
// Dead nodes.  A recomputed sender is live if one of its kept edges leads to the output node or to a
// receiver of a live node (v's own node always counts as live).  Every edge out of a dead sender is
// removed, so every receiver takes the corrupted run's output from it whatever it computes: it is not
// computed at all, the running stream takes its cached corrupted output in its place (its difference
// D_s to the corrupted run is then zero and drops out of every removed-form sum), and its receivers
// get form -1.  The outputs are those of the full computation; a sparse graph costs only its live part.
//
// Per live receiver the cheaper of the two forms of its input; every recomputed sender that some
// receiver needs separately gets a slot for its (output - corrupted output).
// split: the receiver's own layer is shared between candidates except for the investigated head, so
// the other heads of that layer need one slot for all instances instead of one per instance.
inline void plan_receivers(const GraphDims& g, const uint8_t* removed, const int64_t* edge_off, bool pahq_precision,
                           int p0, int v, RecvPlan& out, bool skip_dead = true) {
  out.p0 = p0;
  out.spec.assign(g.Nr, RecvSpec());
  out.slot_of.assign(g.Ns, -1);
  out.shared.assign(g.Ns, 0);
  out.live.assign(g.Ns, 1);
  out.n_slots = 0;
  out.n_shared = 0;
  out.n_dead = 0;
  int vk = -1, vl, vh, vc;
  if (v >= 0) g.receiver_info(v, vk, vl, vh, vc);
  out.split_first = (vk == 0 && pahq_precision);
  const int v_node = v >= 0 ? g.node_of_receiver(v) : -1;
  const int nstat = g.n_static(p0);
  // liveness, from the last sender backwards: the receivers a sender feeds belong to later senders (or are the output)
  if (skip_dead)
    for (int s = g.Ns - 1; s >= nstat; s--) {
      bool lv = (s == v_node);
      const int pa = g.pos_after_sender(s);
      for (int w = g.Nr - 1; w >= 0 && !lv; w--) {
        if (g.pos_of_receiver(w) < pa) break;                 // receiver ids follow the stream
        if (removed[edge_off[w] + s]) continue;
        const int nw = g.node_of_receiver(w);
        lv = nw < 0 || out.live[nw];
      }
      out.live[s] = lv ? 1 : 0;
      out.n_dead += lv ? 0 : 1;
    }
  for (int w = 0; w < g.Nr; w++) {
    if (g.pos_of_receiver(w) < p0) continue;
    RecvSpec& sp = out.spec[w];
    const int nw = g.node_of_receiver(w);
    if (nw >= 0 && !out.live[nw]) { sp.form = -1; continue; }
    const int n_up = g.n_upstream(w);
    const uint8_t* row = removed + edge_off[w];
    int n_rem = 0, n_kept = 0;       // removed edges from live senders; kept edges (dead senders have none)
    for (int s = 0; s < n_up; s++) { n_rem += row[s] && out.live[s]; n_kept += !row[s]; }
    if (n_rem == 0) { sp.form = 0; continue; }
    if (n_rem <= n_kept) {
      sp.form = 1;
      for (int s = 0; s < n_up; s++) if (row[s] && out.live[s]) sp.senders.push_back(s);
    } else {
      sp.form = 2;
      for (int s = 0; s < n_up; s++) if (!row[s]) sp.senders.push_back(s);
    }
    for (int s : sp.senders)
      if (s >= nstat && out.slot_of[s] < 0) {
        bool sh = out.split_first && s != v_node && g.pos_after_sender(s) == p0 + 1;   // another head of v's layer
        out.shared[s] = sh ? 1 : 0;
        out.slot_of[s] = sh ? out.n_shared++ : out.n_slots++;
      }
  }
}

// The accept scan for one receiver with n_up incoming edges, candidates in descending sender order.
//
// The procedure it must reproduce is sequential: evaluate the next edge with all earlier decisions
// applied, remove it iff kl_new - kl_cur < tau, and then kl_cur = kl_new.  A device batch evaluates nb
// candidates at once under one of two assumptions about the candidates before them in the batch:
//   mode 2 (cumulative)  candidate i is scored with candidates 0..i-1 of the batch removed as well:
//                        right as long as all of those were removed, i.e. up to and including the
//                        first kept edge;
//   mode 1 (independent) candidate i is scored with none of them removed: right up to and including
//                        the first removed edge.
// The scan accepts that prefix, has the receiver's input advanced by the removed edges, and issues the
// rest again.  The mode follows the receiver's decision mix so far, the batch size doubles after a
// fully used batch and falls back to twice the used prefix otherwise.
//
//   eval(senders, nb, mode, kl)   scores senders[0..nb) into kl[0..nb); returns 0 or an error code
//   advance(first, count)         applies the removal of candidates first..first+count-1 of the LAST batch
//                                 to the receiver's input; returns 0 or an error code
//   record(sender, kl_new, kl_cur, removed)   one call per decision, in order
// row[s] is set to 1 for every removed sender; kl_cur is updated in place.  max_batch >= 1.
template <class Eval, class Advance, class Record>
int scan_receiver(int n_up, int max_batch, double tau, double& kl_cur, uint8_t* row, int* senders, double* kl,
                  Eval&& eval, Advance&& advance, Record&& record) {
  int pos = 0;                      // candidates are senders n_up-1-pos, descending
  int bs = max_batch;
  int recent_rm = 1, recent_n = 1;  // decision history of this receiver (start optimistic: most edges go)
  while (pos < n_up) {
    const int nb = std::min(std::min(bs, max_batch), n_up - pos);
    const int mode = (2 * recent_rm >= recent_n) ? 2 : 1;
    for (int i = 0; i < nb; i++) senders[i] = n_up - 1 - (pos + i);
    int rc = eval(senders, nb, mode, kl);
    if (rc != 0) return rc;
    int used = 0, n_rm = 0;
    for (int i = 0; i < nb; i++) {
      const double kn = kl[i];
      const bool rm = (kn - kl_cur) < tau;
      const int u = senders[i];
      record(u, kn, kl_cur, rm);
      used++; recent_n++;
      if (rm) { row[u] = 1; kl_cur = kn; n_rm++; recent_rm++; }
      if ((mode == 2 && !rm) || (mode == 1 && rm)) break;
    }
    if (n_rm > 0) {
      // removed edges of this batch: in cumulative mode the first n_rm candidates, in independent mode the last used
      rc = (mode == 2) ? advance(0, n_rm) : advance(used - 1, 1);
      if (rc != 0) return rc;
    }
    pos += used;
    bs = (used == nb) ? std::min(max_batch, std::max(2 * bs, 2)) : std::max(1, std::min(max_batch, 2 * used));
  }
  return 0;
}

// Bookkeeping of the device slots that hold fp32 head weights while the masters stay in host memory
// (paper, Sec. "Selective Precision Allocation Strategy", Hierarchical Weight Scheduling: S_t, the nodes
// in fp32 at step t, must be on the device at t, and Prefetch(t) moves S_{t+1} while step t computes;
// Sec. "Algorithm Implementation in Practice", Scheduler Implementation).
//
// Head id = layer * H + head lives in slot id % n_slots (n_slots = 2 H: all heads of two neighbouring
// layers fit at once, so the heads of the layer the sweep visits next never displace the current one's).
// The caller does the transfers and the event waits; this keeps who is where:
//   acquire(id)   a pass is about to use head id; returns true if a transfer has to be issued now
//                 (a demand transfer: the pass waits for all of it); the slot is busy until release
//   prefetch(id)  the head is expected next; returns true if a transfer should be issued now (false:
//                 already there or on its way, or the slot still serves a running pass)
//   release(id)   the pass has enqueued its last use
// A slot's contents change only through acquire / prefetch returning true.
struct HeadSlots {
  int n_slots = 0;
  std::vector<int> holds;          // per slot: head id it holds or is being filled with, -1 = nothing yet
  std::vector<char> busy;          // per slot: acquired and not yet released
  long long n_acquire = 0, n_demand = 0, n_prefetch = 0;
  void init(int slots) { n_slots = slots; holds.assign(slots, -1); busy.assign(slots, 0); n_acquire = n_demand = n_prefetch = 0; }
  int slot_of(int id) const { return id % n_slots; }
  bool resident(int id) const { return holds[slot_of(id)] == id; }
  // returns 1 = issue a transfer, 0 = nothing to do, -1 = the slot is in use by another head of the same pass
  int acquire(int id) {
    const int s = slot_of(id);
    n_acquire++;
    if (holds[s] == id) { busy[s] = 1; return 0; }
    if (busy[s]) return -1;
    holds[s] = id; busy[s] = 1; n_demand++;
    return 1;
  }
  bool prefetch(int id) {
    const int s = slot_of(id);
    if (holds[s] == id || busy[s]) return false;
    holds[s] = id; n_prefetch++;
    return true;
  }
  void release(int id) { const int s = slot_of(id); if (holds[s] == id) busy[s] = 0; }
  void release_all() { std::fill(busy.begin(), busy.end(), 0); }
};

// The head (or heads) a sweep in descending receiver order needs after head (l, h): the next lower head of the
// layer, and below head 0 every head of the layer underneath (the reference runs of a layer's heads are made
// together).  Returns the layer (-1: none) and sets mask to the heads.
inline int next_heads_in_sweep_order(int H, int l, int h, unsigned long long& mask) {
  if (h > 0) { mask = 1ull << (h - 1); return l; }
  mask = H >= 64 ? ~0ull : ((1ull << H) - 1ull);
  return l - 1;
}

}  // namespace pahq
