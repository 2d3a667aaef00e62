"""ACDC edge scoring and the pruning sweep on the oracle model (test infrastructure).

Paper, Appendix "Preliminaries": an edge is pruned when removing it (its
sender's activation replaced by the corrupted run's) changes the loss by less
than a threshold tau; the loss here is the KL divergence to the clean model's
output distribution (Appendix "Metrics").  Appendix "Integration with ACDC":
each edge evaluation consists of three inferences -- clean, corrupted,
patched.  Sec. "Selective Precision Allocation Strategy": during one edge
evaluation only the investigated head is kept in fp32.

Readings (the paper defers the procedure to ACDC and is silent on them):
* the fp32 head is the head the candidate edge feeds (receiver side); edges
  into an MLP or into the unembedding have no fp32 head.  The policy as Eq. P_t
  prints it (fp32 for the edge's SOURCE) is available next to it
  (pair_sender_policy, sweep_sender_policy) for comparison;
* the reference distribution is computed under the same precision set as the
  patched run, so that patching with clean activations gives KL = 0;
* one pass over receivers in descending id (output first), senders in
  descending id; an edge is removed when kl_new - kl_cur < tau (signed,
  strict), and kl_cur then becomes kl_new;
* a receiver whose node has no kept outgoing edge is skipped and all its
  in-edges are removed (their effect is exactly zero).

Two evaluators are provided: `kl_brute` (three full forwards from the
embedding, the definition) and `kl_fast` (layers before the receiver's layer
come from caches computed once; they do not depend on the precision set nor
on the removed set).  Tests assert they agree.

parity unpinned: the KL values themselves on synthetic models are defined
only by this code; what is pinned are the properties listed in the tests
(clean patch = 0, full ablation = clean-vs-corrupt KL, dead-node edges = 0,
output-receiver closed form, brute force = fast path, plain-forward equality).
"""
from __future__ import annotations
import numpy as np

from .model import Model, ALL, NONE, log_softmax, kl_to_reference

MODE_ALL_FP32, MODE_ALL_FP8, MODE_PAHQ = 0, 1, 2
METRIC_KL, METRIC_LOGIT_DIFF = 0, 1


def logit_diff_drop(ref_logits, logits, answer, distractor):
    """Batch mean of how far the logit difference (answer minus distractor) of `logits` has dropped below
    that of the reference logits.  Paper, Appendix "Task Metrics": the task metric is the difference in
    logit values between the correct answer and a distractor; taken relative to the clean reference, and
    with the sign of a loss (larger = worse), it is 0 for the unpruned graph, like the KL."""
    b = np.arange(len(answer))
    ref = ref_logits[b, answer] - ref_logits[b, distractor]
    cur = logits[b, answer] - logits[b, distractor]
    return float((ref - cur).mean())


class Acdc:
    def __init__(self, model: Model, clean_tokens, corrupt_tokens, mode=MODE_PAHQ, metric=METRIC_KL, answer=None,
                 distractor=None):
        """metric: METRIC_KL (KL to the clean reference) or METRIC_LOGIT_DIFF (needs one answer and one
        distractor token id per sequence)."""
        self.m, self.g, self.mode = model, model.g, mode
        self.metric = metric
        if metric == METRIC_LOGIT_DIFF:
            self.answer, self.distractor = np.asarray(answer), np.asarray(distractor)
            assert self.answer.shape == self.distractor.shape == (len(clean_tokens),)
        self.clean = np.asarray(clean_tokens)
        self.corrupt = np.asarray(corrupt_tokens)
        self.base_pi = ALL if mode == MODE_ALL_FP32 else NONE
        self._base = None
        self._pi_cache = {}
        self.n_forwards = 0

    # precision policy ------------------------------------------------------
    def pi_of(self, receiver):
        if self.mode == MODE_ALL_FP32:
            return ALL
        kind, l, h, _ = self.g.receiver_info(receiver)
        if self.mode == MODE_PAHQ and kind == "headin":
            return frozenset([(l, h)])
        return NONE

    def start_layer_of(self, receiver):
        kind, l, _, _ = self.g.receiver_info(receiver)
        return l            # OUT: l = L, i.e. nothing but the unembedding is recomputed

    # definition: three full forwards -----------------------------------------
    def kl_brute(self, receiver, removed, pi=None):
        pi = self.pi_of(receiver) if pi is None else pi
        C, _ = self.m.forward(self.corrupt, pi)
        _, ref = self.m.forward(self.clean, pi)
        _, lg = self.m.forward(self.clean, pi, removed=removed, C=C)
        self.n_forwards += 3
        return self.score(ref, lg)

    def score(self, ref_logits, logits):
        """The loss of a pruned run against the reference run's logits (0 when they are equal)."""
        if self.metric == METRIC_LOGIT_DIFF:
            return logit_diff_drop(ref_logits, logits, self.answer, self.distractor)
        return kl_to_reference(log_softmax(ref_logits), logits)

    # cached fast path ------------------------------------------------------------
    def base(self):
        if self._base is None:
            oc, lc = self.m.forward(self.clean, self.base_pi)
            ox, lx = self.m.forward(self.corrupt, self.base_pi)
            self._base = (oc, ox, lc, lx)
        return self._base

    def _pi_state(self, receiver):
        pi, l0 = self.pi_of(receiver), self.start_layer_of(receiver)
        key = (pi if pi == ALL else tuple(sorted(pi)), l0)
        if key not in self._pi_cache:
            oc, ox, _, _ = self.base()
            C, _ = self.m.forward(self.corrupt, pi, base=ox, start_layer=l0)
            _, ref = self.m.forward(self.clean, pi, base=oc, start_layer=l0)
            self._pi_cache = {key: (C, ref)}      # keep one entry: they are large
        return self._pi_cache[key]

    def logits_fast(self, receiver, removed):
        C, _ = self._pi_state(receiver)
        oc = self.base()[0]
        _, lg = self.m.forward(self.clean, self.pi_of(receiver), removed=removed, C=C, base=oc,
                               start_layer=self.start_layer_of(receiver))
        self.n_forwards += 1
        return lg

    def kl_fast(self, receiver, removed):
        _, ref = self._pi_state(receiver)
        return self.score(ref, self.logits_fast(receiver, removed))

    def kl_edge(self, receiver, sender, removed=None, brute=False):
        """kl_new of the candidate (sender -> receiver) on top of the removed set."""
        rem = self.g.empty_removed() if removed is None else removed.copy()
        assert sender < self.g.n_upstream(receiver)
        rem[receiver, sender] = True
        return self.kl_brute(receiver, rem) if brute else self.kl_fast(receiver, rem)

    # the paper-literal precision policy -------------------------------------------
    def pi_of_sender(self, sender):
        """Eq. P_t as printed: FP32 for the SOURCE node of the evaluated edge (a head; an MLP or the embedding
        has no attention weights to keep in fp32), FP8 for everything else."""
        kind, l, h = self.g.sender_info(sender)
        if self.mode == MODE_ALL_FP32:
            return ALL
        return frozenset([(l, h)]) if (self.mode == MODE_PAHQ and kind == "head") else NONE

    def pair_sender_policy(self, receiver, sender, removed):
        """(loss of the current graph, loss with the edge sender -> receiver removed as well), both under the
        precision set of the SENDER: corrupted run, reference run and the two pruned runs are recomputed from
        the sender's layer on (below it nothing depends on that set)."""
        pi = self.pi_of_sender(sender)
        kind, l_s, _ = self.g.sender_info(sender)
        l0 = min(l_s, self.start_layer_of(receiver)) if kind == "head" else self.start_layer_of(receiver)
        oc, ox, _, _ = self.base()
        C, _ = self.m.forward(self.corrupt, pi, base=ox, start_layer=l0)
        _, ref = self.m.forward(self.clean, pi, base=oc, start_layer=l0)
        _, cur = self.m.forward(self.clean, pi, removed=removed, C=C, base=oc, start_layer=l0)
        cand = removed.copy()
        cand[receiver, sender] = True
        _, new = self.m.forward(self.clean, pi, removed=cand, C=C, base=oc, start_layer=l0)
        self.n_forwards += 4
        return self.score(ref, cur), self.score(ref, new)

    def sweep_sender_policy(self, tau, receivers=None):
        """The same pass as sweep(), every candidate judged under the precision set of its own sender."""
        g = self.g
        removed = g.empty_removed()
        trace = []
        order = range(g.n_receivers - 1, -1, -1) if receivers is None else sorted(receivers, reverse=True)
        for v in order:
            n_up = g.n_upstream(v)
            if not self.node_is_live(v, removed):
                removed[v, :n_up] = True
                continue
            for u in range(n_up - 1, -1, -1):
                kl_cur, kl_new = self.pair_sender_policy(v, u, removed)
                rm = (kl_new - kl_cur) < tau
                trace.append((v, u, kl_new, kl_cur, bool(rm)))
                if rm:
                    removed[v, u] = True
        return removed, trace

    # the sweep -------------------------------------------------------------------
    def node_is_live(self, receiver, removed):
        s = self.g.node_of_receiver(receiver)
        if s < 0:
            return True
        return any(not removed[r, s] for r in self.g.receivers_downstream_of(s))

    def sweep(self, tau, receivers=None, brute=False, progress=None, start=None):
        """One reverse-topological ACDC pass.

        receivers: restrict evaluation to these receiver ids (others keep all
        their in-edges and are not visited); None = all.
        start: removed matrix to begin from instead of the empty one (the
        state an interrupted pass had reached: the pass decides receiver by
        receiver, each decision given all earlier ones, so that state is the
        removed set alone).
        Returns (removed matrix, trace).  trace rows:
        (receiver, sender, kl_new, kl_cur_before, removed?) for evaluated
        edges, in evaluation order.
        """
        g = self.g
        removed = g.empty_removed() if start is None else np.array(start, dtype=bool, copy=True)
        trace = []
        order = range(g.n_receivers - 1, -1, -1) if receivers is None else sorted(receivers, reverse=True)
        ev = self.kl_brute if brute else self.kl_fast
        for v in order:
            n_up = g.n_upstream(v)
            if not self.node_is_live(v, removed):
                removed[v, :n_up] = True
                continue
            kl_cur = ev(v, removed)
            for u in range(n_up - 1, -1, -1):
                cand = removed.copy()
                cand[v, u] = True
                kl_new = ev(v, cand)
                rm = (kl_new - kl_cur) < tau
                trace.append((v, u, kl_new, kl_cur, bool(rm)))
                if rm:
                    removed = cand
                    kl_cur = kl_new
            if progress:
                progress(v, len(trace), int(g.removed_to_flat(removed).sum()))
        return removed, trace
