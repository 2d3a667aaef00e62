"""Computational graph of the transformer (test infrastructure).

Paper, Appendix "Preliminaries / Circuit Discovery": nodes are the attention
heads and MLP layers (plus the embedding and the unembedding), edges are the
activation pathways, and a node's input is the sum of the outputs of its
predecessors.  The appendix on the edge-cutting process reports about 35 000
starting edges for GPT-2 small, which only the graph with separate query, key
and value inputs per head reaches (32 491 edges), so head inputs are split.

The coarser graph, in which a head has a single input that its query, key and
value projections all read (11 611 edges for GPT-2 small), is available with
split_qkv=False: C = 1 input per head instead of C = 3.

Ids
  senders    0 = EMBED;  HEAD(l,h) = 1 + l*(H+mu) + h;  MLP(l) = 1 + l*(H+mu) + H
  receivers  HEADIN(l,h,c) = l*(C*H+mu) + C*h + c  (C = 3, c: Q=0, K=1, V=2; or C = 1, c ignored)
             MLPIN(l) = l*(C*H+mu) + C*H;  OUT = L*(C*H+mu)
  with mu = 1 when the model has MLPs, else 0.  Receiver ids ascend in
  topological order.  Canonical edge order: receivers ascending, then senders
  ascending.
"""
from __future__ import annotations
import numpy as np

Q, K, V = 0, 1, 2


class Graph:
    def __init__(self, n_layers: int, n_heads: int, has_mlp: bool, split_qkv: bool = True):
        self.L, self.H, self.mu = n_layers, n_heads, 1 if has_mlp else 0
        self.split = bool(split_qkv)
        self.C = 3 if self.split else 1              # inputs per head
        self.n_senders = 1 + self.L * (self.H + self.mu)
        self.n_receivers = self.L * (self.C * self.H + self.mu) + 1
        self.OUT = self.n_receivers - 1

    # ---- senders
    def head(self, l, h):
        return 1 + l * (self.H + self.mu) + h

    def mlp(self, l):
        assert self.mu
        return 1 + l * (self.H + self.mu) + self.H

    def sender_info(self, s):
        """('embed',-1,-1) | ('head',l,h) | ('mlp',l,-1)"""
        if s == 0:
            return ("embed", -1, -1)
        l, r = divmod(s - 1, self.H + self.mu)
        return ("head", l, r) if r < self.H else ("mlp", l, -1)

    # ---- receivers
    def headin(self, l, h, c=0):
        return l * (self.C * self.H + self.mu) + self.C * h + (c if self.split else 0)

    def mlpin(self, l):
        assert self.mu
        return l * (self.C * self.H + self.mu) + self.C * self.H

    def receiver_info(self, r):
        """('headin',l,h,c) | ('mlpin',l,-1,-1) | ('out',L,-1,-1); c = -1 for the single input of an unsplit head"""
        if r == self.OUT:
            return ("out", self.L, -1, -1)
        l, q = divmod(r, self.C * self.H + self.mu)
        if q < self.C * self.H:
            return ("headin", l, q // self.C, q % self.C if self.split else -1)
        return ("mlpin", l, -1, -1)

    def n_upstream(self, r):
        """Senders 0 .. n_upstream(r)-1 are exactly the senders upstream of receiver r."""
        kind, l, _, _ = self.receiver_info(r)
        if kind == "out":
            return self.n_senders
        if kind == "headin":                      # embed + everything in layers < l
            return 1 + l * (self.H + self.mu)
        return 1 + l * (self.H + self.mu) + self.H   # mlpin: + heads of layer l

    def node_of_receiver(self, r):
        """Sender id of the node that receiver r feeds (-1 for OUT)."""
        kind, l, h, _ = self.receiver_info(r)
        if kind == "out":
            return -1
        return self.head(l, h) if kind == "headin" else self.mlp(l)

    def receivers_downstream_of(self, s):
        """Receiver ids r with an edge s -> r, ascending."""
        return [r for r in range(self.n_receivers) if s < self.n_upstream(r)]

    def edge_offsets(self):
        off = np.zeros(self.n_receivers + 1, dtype=np.int64)
        for r in range(self.n_receivers):
            off[r + 1] = off[r] + self.n_upstream(r)
        return off

    def n_edges(self):
        return int(self.edge_offsets()[-1])

    def edge_id(self, s, r):
        assert 0 <= s < self.n_upstream(r)
        return int(self.edge_offsets()[r] + s)

    def empty_removed(self):
        """Boolean [n_receivers][n_senders]; entries beyond n_upstream(r) stay False."""
        return np.zeros((self.n_receivers, self.n_senders), dtype=bool)

    def removed_to_flat(self, removed):
        return np.concatenate([removed[r, :self.n_upstream(r)] for r in range(self.n_receivers)])

    def flat_to_removed(self, flat):
        rem = self.empty_removed()
        off = self.edge_offsets()
        for r in range(self.n_receivers):
            rem[r, :self.n_upstream(r)] = flat[off[r]:off[r + 1]]
        return rem
