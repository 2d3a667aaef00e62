"""A second, independently written mixed-precision forward with edge patching,
for tiny models only (explicit Python loops over layers, heads, channels and
senders).  It pins two parts of oracle/model.py that no closed form covers:

* where the quantisers sit under a precision set (paper, Sec. "Selective
  Precision Allocation Strategy" and Sec. "Mixed-Precision Computation
  Design"): a head in `pi` multiplies unquantised activations with its fp32
  master weights in its query / key / value projections and in its output
  projection; every other head's four projections, both (three with a gate)
  MLP matrix products and the unembedding multiply e4m3-quantised activation
  rows (one scale per row) with e4m3-quantised weights (one scale per head
  slice, per MLP matrix, for the unembedding);
* how a patch is routed (Appendix "Preliminaries"): the input of one receiver
  -- the query, key or value input of one head, an MLP input, the unembedding
  input -- is the sum over its upstream senders of the sender's output, taken
  from the other run where that one edge is removed.

It shares nothing with oracle/model.py except the e4m3 codec (pinned on its own
by tests/test_oracle_e4m3.py); nodes and edges are named by tuples, not by ids:
  senders    ("embed",) ("head", l, h) ("mlp", l)
  receivers  ("q", l, h) ("k", l, h) ("v", l, h) ("mlpin", l) ("out",)
`removed` is a set of (sender, receiver) pairs; `other` maps a sender to its
[T][d] output in the other run.

`drop` names one quantiser to leave out ("act:q", "w:q", ... see SITES); the
tests use it to show that every single one of them is seen by the comparison.
"""
import math
import numpy as np

from oracle import e4m3

SITES = ("act:q", "act:k", "act:v", "w:q", "w:k", "w:v", "act:o", "w:o",
         "act:in", "w:in", "w:gate", "act:out", "w:out", "act:u", "w:u")


_CODEC = [e4m3, e4m3]      # the quantisers of the attention heads' products and of the other products (loop_forward's arguments)


def _qrows(x, q):
    """Dequantised rows: grid points x one scale per row."""
    codes, scale = q.quantize_rows(np.asarray(x, dtype=np.float32))
    return q.decode(codes) * scale.astype(np.float64)[:, None]


def _qall(w, q):
    """Dequantised matrix: grid points x one scale for the whole slice."""
    codes, scale = q.quantize_groups(np.asarray(w, dtype=np.float32), axis=None)
    return q.decode(codes) * np.float64(scale)


def _matmul(x, w, low, drop, act_site, w_site):
    q = _CODEC[0] if w_site in ("w:q", "w:k", "w:v", "w:o") else _CODEC[1]
    a = _qrows(x, q) if (low and drop != act_site) else np.asarray(x, dtype=np.float64)
    b = _qall(w, q) if (low and drop != w_site) else np.asarray(w, dtype=np.float64)
    out = np.zeros((a.shape[0], b.shape[1]))
    for t in range(a.shape[0]):
        for j in range(b.shape[1]):
            out[t, j] = math.fsum(a[t, k] * b[k, j] for k in range(a.shape[1]))
    return out


def _is_upstream(sender, receiver):
    if sender[0] == "embed" or receiver[0] == "out":
        return True
    ls = sender[1]
    if receiver[0] in ("q", "k", "v"):
        return ls < receiver[1]
    return ls < receiver[1] or (ls == receiver[1] and sender[0] == "head")      # MLP input


def loop_forward(shape, w, tokens, pi=frozenset(), quantise=True, removed=frozenset(), other=None, drop=None, codec=None,
                 codec_other=None):
    """Returns (outputs: dict sender -> [T][d], logits [B][vocab] at the last position).
    codec: the quantiser (quantize_rows / quantize_groups / decode) of the attention heads' products, default the
    separately pinned e4m3 codec; codec_other: that of the MLP matrices and the unembedding, default `codec`."""
    _CODEC[0] = e4m3 if codec is None else codec
    _CODEC[1] = _CODEC[0] if codec_other is None else codec_other
    L, H, dh, d, m = shape.n_layers, shape.n_heads, shape.d_head, shape.d_model, shape.d_mlp
    B, S = tokens.shape
    T = B * S
    f = lambda a: np.asarray(a, dtype=np.float64)

    def norm(x, gain, offset):
        y = np.zeros_like(x)
        for t in range(x.shape[0]):
            if shape.norm == 1:
                y[t] = x[t] / math.sqrt(math.fsum(x[t] ** 2) / d + shape.norm_eps) * gain
            else:
                mu = math.fsum(x[t]) / d
                var = math.fsum((x[t] - mu) ** 2) / d
                y[t] = (x[t] - mu) / math.sqrt(var + shape.norm_eps) * gain + offset
        return y

    out = {}
    emb = np.zeros((T, d))
    for b in range(B):
        for p in range(S):
            emb[b * S + p] = f(w["W_E"][tokens[b, p]]) + (f(w["W_pos"][p]) if shape.pos == 0 else 0.0)
    out[("embed",)] = emb
    order = [("embed",)]                                     # senders in the order they are computed

    def receiver_input(receiver):
        x = np.zeros((T, d))
        for s in order:
            if _is_upstream(s, receiver):
                x = x + (other[s] if (s, receiver) in removed else out[s])
        # constant biases of every block upstream of the receiver
        lim = L if receiver[0] == "out" else receiver[1]
        for l in range(L):
            if l < lim or (receiver[0] == "mlpin" and l == lim):
                x = x + f(w["b_O"][l])
            if m > 0 and l < lim:
                x = x + f(w["b_out"][l])
        return x

    def rope(a):
        half = dh // 2
        r = a.copy()
        for t in range(T):
            p = t % S
            for i in range(half):
                th = p * shape.rope_theta ** (-2.0 * i / dh)
                c, s_ = math.cos(th), math.sin(th)
                r[t, i] = a[t, i] * c - a[t, i + half] * s_
                r[t, i + half] = a[t, i + half] * c + a[t, i] * s_
        return r

    for l in range(L):
        heads = {}
        for h in range(H):
            low = quantise and (l, h) not in pi
            proj = {}
            for ch, nm in (("q", "W_Q"), ("k", "W_K"), ("v", "W_V")):
                xn = norm(receiver_input((ch, l, h)), f(w["ln1_g"][l]), f(w["ln1_b"][l]))
                y = _matmul(xn, w[nm][l, h], low, drop, "act:" + ch, "w:" + ch) + f(w["b_" + nm[-1]][l, h])
                proj[ch] = rope(y) if (shape.pos == 1 and ch != "v") else y
            z = np.zeros((T, dh))
            for b in range(B):
                for i in range(S):
                    sc = [math.fsum(proj["q"][b * S + i] * proj["k"][b * S + j]) / math.sqrt(dh) for j in range(i + 1)]
                    mx = max(sc)
                    e = [math.exp(v - mx) for v in sc]
                    tot = math.fsum(e)
                    for j in range(i + 1):
                        z[b * S + i] += e[j] / tot * proj["v"][b * S + j]
            heads[h] = _matmul(z, w["W_O"][l, h], low, drop, "act:o", "w:o")
        for h in range(H):                                   # heads of a layer do not see each other
            out[("head", l, h)] = heads[h]
            order.append(("head", l, h))
        if m > 0:
            xn = norm(receiver_input(("mlpin", l)), f(w["ln2_g"][l]), f(w["ln2_b"][l]))
            up = _matmul(xn, w["W_in"][l], quantise, drop, "act:in", "w:in") + f(w["b_in"][l])
            if shape.act == 2:
                gt = _matmul(xn, w["W_gate"][l], quantise, drop, "act:in", "w:gate")
                hid = gt / (1.0 + np.exp(-gt)) * up
            elif shape.act == 1:
                hid = 0.5 * up * (1.0 + np.tanh(math.sqrt(2.0 / math.pi) * (up + 0.044715 * up ** 3)))
            else:
                hid = up
            out[("mlp", l)] = _matmul(hid, w["W_out"][l], quantise, drop, "act:out", "w:out")
            order.append(("mlp", l))

    x = receiver_input(("out",))
    last = np.stack([x[b * S + S - 1] for b in range(B)])
    xn = norm(last, f(w["lnf_g"]), f(w["lnf_b"]))
    logits = _matmul(xn, w["W_U"], quantise, drop, "act:u", "w:u") + f(w["b_U"])
    return out, logits
