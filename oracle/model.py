"""fp64 transformer forward with per-receiver inputs and simulated e4m3 GEMMs
(test infrastructure).

What is computed, with the passage of the paper that fixes it:

* Graph semantics (Appendix "Preliminaries / Circuit Discovery"): every
  receiver (a head's query, key or value input, an MLP's input, the
  unembedding's input) reads the SUM of the outputs of the senders upstream
  of it (embedding, earlier heads, earlier MLPs) plus the constant biases
  b_O / b_out of the layers before it.  An edge in the removed set R carries
  the sender's output from ANOTHER run (the corrupted prompt) instead of the
  current one ("hybrid activations", same appendix).
* Precision map (Sec. "Selective Precision Allocation Strategy", Eq. P_t; Sec.
  "Mixed-Precision Computation Design"): heads in the set `pi` use the fp32
  master weights and unquantised activations for their Q/K/V projections and
  their output projection; every other head projection, the MLP matmuls and
  the unembedding are fp8 GEMMs: e4m3 codes for both operands (one scale per
  activation row, one scale per weight slice), exact accumulation, result
  rescaled.  pi = "ALL" switches every quantiser off (plain forward).
* Attention scores, softmax, the value mix, norms, activation functions,
  residual sums and log-softmax are never quantised (Sec. "Scheduler
  Implementation", Phase 3: attention core in unified fp32; Sec. "Mantissa
  Loss": sums must not be taken in 8 bits).

All arithmetic is fp64 except the quantiser, which rounds its input to
binary32 and works in binary32 (see e4m3.py).

Readings where the paper is silent: pre-norm blocks, LayerNorm with biased
variance, RMSNorm without offset, tanh-form GELU, SwiGLU = silu(x W_gate) *
(x W_in), rotary embedding on (i, i + d_head/2) pairs applied after the
projection bias, logits at the last position only.
"""
from __future__ import annotations
import numpy as np

from . import e4m3, bf16
from .rtn import Rtn
from .graph import Graph

NORM_LAYER, NORM_RMS = 0, 1
ACT_NONE, ACT_GELU, ACT_SWIGLU = 0, 1, 2
POS_LEARNED, POS_ROPE = 0, 1

ALL = "ALL"            # precision set meaning "nothing is quantised"
NONE = frozenset()     # precision set meaning "no fp32 head"


def layer_norm(x, g, b, eps):
    mu = x.mean(axis=-1, keepdims=True)
    xc = x - mu
    var = (xc * xc).mean(axis=-1, keepdims=True)
    return xc / np.sqrt(var + eps) * g + b


def rms_norm(x, g, eps):
    ms = (x * x).mean(axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * g


def gelu_tanh(x):
    return 0.5 * x * (1.0 + np.tanh(np.sqrt(2.0 / np.pi) * (x + 0.044715 * x ** 3)))


def silu(x):
    return x / (1.0 + np.exp(-x))


def log_softmax(z):
    z = z - z.max(axis=-1, keepdims=True)
    return z - np.log(np.exp(z).sum(axis=-1, keepdims=True))


def kl_to_reference(logp_ref, logits):
    """Batch mean of KL(P_ref || P) with natural logarithms."""
    logp = log_softmax(logits)
    return float((np.exp(logp_ref) * (logp_ref - logp)).sum(axis=-1).mean())


class Model:
    def __init__(self, shape, weights, cache_decoded_bytes=6 << 30, low_bits=8, nonattn_bf16=False, split_qkv=True):
        """shape: any object with the ModelShape attributes; weights: dict of float32 arrays.
        low_bits: the grid of the quantised operands -- 8: e4m3 (the paper's setting); 4: Eq. RTN-Q with
        N = 4 (the 4-bit point of the bit-width ablation, rtn.py); 16: bfloat16 rounding (its 16-bit point,
        bf16.py: the 16-bit format the paper itself uses).
        nonattn_bf16: the MLP matrices and the unembedding multiply bfloat16-rounded operands instead (paper, Sec.
        "Selective Precision Allocation Strategy": bfloat16 for the components that are not attention heads).
        split_qkv: False = the coarser graph in which a head's query, key and value projections read one input."""
        if low_bits not in (4, 8, 16):
            raise ValueError("low_bits")
        self.q = e4m3 if low_bits == 8 else (bf16 if low_bits == 16 else Rtn(low_bits))
        # the quantiser of the matrix products that are not attention heads: the MLP matrices and the unembedding
        self.q_other = bf16 if nonattn_bf16 else self.q
        self.s = shape
        self.L, self.H, self.dh, self.d = shape.n_layers, shape.n_heads, shape.d_head, shape.d_model
        self.m, self.V = shape.d_mlp, shape.vocab
        self.g = Graph(self.L, self.H, self.m > 0, split_qkv)
        self.w = {k: np.asarray(v, dtype=np.float32) for k, v in weights.items()}
        for k, v in self.w.items():
            if not np.isfinite(v).all():
                raise ValueError(f"non-finite weight in {k}")
        self._dec_cache, self._dec_budget = {}, cache_decoded_bytes
        self._quantise_weights()

    # ------------------------------------------------------------------ weights
    def _quantise_weights(self):
        """One scale per slice: each head's W_Q/W_K/W_V/W_O, each layer's W_in/W_gate/W_out, W_U."""
        w, L, H = self.w, self.L, self.H
        self.qc, self.qs = {}, {}
        for nm in ("W_Q", "W_K", "W_V", "W_O"):
            flat = w[nm].reshape(L * H, -1)
            c, s = self.q.quantize_groups(flat, axis=-1)
            self.qc[nm], self.qs[nm] = c.reshape(w[nm].shape), s.reshape(L, H)
        for nm in ("W_in", "W_gate", "W_out"):
            if nm in w:
                flat = w[nm].reshape(L, -1)
                c, s = self.q_other.quantize_groups(flat, axis=-1)
                self.qc[nm], self.qs[nm] = c.reshape(w[nm].shape), s.reshape(L)
        c, s = self.q_other.quantize_groups(w["W_U"], axis=None)
        self.qc["W_U"], self.qs["W_U"] = c, np.float32(s)

    def _wdec(self, nm, *idx):
        """Decoded (unscaled) fp64 grid values of a weight slice."""
        key = (nm,) + idx
        if key in self._dec_cache:
            return self._dec_cache[key]
        a = self._q_of(nm).decode(self.qc[nm][idx])
        if self._dec_budget >= a.nbytes:
            self._dec_budget -= a.nbytes
            self._dec_cache[key] = a
        return a

    def _q_of(self, nm):
        return self.q if nm in ("W_Q", "W_K", "W_V", "W_O") else self.q_other

    def _quant_act(self, x, nm="W_Q"):
        """Row-quantise an activation that multiplies W[nm]: decoded grid values and one scale per row."""
        q = self._q_of(nm)
        ca, sa = q.quantize_rows(x)
        return q.decode(ca), sa

    def _linear(self, x, nm, idx, quantised, bias=None, qa=None):
        """x @ W[nm][idx] (+ bias): fp8 GEMM when `quantised`, else fp32 masters in fp64.
        qa: the result of _quant_act(x) when the caller already has it (several
        projections read the same quantised rows)."""
        if quantised:
            da, sa = self._quant_act(x, nm) if qa is None else qa
            acc = da @ self._wdec(nm, *idx)                        # exact products, fp64 sum
            y = acc * sa.astype(np.float64)[:, None] * np.float64(self.qs[nm][idx] if idx else self.qs[nm])
        else:
            y = x @ self.w[nm][idx].astype(np.float64)
        if bias is not None:
            y = y + bias.astype(np.float64)
        return y

    # ------------------------------------------------------------------ pieces
    def norm(self, x, which, l=None):
        g = self.w[which + "_g"] if l is None else self.w[which + "_g"][l]
        if self.s.norm == NORM_RMS:
            return rms_norm(x, g.astype(np.float64), self.s.norm_eps)
        b = self.w[which + "_b"] if l is None else self.w[which + "_b"][l]
        return layer_norm(x, g.astype(np.float64), b.astype(np.float64), self.s.norm_eps)

    def embed(self, tokens):
        B, S = tokens.shape
        x = self.w["W_E"][tokens.reshape(-1)].astype(np.float64)
        if self.s.pos == POS_LEARNED:
            x = x + np.tile(self.w["W_pos"][:S].astype(np.float64), (B, 1))
        return x

    def _rope(self, a, B, S):
        half = self.dh // 2
        inv = self.s.rope_theta ** (-2.0 * np.arange(half) / self.dh)
        ang = np.arange(S)[:, None] * inv[None, :]                 # [S][half]
        cos, sin = np.tile(np.cos(ang), (B, 1)), np.tile(np.sin(ang), (B, 1))
        a1, a2 = a[:, :half], a[:, half:]
        return np.concatenate([a1 * cos - a2 * sin, a2 * cos + a1 * sin], axis=1)

    def attention(self, q, k, v, B, S):
        """Causal softmax(q k^T / sqrt(d_head)) v per sequence; inputs [B*S][d_head]."""
        q, k, v = (a.reshape(B, S, self.dh) for a in (q, k, v))
        sc = np.einsum("bid,bjd->bij", q, k) / np.sqrt(self.dh)
        sc = np.where(np.tril(np.ones((S, S), dtype=bool))[None], sc, -np.inf)
        sc = sc - sc.max(axis=-1, keepdims=True)
        p = np.exp(sc)
        p = p / p.sum(axis=-1, keepdims=True)
        return np.einsum("bij,bjd->bid", p, v).reshape(B * S, self.dh)

    def bias_prefix(self, r):
        """Sum of the constant output biases of every layer component upstream of receiver r."""
        kind, l, _, _ = self.g.receiver_info(r)
        b = np.zeros(self.d)
        for lp in range(self.L):
            if lp < l or (kind == "mlpin" and lp == l):
                b = b + self.w["b_O"][lp]
            if self.m > 0 and lp < l:
                b = b + self.w["b_out"][lp]
        return b

    def receiver_inputs(self, recv_ids, outs, removed, C):
        """x_w = sum over upstream senders s of (edge s->w removed ? C[s] : outs[s]) + bias prefix.

        outs, C: [n_senders][T*d] (rows of senders not yet computed are never
        read: only the first n_upstream(w) rows enter).  Receivers with the same
        upstream senders and the same removed edges read the same sum; it is
        formed once.  Returns (inputs, which): inputs is a list of distinct
        [T][d] arrays, which[i] the index of recv_ids[i]'s input in it.
        """
        g, T = self.g, outs.shape[1] // self.d
        inputs, which, seen = [], [], {}
        for r in recv_ids:
            n_up = g.n_upstream(r)
            mask = np.zeros(n_up, dtype=bool) if removed is None else removed[r, :n_up]
            kind, l, _, _ = g.receiver_info(r)
            key = (kind, l, mask.tobytes())
            if key not in seen:
                x = np.zeros(T * self.d)
                for s in range(n_up):                              # senders in ascending id
                    x += C[s] if mask[s] else outs[s]
                x = x.reshape(T, self.d) + self.bias_prefix(r)
                seen[key] = len(inputs)
                inputs.append(x)
            which.append(seen[key])
        return inputs, which

    # ------------------------------------------------------------------ forward
    def forward(self, tokens, pi=NONE, removed=None, C=None, base=None, start_layer=0):
        """Run the model on `tokens` [B][S].

        pi       ALL, or a frozenset of (layer, head) computed in fp32
        removed  bool [n_receivers][n_senders] (None = no edge removed)
        C        [n_senders][T*d] sender outputs of the other run, read where an edge is removed
        base     [n_senders][T*d] outputs to reuse for every sender in layers < start_layer
        Returns (outs [n_senders][T*d] fp64, logits [B][vocab] fp64 at the last position).
        """
        g, L, H, d = self.g, self.L, self.H, self.d
        tokens = np.asarray(tokens)
        if tokens.min() < 0 or tokens.max() >= self.V:
            raise ValueError("token id out of range")
        B, S = tokens.shape
        T = B * S
        quant_all = pi != ALL
        pis = frozenset() if pi == ALL else pi
        outs = np.zeros((g.n_senders, T * d))
        if start_layer > 0:
            n0 = g.n_upstream(g.headin(start_layer, 0, 0))
            outs[:n0] = base[:n0]
        else:
            outs[0] = self.embed(tokens).reshape(-1)

        for l in range(start_layer, L):
            rids = [g.headin(l, h, c) for h in range(H) for c in range(3)]
            xs, which = self.receiver_inputs(rids, outs, removed, C)
            normed = [self.norm(x, "ln1", l) for x in xs]
            quant = {}                                             # distinct input -> its quantised rows
            for h in range(H):
                hq = quant_all and (l, h) not in pis
                a = []
                for c, nm in enumerate(("Q", "K", "V")):
                    k = which[3 * h + c]
                    if hq and k not in quant:
                        quant[k] = self._quant_act(normed[k])
                    y = self._linear(normed[k], "W_" + nm, (l, h), hq, self.w["b_" + nm][l, h],
                                     qa=quant[k] if hq else None)
                    if self.s.pos == POS_ROPE and c < 2:
                        y = self._rope(y, B, S)
                    a.append(y)
                z = self.attention(a[0], a[1], a[2], B, S)
                outs[g.head(l, h)] = self._linear(z, "W_O", (l, h), hq).reshape(-1)
            if self.m > 0:
                xs, _ = self.receiver_inputs([g.mlpin(l)], outs, removed, C)
                xn = self.norm(xs[0], "ln2", l)
                qa = self._quant_act(xn, "W_in") if quant_all else None
                up = self._linear(xn, "W_in", (l,), quant_all, self.w["b_in"][l], qa=qa)
                if self.s.act == ACT_SWIGLU:
                    hid = silu(self._linear(xn, "W_gate", (l,), quant_all, qa=qa)) * up
                elif self.s.act == ACT_GELU:
                    hid = gelu_tanh(up)
                else:
                    hid = up
                outs[g.mlp(l)] = self._linear(hid, "W_out", (l,), quant_all).reshape(-1)

        xs, _ = self.receiver_inputs([g.OUT], outs, removed, C)
        last = xs[0].reshape(B, S, d)[:, S - 1, :]
        xn = self.norm(last, "lnf")
        logits = self._linear(xn, "W_U", (), quant_all, self.w["b_U"])
        return outs, logits
