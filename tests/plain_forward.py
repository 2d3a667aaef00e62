"""A textbook fp64 decoder forward, written independently of oracle/ (no
quantisation code, no graph, fused QKV, an ordinary residual stream).  Used to
pin the oracle's all-fp32 configuration."""
import math
import numpy as np


def plain_forward(shape, w, tokens):
    L, H, dh, d, m = shape.n_layers, shape.n_heads, shape.d_head, shape.d_model, shape.d_mlp
    B, S = tokens.shape
    f = lambda a: np.asarray(a, dtype=np.float64)
    x = f(w["W_E"])[tokens]                                    # [B,S,d]
    if shape.pos == 0:
        x = x + f(w["W_pos"])[None, :S]

    def norm(x, g, b):
        if shape.norm == 1:
            return x * g / np.sqrt(np.mean(x ** 2, -1, keepdims=True) + shape.norm_eps)
        mu = np.mean(x, -1, keepdims=True)
        return (x - mu) / np.sqrt(np.var(x, -1, keepdims=True) + shape.norm_eps) * g + b

    def rope(a):                                               # a [B,S,H,dh]
        half = dh // 2
        out = np.empty_like(a)
        for p in range(S):
            for i in range(half):
                th = p * shape.rope_theta ** (-2.0 * i / dh)
                c, s = math.cos(th), math.sin(th)
                out[:, p, :, i] = a[:, p, :, i] * c - a[:, p, :, i + half] * s
                out[:, p, :, i + half] = a[:, p, :, i + half] * c + a[:, p, :, i] * s
        return out

    mask = np.triu(np.full((S, S), -np.inf), 1)
    for l in range(L):
        xn = norm(x, f(w["ln1_g"][l]), f(w["ln1_b"][l]))
        q = np.einsum("bsd,hde->bshe", xn, f(w["W_Q"][l])) + f(w["b_Q"][l])
        k = np.einsum("bsd,hde->bshe", xn, f(w["W_K"][l])) + f(w["b_K"][l])
        v = np.einsum("bsd,hde->bshe", xn, f(w["W_V"][l])) + f(w["b_V"][l])
        if shape.pos == 1:
            q, k = rope(q), rope(k)
        sc = np.einsum("bihe,bjhe->bhij", q, k) / math.sqrt(dh) + mask
        p = np.exp(sc - sc.max(-1, keepdims=True))
        p /= p.sum(-1, keepdims=True)
        z = np.einsum("bhij,bjhe->bihe", p, v)
        x = x + np.einsum("bihe,hed->bid", z, f(w["W_O"][l])) + f(w["b_O"][l])
        if m > 0:
            xn = norm(x, f(w["ln2_g"][l]), f(w["ln2_b"][l]))
            up = xn @ f(w["W_in"][l]) + f(w["b_in"][l])
            if shape.act == 2:
                gt = xn @ f(w["W_gate"][l])
                hid = gt / (1 + np.exp(-gt)) * up
            elif shape.act == 1:
                hid = np.array([0.5 * t * (1 + math.tanh(math.sqrt(2 / math.pi) * (t + 0.044715 * t ** 3)))
                                for t in up.ravel()]).reshape(up.shape)
            else:
                hid = up
            x = x + hid @ f(w["W_out"][l]) + f(w["b_out"][l])
    xn = norm(x[:, -1], f(w["lnf_g"]), f(w["lnf_b"]))
    return xn @ f(w["W_U"]) + f(w["b_U"])
