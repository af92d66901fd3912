"""CPU oracle for the floating-point glue between the integer products of one greedy decode
step of the averaging-attention decoder (arxiv 1805.12096, Section 3.2; the block itself is the
one of the averaging attention network paper it cites: cumulative average, feed-forward network,
gate, residual + layer normalisation), the source attention over precomputed keys / values and
the position-wise feed-forward block of the Transformer (Section 3.1).

TEST INFRASTRUCTURE ONLY, like the rest of this package.  Plain numpy in binary64; every function
takes and returns arrays, nothing is blocked, fused or reordered.  Products go through
``oracle.linear`` (quant_int, dot'_int, dequantize + bias), whose inputs are binary32 by
definition, so a glue result is rounded to binary32 exactly once, where it becomes the input of
the next product.
"""
from __future__ import annotations

import numpy as np

from . import linear as _linear
from . import greedy_output_layer as _greedy_output_layer

LN_EPS = 1e-6


def running_average(g_prev, x, t: int):
    """Cumulative uniform average over the decoder positions seen so far, from the last step only:
    g_t = ((t - 1) g_{t-1} + x_t) / t  (Section 3.2)."""
    if t < 1:
        raise ValueError("positions count from 1")
    g_prev = np.asarray(g_prev, dtype=np.float64)
    x = np.asarray(x, dtype=np.float64)
    return ((t - 1) * g_prev + x) / t


def sigmoid(z):
    z = np.asarray(z, dtype=np.float64)
    return 1.0 / (1.0 + np.exp(-z))


def gate_mix(x, f, z):
    """Gate of the averaging block: z [M x 2d] are the pre-activations of the gate product on
    [x; f]; the first d columns gate the layer input x, the last d the averaged path f."""
    x = np.asarray(x, dtype=np.float64)
    f = np.asarray(f, dtype=np.float64)
    z = np.asarray(z, dtype=np.float64)
    d = x.shape[1]
    if z.shape != (x.shape[0], 2 * d) or f.shape != x.shape:
        raise ValueError("shapes: x, f [M x d], z [M x 2d]")
    return sigmoid(z[:, :d]) * x + sigmoid(z[:, d:]) * f


def layer_norm(h, gamma, beta, eps: float = LN_EPS):
    """Row-wise (h - mean) / sqrt(var + eps) * gamma + beta with the biased variance."""
    h = np.asarray(h, dtype=np.float64)
    mu = h.mean(axis=1, keepdims=True)
    var = ((h - mu) ** 2).mean(axis=1, keepdims=True)
    return (h - mu) / np.sqrt(var + eps) * np.asarray(gamma, dtype=np.float64) + np.asarray(beta, dtype=np.float64)


def add_layer_norm(a, b, gamma, beta, eps: float = LN_EPS):
    """Residual connection followed by layer normalisation."""
    return layer_norm(np.asarray(a, dtype=np.float64) + np.asarray(b, dtype=np.float64), gamma, beta, eps)


def cross_attention(q, K, V, heads: int):
    """Scaled dot-product attention of one query per sentence over that sentence's S source
    positions: q [M x d], K, V [M x S x d]; per head h of width d / heads:
    p = softmax_s(q_h . K_h[s] / sqrt(d / heads)), context_h = sum_s p[s] V_h[s]."""
    q = np.asarray(q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    M, d = q.shape
    S = K.shape[1]
    if d % heads or K.shape != (M, S, d) or V.shape != (M, S, d):
        raise ValueError("shapes: q [M x d], K, V [M x S x d], d divisible by heads")
    dh = d // heads
    ctx = np.empty((M, d), dtype=np.float64)
    for h in range(heads):
        sl = slice(h * dh, (h + 1) * dh)
        scores = np.einsum("md,msd->ms", q[:, sl], K[:, :, sl]) / np.sqrt(dh)
        scores -= scores.max(axis=1, keepdims=True)
        p = np.exp(scores)
        p /= p.sum(axis=1, keepdims=True)
        ctx[:, sl] = np.einsum("ms,msd->md", p, V[:, :, sl])
    return ctx


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _product(A, W, bits, relu=False):
    """One parameter product: A (rounded to binary32 here), W = {"Wt", "bias"}."""
    return _linear(_f32(A), W["Wt"], bits, W["bias"], relu)["Y"]


def aan_decoder_layer(x, g_prev, t: int, P, K, V, heads: int = 8, bits: int = 8, use_ffn: bool = True,
                      use_gate: bool = True, eps: float = LN_EPS):
    """One decoder layer at decode position t for all sentences: averaging block, source attention,
    feed-forward block, each followed by residual + layer normalisation.

    x, g_prev: [M x d] (layer input at this position, running average up to t - 1);
    P: parameters, each product as {"Wt": [N x K], "bias": [N]}, each normalisation as
    {"gamma", "beta"}: aan_ffn1, aan_ffn2, aan_gate, ln1, ctx_q, ctx_o, ln2, ffn1, ffn2, ln3.
    Returns (layer output [M x d] float32, new running average float32).
    use_ffn / use_gate switch off the averaging block's network and gate (the "-ffn", "-gate"
    variants of Table 2)."""
    x = _f32(x)
    g = _f32(running_average(g_prev, x, t))
    f = g
    if use_ffn:
        f = _product(_product(g, P["aan_ffn1"], bits, relu=True), P["aan_ffn2"], bits)
    if use_gate:
        z = _product(np.concatenate([x, _f32(f)], axis=1), P["aan_gate"], bits)
        h = gate_mix(x, f, z)
    else:
        h = np.asarray(f, dtype=np.float64)
    y1 = _f32(add_layer_norm(h, x, P["ln1"]["gamma"], P["ln1"]["beta"], eps))
    q = _product(y1, P["ctx_q"], bits)
    ctx = cross_attention(q, K, V, heads)
    o = _product(ctx, P["ctx_o"], bits)
    y2 = _f32(add_layer_norm(o, y1, P["ln2"]["gamma"], P["ln2"]["beta"], eps))
    ff = _product(_product(y2, P["ffn1"], bits, relu=True), P["ffn2"], bits)
    y3 = _f32(add_layer_norm(ff, y2, P["ln3"]["gamma"], P["ln3"]["beta"], eps))
    return y3, g


def decode_step(x0, g_prev, t: int, layers, KV, E, heads: int = 8, bits: int = 8, use_ffn: bool = True,
                use_gate: bool = True, eps: float = LN_EPS):
    """All layers of one greedy decode step, then the tied output layer with beam-1 arg-max
    (Section 2.3).  g_prev[l], KV[l] = (K, V) belong to layer l.  Returns the tokens, the max
    logits, the last hidden state and the new running averages."""
    x = _f32(x0)
    g_new = []
    for l, P in enumerate(layers):
        x, g = aan_decoder_layer(x, g_prev[l], t, P, KV[l][0], KV[l][1], heads, bits, use_ffn, use_gate, eps)
        g_new.append(g)
    out = _greedy_output_layer(x, E, bits)
    return {"tok": out["tok"], "maxlogit": out["maxlogit"], "hidden": x, "g": g_new}
