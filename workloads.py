"""Seeded synthetic inputs for the five benchmark workloads.

This module holds random number generation and shapes only -- none of the
method's arithmetic -- so that the CPU oracle and the HIP path can be fed the
very same float32 buffers.  The tensors stand in for the batches the paper
decodes (arxiv 1805.12096: 36 000-entry tied vocabulary, Section 2.1; batches
of about 384 words on the CPU and about 8192 words / 300 sentences on the GPU,
Section 2.3; model and FFN widths of Table 1), which need the trained student
models and the news test set and are therefore replaced by Gaussian data of
the same shapes.

Weights are generated directly in the transposed layout Wt = B^T, [N x K], the
layout dot'_int consumes (Section 4.3).
"""
from __future__ import annotations

import numpy as np

BASE_SEED = 180512096


def _normal(rng: np.random.Generator, shape, sigma: float) -> np.ndarray:
    x = rng.standard_normal(size=shape, dtype=np.float32)
    if sigma != 1.0:
        x *= np.float32(sigma)
    return x


def rng_for(config: int, extra: int = 0) -> np.random.Generator:
    return np.random.default_rng(BASE_SEED + config + 1000 * extra)


def config1(seed_extra: int = 0):
    """Single int16 product, 384-word CPU batch through a 512x512 parameter."""
    r = rng_for(1, seed_extra)
    return {"bits": 16, "A": _normal(r, (384, 512), 1.0), "Wt": _normal(r, (512, 512), 0.05),
            "bias": _normal(r, (512,), 0.1)}


def ffn(config: int, M: int, d: int, f: int, w_sigma: float, bits: int, seed_extra: int = 0):
    r = rng_for(config, seed_extra)
    return {"bits": bits, "A": _normal(r, (M, d), 1.0),
            "W1t": _normal(r, (f, d), w_sigma), "b1": _normal(r, (f,), 0.1),
            "W2t": _normal(r, (d, f), w_sigma), "b2": _normal(r, (d,), 0.1)}


def config2(M: int = 8192, seed_extra: int = 0):
    """Transformer-base FFN block in int8 (512 -> 2048 -> 512), M tokens."""
    return ffn(2, M, 512, 2048, 0.04, 8, seed_extra)


def config3(M: int = 300, V: int = 36000, d: int = 512, seed_extra: int = 0):
    """Greedy output layer of one decode step: hidden [M x d], tied embedding [V x d]."""
    r = rng_for(3, seed_extra)
    return {"bits": 8, "Hd": _normal(r, (M, d), 1.0), "E": _normal(r, (V, d), 0.05)}


def config4(M: int = 8192, seed_extra: int = 0):
    """Transformer-big FFN block in int16 (1024 -> 4096 -> 1024), M tokens."""
    return ffn(4, M, 1024, 4096, 0.03, 16, seed_extra)


# (name, N, K, relu) of the parameter products of one AAN decoder layer at a
# decode step (Section 3.2: averaging attention replaces decoder self-attention
# and carries a feed-forward network and a gate; then source attention's query
# and output projections; then the layer's FFN).
AAN_LAYER_GEMMS = (
    ("aan_ffn1", 2048, 512, True),
    ("aan_ffn2", 512, 2048, False),
    ("aan_gate", 1024, 1024, False),
    ("ctx_q", 512, 512, False),
    ("ctx_o", 512, 512, False),
    ("ffn1", 2048, 512, True),
    ("ffn2", 512, 2048, False),
)


def config5(M: int = 300, layers: int = 6, V: int = 36000, seed_extra: int = 0):
    """All parameter products of one greedy decode step of a 6-layer base AAN decoder.

    Every product gets its own N(0,1) input, as the float glue between them
    (running average, gate, attention over the source, layer norm) is not part
    of the integer path.
    """
    r = rng_for(5, seed_extra)
    gemms = []
    for layer in range(layers):
        for name, N, K, relu in AAN_LAYER_GEMMS:
            gemms.append({"name": f"l{layer}.{name}", "relu": relu,
                          "A": _normal(r, (M, K), 1.0), "Wt": _normal(r, (N, K), 0.04),
                          "bias": _normal(r, (N,), 0.1)})
    out = {"Hd": _normal(r, (M, 512), 1.0), "E": _normal(r, (V, 512), 0.05)}
    return {"bits": 8, "gemms": gemms, "output": out}


def config5_chained(M: int = 300, layers: int = 6, d: int = 512, ffn: int = 2048, aan_ffn: int = 2048,
                    S: int = 25, V: int = 36000, t: int = 20, seed_extra: int = 0):
    """The same decode step with its real data dependencies: per layer the parameters of the seven
    products and the three layer normalisations, the running average up to position t - 1, and
    the precomputed source keys / values [M x S x d]; plus the layer-0 input and the tied embedding."""
    r = rng_for(5, 1000 + seed_extra)

    def product(N, K):
        return {"Wt": _normal(r, (N, K), 0.04), "bias": _normal(r, (N,), 0.1)}

    def norm():
        return {"gamma": (np.float32(1) + _normal(r, (d,), 0.1)).astype(np.float32), "beta": _normal(r, (d,), 0.1)}

    L = []
    KV = []
    g_prev = []
    for _ in range(layers):
        L.append({"aan_ffn1": product(aan_ffn, d), "aan_ffn2": product(d, aan_ffn), "aan_gate": product(2 * d, 2 * d),
                  "ln1": norm(), "ctx_q": product(d, d), "ctx_o": product(d, d), "ln2": norm(),
                  "ffn1": product(ffn, d), "ffn2": product(d, ffn), "ln3": norm()})
        KV.append((_normal(r, (M, S, d), 1.0), _normal(r, (M, S, d), 1.0)))
        g_prev.append(_normal(r, (M, d), 1.0 / np.sqrt(max(t - 1, 1))))
    return {"bits": 8, "t": t, "heads": 8, "x0": _normal(r, (M, d), 1.0), "layers": L, "KV": KV, "g_prev": g_prev,
            "E": _normal(r, (V, d), 0.05)}


def random_problem(seed: int, M: int, N: int, K: int, a_sigma: float = 1.0, w_sigma: float = 0.05):
    """Free-shape problem for parity tests (odd sizes, tails)."""
    r = np.random.default_rng(BASE_SEED * 7 + seed)
    return {"A": _normal(r, (M, K), a_sigma), "Wt": _normal(r, (N, K), w_sigma),
            "bias": _normal(r, (N,), 0.1)}
