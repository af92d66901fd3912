"""Pins for the floating-point glue of the averaging-attention decode step (oracle/glue.py):
closed forms, invariants and brute force, none of which retypes the formula under test."""
import math

import numpy as np
import pytest

import workloads
from oracle import glue


def test_running_average_is_the_mean_of_the_positions_seen_so_far():
    # Section 3.2: the cumulative uniform average can be computed from the last step only.
    rng = np.random.default_rng(1)
    xs = rng.standard_normal((7, 5, 12))
    g = np.zeros((5, 12))
    for t in range(1, 8):
        g = glue.running_average(g, xs[t - 1], t)
        assert np.allclose(g, xs[:t].mean(axis=0), rtol=0, atol=1e-14)
    assert np.array_equal(glue.running_average(np.full((2, 3), 123.0), xs[0, :2, :3], 1), xs[0, :2, :3])   # t = 1 ignores g
    c = np.full((2, 3), 0.75)
    assert np.allclose(glue.running_average(c, c, 20), c, atol=1e-16)
    with pytest.raises(ValueError):
        glue.running_average(c, c, 0)


def test_gate_mix_special_cases():
    rng = np.random.default_rng(2)
    x, f = rng.standard_normal((4, 6)), rng.standard_normal((4, 6))
    assert np.allclose(glue.gate_mix(x, f, np.zeros((4, 12))), 0.5 * (x + f), atol=1e-15)       # sigmoid(0) = 1/2
    assert np.allclose(glue.gate_mix(x, f, np.full((4, 12), 50.0)), x + f, atol=1e-12)          # both gates open
    assert np.allclose(glue.gate_mix(x, f, np.full((4, 12), -50.0)), 0.0, atol=1e-12)           # both closed
    z = np.concatenate([np.full((4, 6), 50.0), np.full((4, 6), -50.0)], axis=1)
    assert np.allclose(glue.gate_mix(x, f, z), x, atol=1e-12)                                   # first half gates x
    # one entry against the textbook logistic function
    z = np.zeros((1, 2)); z[0, 0] = math.log(3.0)          # sigmoid(log 3) = 3/4
    assert np.allclose(glue.gate_mix(np.array([[8.0]]), np.array([[2.0]]), z), [[0.75 * 8 + 0.5 * 2]], atol=1e-14)


def test_layer_norm_invariants():
    rng = np.random.default_rng(3)
    h = rng.standard_normal((9, 64)) * 3 + 1.5
    one, zero = np.ones(64), np.zeros(64)
    y = glue.layer_norm(h, one, zero, eps=0.0)
    assert np.allclose(y.mean(axis=1), 0, atol=1e-13) and np.allclose(y.var(axis=1), 1, atol=1e-12)
    # shift and positive scaling of the input do not change the result (eps = 0)
    assert np.allclose(glue.layer_norm(7.0 * h - 3.0, one, zero, eps=0.0), y, atol=1e-12)
    # gamma and beta act per column after normalisation
    gamma, beta = rng.standard_normal(64), rng.standard_normal(64)
    assert np.allclose(glue.layer_norm(h, gamma, beta, eps=0.0), y * gamma + beta, atol=1e-13)
    # a constant row has zero variance: with eps > 0 the output is beta
    assert np.allclose(glue.layer_norm(np.full((2, 64), 4.0), gamma, beta, eps=1e-6), np.tile(beta, (2, 1)), atol=1e-12)
    # two-element row by hand: h = (1, 3): mean 2, biased variance 1 -> (-1, 1) / sqrt(1 + eps)
    assert np.allclose(glue.layer_norm(np.array([[1.0, 3.0]]), np.ones(2), np.zeros(2), eps=3.0), [[-0.5, 0.5]], atol=1e-15)
    assert np.allclose(glue.add_layer_norm(h, -h + np.arange(64.0), one, zero, eps=0.0),
                       glue.layer_norm(np.tile(np.arange(64.0), (9, 1)), one, zero, eps=0.0), atol=1e-12)


def brute_attention(q, K, V, heads):
    M, d = q.shape
    S = K.shape[1]
    dh = d // heads
    out = [[0.0] * d for _ in range(M)]
    for m in range(M):
        for h in range(heads):
            sc = [sum(float(q[m, h * dh + j]) * float(K[m, s, h * dh + j]) for j in range(dh)) / math.sqrt(dh) for s in range(S)]
            mx = max(sc)
            w = [math.exp(v - mx) for v in sc]
            tot = sum(w)
            for j in range(dh):
                out[m][h * dh + j] = sum(w[s] / tot * float(V[m, s, h * dh + j]) for s in range(S))
    return np.array(out)


def test_cross_attention_brute_force_and_special_cases():
    rng = np.random.default_rng(4)
    q, K, V = rng.standard_normal((3, 8)), rng.standard_normal((3, 5, 8)), rng.standard_normal((3, 5, 8))
    assert np.allclose(glue.cross_attention(q, K, V, 2), brute_attention(q, K, V, 2), atol=1e-13)
    assert np.allclose(glue.cross_attention(q, K, V, 8), brute_attention(q, K, V, 8), atol=1e-13)
    # identical keys -> uniform weights -> the context is the mean of the values
    Kc = np.tile(K[:, :1, :], (1, 5, 1))
    assert np.allclose(glue.cross_attention(q, Kc, V, 2), V.mean(axis=1), atol=1e-13)
    # one source position: the context is its value whatever the query
    assert np.allclose(glue.cross_attention(q, K[:, :1], V[:, :1], 4), V[:, 0], atol=1e-15)
    # a key far along the query's direction takes all the weight
    Kb = K.copy()
    Kb[:, 3, :] = 200.0 * q
    assert np.allclose(glue.cross_attention(q, Kb, V, 1), V[:, 3], atol=1e-9)
    # heads do not mix: permuting whole heads of q, K, V permutes the context the same way
    perm = np.r_[4:8, 0:4]
    assert np.allclose(glue.cross_attention(q[:, perm], K[:, :, perm], V[:, :, perm], 2),
                       glue.cross_attention(q, K, V, 2)[:, perm], atol=1e-14)
    # adding a constant to all scores of a head (q orthogonal shift of keys) changes nothing: softmax is shift invariant
    with pytest.raises(ValueError):
        glue.cross_attention(q, K, V, 3)


def test_decoder_layer_variants_reduce_to_their_parts():
    c = workloads.config5_chained(M=6, layers=1, d=32, ffn=64, aan_ffn=48, S=4, V=50, t=5)
    P, (K, V) = c["layers"][0], c["KV"][0]
    x, gp = c["x0"], c["g_prev"][0]
    # without network and gate the averaging block is LN(g + x); rebuild the layer from the parts
    y, g = glue.aan_decoder_layer(x, gp, 5, P, K, V, heads=4, use_ffn=False, use_gate=False)
    g_ref = glue.running_average(gp, x, 5).astype(np.float32)
    assert np.array_equal(g, g_ref)
    y1 = glue.add_layer_norm(g_ref, x, P["ln1"]["gamma"], P["ln1"]["beta"]).astype(np.float32)
    from oracle import linear
    q = linear(y1, P["ctx_q"]["Wt"], 8, P["ctx_q"]["bias"])["Y"]
    o = linear(glue.cross_attention(q, K, V, 4).astype(np.float32), P["ctx_o"]["Wt"], 8, P["ctx_o"]["bias"])["Y"]
    y2 = glue.add_layer_norm(o, y1, P["ln2"]["gamma"], P["ln2"]["beta"]).astype(np.float32)
    h1 = linear(y2, P["ffn1"]["Wt"], 8, P["ffn1"]["bias"], True)["Y"]
    ff = linear(h1, P["ffn2"]["Wt"], 8, P["ffn2"]["bias"])["Y"]
    y3 = glue.add_layer_norm(ff, y2, P["ln3"]["gamma"], P["ln3"]["beta"]).astype(np.float32)
    assert np.array_equal(y, y3)
    # the full block differs from the reduced one (the network and the gate are really applied)
    yf, _ = glue.aan_decoder_layer(x, gp, 5, P, K, V, heads=4)
    assert not np.allclose(yf, y, atol=1e-3)
    # every row of a layer output is a layer-normalised vector: (y - beta) / gamma has mean 0, variance ~ 1
    zrow = (yf.astype(np.float64) - P["ln3"]["beta"]) / P["ln3"]["gamma"]
    assert np.allclose(zrow.mean(axis=1), 0, atol=1e-5) and np.allclose(zrow.var(axis=1), 1, atol=1e-3)


def hand_composed_layer(x, gp, t, P, K, V, heads, use_ffn=True, use_gate=True):
    """The decoder layer of reading R16 / R17 written out step by step from the single operations (each pinned above
    or in test_oracle_pins.py); returns every intermediate."""
    from oracle import linear
    f32 = lambda a: np.ascontiguousarray(a, dtype=np.float32)
    r = {}
    r["g"] = f32(glue.running_average(gp, x, t))
    r["f"] = r["g"]
    if use_ffn:
        r["h1"] = linear(r["g"], P["aan_ffn1"]["Wt"], 8, P["aan_ffn1"]["bias"], True)["Y"]
        r["f"] = linear(r["h1"], P["aan_ffn2"]["Wt"], 8, P["aan_ffn2"]["bias"])["Y"]
    if use_gate:
        r["cat"] = np.concatenate([f32(x), f32(r["f"])], axis=1)             # the layer input first, then the averaged path
        r["z"] = linear(r["cat"], P["aan_gate"]["Wt"], 8, P["aan_gate"]["bias"])["Y"]
        h = glue.gate_mix(x, r["f"], r["z"])
    else:
        h = r["f"].astype(np.float64)
    r["y1"] = f32(glue.add_layer_norm(h, x, P["ln1"]["gamma"], P["ln1"]["beta"]))
    r["q"] = linear(r["y1"], P["ctx_q"]["Wt"], 8, P["ctx_q"]["bias"])["Y"]
    r["ctx"] = f32(glue.cross_attention(r["q"], K, V, heads))
    r["o"] = linear(r["ctx"], P["ctx_o"]["Wt"], 8, P["ctx_o"]["bias"])["Y"]
    r["y2"] = f32(glue.add_layer_norm(r["o"], r["y1"], P["ln2"]["gamma"], P["ln2"]["beta"]))
    r["h2"] = linear(r["y2"], P["ffn1"]["Wt"], 8, P["ffn1"]["bias"], True)["Y"]
    r["ff"] = linear(r["h2"], P["ffn2"]["Wt"], 8, P["ffn2"]["bias"])["Y"]
    r["y3"] = f32(glue.add_layer_norm(r["ff"], r["y2"], P["ln3"]["gamma"], P["ln3"]["beta"]))
    return r


@pytest.mark.parametrize("use_ffn,use_gate", [(True, True), (False, True), (True, False), (False, False)])
def test_decoder_layer_equals_the_hand_composition_of_its_parts(use_ffn, use_gate):
    c = workloads.config5_chained(M=7, layers=1, d=32, ffn=64, aan_ffn=48, S=4, V=50, t=5, seed_extra=3)
    P, (K, V) = c["layers"][0], c["KV"][0]
    x, gp = c["x0"], c["g_prev"][0]
    y, g = glue.aan_decoder_layer(x, gp, 5, P, K, V, heads=4, use_ffn=use_ffn, use_gate=use_gate)
    r = hand_composed_layer(x, gp, 5, P, K, V, 4, use_ffn, use_gate)
    assert np.array_equal(g, r["g"]) and np.array_equal(y, r["y3"])


def planted_gate_case():
    """A layer whose inputs tell the pieces of the gate apart: every sentence has x[0] >= 0.5, the running average's
    first entry is positive too, and the averaging network's output has f[0] ~ -100 (planted in its last bias)."""
    c = workloads.config5_chained(M=9, layers=1, d=32, ffn=64, aan_ffn=48, S=4, V=50, t=5, seed_extra=11)
    P, (K, V) = c["layers"][0], c["KV"][0]
    x, gp = c["x0"].copy(), c["g_prev"][0].copy()
    x[:, 0] = np.abs(x[:, 0]) + np.float32(0.5)
    gp[:, 0] = np.abs(gp[:, 0]) + np.float32(0.5)
    P = {k: dict(v) for k, v in P.items()}
    b = P["aan_ffn2"]["bias"].copy()
    b[0] = -100.0
    P["aan_ffn2"]["bias"] = b
    return c, P, K, V, x, gp


def test_gate_halves_first_columns_gate_the_input_last_columns_the_averaged_path():
    # gate weights zero, biases saturating: z = bias.  (+50 | -50) opens the input's gate only: h = x, the layer is
    # LN(x + x) ..., which is the "-ffn -gate" layer at position 1 (there g = x).  (-50 | +50) opens the averaged
    # path's gate only: h = f, which is the "-gate" layer.  Exact: sigmoid(+-50) is 1 and 2e-22 in binary64.
    c, P, K, V, x, gp = planted_gate_case()
    d = 32
    Pz = dict(P)
    for first, second, same_as in ((50.0, -50.0, "x"), (-50.0, 50.0, "f")):
        Pz["aan_gate"] = {"Wt": np.zeros((2 * d, 2 * d), dtype=np.float32),
                          "bias": np.r_[np.full(d, first), np.full(d, second)].astype(np.float32)}
        y, _ = glue.aan_decoder_layer(x, gp, 5, Pz, K, V, heads=4)
        if same_as == "x":
            want, _ = glue.aan_decoder_layer(x, gp, 1, Pz, K, V, heads=4, use_ffn=False, use_gate=False)
        else:
            want, _ = glue.aan_decoder_layer(x, gp, 5, Pz, K, V, heads=4, use_gate=False)
        assert np.array_equal(y, want), same_as
    other, _ = glue.aan_decoder_layer(x, gp, 5, Pz, K, V, heads=4, use_ffn=False, use_gate=False)
    assert not np.allclose(y, other, atol=1e-3)          # h = f is not h = g


def test_gate_input_is_the_layer_input_followed_by_the_network_output():
    # The gate product reads [x ; f].  Weights on ONE input column, +1000 into every z1 and -1000 into every z2:
    # on column 0 (x[0] >= 0.5 in every sentence) the input's gate saturates open and the other one shut: h = x;
    # on column d (f[0] ~ -100) it is the other way round: h = f.  With the halves of the input swapped, or with
    # the running average g (g[0] > 0) in the place of f, each case would give the other case's result.
    c, P, K, V, x, gp = planted_gate_case()
    d = 32
    f0 = hand_composed_layer(x, gp, 5, P, K, V, 4)["f"][:, 0]
    assert np.all(f0 < -50) and np.all(glue.running_average(gp, x, 5)[:, 0] > 0)
    want_x, _ = glue.aan_decoder_layer(x, gp, 1, P, K, V, heads=4, use_ffn=False, use_gate=False)     # h = x
    want_f, _ = glue.aan_decoder_layer(x, gp, 5, P, K, V, heads=4, use_gate=False)                    # h = f
    assert not np.allclose(want_x, want_f, atol=1e-3)
    for col, want in ((0, want_x), (d, want_f)):
        Wt = np.zeros((2 * d, 2 * d), dtype=np.float32)
        Wt[:d, col] = 1000.0
        Wt[d:, col] = -1000.0
        Pg = dict(P)
        Pg["aan_gate"] = {"Wt": Wt, "bias": np.zeros(2 * d, dtype=np.float32)}
        y, _ = glue.aan_decoder_layer(x, gp, 5, Pg, K, V, heads=4)
        assert np.array_equal(y, want), col


def test_decode_step_chains_layers_and_picks_tokens():
    c = workloads.config5_chained(M=5, layers=2, d=32, ffn=64, aan_ffn=64, S=3, V=40, t=4)
    r = glue.decode_step(c["x0"], c["g_prev"], c["t"], c["layers"], c["KV"], c["E"], heads=4)
    x1, g0 = glue.aan_decoder_layer(c["x0"], c["g_prev"][0], 4, c["layers"][0], *c["KV"][0], heads=4)
    x2, g1 = glue.aan_decoder_layer(x1, c["g_prev"][1], 4, c["layers"][1], *c["KV"][1], heads=4)
    assert np.array_equal(r["hidden"], x2) and np.array_equal(r["g"][0], g0) and np.array_equal(r["g"][1], g1)
    from oracle import greedy_output_layer
    assert np.array_equal(r["tok"], greedy_output_layer(x2, c["E"])["tok"])
    assert r["tok"].shape == (5,) and r["tok"].min() >= 0 and r["tok"].max() < 40
