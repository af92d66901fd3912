"""Pins for the CPU oracle: each test checks an oracle function against
something other than the oracle -- hand-computed values, unbounded Python
integers, numpy library routines, closed forms and error bounds.  CPU only.

Citations are to arxiv 1805.12096: Section 4.2 (quantization, 32-bit sums),
Section 4.3 (dot'_int = A times B transposed), Section 2.3 (beam-1 arg-max
without softmax).
"""
import os

import numpy as np
import pytest

import oracle
import workloads


# ----------------------------------------------------------------- quant_int

def _golden_cases(golden_dir):
    cases = []
    with open(os.path.join(golden_dir, "quant_int_cases.txt")) as fh:
        for line in fh:
            line = line.split("#")[0].strip()
            if not line:
                continue
            bits, mult, expr, want = line.split()
            cases.append((int(bits), float(mult), float(eval(expr, {"__builtins__": {}})), int(want)))
    return cases


def test_quant_int_hand_cases(golden_dir):
    cases = _golden_cases(golden_dir)
    assert len(cases) >= 30
    for bits, mult, x, want in cases:
        got = oracle.quant_int(np.array([x], dtype=np.float32), bits, mult)
        assert got.dtype == (np.int8 if bits == 8 else np.int16)
        assert int(got[0]) == want, (bits, mult, x, want, int(got[0]))


@pytest.mark.parametrize("bits", [8, 16])
def test_quant_int_absmax_invariants(bits):
    rng = np.random.default_rng(11 + bits)
    x = (rng.standard_normal(20011, dtype=np.float32) * np.float32(0.37))
    amax = oracle.absmax(x)
    assert amax == float(np.max(np.abs(x)))          # numpy: independent routine
    s = oracle.scale_from_amax(amax, bits)
    assert s == np.float32(oracle.QMAX[bits]) / np.float32(amax)
    q = oracle.quant_int(x, bits, s)
    qm = oracle.QMAX[bits]
    assert int(np.max(np.abs(q.astype(np.int64)))) == qm  # extreme element hits +-Qmax
    i = int(np.argmax(np.abs(x)))
    assert int(q[i]) == (qm if x[i] > 0 else -qm)
    assert q.min() >= -qm                                  # -128 / -32768 never appear
    # rounding error at most half a step (plus the multiply's own rounding)
    t = x.astype(np.float64) * float(s)
    assert np.all(np.abs(q - t) <= 0.5 + 2.0 ** -22 * np.abs(t))
    # sign symmetry: quant(-x) == -quant(x)
    assert np.array_equal(oracle.quant_int(-x, bits, s), -q)


@pytest.mark.parametrize("bits,scale", [(8, 63.5), (8, 29.0), (16, 1024.0), (16, 777.25)])
def test_quant_int_against_numpy_rint(bits, scale):
    # numpy.rint on float32 is an independent implementation of round-half-even
    rng = np.random.default_rng(5)
    x = rng.standard_normal(50000, dtype=np.float32) * np.float32(3.0)
    # add exact ties
    ties = (np.arange(-300, 300, dtype=np.float32) + np.float32(0.5)) / np.float32(scale)
    x = np.concatenate([x, ties.astype(np.float32)])
    qm = oracle.QMAX[bits]
    want = np.clip(np.rint(x * np.float32(scale)), -qm, qm).astype(np.int64)
    got = oracle.quant_int(x, bits, scale).astype(np.int64)
    assert np.array_equal(got, want)


def test_quant_int_zero_tensor_and_nan():
    z = np.zeros(17, dtype=np.float32)
    assert oracle.absmax(z) == 0.0
    assert oracle.scale_from_amax(0.0, 8) == np.float32(1.0)
    assert not oracle.quant_int(z, 8, 1.0).any()
    x = np.array([1.0, np.nan, -3.0, np.nan], dtype=np.float32)
    assert oracle.absmax(x) == 3.0 and oracle.nan_count(x) == 2
    assert oracle.quant_int(x, 16, 2.0).tolist() == [2, 0, -6, 0]


def test_quant_int_rejects_other_widths():
    with pytest.raises((ValueError, KeyError)):
        oracle.quant_int(np.zeros(3, dtype=np.float32), 4, 1.0)


# ------------------------------------------------------------------ dot'_int

def _brute(qA, qB):
    """Unbounded Python integers, written out from the definition A . B^T."""
    M, K = qA.shape
    N = qB.shape[0]
    out = [[0] * N for _ in range(M)]
    for m in range(M):
        for n in range(N):
            s = 0
            for k in range(K):
                s += int(qA[m, k]) * int(qB[n, k])
            out[m][n] = s
    return out


def _wrap32(v: int) -> int:
    v &= 0xFFFFFFFF
    return v - (1 << 32) if v >= (1 << 31) else v


@pytest.mark.parametrize("dtype,M,N,K", [(np.int8, 3, 5, 7), (np.int8, 8, 2, 1), (np.int16, 4, 6, 5),
                                         (np.int16, 1, 7, 8), (np.int8, 5, 1, 3)])
def test_dot_int_brute_force_tiny(dtype, M, N, K):
    rng = np.random.default_rng(M * 100 + N * 10 + K)
    lim = 127 if dtype == np.int8 else 32767
    qA = rng.integers(-lim, lim + 1, size=(M, K)).astype(dtype)
    qB = rng.integers(-lim, lim + 1, size=(N, K)).astype(dtype)
    want = _brute(qA, qB)
    got, over = oracle.dot_int(qA, qB, return_overflow=True)
    assert got.shape == (M, N)
    n_over = 0
    for m in range(M):
        for n in range(N):
            assert int(got[m, n]) == _wrap32(want[m][n])
            n_over += want[m][n] != _wrap32(want[m][n])
    assert over == n_over


@pytest.mark.parametrize("dtype,M,N,K", [(np.int8, 37, 53, 129), (np.int16, 33, 29, 257), (np.int16, 16, 24, 1024)])
def test_dot_int_against_numpy_int64(dtype, M, N, K):
    rng = np.random.default_rng(K)
    lim = 127 if dtype == np.int8 else 32767
    qA = rng.integers(-lim, lim + 1, size=(M, K)).astype(dtype)
    qB = rng.integers(-lim, lim + 1, size=(N, K)).astype(dtype)
    exact = qA.astype(np.int64) @ qB.astype(np.int64).T
    want = (exact & 0xFFFFFFFF).astype(np.uint32).view(np.int32)
    got, over = oracle.dot_int(qA, qB, return_overflow=True)
    assert np.array_equal(got, want)
    assert over == int(np.count_nonzero(exact != want.astype(np.int64)))


def test_dot_int_closed_forms():
    # constant matrices: every entry is K*a*b
    for dtype, a, b, K in [(np.int8, 127, -127, 513), (np.int16, 1000, 37, 300), (np.int8, -5, -7, 1)]:
        qA = np.full((6, K), a, dtype=dtype)
        qB = np.full((9, K), b, dtype=dtype)
        assert np.all(oracle.dot_int(qA, qB) == K * a * b)
    # identity as B: A . I^T = A
    rng = np.random.default_rng(3)
    qA = rng.integers(-32767, 32768, size=(11, 13)).astype(np.int16)
    eye = np.eye(13, dtype=np.int16)
    assert np.array_equal(oracle.dot_int(qA, eye), qA.astype(np.int32))
    # a permutation matrix picks columns: catches a transposed B
    perm = np.zeros((13, 13), dtype=np.int16)
    order = rng.permutation(13)
    perm[np.arange(13), order] = 1          # row n of B selects column order[n] of A
    assert np.array_equal(oracle.dot_int(qA, perm), qA[:, order].astype(np.int32))
    # one-hot operands: acc[m, n] = A[m, kA] * B[n, kA]
    qB = rng.integers(-32767, 32768, size=(5, 13)).astype(np.int16)
    oneA = np.zeros((2, 13), dtype=np.int16)
    oneA[0, 4] = 3
    oneA[1, 9] = -2
    want = np.stack([3 * qB[:, 4].astype(np.int64), -2 * qB[:, 9].astype(np.int64)])
    assert np.array_equal(oracle.dot_int(oneA, qB), want.astype(np.int32))


def test_dot_int_overflow_wraps_modulo_2_32():
    # 32767^2 * 2 = 2 147 352 578 fits; * 3 = 3 221 028 867 wraps to -1 073 938 429
    for K, want, n_over in [(2, 2147352578, 0), (3, -1073938429, 1)]:
        qA = np.full((1, K), 32767, dtype=np.int16)
        qB = np.full((1, K), 32767, dtype=np.int16)
        got, over = oracle.dot_int(qA, qB, return_overflow=True)
        assert int(got[0, 0]) == want and over == n_over
    assert 32767 * 32767 * 3 - (1 << 32) == -1073938429
    # negative side
    qA = np.full((1, 3), -32767, dtype=np.int16)
    qB = np.full((1, 3), 32767, dtype=np.int16)
    assert int(oracle.dot_int(qA, qB)[0, 0]) == 1073938429
    # int8 can never overflow at these sizes: 127^2 * K < 2^31 for K <= 133 144
    assert 127 * 127 * 133144 < (1 << 31) <= 127 * 127 * 133145


def test_dot_int_k_split_associativity():
    # any split of the contracted range, each part wrapped, sums (mod 2^32) to the whole
    rng = np.random.default_rng(8)
    qA = rng.integers(-32767, 32768, size=(9, 700)).astype(np.int16)
    qB = rng.integers(-32767, 32768, size=(7, 700)).astype(np.int16)
    whole = oracle.dot_int(qA, qB)
    parts = [oracle.dot_int(qA[:, a:b], qB[:, a:b]) for a, b in [(0, 13), (13, 400), (400, 700)]]
    total = sum(p.astype(np.int64) for p in parts)
    assert np.array_equal((total & 0xFFFFFFFF).astype(np.uint32).view(np.int32), whole)


# ---------------------------------------------------------------- error bound

@pytest.mark.parametrize("bits,fixed", [(8, None), (16, 1024.0), (8, 63.5)])
def test_quantized_product_error_bound_vs_fp64(bits, fixed):
    # |sum a_k w_k - acc/(sA sW)| <= (0.5/sW)|a|_1 + (0.5/sA)|w|_1 + K/(4 sA sW)
    # for outputs that neither clipped nor overflowed.
    p = workloads.random_problem(21, 45, 70, 192, a_sigma=0.5, w_sigma=0.05)
    A, Wt = p["A"], p["Wt"]
    if fixed is not None and bits == 8:          # the paper's retrained models clip to [-2, 2]
        A = np.clip(A, -2, 2)
    r = oracle.linear(A, Wt, bits, sA=fixed, sW=fixed)
    assert r["overflow_count"] == 0
    sA, sW = float(r["sA"]), float(r["sW"])
    real = A.astype(np.float64) @ Wt.astype(np.float64).T
    approx = r["acc"].astype(np.float64) / (sA * sW)
    K = A.shape[1]
    bound = (0.5 / sW) * np.abs(A.astype(np.float64)).sum(1)[:, None] \
        + (0.5 / sA) * np.abs(Wt.astype(np.float64)).sum(1)[None, :] + K * 0.25 / (sA * sW)
    err = np.abs(real - approx)
    assert np.all(err <= bound * (1 + 1e-5) + 1e-12)
    # the bound is not vacuous: the error is a visible fraction of it, and int16 beats int8
    assert err.max() > 1e-3 * bound.max()
    if bits == 16:
        assert err.max() < 1e-2
    # dequantized outputs equal the approximation up to binary32 rounding
    assert np.allclose(r["Y"], approx, rtol=2e-6, atol=1e-9)


# ------------------------------------------------------------------- epilogue

def test_dequant_bias_relu_against_fp64():
    rng = np.random.default_rng(17)
    acc = rng.integers(-(1 << 23), 1 << 23, size=(31, 47)).astype(np.int32)   # exactly representable in binary32
    bias = (rng.standard_normal(47) * 0.1).astype(np.float32)
    sA, sW = np.float32(127 / 3.7), np.float32(127 / 0.21)
    u = 1.0 / (float(sA) * float(sW))
    ref = acc.astype(np.float64) * u + bias.astype(np.float64)
    y = oracle.dequant_bias(acc, sA, sW, bias, relu=False)
    tol = 1e-5 * np.maximum(np.abs(acc * u), np.abs(bias)) + 1e-30
    assert np.all(np.abs(y - ref) <= tol)
    yr = oracle.dequant_bias(acc, sA, sW, bias, relu=True)
    assert np.array_equal(yr, np.maximum(y, 0))
    assert not np.signbit(yr).any()                      # -0 never survives ReLU
    y0 = oracle.dequant_bias(acc, sA, sW, None, relu=False)
    assert np.all(np.abs(y0 - acc * u) <= 1e-6 * np.abs(acc * u) + 1e-30)
    # bias is indexed by column, not by row
    acc0 = np.zeros((3, 5), dtype=np.int32)
    b = np.arange(5, dtype=np.float32)
    assert np.array_equal(oracle.dequant_bias(acc0, 1.0, 1.0, b), np.tile(b, (3, 1)))


def test_dequant_is_single_rounding_fma():
    # acc*u + b with one rounding differs from two roundings on suitably chosen values;
    # an exactly rounded result must agree with the fp64 evaluation rounded once.
    rng = np.random.default_rng(23)
    acc = rng.integers(-(1 << 20), 1 << 20, size=(64, 64)).astype(np.int32)
    bias = rng.standard_normal(64).astype(np.float32)
    sA, sW = np.float32(64.0), np.float32(32.0)           # u = 2^-11 exactly
    y = oracle.dequant_bias(acc, sA, sW, bias)
    exact = acc.astype(np.float64) * 2.0 ** -11 + bias.astype(np.float64)  # exact in fp64
    assert np.array_equal(y, exact.astype(np.float32))    # one rounding, to nearest even


# -------------------------------------------------------------------- arg-max

def test_argmax_matches_numpy_and_planted_cases():
    rng = np.random.default_rng(29)
    acc = rng.integers(-50000, 50000, size=(23, 1031)).astype(np.int32)
    sA, sW = np.float32(40.0), np.float32(2500.0)
    tok, val = oracle.argmax_i32(acc, sA, sW)
    assert np.array_equal(tok, np.argmax(acc, axis=1))
    u = np.float32(1.0) / (sA * sW)
    assert np.array_equal(val, acc.max(1).astype(np.float32) * u)
    # planted ties: lowest index wins, wherever the duplicates sit
    acc2 = acc.copy()
    top = acc2.max() + 5
    acc2[3, [900, 17, 400]] = top
    acc2[4, [1030, 1029]] = top
    acc2[5, 0] = top
    tok2, _ = oracle.argmax_i32(acc2, sA, sW)
    assert tok2[3] == 17 and tok2[4] == 1029 and tok2[5] == 0
    # all-equal row -> index 0; most negative values still compare correctly
    acc3 = np.full((2, 9), np.iinfo(np.int32).min, dtype=np.int32)
    acc3[1, 8] = np.iinfo(np.int32).min + 1
    tok3, _ = oracle.argmax_i32(acc3, sA, sW)
    assert tok3.tolist() == [0, 8]


def test_greedy_output_layer_planted_winner_and_softmax_equivalence():
    c = workloads.config3(M=12, V=777, d=64, seed_extra=1)
    Hd, E = c["Hd"].copy(), c["E"].copy()
    # plant: embedding row j becomes hidden row m, rescaled so E's abs-max (and scale) is unchanged
    emax = np.abs(E).max()
    jstar = int(np.unravel_index(np.argmax(np.abs(E)), E.shape)[0])
    plants = {}
    for m, j in [(0, 5), (7, 700), (11, 776)]:
        assert j != jstar
        E[j] = Hd[m] * (emax / np.abs(Hd[m]).max()) * np.float32(0.999)
        plants[m] = j
    r = oracle.greedy_output_layer(Hd, E)
    for m, j in plants.items():
        assert r["tok"][m] == j
    # duplicate a winning row at a lower index: the lower index must win
    E2 = E.copy()
    E2[3] = E2[700]
    r2 = oracle.greedy_output_layer(Hd, E2)
    assert r2["tok"][7] == 3
    # skipping softmax does not change the winner: softmax is monotone
    logits = r["acc"].astype(np.float64) / (float(r["sA"]) * float(r["sW"]))
    soft = np.exp(logits - logits.max(1, keepdims=True))
    soft /= soft.sum(1, keepdims=True)
    assert np.array_equal(np.argmax(soft, axis=1), r["tok"])
    # against the unquantized fp64 product: any disagreement is a near-tie within the error bound
    real = Hd.astype(np.float64) @ E.astype(np.float64).T
    sA, sW = float(r["sA"]), float(r["sW"])
    bound = (0.5 / sW) * np.abs(Hd).sum(1).max() + (0.5 / sA) * np.abs(E).sum(1).max() + 64 * 0.25 / (sA * sW)
    ftok = np.argmax(real, axis=1)
    for m in np.nonzero(ftok != r["tok"])[0]:
        assert real[m, ftok[m]] - real[m, r["tok"][m]] <= 2 * bound


def test_argmax_f32_lowest_index():
    Y = np.array([[0.5, 2.0, 2.0, -1.0], [-3.0, -3.0, -4.0, -3.0]], dtype=np.float32)
    tok, val = oracle.argmax_f32(Y)
    assert tok.tolist() == [1, 0] and val.tolist() == [2.0, -3.0]


# ---------------------------------------------------------- composed pipeline

def test_linear_pipeline_config1_shape_and_overflow_fraction():
    # the full-range int16 workload overflows 32-bit sums in a visible fraction of
    # outputs (Section 4.2 explains why the paper keeps to 2^10); with the
    # paper's multiplier nothing overflows.
    c = workloads.config1()
    r = oracle.linear(c["A"], c["Wt"], 16, c["bias"])
    assert r["Y"].shape == (384, 512)
    frac = r["overflow_count"] / r["acc"].size
    assert 0.02 < frac < 0.2
    exact = r["qA"].astype(np.int64) @ r["qW"].astype(np.int64).T
    assert r["overflow_count"] == int(np.count_nonzero(np.abs(exact) >= 2 ** 31))
    r2 = oracle.linear(c["A"], c["Wt"], 16, c["bias"], sA=1024.0, sW=1024.0)
    assert r2["overflow_count"] == 0
    real = c["A"].astype(np.float64) @ c["Wt"].astype(np.float64).T + c["bias"]
    assert np.abs(r2["Y"] - real).max() < 0.05


def test_memoized_weight_equals_requantizing_every_call():
    # Section 4.3: quant_int(B^T) is a constant node; caching it must not change results
    c = workloads.config2(M=16)
    qW, sW = oracle.quant_int_absmax(c["W1t"], 8)
    outs = []
    for i in range(2):
        A = c["A"] * np.float32(1 + i)
        qA, sA = oracle.quant_int_absmax(A, 8)
        cached = oracle.dequant_bias(oracle.dot_int(qA, qW), sA, sW, c["b1"], True)
        fresh = oracle.linear(A, c["W1t"], 8, c["b1"], True)["Y"]
        assert np.array_equal(cached, fresh)
        outs.append(cached)
    # transposing before or after quantizing commutes for a per-tensor scale
    B = np.ascontiguousarray(c["W1t"].T)
    assert np.array_equal(oracle.quant_int(B, 8, sW).T, qW)


def test_shortlisted_output_layer_is_argmax_over_the_listed_rows():
    # Section 4.1: the output product restricted to a candidate subset.  Pinned against numpy on the
    # full logits: the winner among the listed ids is the masked arg-max of the full product.
    c = workloads.config3(M=9, V=500, d=32, seed_extra=4)
    full = oracle.greedy_output_layer(c["Hd"], c["E"])
    rng = np.random.default_rng(12)
    sl = np.sort(rng.choice(500, size=77, replace=False))
    r = oracle.greedy_output_layer(c["Hd"], c["E"], shortlist=sl)
    masked = np.full(full["acc"].shape, np.iinfo(np.int64).min, dtype=np.int64)
    masked[:, sl] = full["acc"][:, sl]
    assert np.array_equal(r["tok"], np.argmax(masked, axis=1))
    assert np.array_equal(r["maxlogit"], (masked.max(1).astype(np.float32) * (np.float32(1) / (r["sA"] * r["sW"]))))
    # the full vocabulary as a shortlist changes nothing; a one-entry list always returns that entry
    assert np.array_equal(oracle.greedy_output_layer(c["Hd"], c["E"], shortlist=np.arange(500))["tok"], full["tok"])
    assert np.all(oracle.greedy_output_layer(c["Hd"], c["E"], shortlist=[123])["tok"] == 123)
    # if the unrestricted winner is listed it stays the winner
    keep = np.unique(np.concatenate([sl, full["tok"]]))
    assert np.array_equal(oracle.greedy_output_layer(c["Hd"], c["E"], shortlist=keep)["tok"], full["tok"])
    with pytest.raises(ValueError):
        oracle.greedy_output_layer(c["Hd"], c["E"], shortlist=[5, 5, 7])


def test_topk_log_softmax_against_library_routines_and_special_cases():
    # Beam search with beam size k > 1 (Table 2, b = 2 / b = 4) needs the k best words with normalised
    # log-probabilities.  Pinned against scipy's log_softmax on the float product of the quantized integers,
    # against numpy's stable argsort, and by closed forms.
    from scipy.special import log_softmax
    c = workloads.config3(M=7, V=300, d=48, seed_extra=9)
    r = oracle.topk_log_softmax(c["Hd"], c["E"], 4)
    u = np.float32(1) / (r["sA"] * r["sW"])
    y = (r["acc"].astype(np.float32) * u).astype(np.float64)
    lp = log_softmax(y, axis=1)
    order = np.argsort(-r["acc"].astype(np.int64), axis=1, kind="stable")[:, :4]
    assert np.array_equal(r["tok"], order)
    assert np.allclose(r["logprob"], np.take_along_axis(lp, order, axis=1), rtol=0, atol=1e-12)
    # the best word is the greedy arg-max, log-probabilities descend, and all V of them sum to one
    assert np.array_equal(r["tok"][:, 0], oracle.greedy_output_layer(c["Hd"], c["E"])["tok"])
    assert np.all(np.diff(r["logprob"], axis=1) <= 0)
    full = oracle.topk_log_softmax(c["Hd"], c["E"], 300)
    assert np.allclose(np.exp(full["logprob"]).sum(axis=1), 1.0, atol=1e-12)
    assert np.array_equal(np.sort(full["tok"], axis=1), np.tile(np.arange(300), (7, 1)))
    # identical embedding rows: every word has probability 1 / V, ties go to the lowest indices in order
    E = np.tile(c["E"][:1], (16, 1))
    t = oracle.topk_log_softmax(c["Hd"], E, 3)
    assert np.array_equal(t["tok"], np.tile(np.arange(3), (7, 1)))
    assert np.allclose(t["logprob"], -np.log(16.0), atol=1e-12)
    # planted tie between a high and a low index
    E2 = c["E"].copy()
    E2[250] = E2[3]
    t2 = oracle.topk_log_softmax(c["Hd"], E2, 300)
    pos3 = np.argmax(t2["tok"] == 3, axis=1)
    pos250 = np.argmax(t2["tok"] == 250, axis=1)
    assert np.all(pos250 == pos3 + 1)
    with pytest.raises(ValueError):
        oracle.topk_log_softmax(c["Hd"], c["E"], 0)
