"""GPU parity: every stage of the HIP path against the CPU oracle on the same
seeded inputs, through the C boundary.  Integer results (quantized tensors,
32-bit sums, token ids) must match bit for bit; float outputs are produced by
the same single-FMA formula from the same integers and are expected to be
identical, with 1e-5 relative as the stated bar.
"""
import functools

import numpy as np
import pytest
import torch

import oracle
import workloads
import paper_1805_12096_amd as mq

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
QT = {8: torch.int8, 16: torch.int16}


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    assert torch.cuda.is_available(), "GPU tests need a GPU; there is no CPU fallback"
    mq.load_library()


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def host(t):
    torch.cuda.synchronize()
    return t.cpu().numpy()


def gpu_quantize(x, bits, scale=None, want_rowsum=False):
    """abs-max -> scale -> quant_int on the GPU; returns (q, scale, rowsum) device tensors."""
    xd = dev(x) if isinstance(x, np.ndarray) else x
    rows, cols = xd.shape
    s = torch.empty(1, dtype=torch.float32, device=DEV)
    if scale is None:
        mq.mq_absmax_f32(xd, xd.numel(), s)
        mq.mq_scale_from_amax(s, bits, s)
    else:
        s.fill_(float(scale))
    q = torch.empty((rows, cols), dtype=QT[bits], device=DEV)
    rs = torch.empty(rows, dtype=torch.int32, device=DEV) if (want_rowsum or bits == 16) else None
    mq.mq_quantize_f32(xd, rows, cols, bits, s, q, rs)
    return q, s, rs


def gpu_linear(A, Wt, bits, bias=None, relu=False, sA=None, sW=None, amax=False):
    pw = mq.prepare_weight(dev(Wt), bits, transposed=True,
                           scale=None if sW is None else torch.tensor([sW], dtype=torch.float32, device=DEV))
    q, s, rs = gpu_quantize(A, bits, sA)
    M, K = A.shape
    N = Wt.shape[0]
    C = torch.empty((M, N), dtype=torch.int32, device=DEV)
    mq.mq_gemm_i32(q, rs, pw.packed, bits, M, N, K, C)
    Y = torch.empty((M, N), dtype=torch.float32, device=DEV)
    am = torch.zeros(1, dtype=torch.float32, device=DEV) if amax else None
    mq.mq_gemm_dequant(q, rs, pw.packed, bits, M, N, K, s, pw.scale, None if bias is None else dev(bias),
                       relu, Y, am)
    qW = torch.empty((N, K), dtype=QT[bits], device=DEV)
    mq.mq_unpack_weight(pw.packed, bits, N, K, qW)
    return {"qA": host(q), "sA": host(s)[0], "sW": host(pw.scale)[0], "qW": host(qW), "acc": host(C),
            "Y": host(Y), "rowsum": None if rs is None else host(rs),
            "amax": None if am is None else host(am)[0]}


def assert_linear_matches(g, o):
    assert g["sA"] == o["sA"] and g["sW"] == o["sW"]
    assert np.array_equal(g["qA"], o["qA"])
    assert np.array_equal(g["qW"], o["qW"])
    assert np.array_equal(g["acc"], o["acc"])
    if g["rowsum"] is not None:
        assert np.array_equal(g["rowsum"], o["qA"].astype(np.int64).sum(1).astype(np.int32))
    tol = 1e-5 * np.abs(o["Y"]) + 1e-30
    assert np.all(np.abs(g["Y"] - o["Y"]) <= tol)
    assert np.array_equal(g["Y"], o["Y"]), "expected bit-identical float outputs"
    if g["amax"] is not None:
        assert g["amax"] == np.abs(o["Y"]).max()


# ------------------------------------------------------------------ quant_int

@pytest.mark.parametrize("bits", [8, 16])
@pytest.mark.parametrize("shape", [(1, 1), (3, 7), (5, 64), (17, 513), (300, 512), (64, 2048), (1, 100003)])
def test_absmax_scale_quantize(bits, shape):
    rng = np.random.default_rng(shape[0] * 7919 + shape[1] + bits)
    x = rng.standard_normal(shape, dtype=np.float32) * np.float32(0.7)
    for rowsum in (False, True):
        q, s, rs = gpu_quantize(x, bits, want_rowsum=rowsum)
        oq, os_ = oracle.quant_int_absmax(x, bits)
        assert host(s)[0] == os_
        assert np.array_equal(host(q), oq)
        if rs is not None:
            assert np.array_equal(host(rs), oq.astype(np.int64).sum(1).astype(np.int32))


def test_quantize_fixed_multipliers_ties_clip_and_nan():
    # the paper's multipliers: 2^10 for 16 bit, 127/2 for 8 bit after clipping to [-2, 2]
    ties16 = (np.arange(-4000, 4000, dtype=np.float32) + np.float32(0.5)) / np.float32(1024)
    big = np.array([31.99, 32.0, 40.0, -40.0, 1e30, -1e30, np.inf, -np.inf, np.nan, 0.0, -0.0], dtype=np.float32)
    x = np.concatenate([ties16, big])[None, :]
    for bits, scale in [(16, 1024.0), (8, 63.5), (8, 1.0), (16, 1.0)]:
        q, _, _ = gpu_quantize(x, bits, scale=scale)
        assert np.array_equal(host(q), oracle.quant_int(x, bits, scale))
    z = np.zeros((4, 33), dtype=np.float32)
    q, s, _ = gpu_quantize(z, 8)
    assert host(s)[0] == 1.0 and not host(q).any()
    xn = np.array([[1.0, np.nan, -3.0, 2.0]], dtype=np.float32)
    q, s, _ = gpu_quantize(xn, 16)
    assert host(s)[0] == oracle.scale_from_amax(oracle.absmax(xn), 16)
    assert np.array_equal(host(q), oracle.quant_int(xn, 16, host(s)[0]))


@pytest.mark.parametrize("bits", [8, 16])
@pytest.mark.parametrize("N,K", [(1, 1), (33, 65), (70, 50), (512, 512), (100, 1000)])
def test_prepare_weight_both_layouts_and_memoization(bits, N, K):
    rng = np.random.default_rng(N * 31 + K + bits)
    Wt = rng.standard_normal((N, K), dtype=np.float32) * np.float32(0.05)
    oq, os_ = oracle.quant_int_absmax(Wt, bits)
    pa = mq.prepare_weight(dev(Wt), bits, transposed=True)
    pb = mq.prepare_weight(dev(np.ascontiguousarray(Wt.T)), bits, transposed=False)
    pc = mq.prepare_weight(dev(Wt), bits, transposed=True)       # preparing again changes nothing
    assert host(pa.scale)[0] == os_ == host(pb.scale)[0]
    assert torch.equal(pa.packed, pb.packed) and torch.equal(pa.packed, pc.packed)
    q = torch.empty((N, K), dtype=QT[bits], device=DEV)
    mq.mq_unpack_weight(pa.packed, bits, N, K, q)
    assert np.array_equal(host(q), oq)
    if bits == 16:      # appended column sums
        Np = (N + 31) // 32 * 32
        cs = host(pa.packed)[-4 * Np:].view(np.int32)
        want = np.zeros(Np, dtype=np.int32)
        want[:N] = oq.astype(np.int64).sum(1)
        assert np.array_equal(cs, want)


# ------------------------------------------------------------------- dot'_int

def gpu_dot_int(qA, qB):
    """Exact integer operands through the GPU product: integers are fed as floats with multiplier 1."""
    bits = 8 if qA.dtype == np.int8 else 16
    one = torch.ones(1, dtype=torch.float32, device=DEV)
    pw = mq.prepare_weight(dev(qB.astype(np.float32)), bits, transposed=True, scale=one)
    qd = dev(qA)
    M, K = qA.shape
    N = qB.shape[0]
    rs = dev(qA.astype(np.int64).sum(1).astype(np.int32)) if bits == 16 else None
    C = torch.empty((M, N), dtype=torch.int32, device=DEV)
    mq.mq_gemm_i32(qd, rs, pw.packed, bits, M, N, K, C)
    return host(C)


SHAPES = [(1, 1, 1), (1, 5, 3), (7, 1, 16), (5, 3, 1), (32, 32, 32), (33, 31, 65), (64, 64, 64), (128, 128, 128),
          (129, 130, 80), (200, 260, 1000), (300, 70, 512), (45, 517, 96), (2, 1000, 2048)]


@pytest.mark.parametrize("dtype", [np.int8, np.int16])
@pytest.mark.parametrize("M,N,K", SHAPES)
def test_gemm_i32_full_range_integers(dtype, M, N, K):
    rng = np.random.default_rng(M * 1000003 + N * 1009 + K)
    lim = 127 if dtype == np.int8 else 32767
    qA = rng.integers(-lim, lim + 1, size=(M, K)).astype(dtype)
    qB = rng.integers(-lim, lim + 1, size=(N, K)).astype(dtype)
    want, over = oracle.dot_int(qA, qB, return_overflow=True)
    got = gpu_dot_int(qA, qB)
    assert np.array_equal(got, want)
    if dtype == np.int16 and K >= 512:
        assert over > 0          # the wrap-around path is really exercised


def test_gemm_i32_extremes_and_wrap():
    # all operands at +-32767: every sum wraps many times; int16 minimum -32768 as an A operand too
    for a, b, K in [(32767, 32767, 3), (32767, -32767, 4096), (-32768, 32767, 777), (-32768, -32767, 64)]:
        qA = np.full((40, K), a, dtype=np.int16)
        qB = np.full((37, K), b, dtype=np.int16)
        assert np.array_equal(gpu_dot_int(qA, qB), oracle.dot_int(qA, qB))
    qA = np.full((33, 100), -127, dtype=np.int8)
    qB = np.full((5, 100), 127, dtype=np.int8)
    assert np.all(gpu_dot_int(qA, qB) == -127 * 127 * 100)


def test_gemm_i32_one_hot_layout():
    # one non-zero per operand: exposes any mix-up of rows, columns or K slices
    for dtype in (np.int8, np.int16):
        M, N, K = 70, 90, 200
        for (m, n, k) in [(0, 0, 0), (69, 89, 199), (31, 32, 15), (32, 31, 16), (40, 64, 63), (5, 70, 64), (63, 33, 127)]:
            qA = np.zeros((M, K), dtype=dtype)
            qB = np.zeros((N, K), dtype=dtype)
            qA[m, k] = 3
            qB[n, k] = -5
            got = gpu_dot_int(qA, qB)
            want = np.zeros((M, N), dtype=np.int32)
            want[m, n] = -15
            assert np.array_equal(got, want), (dtype, m, n, k)


# ------------------------------------------------------------- fused epilogue

@pytest.mark.parametrize("bits", [8, 16])
@pytest.mark.parametrize("M,N,K,relu,bias", [(1, 1, 1, False, True), (37, 53, 129, True, True),
                                             (130, 200, 192, False, False), (300, 512, 512, True, True),
                                             (64, 96, 2048, False, True)])
def test_linear_pipeline(bits, M, N, K, relu, bias):
    p = workloads.random_problem(M + N + K + bits, M, N, K)
    b = p["bias"] if bias else None
    o = oracle.linear(p["A"], p["Wt"], bits, b, relu)
    g = gpu_linear(p["A"], p["Wt"], bits, b, relu, amax=True)
    assert_linear_matches(g, o)


def test_linear_paper_multipliers():
    # 16 bit with 2^10 on both operands (no overflow), 8 bit with 63.5 on inputs clipped to [-2, 2]
    p = workloads.random_problem(5, 100, 150, 512, a_sigma=1.0, w_sigma=0.05)
    o = oracle.linear(p["A"], p["Wt"], 16, p["bias"], False, sA=1024.0, sW=1024.0)
    assert o["overflow_count"] == 0
    assert_linear_matches(gpu_linear(p["A"], p["Wt"], 16, p["bias"], False, sA=1024.0, sW=1024.0), o)
    A, W = np.clip(p["A"], -2, 2), np.clip(p["Wt"] * 10, -2, 2)
    o = oracle.linear(A, W, 8, p["bias"], True, sA=63.5, sW=63.5)
    assert_linear_matches(gpu_linear(A, W, 8, p["bias"], True, sA=63.5, sW=63.5), o)


def test_mq_linear_f32_is_the_composition():
    for bits in (8, 16):
        p = workloads.random_problem(77 + bits, 90, 130, 256)
        o = oracle.linear(p["A"], p["Wt"], bits, p["bias"], True)
        pw = mq.prepare_weight(dev(p["Wt"]), bits)
        M, K = p["A"].shape
        N = p["Wt"].shape[0]
        nbytes = mq.mq_linear_ws_bytes(bits, M, K)
        ws = torch.empty(nbytes, dtype=torch.uint8, device=DEV)
        Y = torch.empty((M, N), dtype=torch.float32, device=DEV)
        am = torch.zeros(1, dtype=torch.float32, device=DEV)
        mq.mq_linear_f32(dev(p["A"]), M, K, None, pw.packed, pw.scale, bits, N, dev(p["bias"]), True, Y, am, ws, nbytes)
        assert np.array_equal(host(Y), o["Y"])
        assert host(am)[0] == o["Y"].max()


@pytest.mark.parametrize("M,N,K,relu,fixed", [(300, 2048, 512, True, False), (300, 512, 512, False, False),
                                              (300, 1024, 1024, False, False), (1, 1, 32, False, False),
                                              (33, 70, 96, True, False), (512, 100, 768, False, True),
                                              (300, 512, 2048, False, False), (77, 40, 100, True, False),
                                              (290, 333, 992, True, True)])
def test_mq_linear_f32_decode_sizes(M, N, K, relu, fixed):
    # few rows, 8 bit: quant_int runs inside the product kernel when K is a multiple of 32 up to 1024
    # (the other shapes here take the separate quantizer); either way the oracle's linear layer, bit for bit
    p = workloads.random_problem(M * 7 + N * 3 + K, M, N, K)
    A = np.clip(p["A"], -2, 2) if fixed else p["A"]
    o = oracle.linear(A, p["Wt"], 8, p["bias"], relu, sA=63.5 if fixed else None)
    pw = mq.prepare_weight(dev(p["Wt"]), 8)
    nbytes = mq.mq_linear_ws_bytes(8, M, K)
    ws = torch.full((nbytes,), 0x5A, dtype=torch.uint8, device=DEV)
    Y = torch.empty((M, N), dtype=torch.float32, device=DEV)
    am = torch.zeros(1, dtype=torch.float32, device=DEV)
    sA = torch.full((1,), 63.5, dtype=torch.float32, device=DEV) if fixed else None
    for bias in (dev(p["bias"]), None):
        want = o["Y"] if bias is not None else oracle.linear(A, p["Wt"], 8, None, relu, sA=63.5 if fixed else None)["Y"]
        am.zero_()
        mq.mq_linear_f32(dev(A), M, K, sA, pw.packed, pw.scale, 8, N, bias, relu, Y, am, ws, nbytes)
        assert np.array_equal(host(Y), want)
        assert host(am)[0] == np.abs(want).max()


def test_decode_sized_products_random_shapes():
    # seeded random shapes (rows <= 512, any width, K a multiple of 32 up to 1024): the in-kernel quantizer through
    # mq_linear_f32, and the split-K / loader-wave kernels forced through the packed entry point, against the oracle
    rng = np.random.default_rng(20241127)
    qws = torch.empty(mq.mq_quantize_absmax_ws_bytes(), dtype=torch.uint8, device=DEV)
    try:
        for it in range(12):
            M, N, K = int(rng.integers(1, 513)), int(rng.integers(1, 2500)), int(rng.integers(1, 33)) * 32
            relu, fixed = bool(rng.integers(0, 2)), bool(rng.integers(0, 2))
            p = workloads.random_problem(1000 + it, M, N, K)
            A = np.clip(p["A"], -2, 2) if fixed else p["A"]
            o = oracle.linear(A, p["Wt"], 8, p["bias"], relu, sA=63.5 if fixed else None)
            pw = mq.prepare_weight(dev(p["Wt"]), 8)
            nb = mq.mq_linear_ws_bytes(8, M, K)
            ws = torch.full((nb,), 0x77, dtype=torch.uint8, device=DEV)
            Y = torch.empty((M, N), dtype=torch.float32, device=DEV)
            am = torch.zeros(1, dtype=torch.float32, device=DEV)
            sA = torch.full((1,), 63.5, dtype=torch.float32, device=DEV) if fixed else None
            mq.mq_linear_f32(dev(A), M, K, sA, pw.packed, pw.scale, 8, N, dev(p["bias"]), relu, Y, am, ws, nb)
            assert np.array_equal(host(Y), o["Y"]), (M, N, K, relu, fixed)
            assert host(am)[0] == np.abs(o["Y"]).max()
            q = torch.empty(mq.mq_packed_bytes(8, M, K), dtype=torch.uint8, device=DEV)
            s = torch.empty(1, dtype=torch.float32, device=DEV)
            mq.mq_quantize_absmax_pack_f32(dev(p["A"]), M, K, 8, q, s, qws, qws.numel())
            o2 = oracle.linear(p["A"], p["Wt"], 8, p["bias"], relu)
            for v in (10, 11, 12, 13, 14):
                mq.mq_set_gemm_variant(v)
                mq.mq_gemm_dequant_packed(q, pw.packed, 8, M, N, K, s, pw.scale, dev(p["bias"]), relu, Y, None)
                assert np.array_equal(host(Y), o2["Y"]), (M, N, K, relu, v)
    finally:
        mq.mq_set_gemm_variant(0)


def test_mq_linear_f32_decode_sizes_special_values():
    # quant_int inside the product kernel: ties to even, clipping, infinities, NaN -> 0, an all-zero input
    M, N, K = 40, 48, 64
    rng = np.random.default_rng(4242)
    A = rng.standard_normal((M, K), dtype=np.float32)
    A[0, :8] = (np.arange(8, dtype=np.float32) + np.float32(0.5)) / np.float32(63.5)      # x * 63.5 = k + 0.5
    A[1, :6] = [np.inf, -np.inf, np.nan, 1e30, -1e30, -0.0]
    A[2, :] = 0.0
    Wt = rng.standard_normal((N, K), dtype=np.float32) * np.float32(0.05)
    bias = rng.standard_normal(N, dtype=np.float32) * np.float32(0.1)
    pw = mq.prepare_weight(dev(Wt), 8)
    nbytes = mq.mq_linear_ws_bytes(8, M, K)
    ws = torch.empty(nbytes, dtype=torch.uint8, device=DEV)
    Y = torch.empty((M, N), dtype=torch.float32, device=DEV)
    sA = torch.full((1,), 63.5, dtype=torch.float32, device=DEV)
    want = oracle.linear(A, Wt, 8, bias, False, sA=63.5)
    mq.mq_linear_f32(dev(A), M, K, sA, pw.packed, pw.scale, 8, N, dev(bias), False, Y, None, ws, nbytes)
    assert np.array_equal(host(Y), want["Y"])
    Z = np.zeros((M, K), dtype=np.float32)                     # abs-max of zeros: multiplier 1, output = bias
    mq.mq_linear_f32(dev(Z), M, K, None, pw.packed, pw.scale, 8, N, dev(bias), False, Y, None, ws, nbytes)
    assert np.array_equal(host(Y), oracle.linear(Z, Wt, 8, bias, False)["Y"])
    B = A.copy()
    B[1, :6] = [3.0, -3.0, np.nan, 2.5, -2.5, -0.0]            # abs-max skips the NaN
    mq.mq_linear_f32(dev(B), M, K, None, pw.packed, pw.scale, 8, N, dev(bias), False, Y, None, ws, nbytes)
    assert np.array_equal(host(Y), oracle.linear(B, Wt, 8, bias, False)["Y"])


# -------------------------------------------------------------------- arg-max

def gpu_greedy(Hd, E, pw=None):
    pw = pw or mq.prepare_weight(dev(E), 8)
    q, s, _ = gpu_quantize(Hd, 8)
    M, K = Hd.shape
    N = E.shape[0]
    nbytes = mq.mq_argmax_ws_bytes(M, N)
    ws = torch.full((nbytes,), 0xAB, dtype=torch.uint8, device=DEV)     # contents must not matter
    tok = torch.empty(M, dtype=torch.int32, device=DEV)
    val = torch.empty(M, dtype=torch.float32, device=DEV)
    mq.mq_gemm_argmax(q, pw.packed, M, N, K, s, pw.scale, tok, val, ws, nbytes)
    return host(tok), host(val)


# 70 000 words are more units per workgroup than the pipeline holds stages: the loop that refills slots
@pytest.mark.parametrize("M,V,d", [(1, 1, 1), (3, 17, 8), (12, 777, 64), (33, 4100, 96), (300, 3000, 512), (130, 129, 512),
                                   (20, 70000, 64), (40, 150001, 32)])
def test_greedy_output_layer_small(M, V, d):
    c = workloads.config3(M=M, V=V, d=d, seed_extra=M + V)
    o = oracle.greedy_output_layer(c["Hd"], c["E"])
    tok, val = gpu_greedy(c["Hd"], c["E"])
    assert np.array_equal(tok, o["tok"])
    assert np.array_equal(val, o["maxlogit"])


def test_greedy_planted_winner_and_ties():
    c = workloads.config3(M=40, V=2085, d=128, seed_extra=9)
    Hd, E = c["Hd"].copy(), c["E"].copy()
    emax = np.abs(E).max()
    for m, j in [(0, 2084), (7, 5), (39, 1024)]:
        E[j] = Hd[m] * (emax / np.abs(Hd[m]).max()) * np.float32(0.999)
    # duplicates across different tiles and lanes: the lowest index has to win
    E[3] = E[1024]
    E[2080] = E[1024]
    E[1] = E[2084]
    o = oracle.greedy_output_layer(Hd, E)
    assert o["tok"][0] == 1 and o["tok"][7] == 5 and o["tok"][39] == 3
    tok, val = gpu_greedy(Hd, E)
    assert np.array_equal(tok, o["tok"]) and np.array_equal(val, o["maxlogit"])
    # all-equal logits (zero hidden state): index 0 everywhere
    tok, val = gpu_greedy(np.zeros((5, 128), dtype=np.float32), E)
    assert not tok.any() and not val.any()
    # all-negative rows: padding columns (zeros) must never win
    Hneg = np.abs(Hd[:4])
    Eneg = -np.abs(E[:70])           # 70 columns: 58 padded candidates in the last tile
    o = oracle.greedy_output_layer(Hneg, Eneg)
    assert (o["acc"] < 0).all()
    tok, val = gpu_greedy(Hneg, Eneg)
    assert np.array_equal(tok, o["tok"]) and np.array_equal(val, o["maxlogit"])


# ------------------------------------------------ benchmark workloads, full size

def test_config1_int16_single_product():
    c = workloads.config1()
    o = oracle.linear(c["A"], c["Wt"], 16, c["bias"])
    assert o["overflow_count"] > 0
    assert_linear_matches(gpu_linear(c["A"], c["Wt"], 16, c["bias"]), o)


def gpu_ffn(c, bits):
    """The launch sequence bench.py times: quantize, product+ReLU+abs-max, re-quantize, product."""
    A = dev(c["A"])
    M, d = A.shape
    f = c["W1t"].shape[0]
    p1 = mq.prepare_weight(dev(c["W1t"]), bits)
    p2 = mq.prepare_weight(dev(c["W2t"]), bits)
    b1, b2 = dev(c["b1"]), dev(c["b2"])
    s1 = torch.empty(1, dtype=torch.float32, device=DEV)
    mq.mq_absmax_f32(A, A.numel(), s1)
    mq.mq_scale_from_amax(s1, bits, s1)
    p_q1 = torch.empty(mq.mq_packed_bytes(bits, M, d), dtype=torch.uint8, device=DEV)
    mq.mq_quantize_pack_f32(A, M, d, bits, s1, p_q1)
    H = torch.empty((M, f), dtype=torch.float32, device=DEV)
    hmax = torch.zeros(1, dtype=torch.float32, device=DEV)
    mq.mq_gemm_dequant_packed(p_q1, p1.packed, bits, M, f, d, s1, p1.scale, b1, True, H, hmax)
    s2 = torch.empty(1, dtype=torch.float32, device=DEV)
    mq.mq_scale_from_amax(hmax, bits, s2)
    p_q2 = torch.empty(mq.mq_packed_bytes(bits, M, f), dtype=torch.uint8, device=DEV)
    mq.mq_quantize_pack_f32(H, M, f, bits, s2, p_q2)
    Y = torch.empty((M, d), dtype=torch.float32, device=DEV)
    mq.mq_gemm_dequant_packed(p_q2, p2.packed, bits, M, d, f, s2, p2.scale, b2, False, Y, None)
    # plain row-major views of the packed activations, for comparison with the oracle
    q1 = torch.empty((M, d), dtype=QT[bits], device=DEV)
    q2 = torch.empty((M, f), dtype=QT[bits], device=DEV)
    mq.mq_unpack_weight(p_q1, bits, M, d, q1)
    mq.mq_unpack_weight(p_q2, bits, M, f, q2)
    return {"q1": q1, "H": H, "s2": s2, "q2": q2, "Y": Y}


@functools.lru_cache(maxsize=None)
def oracle_ffn_full(cfg):
    """The oracle's whole FFN chain on ALL token rows of config 2 / config 4 (every value, the intermediate's
    multiplier included, comes from the oracle alone); computed once per test session."""
    bits = 8 if cfg == 2 else 16
    c = (workloads.config2 if cfg == 2 else workloads.config4)()
    o1 = oracle.linear(c["A"], c["W1t"], bits, c["b1"], True)
    s2 = oracle.scale_from_amax(oracle.absmax(o1["Y"]), bits)
    o2 = oracle.linear(o1["Y"], c["W2t"], bits, c["b2"], False, sA=s2)
    return c, o1, s2, o2


def oracle_ffn_rows(c, bits, rows, sA, s2):
    """Oracle on a subset of token rows, given the two per-tensor multipliers."""
    A = c["A"][rows]
    o1 = oracle.linear(A, c["W1t"], bits, c["b1"], True, sA=sA)
    o2 = oracle.linear(o1["Y"], c["W2t"], bits, c["b2"], False, sA=s2)
    return o1, o2


@pytest.mark.parametrize("cfg,bits", [(2, 8), (4, 16)])
def test_ffn_reduced_rows_full_chain(cfg, bits):
    c = (workloads.config2 if cfg == 2 else workloads.config4)(M=320)
    g = gpu_ffn(c, bits)
    o1 = oracle.linear(c["A"], c["W1t"], bits, c["b1"], True)
    s2 = oracle.scale_from_amax(oracle.absmax(o1["Y"]), bits)
    o2 = oracle.linear(o1["Y"], c["W2t"], bits, c["b2"], False, sA=s2)
    assert np.array_equal(host(g["q1"]), o1["qA"])
    assert np.array_equal(host(g["H"]), o1["Y"])
    assert host(g["s2"])[0] == s2
    assert np.array_equal(host(g["q2"]), o2["qA"])
    assert np.array_equal(host(g["Y"]), o2["Y"])


@pytest.mark.parametrize("cfg,bits", [(2, 8), (4, 16)])
def test_ffn_full_size_all_rows(cfg, bits):
    # M = 8192 as benchmarked, call by call; the oracle recomputes the whole chain on every token row and
    # supplies the intermediate's multiplier itself.
    c, o1, s2, o2 = oracle_ffn_full(cfg)
    g = gpu_ffn(c, bits)
    assert host(g["s2"])[0] == s2
    assert np.array_equal(host(g["q1"]), o1["qA"])
    assert np.array_equal(host(g["H"]), o1["Y"])
    assert np.array_equal(host(g["q2"]), o2["qA"])
    assert np.array_equal(host(g["Y"]), o2["Y"])


def test_config3_output_layer_full():
    c = workloads.config3()
    o = oracle.greedy_output_layer(c["Hd"], c["E"])
    tok, val = gpu_greedy(c["Hd"], c["E"])
    assert np.array_equal(tok, o["tok"])
    assert np.array_equal(val, o["maxlogit"])


def test_config5_decode_step_products():
    c = workloads.config5(layers=2)     # two of the six identical layers keep the oracle to seconds
    for g in c["gemms"]:
        o = oracle.linear(g["A"], g["Wt"], 8, g["bias"], g["relu"])
        r = gpu_linear(g["A"], g["Wt"], 8, g["bias"], g["relu"])
        assert np.array_equal(r["Y"], o["Y"]), g["name"]
    out = c["output"]
    o = oracle.greedy_output_layer(out["Hd"], out["E"])
    tok, val = gpu_greedy(out["Hd"], out["E"])
    assert np.array_equal(tok, o["tok"]) and np.array_equal(val, o["maxlogit"])


# ------------------------------------------- packed activations + packed product

def gpu_quantize_pack(x, bits, scale=None):
    xd = dev(x)
    rows, cols = xd.shape
    s = torch.empty(1, dtype=torch.float32, device=DEV)
    if scale is None:
        mq.mq_absmax_f32(xd, xd.numel(), s)
        mq.mq_scale_from_amax(s, bits, s)
    else:
        s.fill_(float(scale))
    packed = torch.full((mq.mq_packed_bytes(bits, rows, cols),), 0x5A, dtype=torch.uint8, device=DEV)
    mq.mq_quantize_pack_f32(xd, rows, cols, bits, s, packed)
    return packed, s


@pytest.mark.parametrize("bits", [8, 16])
@pytest.mark.parametrize("shape", [(1, 1), (3, 7), (33, 65), (300, 512), (70, 2048), (257, 100), (8, 4099)])
def test_quantize_pack_matches_oracle(bits, shape):
    rng = np.random.default_rng(shape[0] * 131 + shape[1] + bits)
    x = rng.standard_normal(shape, dtype=np.float32) * np.float32(1.3)
    packed, s = gpu_quantize_pack(x, bits)
    oq, os_ = oracle.quant_int_absmax(x, bits)
    assert host(s)[0] == os_
    q = torch.empty(shape, dtype=QT[bits], device=DEV)
    mq.mq_unpack_weight(packed, bits, shape[0], shape[1], q)
    assert np.array_equal(host(q), oq)
    if bits == 16:
        Mp = (shape[0] + 31) // 32 * 32
        sums = host(packed)[-4 * Mp:].view(np.int32)
        assert np.array_equal(sums[:shape[0]], oq.astype(np.int64).sum(1).astype(np.int32))


def gpu_dot_int_packed(qA, qB):
    bits = 8 if qA.dtype == np.int8 else 16
    one = torch.ones(1, dtype=torch.float32, device=DEV)
    pw = mq.prepare_weight(dev(qB.astype(np.float32)), bits, transposed=True, scale=one)
    pa, _ = gpu_quantize_pack(qA.astype(np.float32), bits, scale=1.0)
    M, K = qA.shape
    N = qB.shape[0]
    C = torch.empty((M, N), dtype=torch.int32, device=DEV)
    mq.mq_gemm_i32_packed(pa, pw.packed, bits, M, N, K, C)
    return host(C)


PACKED_VARIANTS = {8: [0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12, 13, 14], 16: [0, 1, 2, 3, 4, 5, 6, 7, 8]}


@pytest.mark.parametrize("dtype", [np.int8, np.int16])
@pytest.mark.parametrize("M,N,K", [(1, 1, 1), (33, 31, 65), (129, 130, 80), (300, 70, 512), (260, 517, 96),
                                   (2, 1000, 2048), (513, 258, 320), (300, 64, 4100), (70, 40, 9000),
                                   (320, 1030, 1024)])
def test_gemm_packed_full_range_all_variants(dtype, M, N, K):
    rng = np.random.default_rng(M * 1000003 + N * 1009 + K + 1)
    lim = 127 if dtype == np.int8 else 32767
    qA = rng.integers(-lim, lim + 1, size=(M, K)).astype(dtype)
    qB = rng.integers(-lim, lim + 1, size=(N, K)).astype(dtype)
    want = oracle.dot_int(qA, qB)
    try:
        for v in PACKED_VARIANTS[8 if dtype == np.int8 else 16]:
            mq.mq_set_gemm_variant(v)
            assert np.array_equal(gpu_dot_int_packed(qA, qB), want), f"variant {v}"
    finally:
        mq.mq_set_gemm_variant(0)


@pytest.mark.parametrize("dtype", [np.int8, np.int16])
@pytest.mark.parametrize("K", [129, 192, 256, 320, 384, 448, 576, 640])
def test_gemm_packed_pipeline_boundaries_all_variants(dtype, K):
    # 3 to 10 K steps of 64: around every variant's ring depth (3, 4, 6 or 8 stages), where the main loop changes from
    # "everything issued by the prologue" to one peeled step to the steady loop
    M, N = 150, 140
    rng = np.random.default_rng(K * 7919 + (8 if dtype == np.int8 else 16))
    lim = 127 if dtype == np.int8 else 32767
    qA = rng.integers(-lim, lim + 1, size=(M, K)).astype(dtype)
    qB = rng.integers(-lim, lim + 1, size=(N, K)).astype(dtype)
    want = oracle.dot_int(qA, qB)
    try:
        for v in PACKED_VARIANTS[8 if dtype == np.int8 else 16]:
            mq.mq_set_gemm_variant(v)
            assert np.array_equal(gpu_dot_int_packed(qA, qB), want), f"variant {v}"
    finally:
        mq.mq_set_gemm_variant(0)


@pytest.mark.parametrize("M,N,K,relu", [(1, 1, 1, False), (37, 53, 64, True), (384, 512, 512, False), (130, 260, 1100, True)])
def test_int16_vector_alu_product_matches_oracle(M, N, K, relu):
    # variant 7 of the 16-bit packed products: the 16-bit dot instruction on the vector ALU instead of four 8-bit
    # matrix products.  Raw sums on full-range integers (runs of the extreme values planted, so that a pair of
    # products reaches 2 x 32767^2 and the sums wrap), then the dequantizing epilogue with bias, ReLU and the
    # abs-max by-product.
    rng = np.random.default_rng(M * 31 + N * 7 + K)
    qA = rng.integers(-32767, 32768, size=(M, K)).astype(np.int16)
    qB = rng.integers(-32767, 32768, size=(N, K)).astype(np.int16)
    qA[0, : min(K, 6)] = -32767
    qB[0, : min(K, 6)] = -32767
    qA[-1, -1], qB[-1, -1] = 32767, -32767
    p = workloads.random_problem(M + N + K + 7, M, N, K)
    o = oracle.linear(p["A"], p["Wt"], 16, p["bias"], relu)
    pw = mq.prepare_weight(dev(p["Wt"]), 16)
    pa, s = gpu_quantize_pack(p["A"], 16)
    Y = torch.empty((M, N), dtype=torch.float32, device=DEV)
    am = torch.zeros(1, dtype=torch.float32, device=DEV)
    try:
        mq.mq_set_gemm_variant(7)
        assert np.array_equal(gpu_dot_int_packed(qA, qB), oracle.dot_int(qA, qB))
        mq.mq_gemm_dequant_packed(pa, pw.packed, 16, M, N, K, s, pw.scale, dev(p["bias"]), relu, Y, am)
    finally:
        mq.mq_set_gemm_variant(0)
    assert np.array_equal(host(Y), o["Y"])
    assert host(am)[0] == np.abs(o["Y"]).max()


@pytest.mark.parametrize("M,N,K,relu,with_bias", [(4200, 2100, 200, True, True), (4097, 2049, 128, False, False),
                                                  (8200, 1100, 130, True, True), (300, 140, 1100, False, True),
                                                  (2100, 4200, 64, True, True)])
def test_int16_product_walking_through_several_tiles_matches_oracle(M, N, K, relu, with_bias):
    # variant 8 of the 16-bit packed products: one workgroup per compute unit that takes its tiles one after the other
    # and loads across tile boundaries.  The first three shapes have more 256 x 128 tiles than the chip has compute
    # units (289, 289 and 297, ragged in both directions), so workgroups take two tiles, with 4, 2 and 3 K steps per
    # tile (2 = the ring's look-ahead: every step of a tile already loads the next tile); then the one-tile case, and
    # a single K step, which the tile kernel takes over.
    rng = np.random.default_rng(M * 31 + N * 7 + K)
    qA = rng.integers(-32767, 32768, size=(M, K)).astype(np.int16)
    qB = rng.integers(-32767, 32768, size=(N, K)).astype(np.int16)
    qA[0, : min(K, 6)] = -32767
    qB[0, : min(K, 6)] = -32767
    qA[-1, -1], qB[-1, -1] = 32767, -32767
    p = workloads.random_problem(M + N + K + 8, M, N, K)
    bias = p["bias"] if with_bias else None
    o = oracle.linear(p["A"], p["Wt"], 16, bias, relu)
    pw = mq.prepare_weight(dev(p["Wt"]), 16)
    pa, s = gpu_quantize_pack(p["A"], 16)
    Y = torch.empty((M, N), dtype=torch.float32, device=DEV)
    am = torch.zeros(1, dtype=torch.float32, device=DEV)
    try:
        mq.mq_set_gemm_variant(8)
        assert np.array_equal(gpu_dot_int_packed(qA, qB), oracle.dot_int(qA, qB))
        mq.mq_gemm_dequant_packed(pa, pw.packed, 16, M, N, K, s, pw.scale, dev(bias) if with_bias else None, relu, Y, am)
    finally:
        mq.mq_set_gemm_variant(0)
    assert np.array_equal(host(Y), o["Y"])
    assert host(am)[0] == np.abs(o["Y"]).max()


def _seeded_shapes():
    rng = np.random.default_rng(2024)
    out = [(int(rng.integers(1, 1500)), int(rng.integers(1, 1500)), int(rng.integers(1, 700))) for _ in range(6)]
    out += [(int(rng.integers(3900, 4600)), int(rng.integers(2050, 2300)), int(rng.integers(65, 400))) for _ in range(4)]
    out += [(int(rng.integers(8100, 8300)), int(rng.integers(2050, 2200)), int(rng.integers(65, 200))) for _ in range(2)]
    return out


@pytest.mark.parametrize("idx,shape", list(enumerate(_seeded_shapes())))
def test_int16_walking_product_seeded_shapes(idx, shape):
    # variant 8 on shapes drawn from a seeded generator (ragged in every direction; the last six have more tiles than
    # compute units), through the library's own quantizer: 32-bit sums, dequantized outputs and max|y| against the oracle
    M, N, K = shape
    p = workloads.random_problem(1000 + idx, M, N, K)
    relu, with_bias = bool(idx % 2), idx % 3 != 0
    bias = p["bias"] if with_bias else None
    o = oracle.linear(p["A"], p["Wt"], 16, bias, relu)
    pw = mq.prepare_weight(dev(p["Wt"]), 16)
    pa, s = gpu_quantize_pack(p["A"], 16)
    Y = torch.empty((M, N), dtype=torch.float32, device=DEV)
    C = torch.empty((M, N), dtype=torch.int32, device=DEV)
    am = torch.zeros(1, dtype=torch.float32, device=DEV)
    try:
        mq.mq_set_gemm_variant(8)
        mq.mq_gemm_i32_packed(pa, pw.packed, 16, M, N, K, C)
        mq.mq_gemm_dequant_packed(pa, pw.packed, 16, M, N, K, s, pw.scale, dev(bias) if with_bias else None, relu, Y, am)
    finally:
        mq.mq_set_gemm_variant(0)
    assert np.array_equal(host(C), o["acc"])
    assert np.array_equal(host(Y), o["Y"])
    assert host(am)[0] == np.abs(o["Y"]).max()


def test_gemm_packed_one_hot_layout():
    # one non-zero per operand: checks where the direct-to-LDS copy puts each lane's bytes
    for dtype in (np.int8, np.int16):
        M, N, K = 70, 90, 200
        for (m, n, k) in [(0, 0, 0), (69, 89, 199), (31, 32, 15), (32, 31, 16), (40, 64, 63), (5, 70, 64), (63, 33, 127)]:
            qA = np.zeros((M, K), dtype=dtype)
            qB = np.zeros((N, K), dtype=dtype)
            qA[m, k] = 3
            qB[n, k] = -5
            want = np.zeros((M, N), dtype=np.int32)
            want[m, n] = -15
            assert np.array_equal(gpu_dot_int_packed(qA, qB), want), (dtype, m, n, k)


@pytest.mark.parametrize("M,N,K,relu", [(37, 53, 64, True), (300, 200, 320, False), (513, 258, 448, True),
                                        (1000, 130, 2048, False), (129, 512, 4100, True)])
def test_linear_pipeline_packed_k_split_over_wave_groups(M, N, K, relu):
    # variant 14: an odd number of 64-element K steps leaves the second wave group's last step empty; the
    # dequantizing epilogue with bias, ReLU and the abs-max by-product runs on the first group only
    p = workloads.random_problem(M + N + K + 14, M, N, K)
    o = oracle.linear(p["A"], p["Wt"], 8, p["bias"], relu)
    pw = mq.prepare_weight(dev(p["Wt"]), 8)
    pa, s = gpu_quantize_pack(p["A"], 8)
    Y = torch.empty((M, N), dtype=torch.float32, device=DEV)
    am = torch.zeros(1, dtype=torch.float32, device=DEV)
    try:
        mq.mq_set_gemm_variant(14)
        mq.mq_gemm_dequant_packed(pa, pw.packed, 8, M, N, K, s, pw.scale, dev(p["bias"]), relu, Y, am)
    finally:
        mq.mq_set_gemm_variant(0)
    assert np.array_equal(host(Y), o["Y"])
    assert host(am)[0] == np.abs(o["Y"]).max()


@pytest.mark.parametrize("bits", [8, 16])
@pytest.mark.parametrize("M,N,K,relu", [(37, 53, 129, True), (300, 512, 512, True), (520, 300, 1024, False)])
def test_linear_pipeline_packed(bits, M, N, K, relu):
    p = workloads.random_problem(M + N + K + bits + 3, M, N, K)
    o = oracle.linear(p["A"], p["Wt"], bits, p["bias"], relu)
    pw = mq.prepare_weight(dev(p["Wt"]), bits)
    pa, s = gpu_quantize_pack(p["A"], bits)
    Y = torch.empty((M, N), dtype=torch.float32, device=DEV)
    am = torch.zeros(1, dtype=torch.float32, device=DEV)
    mq.mq_gemm_dequant_packed(pa, pw.packed, bits, M, N, K, s, pw.scale, dev(p["bias"]), relu, Y, am)
    assert np.array_equal(host(Y), o["Y"])
    assert host(am)[0] == np.abs(o["Y"]).max()


# ------------------------------------------------ decode-step arg-max kernel

def gpu_greedy_packed(Hd, E):
    pw = mq.prepare_weight(dev(E), 8)
    pa, s = gpu_quantize_pack(Hd, 8)
    M, K = Hd.shape
    N = E.shape[0]
    nbytes = mq.mq_argmax_ws_bytes(M, N)
    ws = torch.full((nbytes,), 0xCD, dtype=torch.uint8, device=DEV)     # contents must not matter
    tok = torch.full((M,), -7, dtype=torch.int32, device=DEV)
    val = torch.empty(M, dtype=torch.float32, device=DEV)
    mq.mq_gemm_argmax_packed(pa, pw.packed, M, N, K, s, pw.scale, tok, val, ws, nbytes)
    return host(tok), host(val)


@pytest.mark.parametrize("M,V,d", [(1, 1, 1), (3, 17, 8), (12, 777, 64), (33, 4100, 96), (130, 129, 512), (300, 3000, 512),
                                   (384, 9000, 192), (97, 20000, 128), (257, 33, 300), (320, 5000, 448),
                                   (261, 40000, 512)])
def test_greedy_packed_small(M, V, d):
    c = workloads.config3(M=M, V=V, d=d, seed_extra=M + V + 5)
    o = oracle.greedy_output_layer(c["Hd"], c["E"])
    tok, val = gpu_greedy_packed(c["Hd"], c["E"])
    assert np.array_equal(tok, o["tok"])
    assert np.array_equal(val, o["maxlogit"])


def test_greedy_packed_ties_padding_and_limits():
    c = workloads.config3(M=40, V=9000, d=128, seed_extra=11)
    Hd, E = c["Hd"].copy(), c["E"].copy()
    emax = np.abs(E).max()
    for m, j in [(0, 8999), (7, 5), (39, 4096)]:
        E[j] = Hd[m] * (emax / np.abs(Hd[m]).max()) * np.float32(0.999)
    E[3] = E[4096]          # duplicates in other vocabulary blocks, handled by other workgroups
    E[8990] = E[4096]
    E[1] = E[8999]
    o = oracle.greedy_output_layer(Hd, E)
    assert o["tok"][0] == 1 and o["tok"][7] == 5 and o["tok"][39] == 3
    tok, val = gpu_greedy_packed(Hd, E)
    assert np.array_equal(tok, o["tok"]) and np.array_equal(val, o["maxlogit"])
    tok, val = gpu_greedy_packed(np.zeros((5, 128), dtype=np.float32), E)
    assert not tok.any() and not val.any()
    Hneg, Eneg = np.abs(Hd[:4]), -np.abs(E[:70])      # all sums negative: zero padding must never win
    o = oracle.greedy_output_layer(Hneg, Eneg)
    tok, val = gpu_greedy_packed(Hneg, Eneg)
    assert np.array_equal(tok, o["tok"]) and np.array_equal(val, o["maxlogit"])
    # beyond the kernel's limits the call refuses instead of computing something else
    # (K = 576 > 512: the 32-bit keys of the streaming kernel could no longer hold the sums)
    wide = np.zeros((64, 576), dtype=np.float32)
    pw = mq.prepare_weight(dev(wide), 8)
    pa, s = gpu_quantize_pack(np.zeros((5, 576), dtype=np.float32), 8)
    nbytes = mq.mq_argmax_ws_bytes(5, 64)
    ws = torch.empty(nbytes, dtype=torch.uint8, device=DEV)
    tok_t = torch.empty(5, dtype=torch.int32, device=DEV)
    val_t = torch.empty(5, dtype=torch.float32, device=DEV)
    with pytest.raises(mq.MqError) as e:
        mq.mq_gemm_argmax_packed(pa, pw.packed, 5, 64, 576, s, pw.scale, tok_t, val_t, ws, nbytes)
    assert e.value.status == 6


def test_config3_output_layer_full_packed():
    c = workloads.config3()
    o = oracle.greedy_output_layer(c["Hd"], c["E"])
    tok, val = gpu_greedy_packed(c["Hd"], c["E"])
    assert np.array_equal(tok, o["tok"])
    assert np.array_equal(val, o["maxlogit"])


def test_greedy_packed_more_rows_than_one_pass_holds():
    # 1000 rows: three passes of 384 rows each stream the embedding
    c = workloads.config3(M=1000, V=5000, d=128, seed_extra=11)
    o = oracle.greedy_output_layer(c["Hd"], c["E"])
    tok, val = gpu_greedy_packed(c["Hd"], c["E"])
    assert np.array_equal(tok, o["tok"])
    assert np.array_equal(val, o["maxlogit"])


# ----------------------------------------------------------- fused FFN (8 bit)

def gpu_ffn_fused(c):
    A = dev(c["A"])
    M, d = A.shape
    f = c["W1t"].shape[0]
    p1 = mq.prepare_weight(dev(c["W1t"]), 8)
    p2 = mq.prepare_weight(dev(c["W2t"]), 8)
    nbytes = mq.mq_ffn_ws_bytes(M, d, f)
    ws = torch.full((nbytes,), 0x3C, dtype=torch.uint8, device=DEV)     # contents must not matter
    Y = torch.empty((M, d), dtype=torch.float32, device=DEV)
    mq.mq_ffn_i8_f32(A, M, d, f, p1.packed, p1.scale, dev(c["b1"]), p2.packed, p2.scale, dev(c["b2"]), Y, ws, nbytes)
    return host(Y)


@pytest.mark.parametrize("M,d,f", [(1, 1, 1), (37, 64, 200), (320, 512, 2048), (130, 96, 100), (513, 256, 384)])
def test_ffn_fused_matches_oracle_chain(M, d, f):
    c = workloads.ffn(2, M, d, f, 0.04, 8, seed_extra=M + d + f)
    o1 = oracle.linear(c["A"], c["W1t"], 8, c["b1"], True)
    s2 = oracle.scale_from_amax(oracle.absmax(o1["Y"]), 8)
    o2 = oracle.linear(o1["Y"], c["W2t"], 8, c["b2"], False, sA=s2)
    for v in (0, 1, 3, 4, 5, 7):
        try:
            mq.mq_set_gemm_variant(v)
            assert np.array_equal(gpu_ffn_fused(c), o2["Y"]), f"variant {v}"
        finally:
            mq.mq_set_gemm_variant(0)


@pytest.mark.parametrize("M,d,f", [(37, 64, 200), (700, 128, 600), (4352, 64, 4096)])
def test_ffn_single_pass_and_two_pass_agree_with_oracle(M, d, f):
    # The intermediate's multiplier needs max|H| over the whole tensor: one launch with a grid-wide
    # barrier when every tile is resident at once, two passes otherwise (the last shape has 272
    # tiles of 256 x 256, more than the chip holds).  Repeated calls reuse the workspace's counter.
    c = workloads.ffn(2, M, d, f, 0.04, 8, seed_extra=M + 2 * d + f)
    o1 = oracle.linear(c["A"], c["W1t"], 8, c["b1"], True)
    s2 = oracle.scale_from_amax(oracle.absmax(o1["Y"]), 8)
    o2 = oracle.linear(o1["Y"], c["W2t"], 8, c["b2"], False, sA=s2)
    try:
        for single in (1, 0, 1, 1):
            mq.mq_set_ffn_single_pass(single)
            assert np.array_equal(gpu_ffn_fused(c), o2["Y"]), f"single_pass={single}"
    finally:
        mq.mq_set_ffn_single_pass(1)


@pytest.mark.parametrize("M,d,f", [(1, 1, 1), (37, 64, 200), (300, 256, 520), (2100, 512, 96)])
def test_ffn_int16_one_call_matches_oracle_chain(M, d, f):
    c = workloads.ffn(4, M, d, f, 0.03, 16, seed_extra=M + d + 3 * f)
    o1 = oracle.linear(c["A"], c["W1t"], 16, c["b1"], True)
    s2 = oracle.scale_from_amax(oracle.absmax(o1["Y"]), 16)
    o2 = oracle.linear(o1["Y"], c["W2t"], 16, c["b2"], False, sA=s2)
    A = dev(c["A"])
    p1 = mq.prepare_weight(dev(c["W1t"]), 16)
    p2 = mq.prepare_weight(dev(c["W2t"]), 16)
    nbytes = mq.mq_ffn_i16_ws_bytes(M, d, f)
    ws = torch.full((nbytes,), 0x3C, dtype=torch.uint8, device=DEV)     # contents must not matter
    for _ in range(2):
        Y = torch.empty((M, d), dtype=torch.float32, device=DEV)
        mq.mq_ffn_i16_f32(A, M, d, f, p1.packed, p1.scale, dev(c["b1"]), p2.packed, p2.scale, dev(c["b2"]), Y, ws,
                          nbytes)
        assert np.array_equal(host(Y), o2["Y"])


def test_ffn_fused_full_size_equals_oracle_on_all_rows():
    # the one-call int8 block at M = 8192 against the oracle's whole chain, every row
    c, _, _, o2 = oracle_ffn_full(2)
    assert np.array_equal(gpu_ffn_fused(c), o2["Y"])


def test_ffn_int16_one_call_full_size_equals_oracle_on_all_rows():
    # mq_ffn_i16_f32 at the benchmark's 8192 x 1024 x 4096 against the oracle's whole chain, every row
    c, _, _, o2 = oracle_ffn_full(4)
    M, d = c["A"].shape
    f = c["W1t"].shape[0]
    p1 = mq.prepare_weight(dev(c["W1t"]), 16)
    p2 = mq.prepare_weight(dev(c["W2t"]), 16)
    nbytes = mq.mq_ffn_i16_ws_bytes(M, d, f)
    ws = torch.full((nbytes,), 0x3C, dtype=torch.uint8, device=DEV)
    Y = torch.empty((M, d), dtype=torch.float32, device=DEV)
    mq.mq_ffn_i16_f32(dev(c["A"]), M, d, f, p1.packed, p1.scale, dev(c["b1"]), p2.packed, p2.scale, dev(c["b2"]), Y, ws,
                      nbytes)
    assert np.array_equal(host(Y), o2["Y"])


def capture_graph(fn, reps):
    """HIP graph of `reps` consecutive calls of fn, captured the way bench.py does it."""
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        fn()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        for _ in range(reps):
            fn()
    return g


def test_ffn_block_replayed_as_a_graph_of_several_steps():
    # the launch configuration bench.py times: graphs of consecutive mq_ffn_i8_f32 calls at config 2's size.
    # Every replay (with eager work of the program's own and synchronizations in between, and a different input
    # each time) must give the eager call's bits; the eager result is pinned to the oracle on sampled rows.
    c = workloads.config2()
    M, d = c["A"].shape
    f = c["W1t"].shape[0]
    p1 = mq.prepare_weight(dev(c["W1t"]), 8)
    p2 = mq.prepare_weight(dev(c["W2t"]), 8)
    b1, b2 = dev(c["b1"]), dev(c["b2"])
    nbytes = mq.mq_ffn_ws_bytes(M, d, f)
    ws = torch.full((nbytes,), 0x3C, dtype=torch.uint8, device=DEV)
    A = dev(c["A"])
    Y = torch.empty((M, d), dtype=torch.float32, device=DEV)

    def step():
        mq.mq_ffn_i8_f32(A, M, d, f, p1.packed, p1.scale, b1, p2.packed, p2.scale, b2, Y, ws, nbytes)

    g = capture_graph(step, 3)
    base = dev(c["A"])
    for r, factor in enumerate((1.0, 0.5, -1.25, 1.0)):
        A.copy_(base * factor)                       # eager work between the replays
        step()
        torch.cuda.synchronize()
        want = Y.clone()
        Y.fill_(float("nan"))
        ws.fill_(0xA7 + r)                           # the workspace's contents must not matter either
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(Y, want), f"replay {r}"
    _, _, _, o2 = oracle_ffn_full(2)               # the last replay ran on the unscaled input
    assert np.array_equal(host(Y), o2["Y"])


@pytest.mark.parametrize("M,d,f", [(1, 1, 1), (37, 64, 200), (320, 512, 2048), (2048, 512, 2048), (2048, 512, 16384),
                                   (2100, 512, 300), (8192, 512, 2048)])
def test_ffn_block_on_a_prepared_workspace(M, d, f):
    # mq_ffn_ws_prepare once, then calls that leave the agreement words as they found them: repeated calls with
    # changing inputs, the plain entry point mixed in, both switch positions of the single-pass kernels.  The
    # sizes cover: nothing single-pass (small), single-pass product only, both single-pass kernels (the last
    # ones), and a first product too large for one launch behind a single-pass quantizer (f = 16384).
    c = workloads.ffn(2, M, d, f, 0.04, 8, seed_extra=M + d + f + 5)
    p1 = mq.prepare_weight(dev(c["W1t"]), 8)
    p2 = mq.prepare_weight(dev(c["W2t"]), 8)
    b1, b2 = dev(c["b1"]), dev(c["b2"])
    nbytes = mq.mq_ffn_ws_bytes(M, d, f)
    ws = torch.full((nbytes,), 0x5B, dtype=torch.uint8, device=DEV)
    ws_plain = torch.full((nbytes,), 0x11, dtype=torch.uint8, device=DEV)
    Y = torch.empty((M, d), dtype=torch.float32, device=DEV)
    W = torch.empty((M, d), dtype=torch.float32, device=DEV)
    base = dev(c["A"])
    A = base.clone()
    mq.mq_ffn_ws_prepare(ws, nbytes, M, d, f)
    try:
        for r, (factor, kind) in enumerate([(1.0, "p"), (0.5, "p"), (-2.0, "plain"), (3.0, "p"), (1.0, "off"), (0.25, "p"),
                                            (1.0, "p")]):
            A.copy_(base * factor)
            mq.mq_ffn_i8_f32(A, M, d, f, p1.packed, p1.scale, b1, p2.packed, p2.scale, b2, W, ws_plain, nbytes)
            Y.fill_(float("nan"))
            if kind == "plain":        # the plain entry point on the prepared workspace: leaves it prepared
                mq.mq_ffn_i8_f32(A, M, d, f, p1.packed, p1.scale, b1, p2.packed, p2.scale, b2, Y, ws, nbytes)
            else:
                mq.mq_set_ffn_single_pass(0 if kind == "off" else 1)
                mq.mq_ffn_i8_f32_prepared(A, M, d, f, p1.packed, p1.scale, b1, p2.packed, p2.scale, b2, Y, ws, nbytes)
                mq.mq_set_ffn_single_pass(1)
            torch.cuda.synchronize()
            assert torch.equal(Y, W), f"call {r} ({kind})"
    finally:
        mq.mq_set_ffn_single_pass(1)
    # the last call ran on the unscaled input: pin it to the oracle's whole chain, every row, at every size
    o1 = oracle.linear(c["A"], c["W1t"], 8, c["b1"], True)
    s2 = oracle.scale_from_amax(oracle.absmax(o1["Y"]), 8)
    o2 = oracle.linear(o1["Y"], c["W2t"], 8, c["b2"], False, sA=s2)
    assert np.array_equal(host(Y), o2["Y"])


def test_ffn_block_on_a_prepared_workspace_replayed_as_a_graph():
    c = workloads.config2()
    M, d = c["A"].shape
    f = c["W1t"].shape[0]
    p1 = mq.prepare_weight(dev(c["W1t"]), 8)
    p2 = mq.prepare_weight(dev(c["W2t"]), 8)
    b1, b2 = dev(c["b1"]), dev(c["b2"])
    nbytes = mq.mq_ffn_ws_bytes(M, d, f)
    ws = torch.full((nbytes,), 0x3C, dtype=torch.uint8, device=DEV)
    ws_plain = torch.full((nbytes,), 0x3C, dtype=torch.uint8, device=DEV)
    A = dev(c["A"])
    Y = torch.empty((M, d), dtype=torch.float32, device=DEV)
    mq.mq_ffn_ws_prepare(ws, nbytes, M, d, f)

    def step():
        mq.mq_ffn_i8_f32_prepared(A, M, d, f, p1.packed, p1.scale, b1, p2.packed, p2.scale, b2, Y, ws, nbytes)

    g = capture_graph(step, 3)          # three consecutive blocks per replay: each relies on what the one before left
    base = dev(c["A"])
    for r, factor in enumerate((1.0, 0.5, -1.25, 1.0)):
        A.copy_(base * factor)           # eager work between the replays
        mq.mq_ffn_i8_f32(A, M, d, f, p1.packed, p1.scale, b1, p2.packed, p2.scale, b2, Y, ws_plain, nbytes)
        torch.cuda.synchronize()
        want = Y.clone()
        Y.fill_(float("nan"))
        g.replay()
        if r == 1:
            step()                       # an eager prepared call between replays
        torch.cuda.synchronize()
        assert torch.equal(Y, want), f"replay {r}"


@pytest.mark.parametrize("bits", [8, 16])
@pytest.mark.parametrize("shape", [(1, 1), (33, 65), (300, 512), (300, 2048), (2000, 1024), (8192, 512), (70, 1030),
                                   (17000, 96), (384, 512), (48, 4096), (1000, 700), (8192, 1024)])
def test_quantize_absmax_pack(bits, shape):
    # Tensors that fit the registers of one resident grid are read once (the last shapes do not fit and take
    # the two-pass form anyway); with the switch off it is always two passes.  Both forms must give the
    # oracle's integers and multiplier and the same bytes, padding and appended row sums included.  Each
    # form is called twice on one workspace whose contents do not matter.
    rng = np.random.default_rng(shape[0] + shape[1] * 3 + bits)
    x = rng.standard_normal(shape, dtype=np.float32) * np.float32(0.3)
    oq, os_ = oracle.quant_int_absmax(x, bits)
    nb = mq.mq_quantize_absmax_ws_bytes()
    ws = torch.full((nb,), 0x7F, dtype=torch.uint8, device=DEV)
    outs = []
    try:
        for single in (2, 0, 2, 1):
            mq.mq_set_quantize_single_pass(single)
            s = torch.empty(1, dtype=torch.float32, device=DEV)
            packed = torch.full((mq.mq_packed_bytes(bits, *shape),), 0x5A, dtype=torch.uint8, device=DEV)
            mq.mq_quantize_absmax_pack_f32(dev(x), shape[0], shape[1], bits, packed, s, ws, nb)
            q = torch.empty(shape, dtype=QT[bits], device=DEV)
            mq.mq_unpack_weight(packed, bits, shape[0], shape[1], q)
            assert host(s)[0] == os_ and np.array_equal(host(q), oq)
            outs.append(packed)
    finally:
        mq.mq_set_quantize_single_pass(1)
    for o in outs[1:]:
        assert torch.equal(o, outs[0])


@pytest.mark.parametrize("bits", [8, 16])
@pytest.mark.parametrize("shape", [(1, 1), (33, 65), (300, 512), (300, 2048), (2000, 1024), (8192, 512), (70, 1030),
                                   (17000, 96)])
def test_quantize_absmax_pack_on_a_prepared_workspace(bits, shape):
    # the workspace's agreement words are zeroed once; every call leaves them zero (the kernel that reads x once
    # cleans up after itself, the two-pass form never touches them): five calls in a row with changing inputs,
    # with the one-kernel form switched off in between, then three replays of a graph of two calls
    rng = np.random.default_rng(shape[0] * 7 + shape[1] + bits)
    base = rng.standard_normal(shape, dtype=np.float32) * np.float32(0.3)
    nb = mq.mq_quantize_absmax_ws_bytes()
    ws = torch.full((nb,), 0x6D, dtype=torch.uint8, device=DEV)
    ws_plain = torch.full((nb,), 0x6D, dtype=torch.uint8, device=DEV)
    mq.mq_quantize_absmax_ws_prepare(ws, nb)
    x = dev(base)
    s = torch.empty(1, dtype=torch.float32, device=DEV)
    s_plain = torch.empty(1, dtype=torch.float32, device=DEV)
    packed = torch.empty(mq.mq_packed_bytes(bits, *shape), dtype=torch.uint8, device=DEV)
    packed_plain = torch.empty_like(packed)

    def call():
        mq.mq_quantize_absmax_pack_f32_prepared(x, shape[0], shape[1], bits, packed, s, ws, nb)

    def check(tag):
        mq.mq_quantize_absmax_pack_f32(x, shape[0], shape[1], bits, packed_plain, s_plain, ws_plain, nb)
        torch.cuda.synchronize()
        assert torch.equal(s, s_plain) and torch.equal(packed, packed_plain), tag

    try:
        for r, (factor, single) in enumerate([(1.0, 1), (0.5, 1), (-3.0, 0), (2.0, 1), (1.0, 1)]):
            x.copy_(dev(base) * factor)
            packed.fill_(0x5A)
            mq.mq_set_quantize_single_pass(single)
            call()
            mq.mq_set_quantize_single_pass(1)
            check(f"call {r}")
    finally:
        mq.mq_set_quantize_single_pass(1)
    oq, os_ = oracle.quant_int_absmax(base, bits)
    q = torch.empty(shape, dtype=QT[bits], device=DEV)
    mq.mq_unpack_weight(packed, bits, shape[0], shape[1], q)
    assert host(s)[0] == os_ and np.array_equal(host(q), oq)
    g = capture_graph(call, 2)
    for r, factor in enumerate((0.75, -1.5, 1.0)):
        x.copy_(dev(base) * factor)
        packed.fill_(0x33)
        g.replay()
        check(f"replay {r}")


def test_prepared_quantizer_cleans_up_after_a_timed_out_agreement():
    # every workgroup gives up at once: the multiplier is NaN, all kernels end, and since the workgroups still count
    # themselves out the last one leaves the agreement words zero: the next call is right without preparing again
    shape = (2000, 1024)
    rng = np.random.default_rng(99)
    xh = rng.standard_normal(shape, dtype=np.float32)
    oq, os_ = oracle.quant_int_absmax(xh, 8)
    nb = mq.mq_quantize_absmax_ws_bytes()
    ws = torch.full((nb,), 0x42, dtype=torch.uint8, device=DEV)
    mq.mq_quantize_absmax_ws_prepare(ws, nb)
    x = dev(xh)
    s = torch.empty(1, dtype=torch.float32, device=DEV)
    packed = torch.empty(mq.mq_packed_bytes(8, *shape), dtype=torch.uint8, device=DEV)
    try:
        mq.mq_set_barrier_timeout_us(0)
        mq.mq_quantize_absmax_pack_f32_prepared(x, shape[0], shape[1], 8, packed, s, ws, nb)
        assert np.isnan(host(s)[0])
    finally:
        mq.mq_set_barrier_timeout_us(500000)
    assert not ws[: 4 * (8 * 256 + 64)].any().item()
    for _ in range(2):
        mq.mq_quantize_absmax_pack_f32_prepared(x, shape[0], shape[1], 8, packed, s, ws, nb)
        q = torch.empty(shape, dtype=torch.int8, device=DEV)
        mq.mq_unpack_weight(packed, 8, shape[0], shape[1], q)
        assert host(s)[0] == os_ and np.array_equal(host(q), oq)


def test_quantize_absmax_pack_skips_nan_and_handles_zero_tensor():
    x = np.zeros((40, 70), dtype=np.float32)
    nb = mq.mq_quantize_absmax_ws_bytes()
    ws = torch.empty(nb, dtype=torch.uint8, device=DEV)
    s = torch.empty(1, dtype=torch.float32, device=DEV)
    packed = torch.empty(mq.mq_packed_bytes(8, 40, 70), dtype=torch.uint8, device=DEV)
    mq.mq_quantize_absmax_pack_f32(dev(x), 40, 70, 8, packed, s, ws, nb)
    assert host(s)[0] == 1.0
    x[3, 5] = np.nan
    x[7, 9] = -2.5
    oq, os_ = oracle.quant_int_absmax(x, 8)
    mq.mq_quantize_absmax_pack_f32(dev(x), 40, 70, 8, packed, s, ws, nb)
    q = torch.empty((40, 70), dtype=torch.int8, device=DEV)
    mq.mq_unpack_weight(packed, 8, 40, 70, q)
    assert host(s)[0] == os_ and np.array_equal(host(q), oq)


def test_two_pass_requantizing_product():
    p = workloads.random_problem(404, 300, 520, 256)
    o = oracle.linear(p["A"], p["Wt"], 8, p["bias"], True)
    os2 = oracle.scale_from_amax(oracle.absmax(o["Y"]), 8)
    oq = oracle.quant_int(o["Y"], 8, os2)
    M, K = p["A"].shape
    N = p["Wt"].shape[0]
    pw = mq.prepare_weight(dev(p["Wt"]), 8)
    pa, s = gpu_quantize_pack(p["A"], 8)
    nb = mq.mq_gemm_amax_ws_bytes(M, N)
    ws = torch.full((nb,), 0x11, dtype=torch.uint8, device=DEV)
    bias = dev(p["bias"])
    s2 = torch.empty(1, dtype=torch.float32, device=DEV)
    out = torch.full((mq.mq_packed_bytes(8, M, N),), 0x22, dtype=torch.uint8, device=DEV)
    mq.mq_gemm_amax_packed(pa, pw.packed, M, N, K, s, pw.scale, bias, True, ws, nb)
    mq.mq_gemm_requant_packed(pa, pw.packed, M, N, K, s, pw.scale, bias, True, ws, nb, s2, out)
    q = torch.empty((M, N), dtype=torch.int8, device=DEV)
    mq.mq_unpack_weight(out, 8, M, N, q)
    assert host(s2)[0] == os2
    assert np.array_equal(host(q), oq)
    # padding of the packed output is zero: a prepared copy of the same integers has identical bytes
    ref = mq.prepare_weight(dev(oq.astype(np.float32)), 8, scale=torch.ones(1, dtype=torch.float32, device=DEV))
    assert torch.equal(out, ref.packed)


@pytest.mark.parametrize("shape", [(1, 1, 1), (300, 520, 256), (1000, 1100, 128), (512, 768, 192), (256, 256, 64)])
def test_single_pass_requantizing_product(shape):
    # one pass over the operands, the sums waiting in registers while the grid agrees on max|y|;
    # called twice on one workspace (it clears its two words itself)
    M, N, K = shape
    p = workloads.random_problem(405 + M, M, N, K)
    o = oracle.linear(p["A"], p["Wt"], 8, p["bias"], True)
    os2 = oracle.scale_from_amax(oracle.absmax(o["Y"]), 8)
    oq = oracle.quant_int(o["Y"], 8, os2)
    pw = mq.prepare_weight(dev(p["Wt"]), 8)
    pa, s = gpu_quantize_pack(p["A"], 8)
    nb = mq.mq_gemm_amax_ws_bytes(M, N)
    ws = torch.full((nb,), 0xA5, dtype=torch.uint8, device=DEV)
    bias = dev(p["bias"])
    ref = mq.prepare_weight(dev(oq.astype(np.float32)), 8, scale=torch.ones(1, dtype=torch.float32, device=DEV))
    for _ in range(2):
        s2 = torch.empty(1, dtype=torch.float32, device=DEV)
        out = torch.full((mq.mq_packed_bytes(8, M, N),), 0x22, dtype=torch.uint8, device=DEV)
        mq.mq_gemm_requant_single_packed(pa, pw.packed, M, N, K, s, pw.scale, bias, True, ws, nb, s2, out)
        assert host(s2)[0] == os2
        assert torch.equal(out, ref.packed)


@pytest.mark.parametrize("shape", [(512, 768, 192), (300, 520, 256)])
def test_single_pass_requantizing_product_special_bias(shape):
    # whole tiles + ReLU take the kernel whose re-quantization is a single rounding addition per element;
    # a NaN bias (ReLU turns it into 0) and an infinite one (max = inf, multiplier 0, every output 0)
    # must come out as the clamp-and-NaN rule gives them.  The second shape takes the general kernel.
    M, N, K = shape
    p = workloads.random_problem(911 + M, M, N, K)
    pw = mq.prepare_weight(dev(p["Wt"]), 8)
    pa, s = gpu_quantize_pack(p["A"], 8)
    nb = mq.mq_gemm_amax_ws_bytes(M, N)
    ws = torch.full((nb,), 0xA5, dtype=torch.uint8, device=DEV)
    for special in (np.nan, np.inf):
        bias = p["bias"].copy()
        bias[N // 3] = special
        o = oracle.linear(p["A"], p["Wt"], 8, bias, True)
        os2 = oracle.scale_from_amax(oracle.absmax(o["Y"]), 8)
        oq = oracle.quant_int(o["Y"], 8, os2)
        ref = mq.prepare_weight(dev(oq.astype(np.float32)), 8, scale=torch.ones(1, dtype=torch.float32, device=DEV))
        s2 = torch.empty(1, dtype=torch.float32, device=DEV)
        out = torch.full((mq.mq_packed_bytes(8, M, N),), 0x22, dtype=torch.uint8, device=DEV)
        mq.mq_gemm_requant_single_packed(pa, pw.packed, M, N, K, s, pw.scale, dev(bias), True, ws, nb, s2, out)
        assert host(s2)[0] == os2
        assert torch.equal(out, ref.packed)


def test_single_pass_barrier_timeout_is_loud_and_recoverable():
    # With a zero time limit every workgroup that has to wait gives up at once: all kernels still end,
    # the output's multiplier is NaN (and so is everything a caller computes from it), and the next
    # call with the normal limit is correct again on the same workspace.
    c = workloads.ffn(2, 1000, 128, 1100, 0.04, 8, seed_extra=77)
    o1 = oracle.linear(c["A"], c["W1t"], 8, c["b1"], True)
    s2 = oracle.scale_from_amax(oracle.absmax(o1["Y"]), 8)
    o2 = oracle.linear(o1["Y"], c["W2t"], 8, c["b2"], False, sA=s2)
    try:
        mq.mq_set_barrier_timeout_us(0)
        assert np.all(np.isnan(gpu_ffn_fused(c)))
    finally:
        mq.mq_set_barrier_timeout_us(500000)
    assert np.array_equal(gpu_ffn_fused(c), o2["Y"])


def test_prepared_workspace_after_a_timed_out_agreement():
    # The same failure on a prepared workspace: the call that gave up is loud (NaN) and may leave the agreement words
    # in any state; after mq_ffn_ws_prepare the calls are right again.  (M d >= 2^20, so both single-pass kernels run.)
    M, d, f = 2048, 512, 640
    c = workloads.ffn(2, M, d, f, 0.04, 8, seed_extra=78)
    o1 = oracle.linear(c["A"], c["W1t"], 8, c["b1"], True)
    s2 = oracle.scale_from_amax(oracle.absmax(o1["Y"]), 8)
    o2 = oracle.linear(o1["Y"], c["W2t"], 8, c["b2"], False, sA=s2)
    p1 = mq.prepare_weight(dev(c["W1t"]), 8)
    p2 = mq.prepare_weight(dev(c["W2t"]), 8)
    A, b1, b2 = dev(c["A"]), dev(c["b1"]), dev(c["b2"])
    nbytes = mq.mq_ffn_ws_bytes(M, d, f)
    ws = torch.full((nbytes,), 0x77, dtype=torch.uint8, device=DEV)
    Y = torch.empty((M, d), dtype=torch.float32, device=DEV)

    def call():
        mq.mq_ffn_i8_f32_prepared(A, M, d, f, p1.packed, p1.scale, b1, p2.packed, p2.scale, b2, Y, ws, nbytes)
        torch.cuda.synchronize()
        return host(Y)

    mq.mq_ffn_ws_prepare(ws, nbytes, M, d, f)
    assert np.array_equal(call(), o2["Y"])
    try:
        mq.mq_set_barrier_timeout_us(0)
        assert np.all(np.isnan(call()))
    finally:
        mq.mq_set_barrier_timeout_us(500000)
    mq.mq_ffn_ws_prepare(ws, nbytes, M, d, f)
    assert np.array_equal(call(), o2["Y"])
    assert np.array_equal(call(), o2["Y"])


def test_single_pass_requantizing_product_refuses_what_does_not_fit():
    M, N, K = 4352, 4096, 64           # 272 tiles of 256 x 256
    pa = torch.zeros(mq.mq_packed_bytes(8, M, K), dtype=torch.uint8, device=DEV)
    pw = torch.zeros(mq.mq_packed_bytes(8, N, K), dtype=torch.uint8, device=DEV)
    one = torch.ones(1, dtype=torch.float32, device=DEV)
    nb = mq.mq_gemm_amax_ws_bytes(M, N)
    ws = torch.zeros(nb, dtype=torch.uint8, device=DEV)
    out = torch.zeros(mq.mq_packed_bytes(8, M, N), dtype=torch.uint8, device=DEV)
    with pytest.raises(mq.MqError):
        mq.mq_gemm_requant_single_packed(pa, pw, M, N, K, one, one, None, False, ws, nb, one.clone(), out)


# ------------------------------------------------ short-listed output layer

def gpu_greedy_shortlist(Hd, E, shortlist):
    pw = mq.prepare_weight(dev(E), 8)
    pa, s = gpu_quantize_pack(Hd, 8)
    M, K = Hd.shape
    N = E.shape[0]
    sl = dev(np.asarray(shortlist, dtype=np.int32))
    nbytes = mq.mq_argmax_ws_bytes(M, N)
    ws = torch.full((nbytes,), 0xEE, dtype=torch.uint8, device=DEV)
    tok = torch.full((M,), -7, dtype=torch.int32, device=DEV)
    val = torch.empty(M, dtype=torch.float32, device=DEV)
    mq.mq_gemm_argmax_shortlist(pa, pw.packed, sl, sl.numel(), M, N, K, s, pw.scale, tok, val, ws, nbytes)
    return host(tok), host(val)


@pytest.mark.parametrize("M,V,d,L", [(1, 1, 1, 1), (12, 777, 64, 1), (12, 777, 64, 15), (33, 4100, 96, 1000),
                                     (300, 36000, 512, 4321), (300, 36000, 512, 36000), (130, 9000, 192, 8999),
                                     (20, 150001, 32, 70000)])       # a list longer than the ring: slots refilled
def test_greedy_shortlist(M, V, d, L):
    c = workloads.config3(M=M, V=V, d=d, seed_extra=M + V + L)
    rng = np.random.default_rng(L + V)
    sl = np.sort(rng.choice(V, size=L, replace=False))
    o = oracle.greedy_output_layer(c["Hd"], c["E"], shortlist=sl)
    tok, val = gpu_greedy_shortlist(c["Hd"], c["E"], sl)
    assert np.array_equal(tok, o["tok"])
    assert np.array_equal(val, o["maxlogit"])


def test_greedy_shortlist_ties_and_frequent_plus_translations_shape():
    # list shaped like the paper's: the 100 most frequent ids plus 100 candidates per source word
    V, d, M = 36000, 512, 15
    c = workloads.config3(M=M, V=V, d=d, seed_extra=77)
    rng = np.random.default_rng(5)
    sl = np.unique(np.concatenate([np.arange(100), rng.integers(0, V, size=384 * 100 // 8)]))
    E = c["E"].copy()
    E[sl[40]] = E[sl[3000]]          # duplicate rows inside the list: the smaller id has to win
    E[sl[-1]] = E[sl[3000]]
    o = oracle.greedy_output_layer(c["Hd"], E, shortlist=sl)
    tok, val = gpu_greedy_shortlist(c["Hd"], E, sl)
    assert np.array_equal(tok, o["tok"]) and np.array_equal(val, o["maxlogit"])
    assert np.all(np.isin(tok, sl))


def test_greedy_shortlist_ids_outside_the_vocabulary_do_not_fault():
    # an id outside [0, N) is the caller's mistake; the kernel scores the nearest row in its place instead of reading
    # outside the embedding, and reports the id as listed if that candidate wins
    c = workloads.config3(M=9, V=500, d=64, seed_extra=3)
    bad = np.array([-7, 3, 17, 250, 100000], dtype=np.int32)
    good_clamped = np.array([0, 3, 17, 250, 499])
    o = oracle.greedy_output_layer(c["Hd"], c["E"], shortlist=np.unique(good_clamped))
    tok_bad, val_bad = gpu_greedy_shortlist(c["Hd"], c["E"], bad)
    assert np.array_equal(val_bad, o["maxlogit"])                       # rows 0 and 499 were scored in their place
    back = {-7: 0, 100000: 499}
    assert np.array_equal(np.array([back.get(int(t), int(t)) for t in tok_bad]), o["tok"])


# ---------------------------------- fixed multipliers (the paper's scheme) and auto-tuning

@pytest.mark.parametrize("M,d,f", [(1, 1, 1), (37, 64, 200), (300, 256, 520), (130, 96, 1000)])
def test_ffn_int16_with_the_fixed_multiplier(M, d, f):
    # the paper's 16-bit scheme (Section 4.2): every tensor multiplied by 2^10; the first product writes the
    # second one's input as packed 16-bit activations (byte planes + row sums) from its epilogue
    c = workloads.ffn(4, M, d, f, 0.03, 16, seed_extra=M + d + 7 * f)
    S = np.float32(1024.0)
    o1 = oracle.linear(c["A"], c["W1t"], 16, c["b1"], True, sA=S, sW=S)
    o2 = oracle.linear(o1["Y"], c["W2t"], 16, c["b2"], False, sA=S, sW=S)
    assert o1["overflow_count"] == 0 and o2["overflow_count"] == 0
    sc = torch.full((1,), 1024.0, dtype=torch.float32, device=DEV)
    p1 = mq.prepare_weight(dev(c["W1t"]), 16, scale=sc)
    p2 = mq.prepare_weight(dev(c["W2t"]), 16, scale=sc)
    qA = torch.empty(mq.mq_packed_bytes(16, M, d), dtype=torch.uint8, device=DEV)
    mq.mq_quantize_pack_f32(dev(c["A"]), M, d, 16, sc, qA)
    for _ in range(2):                                            # the row sums are cleared by the call itself
        qH = torch.full((mq.mq_packed_bytes(16, M, f),), 0x5D, dtype=torch.uint8, device=DEV)
        mq.mq_gemm_requant_fixed_packed_i16(qA, p1.packed, M, f, d, sc, sc, dev(c["b1"]), True, sc, qH)
        # identical bytes to the quantizer's packing of the oracle's intermediate (planes, padding, row sums)
        ref = torch.empty_like(qH)
        mq.mq_quantize_pack_f32(dev(o1["Y"]), M, f, 16, sc, ref)
        assert torch.equal(qH, ref)
        q = torch.empty((M, f), dtype=torch.int16, device=DEV)
        mq.mq_unpack_weight(qH, 16, M, f, q)
        assert np.array_equal(host(q), o2["qA"])
        Y = torch.empty((M, d), dtype=torch.float32, device=DEV)
        mq.mq_gemm_dequant_packed(qH, p2.packed, 16, M, d, f, sc, sc, dev(c["b2"]), False, Y, None)
        assert np.array_equal(host(Y), o2["Y"])
    # the same block in one call
    nb = mq.mq_ffn_i16_fixed_ws_bytes(M, d, f)
    ws = torch.full((nb,), 0x6E, dtype=torch.uint8, device=DEV)
    for _ in range(2):
        Y = torch.full((M, d), float("nan"), dtype=torch.float32, device=DEV)
        mq.mq_ffn_i16_fixed_f32(dev(c["A"]), M, d, f, sc, p1.packed, sc, dev(c["b1"]), sc, p2.packed, sc, dev(c["b2"]), Y,
                                ws, nb)
        assert np.array_equal(host(Y), o2["Y"])


def test_ffn_int16_fixed_multiplier_full_size_equals_oracle_on_all_rows():
    # the paper's 16-bit scheme at the benchmark's 8192 x 1024 x 4096, one call, every row against the oracle;
    # with 2^10 no 32-bit sum wraps (Section 4.2 chose the multiplier for that)
    c = workloads.config4()
    M, d = c["A"].shape
    f = c["W1t"].shape[0]
    S = np.float32(1024.0)
    o1 = oracle.linear(c["A"], c["W1t"], 16, c["b1"], True, sA=S, sW=S)
    o2 = oracle.linear(o1["Y"], c["W2t"], 16, c["b2"], False, sA=S, sW=S)
    assert o1["overflow_count"] == 0 and o2["overflow_count"] == 0
    sc = torch.full((1,), 1024.0, dtype=torch.float32, device=DEV)
    p1 = mq.prepare_weight(dev(c["W1t"]), 16, scale=sc)
    p2 = mq.prepare_weight(dev(c["W2t"]), 16, scale=sc)
    nb = mq.mq_ffn_i16_fixed_ws_bytes(M, d, f)
    ws = torch.full((nb,), 0x6E, dtype=torch.uint8, device=DEV)
    Y = torch.full((M, d), float("nan"), dtype=torch.float32, device=DEV)
    mq.mq_ffn_i16_fixed_f32(dev(c["A"]), M, d, f, sc, p1.packed, sc, dev(c["b1"]), sc, p2.packed, sc, dev(c["b2"]), Y, ws, nb)
    assert np.array_equal(host(Y), o2["Y"])


def test_ffn_with_fixed_multipliers_single_pass():
    # Section 4.2: 8-bit inputs clipped to [-2, 2] and scaled by 127/2; no abs-max anywhere.  The
    # intermediate is quantized in the epilogue of the product that creates it.
    c = workloads.ffn(2, 200, 128, 384, 0.04, 8, seed_extra=5)
    A = c["A"] * np.float32(1.5)                  # some values beyond +-2: they saturate at +-127
    W1, W2 = c["W1t"] * np.float32(8), c["W2t"] * np.float32(8)
    fixed = np.float32(63.5)
    o1 = oracle.linear(A, W1, 8, c["b1"], True, sA=fixed, sW=fixed)
    assert np.abs(o1["qA"]).max() == 127 and (np.abs(A) > 2).any()
    oqH = oracle.quant_int(o1["Y"], 8, fixed)
    o2 = oracle.dequant_bias(oracle.dot_int(oqH, oracle.quant_int(W2, 8, fixed)), fixed, fixed, c["b2"], False)
    M, d = A.shape
    f = W1.shape[0]
    sc = torch.full((1,), 63.5, dtype=torch.float32, device=DEV)
    p1 = mq.prepare_weight(dev(W1), 8, scale=sc)
    p2 = mq.prepare_weight(dev(W2), 8, scale=sc)
    qA = torch.empty(mq.mq_packed_bytes(8, M, d), dtype=torch.uint8, device=DEV)
    mq.mq_quantize_pack_f32(dev(A), M, d, 8, sc, qA)
    qH = torch.full((mq.mq_packed_bytes(8, M, f),), 0x44, dtype=torch.uint8, device=DEV)
    mq.mq_gemm_requant_fixed_packed(qA, p1.packed, M, f, d, sc, p1.scale, dev(c["b1"]), True, sc, qH)
    Y = torch.empty((M, d), dtype=torch.float32, device=DEV)
    mq.mq_gemm_dequant_packed(qH, p2.packed, 8, M, d, f, sc, p2.scale, dev(c["b2"]), False, Y, None)
    q = torch.empty((M, f), dtype=torch.int8, device=DEV)
    mq.mq_unpack_weight(qH, 8, M, f, q)
    assert np.array_equal(host(q), oqH)
    assert np.array_equal(host(Y), o2)


def test_autotune_freezes_a_variant_and_results_stay_identical():
    M, N, K = 300, 512, 256
    p = workloads.random_problem(909, M, N, K)
    o = oracle.linear(p["A"], p["Wt"], 8, p["bias"], False)
    nbytes = mq.mq_autotune_ws_bytes(8, M, N, K)
    ws = torch.empty(nbytes, dtype=torch.uint8, device=DEV)
    best, us = mq.mq_autotune_gemm(8, M, N, K, 20, ws, nbytes)
    assert 1 <= best <= 14 and us > 0
    pw = mq.prepare_weight(dev(p["Wt"]), 8)
    pa, s = gpu_quantize_pack(p["A"], 8)
    Y = torch.empty((M, N), dtype=torch.float32, device=DEV)
    mq.mq_gemm_dequant_packed(pa, pw.packed, 8, M, N, K, s, pw.scale, dev(p["bias"]), False, Y, None)
    assert np.array_equal(host(Y), o["Y"])
    best16, _ = mq.mq_autotune_gemm(16, 64, 96, 128, 5, torch.empty(mq.mq_autotune_ws_bytes(16, 64, 96, 128),
                                                                      dtype=torch.uint8, device=DEV),
                                    mq.mq_autotune_ws_bytes(16, 64, 96, 128))
    assert 1 <= best16 <= 6


# ------------------------------------------------ beam-search output layer

def gpu_topk(Hd, E, k, shortlist=None):
    pw = mq.prepare_weight(dev(E), 8)
    pa, s = gpu_quantize_pack(Hd, 8)
    M, K = Hd.shape
    N = E.shape[0]
    sl = None if shortlist is None else dev(np.asarray(shortlist, dtype=np.int32))
    nbytes = mq.mq_topk_ws_bytes(M, N, k)
    ws = torch.full((nbytes,), 0xC3, dtype=torch.uint8, device=DEV)
    tok = torch.full((M, k), -7, dtype=torch.int32, device=DEV)
    lp = torch.empty((M, k), dtype=torch.float32, device=DEV)
    mq.mq_gemm_topk_packed(pa, pw.packed, sl, 0 if sl is None else sl.numel(), M, N, K, s, pw.scale, k, tok, lp, ws,
                           nbytes)
    return host(tok), host(lp)


@pytest.mark.parametrize("k", [1, 2, 3, 4])
@pytest.mark.parametrize("M,V,d", [(1, 4, 1), (12, 777, 64), (33, 4100, 96), (300, 36000, 512), (130, 9000, 192),
                                   (600, 5000, 128), (12, 70000, 64), (1200, 3000, 64)])
def test_beam_output_layer_topk(M, V, d, k):
    # Table 2's b = 2 / b = 4 rows: the k best words per row, exact, with log-probabilities within 1e-4
    # (binary32 logits of magnitude <= ~30 here; the normaliser sums V terms in binary32).  M = 600 and 1200 go
    # through three and five chunks of rows (the last ones ragged), all in one launch.
    c = workloads.config3(M=M, V=V, d=d, seed_extra=M + V + k)
    o = oracle.topk_log_softmax(c["Hd"], c["E"], k)
    tok, lp = gpu_topk(c["Hd"], c["E"], k)
    assert np.array_equal(tok, o["tok"])
    assert np.allclose(lp, o["logprob"], rtol=0, atol=1e-4)


def test_beam_output_layer_ties_and_crowded_lanes():
    # all k best words in one accumulator register's stream: duplicates of the winning embedding row placed
    # one workgroup-stride (256 units of 16 words) apart land in the same register of the same lane
    c = workloads.config3(M=20, V=36000, d=64, seed_extra=123)
    E = c["E"].copy()
    h = c["Hd"][0] / np.abs(c["Hd"][0]).max() * np.abs(E).max()     # aligned with sentence 0, inside the abs-max
    for j in range(4):
        E[5 + 4096 * j] = h * (1.0 - 0.01 * j)
    E[5 + 4096 * 4] = h                                              # exact tie with the first, higher index
    o = oracle.topk_log_softmax(c["Hd"], E, 4)
    tok, lp = gpu_topk(c["Hd"], E, 4)
    assert list(o["tok"][0][:2]) == [5, 5 + 4096 * 4]
    assert np.array_equal(tok, o["tok"])
    assert np.allclose(lp, o["logprob"], rtol=0, atol=1e-4)


@pytest.mark.parametrize("k", [2, 4])
@pytest.mark.parametrize("V,L", [(9000, 1234), (120000, 60000)])     # the longer list refills the ring's slots
def test_beam_output_layer_with_shortlist(k, V, L):
    c = workloads.config3(M=64, V=V, d=128 if V < 10000 else 32, seed_extra=77)
    rng = np.random.default_rng(5)
    sl = np.sort(rng.choice(V, size=L, replace=False)).astype(np.int32)
    qE = c["E"][sl]
    # the short list is scored with the whole embedding's multiplier: quantize the whole, then gather
    full = oracle.greedy_output_layer(c["Hd"], c["E"])
    acc = oracle.dot_int(full["qA"], np.ascontiguousarray(full["qW"][sl]))
    y = oracle.dequant_bias(acc, full["sA"], full["sW"]).astype(np.float64)
    lse = np.log(np.exp(y - y.max(1, keepdims=True)).sum(1, keepdims=True)) + y.max(1, keepdims=True)
    order = np.argsort(-acc.astype(np.int64), axis=1, kind="stable")[:, :k]
    tok, lp = gpu_topk(c["Hd"], c["E"], k, shortlist=sl)
    assert np.array_equal(tok, sl[order])
    assert np.allclose(lp, np.take_along_axis(y, order, axis=1) - lse, rtol=0, atol=1e-4)
    del qE
