"""CPU-only checks of the C boundary: the library loads without a GPU, exports
every symbol include/mq.h declares, and rejects bad arguments before touching
the device."""
import ctypes
import os
import re

import pytest

import paper_1805_12096_amd as mq

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(mq.lib_path()):
        from paper_1805_12096_amd import build
        build.build()
    return mq.load_library()


def test_header_symbols_are_exported(lib):
    header = open(os.path.join(ROOT, "include", "mq.h")).read()
    body = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(mq_[a-z0-9_]+)\s*\(", body))
    assert declared == set(mq.exported_symbols())
    for name in declared:
        assert hasattr(lib, name), name


def test_version_and_status_strings(lib):
    assert mq.mq_version() >= 100
    seen = {mq.mq_status_string(i) for i in range(8)}
    assert len(seen) == 8 and "ok" in seen
    assert mq.mq_status_string(99) == "unknown status"


def test_size_queries(lib):
    # int8: N padded to 32 rows, K to 64 elements
    assert mq.mq_packed_bytes(8, 36000, 512) == 36000 * 512
    assert mq.mq_packed_bytes(8, 1, 1) == 32 * 64
    assert mq.mq_packed_bytes(16, 512, 512) == 2 * 512 * 512 + 4 * 512
    assert mq.mq_packed_bytes(4, 8, 8) == 0 and mq.mq_packed_bytes(8, 0, 8) == 0
    assert mq.mq_argmax_ws_bytes(300, 36000) >= 300 * 8
    assert mq.mq_argmax_ws_bytes(0, 5) == 0
    assert mq.mq_linear_ws_bytes(8, 300, 512) >= 300 * 512
    assert mq.mq_linear_ws_bytes(16, 300, 512) >= 2 * 300 * 512 + 4 * 300
    assert mq.mq_linear_ws_bytes(7, 300, 512) == 0


def test_argument_checks_enqueue_nothing(lib):
    P = ctypes.c_void_p
    good, odd = P(4096), P(4100)      # never dereferenced: checks fail first
    OK, NULL, SHAPE, DTYPE, ALIGN, WS = 0, 1, 2, 3, 4, 5
    assert lib.mq_absmax_f32(None, 8, good, None) == NULL
    assert lib.mq_absmax_f32(good, 0, good, None) == SHAPE
    assert lib.mq_absmax_f32(odd, 8, good, None) == ALIGN
    assert lib.mq_scale_from_amax(good, 12, good, None) == DTYPE
    assert lib.mq_scale_from_amax(None, 8, good, None) == NULL
    assert lib.mq_quantize_f32(good, 4, 4, 32, good, good, None, None) == DTYPE
    assert lib.mq_quantize_f32(good, 4, 0, 8, good, good, None, None) == SHAPE
    assert lib.mq_quantize_f32(good, 4, 4, 8, None, good, None, None) == NULL
    assert lib.mq_quantize_f32(good, 4, 4, 8, good, odd, None, None) == ALIGN
    assert lib.mq_prepare_weight(good, 1, 8, 8, 8, None, None, good, None) == NULL
    assert lib.mq_prepare_weight(good, 1, 0, 8, 8, None, good, good, None) == SHAPE
    assert lib.mq_prepare_weight(good, 1, 8, 8, 9, None, good, good, None) == DTYPE
    assert lib.mq_unpack_weight(good, 8, 8, 8, None, None) == NULL
    assert lib.mq_gemm_i32(good, None, good, 16, 4, 4, 4, good, None) == NULL      # int16 needs row sums
    assert lib.mq_gemm_i32(good, None, good, 8, 4, 4, 4, None, None) == NULL
    assert lib.mq_gemm_i32(good, None, good, 8, 4, 0, 4, good, None) == SHAPE
    assert lib.mq_gemm_i32(good, None, good, 8, 1 << 31, 4, 4, good, None) == SHAPE
    assert lib.mq_gemm_i32(odd, None, good, 8, 4, 4, 4, good, None) == ALIGN
    assert lib.mq_gemm_i32(good, None, good, 3, 4, 4, 4, good, None) == DTYPE
    assert lib.mq_gemm_dequant(good, None, good, 8, 4, 4, 4, None, good, None, 0, good, None, None) == NULL
    assert lib.mq_gemm_dequant(good, None, good, 8, 4, 4, 4, good, good, P(4098), 0, good, None, None) == ALIGN
    assert lib.mq_gemm_argmax(good, good, 4, 4, 4, good, good, good, good, None, 1 << 20, None) == NULL
    assert lib.mq_gemm_argmax(good, good, 4, 4, 4, good, good, good, good, good, 8, None) == WS
    assert lib.mq_linear_f32(good, 4, 4, None, good, good, 8, 4, None, 0, good, None, good, 16, None) == WS
    assert lib.mq_linear_f32(good, 4, 4, None, good, good, 5, 4, None, 0, good, None, good, 1 << 20, None) == DTYPE
    assert OK == 0


def test_binding_raises_on_error_status(lib):
    with pytest.raises(mq.MqError) as e:
        mq.binding._check(4, "somewhere")
    assert "aligned" in str(e.value)


# ---- every entry point that takes pointers: bad arguments are refused before anything touches a device ----------
# Each row is a call that WOULD be valid (it is never made), as (name, argument list); the test replaces one
# argument at a time by a bad value and expects the matching status.  G is a fake, well aligned device pointer that
# is never dereferenced.  Roles: "p16" / "p4" = required pointer with that alignment, "opt" = optional pointer (4-byte
# aligned if given), "n" = size that must not be zero, "bits", "ws" = workspace pointer (256-byte aligned is always
# enough), "wsb" = workspace bytes, "-" = not varied.
G, BIG = 1 << 20, 1 << 40
NULL, SHAPE, DTYPE, ALIGN, WS, UNSUP, LIMIT = 1, 2, 3, 4, 5, 6, 8


def _rows():
    P16, P4, OPT, N_, BITS, WSP, WSB, X = "p16", "p4", "opt", "n", "bits", "ws", "wsb", "-"
    ffn = [(G, P16), (64, N_), (64, N_), (64, N_), (G, P16), (G, P4), (G, OPT), (G, P16), (G, P4), (G, OPT), (G, P4),
           (G, WSP), (BIG, WSB), (None, X)]
    fused = [(G, P16), (G, P16), (64, N_), (64, N_), (64, N_), (G, P4), (G, P4), (G, OPT), (1, X)]
    return {
        "mq_absmax_f32": [(G, P16), (8, N_), (G, P4), (None, X)],
        "mq_scale_from_amax": [(G, P4), (8, BITS), (G, P4), (None, X)],
        "mq_quantize_f32": [(G, P16), (4, N_), (4, N_), (8, BITS), (G, P4), (G, P16), (G, OPT), (None, X)],
        "mq_quantize_pack_f32": [(G, P16), (4, N_), (4, N_), (8, BITS), (G, P4), (G, P16), (None, X)],
        "mq_quantize_absmax_pack_f32": [(G, P16), (4, N_), (4, N_), (8, BITS), (G, P16), (G, P4), (G, WSP), (BIG, WSB),
                                        (None, X)],
        "mq_quantize_absmax_pack_f32_prepared": [(G, P16), (4, N_), (4, N_), (8, BITS), (G, P16), (G, P4), (G, WSP),
                                                 (BIG, WSB), (None, X)],
        "mq_quantize_absmax_ws_prepare": [(G, WSP), (BIG, WSB), (None, X)],
        "mq_prepare_weight": [(G, P16), (1, X), (8, N_), (8, N_), (8, BITS), (G, OPT), (G, P4), (G, P16), (None, X)],
        "mq_unpack_weight": [(G, P16), (8, BITS), (8, N_), (8, N_), (G, "p2"), (None, X)],
        "mq_gemm_i32": [(G, P16), (G, OPT), (G, P16), (8, BITS), (4, N_), (4, N_), (4, N_), (G, P4), (None, X)],
        "mq_gemm_dequant": [(G, P16), (G, OPT), (G, P16), (8, BITS), (4, N_), (4, N_), (4, N_), (G, P4), (G, P4), (G, OPT),
                            (0, X), (G, P4), (G, OPT), (None, X)],
        "mq_gemm_i32_packed": [(G, P16), (G, P16), (8, BITS), (4, N_), (4, N_), (4, N_), (G, P4), (None, X)],
        "mq_gemm_dequant_packed": [(G, P16), (G, P16), (8, BITS), (4, N_), (4, N_), (4, N_), (G, P4), (G, P4), (G, OPT),
                                   (0, X), (G, P4), (G, OPT), (None, X)],
        "mq_gemm_amax_packed": fused + [(G, WSP), (BIG, WSB), (None, X)],
        "mq_gemm_requant_packed": fused + [(G, WSP), (BIG, WSB), (G, P4), (G, P16), (None, X)],
        "mq_gemm_requant_single_packed": fused + [(G, WSP), (BIG, WSB), (G, P4), (G, P16), (None, X)],
        "mq_gemm_requant_fixed_packed": fused + [(G, P4), (G, P16), (None, X)],
        "mq_gemm_requant_fixed_packed_i16": fused + [(G, P4), (G, P16), (None, X)],
        "mq_autotune_gemm": [(8, BITS), (64, N_), (64, N_), (64, N_), (3, N_), (G, WSP), (BIG, WSB), (None, X), (None, X),
                             (None, X)],
        "mq_gemm_argmax": [(G, P16), (G, P16), (4, N_), (4, N_), (4, N_), (G, P4), (G, P4), (G, P4), (G, P4), (G, WSP),
                           (BIG, WSB), (None, X)],
        "mq_gemm_argmax_packed": [(G, P16), (G, P16), (4, N_), (4, N_), (4, N_), (G, P4), (G, P4), (G, P4), (G, P4),
                                  (G, WSP), (BIG, WSB), (None, X)],
        "mq_gemm_argmax_packed_static": [(G, P16), (G, P16), (4, N_), (4, N_), (4, N_), (G, P4), (G, P4), (G, P4), (G, P4),
                                         (None, X)],
        "mq_gemm_argmax_shortlist": [(G, P16), (G, P16), (G, P4), (2, N_), (4, N_), (4, N_), (4, N_), (G, P4), (G, P4),
                                     (G, P4), (G, P4), (G, WSP), (BIG, WSB), (None, X)],
        "mq_linear_f32": [(G, P16), (4, N_), (4, N_), (G, OPT), (G, P16), (G, P4), (8, BITS), (4, N_), (G, OPT), (0, X),
                          (G, P4), (G, OPT), (G, WSP), (BIG, WSB), (None, X)],
        "mq_ffn_i8_f32": ffn,
        "mq_ffn_i8_f32_prepared": ffn,
        "mq_ffn_i16_f32": ffn,
        "mq_ffn_i16_fixed_f32": [(G, P16), (64, N_), (64, N_), (64, N_), (G, P4), (G, P16), (G, P4), (G, OPT), (G, P4),
                                 (G, P16), (G, P4), (G, OPT), (G, P4), (G, WSP), (BIG, WSB), (None, X)],
        "mq_ffn_ws_prepare": [(G, WSP), (BIG, WSB), (64, N_), (64, N_), (64, N_), (None, X)],
        "mq_gemm_topk_packed": [(G, P16), (G, P16), (G, OPT), (8, X), (4, N_), (16, N_), (4, N_), (G, P4), (G, P4), (2, X),
                                (G, P4), (G, P4), (G, WSP), (BIG, WSB), (None, X)],
        "mq_running_average_f32": [(G, P4), (G, P4), (8, N_), (1, N_), (G, P4), (None, X)],
        "mq_concat2_f32": [(G, P4), (4, N_), (G, P4), (4, N_), (4, N_), (G, P4), (None, X)],
        "mq_add_layer_norm_f32": [(G, P4), (G, P4), (G, P4), (G, P4), (4, N_), (4, N_), (1e-6, X), (G, P4), (None, X)],
        "mq_gate_mix_layer_norm_f32": [(G, P4), (G, P4), (G, P4), (G, P4), (G, P4), (4, N_), (4, N_), (1e-6, X), (G, P4),
                                       (None, X)],
        "mq_cross_attention_f32": [(G, P4), (G, P4), (G, P4), (4, N_), (4, N_), (8, N_), (2, N_), (G, P4), (None, X)],
    }


QUERIES_AND_SETTERS = {"mq_version", "mq_autotune_report", "mq_status_string", "mq_last_hip_error", "mq_set_gemm_variant", "mq_packed_bytes",
                       "mq_set_quantize_single_pass", "mq_quantize_absmax_ws_bytes", "mq_gemm_amax_ws_bytes",
                       "mq_set_barrier_timeout_us", "mq_single_pass_fits", "mq_autotune_ws_bytes", "mq_argmax_ws_bytes",
                       "mq_linear_ws_bytes", "mq_ffn_ws_bytes", "mq_set_ffn_single_pass", "mq_ffn_i16_ws_bytes", "mq_ffn_i16_fixed_ws_bytes",
                       "mq_topk_ws_bytes", "mq_aan_layer_ws_bytes"}


def test_every_export_has_a_cpu_side_check():
    covered = set(_rows()) | QUERIES_AND_SETTERS | {"mq_aan_layer_f32"}
    assert covered == set(mq.exported_symbols())


@pytest.mark.parametrize("name", sorted(_rows()))
def test_bad_arguments_are_refused_before_any_launch(lib, name):
    row = _rows()[name]
    fn = getattr(lib, name)
    good = [v for v, _ in row]
    tried = 0
    for i, (_, role) in enumerate(row):
        bad = []
        if role in ("p16", "p4", "p2", "ws"):
            bad.append((None, NULL))
            bad.append((G + {"p16": 4, "p4": 2, "p2": 1, "ws": 4}[role], ALIGN))
        elif role == "opt":
            bad.append((G + 2, ALIGN))
        elif role == "n":
            bad.append((0, SHAPE))
        elif role == "bits":
            bad.append((7, DTYPE))
        elif role == "wsb":
            bad.append((8, WS))
        for value, want in bad:
            args = list(good)
            args[i] = value
            got = fn(*args)
            assert got == want, f"{name}: argument {i} ({role}) = {value!r}: status {got}, expected {want}"
            tried += 1
    assert tried >= 3


def test_limits_of_single_entry_points(lib):
    # sizes a particular kernel cannot serve, still refused on the host
    assert lib.mq_gemm_argmax_packed(G, G, 4, 4, 1024, G, G, G, G, G, BIG, None) == UNSUP        # K beyond 512
    assert lib.mq_gemm_argmax_packed_static(G, G, 4, 4, 1024, G, G, G, G, None) == UNSUP
    assert lib.mq_gemm_argmax_packed_static(G, G, 24577, 4, 64, G, G, G, G, None) == LIMIT       # rows beyond the array
    assert "static scratch" in mq.mq_status_string(LIMIT)
    assert lib.mq_gemm_argmax_shortlist(G, G, G, 9, 4, 4, 4, G, G, G, G, G, BIG, None) == SHAPE  # list longer than N
    assert lib.mq_gemm_topk_packed(G, G, None, 0, 4, 16, 4, G, G, 5, G, G, G, BIG, None) == SHAPE   # k beyond 4
    assert lib.mq_gemm_topk_packed(G, G, G, 1, 4, 16, 4, G, G, 2, G, G, G, BIG, None) == SHAPE      # list shorter than k
    assert lib.mq_running_average_f32(G, G, 8, 0, G, None) == SHAPE                                 # positions from 1
    assert lib.mq_cross_attention_f32(G, G, G, 4, 4, 8, 3, G, None) == SHAPE                        # 8 not divisible by 3
    assert lib.mq_autotune_gemm(8, 64, 64, 64, 0, G, BIG, None, None, None) == SHAPE                # no runs
    assert lib.mq_set_gemm_variant(99) == UNSUP and lib.mq_set_gemm_variant(0) == 0
    assert lib.mq_autotune_report(None, 8) == NULL
    buf = (ctypes.c_float * 8)()
    assert lib.mq_autotune_report(buf, 0) == SHAPE and lib.mq_autotune_report(buf, 8) == 0 and buf[0] == -1.0
    assert lib.mq_set_barrier_timeout_us(20_000_000) == SHAPE and lib.mq_set_barrier_timeout_us(500_000) == 0


def test_decoder_layer_argument_checks(lib):
    from paper_1805_12096_amd import binding
    prod = binding._CProduct(G, G, G)
    norm = binding._CNorm(G, G)
    P = binding._CAanLayer(prod, prod, prod, norm, prod, prod, norm, prod, prod, norm, 64, 128, 128)
    call = lambda **kw: lib.mq_aan_layer_f32(*[kw.get(k, v) for k, v in (
        ("P", ctypes.byref(P)), ("x", G), ("g_prev", G), ("t", 3), ("K", G), ("V", G), ("M", 4), ("S", 5), ("heads", 4),
        ("use_ffn", 1), ("use_gate", 1), ("eps", 1e-6), ("y", G), ("g_out", G), ("ws", G), ("wsb", BIG), ("stream", None))])
    assert call(P=None) == NULL and call(x=None) == NULL and call(ws=None) == NULL
    assert call(t=0) == SHAPE and call(M=0) == SHAPE and call(heads=3) == SHAPE and call(S=0) == SHAPE
    assert call(x=G + 4) == ALIGN and call(ws=G + 16) == ALIGN
    assert call(wsb=64) == WS
    bad = binding._CAanLayer(prod, prod, binding._CProduct(None, G, G), norm, prod, prod, norm, prod, prod, norm, 64, 128, 128)
    assert call(P=ctypes.byref(bad)) == NULL                  # the gate's parameter is missing ...
    assert call(P=ctypes.byref(bad), use_gate=0, wsb=64) == WS         # ... and not asked for without the gate


def test_single_pass_size_test_and_workspace_queries(lib):
    # the launcher's choice between one launch with a grid-wide agreement and the two-pass form, as a pure function
    assert mq.mq_single_pass_fits(8192, 2048, 256)             # config 2's first product: 32 x 8 tiles = 256
    assert not mq.mq_single_pass_fits(8192, 2048, 255)         # one workgroup would not be resident
    assert not mq.mq_single_pass_fits(8192, 2049, 256)         # 288 tiles
    assert not mq.mq_single_pass_fits(8192, 4096, 1024)        # fits the device but not the 256 slots
    assert mq.mq_single_pass_fits(1, 1, 1) and not mq.mq_single_pass_fits(0, 5, 256)
    # workspace queries: zero for invalid sizes, monotonic in the problem size
    assert mq.mq_ffn_ws_bytes(0, 4, 4) == 0 and mq.mq_ffn_i16_ws_bytes(4, 0, 4) == 0
    assert mq.mq_ffn_ws_bytes(8192, 512, 2048) >= 8192 * 512 + 8192 * 2048
    assert mq.mq_ffn_i16_ws_bytes(8192, 1024, 4096) >= 4 * 8192 * 4096 + 2 * 8192 * 4096
    assert mq.mq_gemm_amax_ws_bytes(8192, 2048) >= 2112 * 4 and mq.mq_gemm_amax_ws_bytes(0, 1) == 0
    assert mq.mq_quantize_absmax_ws_bytes() >= 2112 * 4 + 4096
    assert mq.mq_topk_ws_bytes(300, 36000, 5) == 0 and mq.mq_topk_ws_bytes(300, 36000, 4) > 0
    assert mq.mq_autotune_ws_bytes(9, 4, 4, 4) == 0 and mq.mq_autotune_ws_bytes(8, 64, 64, 64) > 0
    assert mq.mq_aan_layer_ws_bytes(300, 512, 2048, 2048) > 300 * 2048 * 4 and mq.mq_aan_layer_ws_bytes(0, 512, 8, 8) == 0
