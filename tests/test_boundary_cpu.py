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
