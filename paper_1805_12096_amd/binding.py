"""ctypes binding of libmq.so.  Argument marshalling only: every function below
has the name and the argument order of the C entry point it calls (see
include/mq.h) and takes torch CUDA tensors where C takes device pointers.
PyTorch supplies device memory and the current HIP stream, nothing else.

There is no fallback: if the library has not been built, importing fails with
instructions, and every non-zero status raises MqError.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

import torch

__all__ = [
    "MqError", "lib_path", "load_library", "exported_symbols",
    "mq_version", "mq_status_string", "mq_last_hip_error", "mq_set_gemm_variant",
    "mq_absmax_f32", "mq_scale_from_amax", "mq_quantize_f32", "mq_quantize_pack_f32", "mq_packed_bytes",
    "mq_prepare_weight", "mq_unpack_weight", "mq_gemm_i32", "mq_gemm_dequant",
    "mq_gemm_i32_packed", "mq_gemm_dequant_packed", "mq_argmax_ws_bytes", "mq_gemm_argmax", "mq_gemm_argmax_packed", "mq_gemm_argmax_packed_static", "mq_gemm_argmax_shortlist", "mq_linear_ws_bytes", "mq_linear_f32", "mq_ffn_ws_bytes", "mq_ffn_i8_f32", "mq_ffn_ws_prepare", "mq_ffn_i8_f32_prepared", "mq_set_ffn_single_pass", "mq_gemm_requant_single_packed", "mq_single_pass_fits", "mq_set_barrier_timeout_us", "mq_set_quantize_single_pass", "mq_ffn_i16_ws_bytes", "mq_ffn_i16_f32", "mq_ffn_i16_fixed_ws_bytes", "mq_ffn_i16_fixed_f32",
    "mq_quantize_absmax_ws_bytes", "mq_quantize_absmax_pack_f32", "mq_quantize_absmax_ws_prepare", "mq_quantize_absmax_pack_f32_prepared", "mq_gemm_amax_ws_bytes", "mq_gemm_amax_packed",
    "mq_gemm_requant_packed", "mq_gemm_requant_fixed_packed", "mq_gemm_requant_fixed_packed_i16",
    "mq_autotune_ws_bytes", "mq_autotune_gemm", "mq_autotune_report",
    "mq_topk_ws_bytes", "mq_gemm_topk_packed",
    "mq_running_average_f32", "mq_concat2_f32", "mq_add_layer_norm_f32", "mq_gate_mix_layer_norm_f32",
    "mq_cross_attention_f32", "mq_aan_layer_ws_bytes", "mq_aan_layer_f32", "AanLayer", "aan_layer",
    "PreparedWeight", "prepare_weight",
]

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libmq.so")
_lib = None

MQ_OK = 0


class MqError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = load_library().mq_status_string(status).decode()
        extra = ""
        if status == 7:
            extra = f" (hipError {load_library().mq_last_hip_error()})"
        super().__init__(f"{where}: status {status}: {msg}{extra}")


def lib_path() -> str:
    return _LIB_PATH


def exported_symbols():
    """Names include/mq.h declares; used by the CPU-only load test."""
    return ["mq_version", "mq_status_string", "mq_last_hip_error", "mq_set_gemm_variant", "mq_absmax_f32",
            "mq_scale_from_amax", "mq_quantize_f32", "mq_quantize_pack_f32", "mq_packed_bytes", "mq_prepare_weight",
            "mq_unpack_weight", "mq_gemm_i32", "mq_gemm_dequant", "mq_gemm_i32_packed",
            "mq_gemm_dequant_packed", "mq_argmax_ws_bytes",
            "mq_gemm_argmax", "mq_gemm_argmax_packed", "mq_gemm_argmax_packed_static", "mq_gemm_argmax_shortlist", "mq_linear_ws_bytes", "mq_linear_f32", "mq_ffn_ws_bytes", "mq_ffn_i8_f32", "mq_ffn_ws_prepare", "mq_ffn_i8_f32_prepared", "mq_set_ffn_single_pass", "mq_gemm_requant_single_packed", "mq_single_pass_fits", "mq_set_barrier_timeout_us", "mq_set_quantize_single_pass", "mq_ffn_i16_ws_bytes", "mq_ffn_i16_f32", "mq_ffn_i16_fixed_ws_bytes", "mq_ffn_i16_fixed_f32",
            "mq_quantize_absmax_ws_bytes", "mq_quantize_absmax_pack_f32", "mq_quantize_absmax_ws_prepare", "mq_quantize_absmax_pack_f32_prepared", "mq_gemm_amax_ws_bytes",
            "mq_gemm_amax_packed", "mq_gemm_requant_packed", "mq_gemm_requant_fixed_packed",
            "mq_gemm_requant_fixed_packed_i16",
            "mq_autotune_ws_bytes", "mq_autotune_gemm", "mq_autotune_report", "mq_topk_ws_bytes", "mq_gemm_topk_packed", "mq_running_average_f32", "mq_concat2_f32",
            "mq_add_layer_norm_f32", "mq_gate_mix_layer_norm_f32", "mq_cross_attention_f32",
            "mq_aan_layer_ws_bytes", "mq_aan_layer_f32"]



# ---- C structs of the decoder-layer entry point (plain device pointers) -----

class _CProduct(ctypes.Structure):
    _fields_ = [("packed", ctypes.c_void_p), ("scale", ctypes.c_void_p), ("bias", ctypes.c_void_p)]


class _CNorm(ctypes.Structure):
    _fields_ = [("gamma", ctypes.c_void_p), ("beta", ctypes.c_void_p)]


class _CAanLayer(ctypes.Structure):
    _fields_ = [("aan_ffn1", _CProduct), ("aan_ffn2", _CProduct), ("aan_gate", _CProduct), ("ln1", _CNorm),
                ("ctx_q", _CProduct), ("ctx_o", _CProduct), ("ln2", _CNorm), ("ffn1", _CProduct), ("ffn2", _CProduct),
                ("ln3", _CNorm), ("d", ctypes.c_size_t), ("ffn", ctypes.c_size_t), ("aan_ffn", ctypes.c_size_t)]


def load_library():
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(
            f"{_LIB_PATH} is missing: build it with `python -m paper_1805_12096_amd.build` "
            "(or __graft_entry__.build()).  There is no CPU fallback.")
    lib = ctypes.CDLL(_LIB_PATH)
    vp, sz, ci = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int
    lib.mq_version.restype = ci
    lib.mq_status_string.restype = ctypes.c_char_p
    lib.mq_status_string.argtypes = [ci]
    lib.mq_last_hip_error.restype = ci
    lib.mq_set_gemm_variant.argtypes = [ci]
    lib.mq_absmax_f32.argtypes = [vp, sz, vp, vp]
    lib.mq_scale_from_amax.argtypes = [vp, ci, vp, vp]
    lib.mq_quantize_f32.argtypes = [vp, sz, sz, ci, vp, vp, vp, vp]
    lib.mq_quantize_pack_f32.argtypes = [vp, sz, sz, ci, vp, vp, vp]
    lib.mq_gemm_i32_packed.argtypes = [vp, vp, ci, sz, sz, sz, vp, vp]
    lib.mq_gemm_dequant_packed.argtypes = [vp, vp, ci, sz, sz, sz, vp, vp, vp, ci, vp, vp, vp]
    lib.mq_packed_bytes.restype = sz
    lib.mq_packed_bytes.argtypes = [ci, sz, sz]
    lib.mq_prepare_weight.argtypes = [vp, ci, sz, sz, ci, vp, vp, vp, vp]
    lib.mq_unpack_weight.argtypes = [vp, ci, sz, sz, vp, vp]
    lib.mq_gemm_i32.argtypes = [vp, vp, vp, ci, sz, sz, sz, vp, vp]
    lib.mq_gemm_dequant.argtypes = [vp, vp, vp, ci, sz, sz, sz, vp, vp, vp, ci, vp, vp, vp]
    lib.mq_argmax_ws_bytes.restype = sz
    lib.mq_argmax_ws_bytes.argtypes = [sz, sz]
    lib.mq_gemm_argmax.argtypes = [vp, vp, sz, sz, sz, vp, vp, vp, vp, vp, sz, vp]
    lib.mq_gemm_argmax_packed.argtypes = [vp, vp, sz, sz, sz, vp, vp, vp, vp, vp, sz, vp]
    lib.mq_gemm_argmax_packed_static.argtypes = [vp, vp, sz, sz, sz, vp, vp, vp, vp, vp]
    lib.mq_gemm_argmax_shortlist.argtypes = [vp, vp, vp, sz, sz, sz, sz, vp, vp, vp, vp, vp, sz, vp]
    lib.mq_quantize_absmax_ws_bytes.restype = sz
    lib.mq_quantize_absmax_ws_bytes.argtypes = []
    lib.mq_quantize_absmax_pack_f32.argtypes = [vp, sz, sz, ci, vp, vp, vp, sz, vp]
    lib.mq_quantize_absmax_pack_f32_prepared.argtypes = [vp, sz, sz, ci, vp, vp, vp, sz, vp]
    lib.mq_quantize_absmax_ws_prepare.argtypes = [vp, sz, vp]
    lib.mq_gemm_amax_ws_bytes.restype = sz
    lib.mq_gemm_amax_ws_bytes.argtypes = [sz, sz]
    lib.mq_gemm_amax_packed.argtypes = [vp, vp, sz, sz, sz, vp, vp, vp, ci, vp, sz, vp]
    lib.mq_gemm_requant_packed.argtypes = [vp, vp, sz, sz, sz, vp, vp, vp, ci, vp, sz, vp, vp, vp]
    lib.mq_gemm_requant_single_packed.argtypes = [vp, vp, sz, sz, sz, vp, vp, vp, ci, vp, sz, vp, vp, vp]
    lib.mq_gemm_requant_fixed_packed.argtypes = [vp, vp, sz, sz, sz, vp, vp, vp, ci, vp, vp, vp]
    lib.mq_gemm_requant_fixed_packed_i16.argtypes = [vp, vp, sz, sz, sz, vp, vp, vp, ci, vp, vp, vp]
    lib.mq_autotune_ws_bytes.restype = sz
    lib.mq_autotune_ws_bytes.argtypes = [ci, sz, sz, sz]
    lib.mq_autotune_gemm.argtypes = [ci, sz, sz, sz, ci, vp, sz, vp, ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_float)]
    lib.mq_autotune_report.argtypes = [ctypes.POINTER(ctypes.c_float), ci]
    lib.mq_set_ffn_single_pass.argtypes = [ci]
    lib.mq_set_quantize_single_pass.argtypes = [ci]
    lib.mq_set_barrier_timeout_us.argtypes = [ctypes.c_uint]
    lib.mq_single_pass_fits.argtypes = [sz, sz, sz]
    lib.mq_ffn_ws_bytes.restype = sz
    lib.mq_ffn_ws_bytes.argtypes = [sz, sz, sz]
    lib.mq_ffn_i8_f32.argtypes = [vp, sz, sz, sz, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.mq_ffn_i8_f32_prepared.argtypes = [vp, sz, sz, sz, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.mq_ffn_ws_prepare.argtypes = [vp, sz, sz, sz, sz, vp]
    lib.mq_ffn_i16_fixed_ws_bytes.restype = sz
    lib.mq_ffn_i16_fixed_ws_bytes.argtypes = [sz, sz, sz]
    lib.mq_ffn_i16_fixed_f32.argtypes = [vp, sz, sz, sz, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.mq_ffn_i16_ws_bytes.restype = sz
    lib.mq_ffn_i16_ws_bytes.argtypes = [sz, sz, sz]
    lib.mq_ffn_i16_f32.argtypes = [vp, sz, sz, sz, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    cf = ctypes.c_float
    lib.mq_topk_ws_bytes.restype = sz
    lib.mq_topk_ws_bytes.argtypes = [sz, sz, ci]
    lib.mq_gemm_topk_packed.argtypes = [vp, vp, vp, sz, sz, sz, sz, vp, vp, ci, vp, vp, vp, sz, vp]
    lib.mq_running_average_f32.argtypes = [vp, vp, sz, ci, vp, vp]
    lib.mq_concat2_f32.argtypes = [vp, sz, vp, sz, sz, vp, vp]
    lib.mq_add_layer_norm_f32.argtypes = [vp, vp, vp, vp, sz, sz, cf, vp, vp]
    lib.mq_gate_mix_layer_norm_f32.argtypes = [vp, vp, vp, vp, vp, sz, sz, cf, vp, vp]
    lib.mq_cross_attention_f32.argtypes = [vp, vp, vp, sz, sz, sz, ci, vp, vp]
    lib.mq_aan_layer_ws_bytes.restype = sz
    lib.mq_aan_layer_ws_bytes.argtypes = [sz, sz, sz, sz]
    lib.mq_aan_layer_f32.argtypes = [ctypes.POINTER(_CAanLayer), vp, vp, ci, vp, vp, sz, sz, ci, ci, ci, cf, vp, vp, vp, sz, vp]
    lib.mq_linear_ws_bytes.restype = sz
    lib.mq_linear_ws_bytes.argtypes = [ci, sz, sz]
    lib.mq_linear_f32.argtypes = [vp, sz, sz, vp, vp, vp, ci, sz, vp, ci, vp, vp, vp, sz, vp]
    for name in exported_symbols():
        fn = getattr(lib, name)
        if fn.restype is None:
            fn.restype = ci
    _lib = lib
    return lib


def _p(t):
    """Device pointer of a tensor (None -> NULL); raw ints pass through."""
    if t is None:
        return None
    if isinstance(t, int):
        return ctypes.c_void_p(t)
    return ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    if isinstance(stream, int):
        return ctypes.c_void_p(stream)
    return ctypes.c_void_p(stream.cuda_stream)


def _check(status: int, where: str):
    if status != MQ_OK:
        raise MqError(status, where)


def mq_version() -> int:
    return int(load_library().mq_version())


def mq_status_string(status: int) -> str:
    return load_library().mq_status_string(int(status)).decode()


def mq_last_hip_error() -> int:
    return int(load_library().mq_last_hip_error())


def mq_set_gemm_variant(variant: int) -> None:
    _check(load_library().mq_set_gemm_variant(int(variant)), "mq_set_gemm_variant")


def mq_absmax_f32(x, n, amax, stream=None):
    _check(load_library().mq_absmax_f32(_p(x), n, _p(amax), _stream(stream)), "mq_absmax_f32")


def mq_scale_from_amax(amax, bits, scale, stream=None):
    _check(load_library().mq_scale_from_amax(_p(amax), bits, _p(scale), _stream(stream)), "mq_scale_from_amax")


def mq_quantize_f32(x, rows, cols, bits, scale, q, rowsum=None, stream=None):
    _check(load_library().mq_quantize_f32(_p(x), rows, cols, bits, _p(scale), _p(q), _p(rowsum),
                                          _stream(stream)), "mq_quantize_f32")


def mq_quantize_pack_f32(x, rows, cols, bits, scale, packed, stream=None):
    _check(load_library().mq_quantize_pack_f32(_p(x), rows, cols, bits, _p(scale), _p(packed), _stream(stream)),
           "mq_quantize_pack_f32")


def mq_gemm_i32_packed(packedA, packedW, bits, M, N, K, C, stream=None):
    _check(load_library().mq_gemm_i32_packed(_p(packedA), _p(packedW), bits, M, N, K, _p(C), _stream(stream)),
           "mq_gemm_i32_packed")


def mq_gemm_dequant_packed(packedA, packedW, bits, M, N, K, sA, sW, bias, relu, Y, out_amax=None, stream=None):
    _check(load_library().mq_gemm_dequant_packed(_p(packedA), _p(packedW), bits, M, N, K, _p(sA), _p(sW), _p(bias),
                                                 int(relu), _p(Y), _p(out_amax), _stream(stream)),
           "mq_gemm_dequant_packed")


def mq_packed_bytes(bits, N, K) -> int:
    return int(load_library().mq_packed_bytes(bits, N, K))


def mq_prepare_weight(B, b_is_transposed, N, K, bits, scale_or_null, scale_out, packed, stream=None):
    _check(load_library().mq_prepare_weight(_p(B), int(b_is_transposed), N, K, bits, _p(scale_or_null),
                                            _p(scale_out), _p(packed), _stream(stream)), "mq_prepare_weight")


def mq_unpack_weight(packed, bits, N, K, q_out, stream=None):
    _check(load_library().mq_unpack_weight(_p(packed), bits, N, K, _p(q_out), _stream(stream)), "mq_unpack_weight")


def mq_gemm_i32(qA, rowsumA, packedW, bits, M, N, K, C, stream=None):
    _check(load_library().mq_gemm_i32(_p(qA), _p(rowsumA), _p(packedW), bits, M, N, K, _p(C),
                                      _stream(stream)), "mq_gemm_i32")


def mq_gemm_dequant(qA, rowsumA, packedW, bits, M, N, K, sA, sW, bias, relu, Y, out_amax=None, stream=None):
    _check(load_library().mq_gemm_dequant(_p(qA), _p(rowsumA), _p(packedW), bits, M, N, K, _p(sA), _p(sW),
                                          _p(bias), int(relu), _p(Y), _p(out_amax), _stream(stream)),
           "mq_gemm_dequant")


def mq_argmax_ws_bytes(M, N) -> int:
    return int(load_library().mq_argmax_ws_bytes(M, N))


def mq_gemm_argmax(qA, packedW, M, N, K, sA, sW, tok, maxlogit, ws, ws_bytes, stream=None):
    _check(load_library().mq_gemm_argmax(_p(qA), _p(packedW), M, N, K, _p(sA), _p(sW), _p(tok), _p(maxlogit),
                                         _p(ws), ws_bytes, _stream(stream)), "mq_gemm_argmax")


def mq_gemm_argmax_packed(packedA, packedW, M, N, K, sA, sW, tok, maxlogit, ws, ws_bytes, stream=None):
    _check(load_library().mq_gemm_argmax_packed(_p(packedA), _p(packedW), M, N, K, _p(sA), _p(sW), _p(tok),
                                                _p(maxlogit), _p(ws), ws_bytes, _stream(stream)),
           "mq_gemm_argmax_packed")


def mq_gemm_argmax_packed_static(packedA, packedW, M, N, K, sA, sW, tok, maxlogit, stream=None):
    _check(load_library().mq_gemm_argmax_packed_static(_p(packedA), _p(packedW), M, N, K, _p(sA), _p(sW), _p(tok),
                                                       _p(maxlogit), _stream(stream)),
           "mq_gemm_argmax_packed_static")


def mq_gemm_argmax_shortlist(packedA, packedW, shortlist, shortlist_len, M, N, K, sA, sW, tok, maxlogit, ws, ws_bytes,
                             stream=None):
    _check(load_library().mq_gemm_argmax_shortlist(_p(packedA), _p(packedW), _p(shortlist), shortlist_len, M, N, K,
                                                   _p(sA), _p(sW), _p(tok), _p(maxlogit), _p(ws), ws_bytes,
                                                   _stream(stream)), "mq_gemm_argmax_shortlist")


def mq_linear_ws_bytes(bits, M, K) -> int:
    return int(load_library().mq_linear_ws_bytes(bits, M, K))


def mq_linear_f32(A, M, K, sA_or_null, packedW, sW, bits, N, bias, relu, Y, out_amax, ws, ws_bytes, stream=None):
    _check(load_library().mq_linear_f32(_p(A), M, K, _p(sA_or_null), _p(packedW), _p(sW), bits, N, _p(bias),
                                        int(relu), _p(Y), _p(out_amax), _p(ws), ws_bytes, _stream(stream)),
           "mq_linear_f32")


def mq_quantize_absmax_ws_bytes() -> int:
    return int(load_library().mq_quantize_absmax_ws_bytes())


def mq_quantize_absmax_pack_f32(x, rows, cols, bits, packed, scale_out, ws, ws_bytes, stream=None):
    _check(load_library().mq_quantize_absmax_pack_f32(_p(x), rows, cols, bits, _p(packed), _p(scale_out), _p(ws),
                                                      ws_bytes, _stream(stream)), "mq_quantize_absmax_pack_f32")


def mq_quantize_absmax_ws_prepare(ws, ws_bytes, stream=None):
    _check(load_library().mq_quantize_absmax_ws_prepare(_p(ws), ws_bytes, _stream(stream)),
           "mq_quantize_absmax_ws_prepare")


def mq_quantize_absmax_pack_f32_prepared(x, rows, cols, bits, packed, scale_out, ws, ws_bytes, stream=None):
    _check(load_library().mq_quantize_absmax_pack_f32_prepared(_p(x), rows, cols, bits, _p(packed), _p(scale_out),
                                                               _p(ws), ws_bytes, _stream(stream)),
           "mq_quantize_absmax_pack_f32_prepared")


def mq_gemm_amax_ws_bytes(M, N) -> int:
    return int(load_library().mq_gemm_amax_ws_bytes(M, N))


def mq_gemm_amax_packed(packedA, packedW, M, N, K, sA, sW, bias, relu, ws, ws_bytes, stream=None):
    _check(load_library().mq_gemm_amax_packed(_p(packedA), _p(packedW), M, N, K, _p(sA), _p(sW), _p(bias),
                                              int(relu), _p(ws), ws_bytes, _stream(stream)), "mq_gemm_amax_packed")


def mq_gemm_requant_packed(packedA, packedW, M, N, K, sA, sW, bias, relu, ws, ws_bytes, scale_out, packed_out,
                           stream=None):
    _check(load_library().mq_gemm_requant_packed(_p(packedA), _p(packedW), M, N, K, _p(sA), _p(sW), _p(bias),
                                                 int(relu), _p(ws), ws_bytes, _p(scale_out), _p(packed_out),
                                                 _stream(stream)), "mq_gemm_requant_packed")


def mq_gemm_requant_single_packed(packedA, packedW, M, N, K, sA, sW, bias, relu, ws, ws_bytes, scale_out,
                                  packed_out, stream=None):
    _check(load_library().mq_gemm_requant_single_packed(_p(packedA), _p(packedW), M, N, K, _p(sA), _p(sW),
                                                        _p(bias), int(relu), _p(ws), ws_bytes, _p(scale_out),
                                                        _p(packed_out), _stream(stream)),
           "mq_gemm_requant_single_packed")


def mq_gemm_requant_fixed_packed(packedA, packedW, M, N, K, sA, sW, bias, relu, s_out, packed_out, stream=None):
    _check(load_library().mq_gemm_requant_fixed_packed(_p(packedA), _p(packedW), M, N, K, _p(sA), _p(sW), _p(bias),
                                                       int(relu), _p(s_out), _p(packed_out), _stream(stream)),
           "mq_gemm_requant_fixed_packed")


def mq_gemm_requant_fixed_packed_i16(packedA, packedW, M, N, K, sA, sW, bias, relu, s_out, packed_out, stream=None):
    _check(load_library().mq_gemm_requant_fixed_packed_i16(_p(packedA), _p(packedW), M, N, K, _p(sA), _p(sW),
                                                           _p(bias), int(relu), _p(s_out), _p(packed_out),
                                                           _stream(stream)),
           "mq_gemm_requant_fixed_packed_i16")


def mq_autotune_ws_bytes(bits, M, N, K) -> int:
    return int(load_library().mq_autotune_ws_bytes(bits, M, N, K))


def mq_autotune_gemm(bits, M, N, K, runs, ws, ws_bytes, stream=None):
    """Returns (best_variant, average_microseconds)."""
    best = ctypes.c_int(0)
    us = ctypes.c_float(0.0)
    _check(load_library().mq_autotune_gemm(bits, M, N, K, runs, _p(ws), ws_bytes, _stream(stream),
                                           ctypes.byref(best), ctypes.byref(us)), "mq_autotune_gemm")
    return int(best.value), float(us.value)


def mq_autotune_report(n=16):
    """Microseconds per launch of every variant in the last mq_autotune_gemm run: {variant: us}."""
    buf = (ctypes.c_float * n)()
    _check(load_library().mq_autotune_report(buf, n), "mq_autotune_report")
    return {v: float(buf[v]) for v in range(1, n) if buf[v] >= 0.0}


def mq_set_ffn_single_pass(enable) -> None:
    _check(load_library().mq_set_ffn_single_pass(int(bool(enable))), "mq_set_ffn_single_pass")


def mq_set_quantize_single_pass(enable) -> None:
    _check(load_library().mq_set_quantize_single_pass(int(enable)), "mq_set_quantize_single_pass")


def mq_single_pass_fits(M, N, resident) -> bool:
    return bool(load_library().mq_single_pass_fits(M, N, resident))


def mq_set_barrier_timeout_us(us) -> None:
    _check(load_library().mq_set_barrier_timeout_us(int(us)), "mq_set_barrier_timeout_us")


def mq_ffn_ws_bytes(M, d, f) -> int:
    return int(load_library().mq_ffn_ws_bytes(M, d, f))


def mq_ffn_i8_f32(A, M, d, f, packedW1, sW1, b1, packedW2, sW2, b2, Y, ws, ws_bytes, stream=None):
    _check(load_library().mq_ffn_i8_f32(_p(A), M, d, f, _p(packedW1), _p(sW1), _p(b1), _p(packedW2), _p(sW2),
                                        _p(b2), _p(Y), _p(ws), ws_bytes, _stream(stream)), "mq_ffn_i8_f32")


def mq_ffn_ws_prepare(ws, ws_bytes, M, d, f, stream=None):
    _check(load_library().mq_ffn_ws_prepare(_p(ws), ws_bytes, M, d, f, _stream(stream)), "mq_ffn_ws_prepare")


def mq_ffn_i8_f32_prepared(A, M, d, f, packedW1, sW1, b1, packedW2, sW2, b2, Y, ws, ws_bytes, stream=None):
    _check(load_library().mq_ffn_i8_f32_prepared(_p(A), M, d, f, _p(packedW1), _p(sW1), _p(b1), _p(packedW2),
                                                 _p(sW2), _p(b2), _p(Y), _p(ws), ws_bytes, _stream(stream)),
           "mq_ffn_i8_f32_prepared")


def mq_ffn_i16_ws_bytes(M, d, f) -> int:
    return int(load_library().mq_ffn_i16_ws_bytes(M, d, f))


def mq_ffn_i16_f32(A, M, d, f, packedW1, sW1, b1, packedW2, sW2, b2, Y, ws, ws_bytes, stream=None):
    _check(load_library().mq_ffn_i16_f32(_p(A), M, d, f, _p(packedW1), _p(sW1), _p(b1), _p(packedW2), _p(sW2),
                                         _p(b2), _p(Y), _p(ws), ws_bytes, _stream(stream)), "mq_ffn_i16_f32")


def mq_ffn_i16_fixed_ws_bytes(M, d, f) -> int:
    return int(load_library().mq_ffn_i16_fixed_ws_bytes(M, d, f))


def mq_ffn_i16_fixed_f32(A, M, d, f, sA, packedW1, sW1, b1, sH, packedW2, sW2, b2, Y, ws, ws_bytes, stream=None):
    _check(load_library().mq_ffn_i16_fixed_f32(_p(A), M, d, f, _p(sA), _p(packedW1), _p(sW1), _p(b1), _p(sH),
                                               _p(packedW2), _p(sW2), _p(b2), _p(Y), _p(ws), ws_bytes, _stream(stream)),
           "mq_ffn_i16_fixed_f32")


def mq_topk_ws_bytes(M, N, k) -> int:
    return int(load_library().mq_topk_ws_bytes(M, N, int(k)))


def mq_gemm_topk_packed(packedA, packedW, shortlist, shortlist_len, M, N, K, sA, sW, k, tok, logprob, ws, ws_bytes,
                        stream=None):
    _check(load_library().mq_gemm_topk_packed(_p(packedA), _p(packedW), _p(shortlist), shortlist_len, M, N, K, _p(sA),
                                              _p(sW), int(k), _p(tok), _p(logprob), _p(ws), ws_bytes, _stream(stream)),
           "mq_gemm_topk_packed")


def mq_running_average_f32(g_prev, x, n, t, g, stream=None):
    _check(load_library().mq_running_average_f32(_p(g_prev), _p(x), n, int(t), _p(g), _stream(stream)),
           "mq_running_average_f32")


def mq_concat2_f32(a, da, b, db, M, out, stream=None):
    _check(load_library().mq_concat2_f32(_p(a), da, _p(b), db, M, _p(out), _stream(stream)), "mq_concat2_f32")


def mq_add_layer_norm_f32(a, r, gamma, beta, M, d, eps, y, stream=None):
    _check(load_library().mq_add_layer_norm_f32(_p(a), _p(r), _p(gamma), _p(beta), M, d, float(eps), _p(y),
                                                _stream(stream)), "mq_add_layer_norm_f32")


def mq_gate_mix_layer_norm_f32(x, f, z, gamma, beta, M, d, eps, y, stream=None):
    _check(load_library().mq_gate_mix_layer_norm_f32(_p(x), _p(f), _p(z), _p(gamma), _p(beta), M, d, float(eps), _p(y),
                                                     _stream(stream)), "mq_gate_mix_layer_norm_f32")


def mq_cross_attention_f32(q, K, V, M, S, d, heads, ctx, stream=None):
    _check(load_library().mq_cross_attention_f32(_p(q), _p(K), _p(V), M, S, d, int(heads), _p(ctx), _stream(stream)),
           "mq_cross_attention_f32")


def mq_aan_layer_ws_bytes(M, d, ffn, aan_ffn) -> int:
    return int(load_library().mq_aan_layer_ws_bytes(M, d, ffn, aan_ffn))


def mq_aan_layer_f32(layer, x, g_prev, t, K, V, M, S, heads, use_ffn, use_gate, eps, y, g_out, ws, ws_bytes,
                     stream=None):
    """layer: an AanLayer (see aan_layer); everything else as in include/mq.h."""
    _check(load_library().mq_aan_layer_f32(ctypes.byref(layer.c), _p(x), _p(g_prev), int(t), _p(K), _p(V), M, S,
                                           int(heads), int(bool(use_ffn)), int(bool(use_gate)), float(eps), _p(y),
                                           _p(g_out), _p(ws), ws_bytes, _stream(stream)), "mq_aan_layer_f32")


# ---- allocation helper (no arithmetic) --------------------------------------

@dataclass
class PreparedWeight:
    """Device buffers of one memoized parameter: packed bytes and its multiplier."""
    packed: torch.Tensor
    scale: torch.Tensor
    bits: int
    N: int
    K: int


def prepare_weight(W: torch.Tensor, bits: int, transposed: bool = True, scale: torch.Tensor | None = None,
                   stream=None) -> PreparedWeight:
    """Allocate the packed buffer and call mq_prepare_weight.  W is a float32 CUDA
    tensor, [N x K] if transposed else [K x N]."""
    if not W.is_cuda or W.dtype != torch.float32 or not W.is_contiguous():
        raise ValueError("W must be a contiguous float32 CUDA tensor")
    N, K = (W.shape if transposed else W.shape[::-1])
    packed = torch.empty(mq_packed_bytes(bits, N, K), dtype=torch.uint8, device=W.device)
    scale_out = torch.empty(1, dtype=torch.float32, device=W.device)
    mq_prepare_weight(W, transposed, N, K, bits, scale, scale_out, packed, stream)
    return PreparedWeight(packed, scale_out, bits, int(N), int(K))


@dataclass
class AanLayer:
    """The C struct of one decoder layer plus the tensors that keep its device memory alive."""
    c: object
    keep: list


def aan_layer(products: dict, norms: dict, d: int, ffn: int, aan_ffn: int) -> AanLayer:
    """Fill an mq_aan_layer from prepared parameters (marshalling only).

    products: name -> (PreparedWeight, bias tensor or None) for aan_ffn1, aan_ffn2, aan_gate, ctx_q, ctx_o, ffn1,
    ffn2 (the averaging block's entries may be missing for the "-ffn" / "-gate" variants);
    norms: name -> (gamma, beta) for ln1, ln2, ln3."""
    c = _CAanLayer()
    keep = []
    for name in ("aan_ffn1", "aan_ffn2", "aan_gate", "ctx_q", "ctx_o", "ffn1", "ffn2"):
        if name in products:
            pw, bias = products[name]
            setattr(c, name, _CProduct(pw.packed.data_ptr(), pw.scale.data_ptr(), None if bias is None else bias.data_ptr()))
            keep += [pw, bias]
    for name in ("ln1", "ln2", "ln3"):
        gamma, beta = norms[name]
        setattr(c, name, _CNorm(gamma.data_ptr(), beta.data_ptr()))
        keep += [gamma, beta]
    c.d, c.ffn, c.aan_ffn = d, ffn, aan_ffn
    return AanLayer(c, keep)
