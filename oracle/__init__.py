"""CPU oracle for the quantize -> integer product -> epilogue / arg-max path.

TEST INFRASTRUCTURE ONLY: tests, the smoke check and the benchmark's
CPU-baseline leg may import this package; the product never does.  The
arithmetic lives in ``mq_oracle.c`` (plain C, compiled with gcc); this module
only marshals numpy arrays into it.  Nothing here touches the HIP library.

Function names follow arxiv 1805.12096: ``quant_int`` (Section 4.2),
``dot_int`` for dot'_int (Section 4.3), the greedy arg-max of Section 2.3.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
import time

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "mq_oracle.c")
_LIB = os.path.join(_HERE, "libmq_oracle.so")

QMAX = {8: 127, 16: 32767}
_QDTYPE = {8: np.int8, 16: np.int16}


def build(force: bool = False) -> str:
    """Compile mq_oracle.c with gcc.  No fast-math, no FP contraction."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
               "-fno-fast-math", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        c_sz, c_f, c_p = ctypes.c_size_t, ctypes.c_float, ctypes.c_void_p
        lib.orc_num_threads.restype = ctypes.c_int
        lib.orc_set_num_threads.argtypes = [ctypes.c_int]
        lib.orc_absmax_f32.restype = c_f
        lib.orc_absmax_f32.argtypes = [c_p, c_sz, c_p]
        lib.orc_scale_from_amax.restype = c_f
        lib.orc_scale_from_amax.argtypes = [c_f, ctypes.c_int]
        lib.orc_quant_int.argtypes = [c_p, c_sz, ctypes.c_int, c_f, c_p, c_p]
        lib.orc_dot_int.argtypes = [c_p, c_p, ctypes.c_int, c_sz, c_sz, c_sz, c_p, c_p]
        lib.orc_dequant_bias.argtypes = [c_p, c_sz, c_sz, c_f, c_f, c_p, ctypes.c_int, c_p]
        lib.orc_argmax_i32.argtypes = [c_p, c_sz, c_sz, c_f, c_f, c_p, c_p]
        lib.orc_argmax_f32.argtypes = [c_p, c_sz, c_sz, c_p, c_p]
        _lib = lib
    return _lib


def _ptr(a: np.ndarray) -> ctypes.c_void_p:
    return ctypes.c_void_p(a.ctypes.data)


def _f32(x) -> np.ndarray:
    return np.ascontiguousarray(x, dtype=np.float32)


def num_threads() -> int:
    return int(_load().orc_num_threads())


def set_num_threads(n: int) -> None:
    _load().orc_set_num_threads(int(n))


def absmax(x) -> float:
    """max |x| in binary32, NaNs skipped."""
    x = _f32(x)
    return float(_load().orc_absmax_f32(_ptr(x), x.size, None))


def nan_count(x) -> int:
    x = _f32(x)
    c = ctypes.c_uint64(0)
    _load().orc_absmax_f32(_ptr(x), x.size, ctypes.byref(c))
    return int(c.value)


def scale_from_amax(amax: float, bits: int) -> np.float32:
    """Qmax / amax as one binary32 division (1 for an all-zero tensor)."""
    return np.float32(_load().orc_scale_from_amax(ctypes.c_float(float(amax)), int(bits)))


def quant_int(x, bits: int, scale) -> np.ndarray:
    """clamp(rint(x * scale), +-Qmax) as int8 / int16, same shape as x."""
    x = _f32(x)
    q = np.empty(x.shape, dtype=_QDTYPE[bits])
    rc = _load().orc_quant_int(_ptr(x), x.size, int(bits), ctypes.c_float(float(scale)), _ptr(q), None)
    if rc != 0:
        raise ValueError("bits must be 8 or 16")
    return q


def quant_int_absmax(x, bits: int):
    """Per-tensor abs-max quantization: returns (q, scale)."""
    s = scale_from_amax(absmax(x), bits)
    return quant_int(x, bits, s), s


def dot_int(qA: np.ndarray, qB: np.ndarray, return_overflow: bool = False):
    """dot'_int(A, B) = A . B^T with exact sums stored modulo 2^32.

    qA is [M x K], qB is [N x K], both int8 or both int16.
    """
    if qA.dtype != qB.dtype or qA.dtype not in (np.int8, np.int16):
        raise ValueError("operands must both be int8 or both int16")
    qA = np.ascontiguousarray(qA)
    qB = np.ascontiguousarray(qB)
    M, K = qA.shape
    N, K2 = qB.shape
    if K != K2:
        raise ValueError("contracted sizes differ")
    acc = np.empty((M, N), dtype=np.int32)
    over = ctypes.c_uint64(0)
    bits = 8 if qA.dtype == np.int8 else 16
    rc = _load().orc_dot_int(_ptr(qA), _ptr(qB), bits, M, N, K, _ptr(acc), ctypes.byref(over))
    assert rc == 0
    return (acc, int(over.value)) if return_overflow else acc


def dequant_bias(acc: np.ndarray, sA, sW, bias=None, relu: bool = False) -> np.ndarray:
    """y = fma(float(acc), 1/(sA*sW), bias), optional ReLU, binary32."""
    acc = np.ascontiguousarray(acc, dtype=np.int32)
    M, N = acc.shape
    Y = np.empty((M, N), dtype=np.float32)
    b = None if bias is None else _f32(bias)
    if b is not None and b.shape != (N,):
        raise ValueError("bias must have N entries")
    _load().orc_dequant_bias(_ptr(acc), M, N, ctypes.c_float(float(sA)), ctypes.c_float(float(sW)),
                             None if b is None else _ptr(b), int(bool(relu)), _ptr(Y))
    return Y


def argmax_i32(acc: np.ndarray, sA, sW):
    """Greedy arg-max on integer sums: (token ids int32[M], max logit float32[M])."""
    acc = np.ascontiguousarray(acc, dtype=np.int32)
    M, N = acc.shape
    tok = np.empty(M, dtype=np.int32)
    val = np.empty(M, dtype=np.float32)
    rc = _load().orc_argmax_i32(_ptr(acc), M, N, ctypes.c_float(float(sA)), ctypes.c_float(float(sW)),
                                _ptr(tok), _ptr(val))
    if rc != 0:
        raise ValueError("N must be positive")
    return tok, val


def argmax_f32(Y: np.ndarray):
    Y = _f32(Y)
    M, N = Y.shape
    tok = np.empty(M, dtype=np.int32)
    val = np.empty(M, dtype=np.float32)
    rc = _load().orc_argmax_f32(_ptr(Y), M, N, _ptr(tok), _ptr(val))
    if rc != 0:
        raise ValueError("N must be positive")
    return tok, val


# ---- compositions of the steps above, in the order the path takes them ------

def linear(A, Wt, bits: int, bias=None, relu: bool = False, sA=None, sW=None):
    """quant_int both operands, dot'_int, dequantize + bias (+ReLU).

    A is [M x K] float, Wt is [N x K] float (the transposed parameter).
    Scales default to per-tensor Qmax / max|x|.  Returns a dict with every
    intermediate so a test can compare each stage.
    """
    if sA is None:
        sA = scale_from_amax(absmax(A), bits)
    if sW is None:
        sW = scale_from_amax(absmax(Wt), bits)
    qA = quant_int(A, bits, sA)
    qW = quant_int(Wt, bits, sW)
    acc, over = dot_int(qA, qW, return_overflow=True)
    Y = dequant_bias(acc, sA, sW, bias, relu)
    return {"sA": np.float32(sA), "sW": np.float32(sW), "qA": qA, "qW": qW, "acc": acc,
            "overflow_count": over, "Y": Y}


def greedy_output_layer(Hd, E, bits: int = 8, sA=None, sW=None, shortlist=None):
    """Output layer with tied embedding E [V x d] and beam-1 arg-max, no softmax.

    shortlist (Section 4.1): ascending vocabulary ids; the product is restricted to those rows
    of the quantized embedding (the whole embedding is quantized once, with its own multiplier)
    and the winning position is mapped back to its vocabulary id.
    """
    if sA is None:
        sA = scale_from_amax(absmax(Hd), bits)
    if sW is None:
        sW = scale_from_amax(absmax(E), bits)
    qA = quant_int(Hd, bits, sA)
    qW = quant_int(E, bits, sW)
    if shortlist is not None:
        shortlist = np.asarray(shortlist, dtype=np.int64)
        if shortlist.ndim != 1 or shortlist.size == 0 or np.any(np.diff(shortlist) <= 0) \
                or shortlist[0] < 0 or shortlist[-1] >= qW.shape[0]:
            raise ValueError("shortlist must be strictly ascending ids inside the vocabulary")
        rows = np.ascontiguousarray(qW[shortlist])          # gather only, no arithmetic
    else:
        rows = qW
    acc = dot_int(qA, rows)
    pos, val = argmax_i32(acc, sA, sW)
    tok = pos if shortlist is None else shortlist[pos].astype(np.int32)
    return {"sA": np.float32(sA), "sW": np.float32(sW), "qA": qA, "qW": qW, "acc": acc,
            "tok": tok, "maxlogit": val}


def topk_log_softmax(Hd, E, k: int, bits: int = 8, sA=None, sW=None):
    """Output layer for beam search with beam size k > 1 (Table 2, the b = 2 and b = 4 rows): the k most
    probable words of every row with their log-probabilities, log p[n] = y[n] - log sum_n' exp(y[n']).

    Logits y = (float) acc * u with u = 1 / (sA * sW) as in dequant_bias (no bias: tied output layer);
    the normaliser is evaluated in binary64 from those binary32 logits.  The k best are chosen on the
    integer sums (u > 0), ties towards the lower vocabulary index, best first."""
    if sA is None:
        sA = scale_from_amax(absmax(Hd), bits)
    if sW is None:
        sW = scale_from_amax(absmax(E), bits)
    qA = quant_int(Hd, bits, sA)
    qW = quant_int(E, bits, sW)
    acc = dot_int(qA, qW)
    M, N = acc.shape
    if not 1 <= k <= N:
        raise ValueError("k must be between 1 and the vocabulary size")
    y32 = dequant_bias(acc, sA, sW)                       # binary32 logits, one rounding each
    y = y32.astype(np.float64)
    mx = y.max(axis=1, keepdims=True)
    lse = np.log(np.exp(y - mx).sum(axis=1, keepdims=True)) + mx
    tok = np.empty((M, k), dtype=np.int32)
    for m in range(M):
        order = np.lexsort((np.arange(N), -acc[m].astype(np.int64)))      # sum descending, index ascending
        tok[m] = order[:k]
    logprob = np.take_along_axis(y, tok.astype(np.int64), axis=1) - lse
    return {"sA": np.float32(sA), "sW": np.float32(sW), "acc": acc, "tok": tok, "logprob": logprob, "lse": lse[:, 0]}


def timed(fn, *args, **kw):
    t0 = time.perf_counter()
    out = fn(*args, **kw)
    return out, time.perf_counter() - t0
