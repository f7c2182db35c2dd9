"""CPU oracle for the MoE expert FFN layer (arXiv 2211.10017, Sec. 3.3-3.4).

TEST INFRASTRUCTURE ONLY: numpy marshalling around ``moe_oracle.c``.  Only the tests, the
smoke check and the benchmark's cpu_baseline leg may import this package; the product path
never does, and this package never imports the product.

All real tensors are float32 numpy arrays whose values are representable in the dtype the
method stores them in (fp16 / bf16).  dtype codes: 0 = fp16, 1 = bf16, 2 = fp32.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

F16, BF16, F32 = 0, 1, 2

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "moe_oracle.c")
_LIB = os.path.join(_HERE, "libmoe_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile moe_oracle.c with gcc (-O2, no fast-math, OpenMP over rows/experts)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-Wall", "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _c():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        lib.orc_f32_to_f16_bits.restype = ctypes.c_uint16
        lib.orc_f32_to_f16_bits.argtypes = [ctypes.c_float]
        lib.orc_f16_bits_to_f32.restype = ctypes.c_float
        lib.orc_f16_bits_to_f32.argtypes = [ctypes.c_uint16]
        lib.orc_f32_to_bf16_bits.restype = ctypes.c_uint16
        lib.orc_f32_to_bf16_bits.argtypes = [ctypes.c_float]
        lib.orc_i2f_magic.restype = ctypes.c_uint16
        lib.orc_i2f_magic.argtypes = [ctypes.c_uint, ctypes.c_uint, ctypes.c_void_p]
        lib.orc_num_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def _p(a: np.ndarray):
    return ctypes.c_void_p(a.ctypes.data)


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def num_threads() -> int:
    return int(_c().orc_num_threads())


def set_num_threads(n: int) -> None:
    """Threads the oracle's loops use from now on (for timing it on one core)."""
    _c().orc_set_num_threads(ctypes.c_int(int(n)))


# ------------------------------------------------------------------ number formats
def f32_to_f16_bits(v: float) -> int:
    return int(_c().orc_f32_to_f16_bits(ctypes.c_float(v)))


def f16_bits_to_f32(b: int) -> float:
    return float(_c().orc_f16_bits_to_f32(ctypes.c_uint16(b)))


def f32_to_bf16_bits(v: float) -> int:
    return int(_c().orc_f32_to_bf16_bits(ctypes.c_float(v)))


def round_to(a, dtype: int) -> np.ndarray:
    """Round every element to fp16 / bf16 (ties to even); result stays float32."""
    a = _f32(a)
    out = np.empty_like(a)
    _c().orc_round_array(_p(a), ctypes.c_size_t(a.size), ctypes.c_int(dtype), _p(out))
    return out


def i2f_magic(code_plus: int, offset: int):
    """Sec. 3.4.1: returns (fp16 bits of 1024+code_plus, fp16 bits of code_plus-offset)."""
    biased = ctypes.c_uint16(0)
    res = _c().orc_i2f_magic(ctypes.c_uint(code_plus), ctypes.c_uint(offset), ctypes.byref(biased))
    return int(biased.value), int(res)


def int4_interleave8(codes) -> np.ndarray:
    a = np.ascontiguousarray(codes, dtype=np.int8)
    assert a.size == 8
    out = np.empty(8, dtype=np.int8)
    _c().orc_int4_interleave8(_p(a), _p(out))
    return out


# ------------------------------------------------------------------ quantisation
def quantize(w, bits: int, group_size: int = 0):
    """w float32 [E,K,N] -> (q int8 [E,K,N], s_bits uint16 [E,K/g,N] fp16 bit patterns)."""
    w = _f32(w)
    E, K, N = w.shape
    g = K if group_size in (0, K) else group_size
    assert bits in (4, 8) and K % g == 0
    q = np.empty((E, K, N), dtype=np.int8)
    s = np.empty((E, K // g, N), dtype=np.uint16)
    _c().orc_quantize(_p(w), E, K, N, bits, g, _p(q), _p(s))
    return q, s


def pack_int4(q) -> np.ndarray:
    q = np.ascontiguousarray(q, dtype=np.int8)
    assert q.shape[-1] % 2 == 0
    out = np.empty(q.shape[:-1] + (q.shape[-1] // 2,), dtype=np.uint8)
    _c().orc_pack_int4(_p(q), ctypes.c_size_t(q.size), _p(out))
    return out


def unpack_int4(b) -> np.ndarray:
    b = np.ascontiguousarray(b, dtype=np.uint8)
    q = np.empty(b.shape[:-1] + (b.shape[-1] * 2,), dtype=np.int8)
    _c().orc_unpack_int4(_p(b), ctypes.c_size_t(q.size), _p(q))
    return q


def scales_to_f32(s_bits) -> np.ndarray:
    return np.ascontiguousarray(s_bits, dtype=np.uint16).view(np.float16).astype(np.float32)


def dequantize(q, s_bits, group_size: int = 0) -> np.ndarray:
    """Algorithm 1.  q int8 [E,K,N], s_bits uint16 [E,K/g,N] -> float32 [E,K,N]."""
    q = np.ascontiguousarray(q, dtype=np.int8)
    s_bits = np.ascontiguousarray(s_bits, dtype=np.uint16)
    E, K, N = q.shape
    g = K if group_size in (0, K) else group_size
    assert s_bits.shape == (E, K // g, N)
    out = np.empty((E, K, N), dtype=np.float32)
    _c().orc_dequantize(_p(q), _p(s_bits), E, K, N, g, _p(out))
    return out


# ------------------------------------------------------------------ gate / routing
def gate(x, wg, bias, k: int, renormalize: bool = True, return_logits: bool = False, finished=None):
    """finished [T] (nonzero = pruned row, Sec. 3.5): such rows get expert index E and scale 0."""
    x, wg = _f32(x), _f32(wg)
    T, d = x.shape
    E = wg.shape[1]
    assert wg.shape[0] == d and 1 <= k <= min(E, 8)
    b = None if bias is None else _f32(bias)
    idx = np.empty((T, k), dtype=np.int32)
    scale = np.empty((T, k), dtype=np.float32)
    logits = np.empty((T, E), dtype=np.float32) if return_logits else None
    fin = None if finished is None else np.ascontiguousarray(finished, dtype=np.uint8)
    _c().orc_gate(_p(x), _p(wg), None if b is None else _p(b), None if fin is None else _p(fin),
                  T, d, E, k, int(renormalize),
                  _p(idx), _p(scale), None if logits is None else _p(logits))
    return (idx, scale, logits) if return_logits else (idx, scale)


def permute(expert_idx, E: int):
    """expert_idx int32 [T,k] -> (perm_src [R], inv_perm [R], offsets [E+1]).
    Index E marks pruned rows: they sort last and offsets[E] counts the active rows."""
    idx = _i32(expert_idx)
    T, k = idx.shape
    R = T * k
    perm_src = np.empty(R, dtype=np.int32)
    inv_perm = np.empty(R, dtype=np.int32)
    offsets = np.empty(E + 1, dtype=np.int32)
    _c().orc_permute(_p(idx), T, k, E, _p(perm_src), _p(inv_perm), _p(offsets))
    return perm_src, inv_perm, offsets


def gather_rows(x, perm_src, k: int) -> np.ndarray:
    x, perm_src = _f32(x), _i32(perm_src)
    R, d = perm_src.shape[0], x.shape[1]
    out = np.empty((R, d), dtype=np.float32)
    _c().orc_gather_rows(_p(x), _p(perm_src), R, k, d, _p(out))
    return out


# ------------------------------------------------------------------ FFN / combine
RELU, GELU = 0, 1


def expert_ffn(x_rows, w1dq, w2dq, act_dtype: int, b1=None, b2=None, return_h: bool = False, activation: int = RELU):
    """One expert: relu(x @ w1dq + b1) rounded to act_dtype, then @ w2dq + b2 (unrounded)."""
    x_rows, w1dq, w2dq = _f32(x_rows), _f32(w1dq), _f32(w2dq)
    m, d = x_rows.shape
    F = w1dq.shape[1]
    assert w1dq.shape == (d, F) and w2dq.shape == (F, d)
    b1 = None if b1 is None else _f32(b1)
    b2 = None if b2 is None else _f32(b2)
    y = np.empty((m, d), dtype=np.float32)
    h = np.empty((m, F), dtype=np.float32) if return_h else None
    if m:
        _c().orc_expert_ffn(_p(x_rows), m, d, F, _p(w1dq), None if b1 is None else _p(b1),
                            _p(w2dq), None if b2 is None else _p(b2), act_dtype, int(activation),
                            None if h is None else _p(h), _p(y))
    return (y, h) if return_h else y


def combine(y_perm, inv_perm, scale, T: int, k: int, active_rows=None) -> np.ndarray:
    y_perm, inv_perm, scale = _f32(y_perm), _i32(inv_perm), _f32(scale)
    d = y_perm.shape[1]
    out = np.empty((T, d), dtype=np.float32)
    _c().orc_combine(_p(y_perm), _p(inv_perm), _p(scale), T, k, d,
                     T * k if active_rows is None else int(active_rows), _p(out))
    return out


def grouped_ffn(x_perm, offsets, q1, s1, q2, s2, group_size: int, act_dtype: int,
                b1=None, b2=None, rows=None, return_h: bool = False, activation: int = RELU):
    """Grouped expert FFN over expert-contiguous rows (Sec. 3.3, Fig. 1).

    q1 [E,d,F] / q2 [E,F,d] int8 codes with fp16-bit scales; expert e owns rows
    offsets[e]:offsets[e+1].  ``rows`` (sorted row numbers) restricts the work to a subset;
    rows are independent given the routing, so the subset is exact.  Experts are dequantised
    one at a time (Algorithm 1).  Returns y float32 [R,d] (rows not asked for stay zero).
    """
    x_perm = _f32(x_perm)
    R, d = x_perm.shape
    E, _, F = q1.shape
    y = np.zeros((R, d), dtype=np.float32)
    h = np.zeros((R, F), dtype=np.float32) if return_h else None
    want = None if rows is None else np.asarray(rows, dtype=np.int64)
    for e in range(E):
        lo, hi = int(offsets[e]), int(offsets[e + 1])
        if hi <= lo:
            continue
        sel = np.arange(lo, hi) if want is None else want[(want >= lo) & (want < hi)]
        if sel.size == 0:
            continue
        w1 = dequantize(q1[e:e + 1], s1[e:e + 1], group_size)[0]
        w2 = dequantize(q2[e:e + 1], s2[e:e + 1], group_size)[0]
        res = expert_ffn(x_perm[sel], w1, w2, act_dtype,
                         None if b1 is None else b1[e], None if b2 is None else b2[e],
                         return_h=return_h, activation=activation)
        if return_h:
            y[sel], h[sel] = res
        else:
            y[sel] = res
    return (y, h) if return_h else y


def grouped_gemm(x_perm, offsets, w_dq):
    """One grouped GEMM (the operation Table 1 times): y[r] = x_perm[r] @ w_dq[e] for the rows r of
    expert e, accumulated in fp64.  w_dq float32 [E,K,N] (dequantised or plain weights)."""
    x_perm = _f32(x_perm)
    R = x_perm.shape[0]
    E, K, N = w_dq.shape
    y = np.zeros((R, N), dtype=np.float64)
    for e in range(E):
        lo, hi = int(offsets[e]), int(offsets[e + 1])
        for r in range(lo, hi):
            acc = np.zeros(N, dtype=np.float64)
            for i in range(K):
                acc += float(x_perm[r, i]) * w_dq[e, i].astype(np.float64)
            y[r] = acc
    return y.astype(np.float32)


def moe_layer(x, wg, gate_bias, q1, s1, q2, s2, k: int, group_size: int, act_dtype: int,
              renormalize: bool = True, y_dtype: int = F32, b1=None, b2=None, finished=None,
              activation: int = RELU):
    """Gate -> permute -> grouped FFN -> combine; returns a dict of every intermediate.
    finished [T]: rows pruned from the batch (Sec. 3.5); their output rows are zero."""
    E = q1.shape[0]
    T = x.shape[0]
    idx, scale = gate(x, wg, gate_bias, k, renormalize, finished=finished)
    perm_src, inv_perm, offsets = permute(idx, E)
    x_perm = gather_rows(x, perm_src, k)
    y_perm = grouped_ffn(x_perm, offsets, q1, s1, q2, s2, group_size, act_dtype, b1, b2, activation=activation)
    y_perm = round_to(y_perm, y_dtype)
    out = combine(y_perm, inv_perm, scale, T, k, active_rows=int(offsets[E]))
    return dict(expert_idx=idx, expert_scale=scale, perm_src=perm_src, inv_perm=inv_perm,
                expert_offsets=offsets, x_perm=x_perm, y_perm=y_perm, out=out)


def moe_layer_dense_masked(x, wg, gate_bias, q1, s1, q2, s2, k: int, group_size: int,
                           act_dtype: int, renormalize: bool = True, y_dtype: int = F32):
    """Same layer without sorting: out[t] = sum_e G[t,e] * FFN_e(x[t]), every expert applied
    to every token and masked by the gate matrix G.  Independent of permute/combine."""
    x = _f32(x)
    T, d = x.shape
    E = q1.shape[0]
    idx, scale = gate(x, wg, gate_bias, k, renormalize)
    out = np.zeros((T, d), dtype=np.float64)
    for e in range(E):
        w1 = dequantize(q1[e:e + 1], s1[e:e + 1], group_size)[0]
        w2 = dequantize(q2[e:e + 1], s2[e:e + 1], group_size)[0]
        y = round_to(expert_ffn(x, w1, w2, act_dtype), y_dtype).astype(np.float64)
        for j in range(k):
            g = np.where(idx[:, j] == e, scale[:, j], 0.0).astype(np.float64)
            out += g[:, None] * y
    return out.astype(np.float32)
