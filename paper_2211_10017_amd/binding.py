"""Thin ctypes binding of the C-ABI HIP library (include/moe_wq.h).

Argument marshalling only: every function takes torch CUDA tensors, checks their dtype,
device and contiguity, and passes raw device pointers plus the current stream.  No step of
the layer runs in Python or in torch ops.  If the library has not been built the first call
raises: there is no fallback path.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmoe_wq.so")

MOE_F16, MOE_BF16, MOE_F32 = 0, 1, 2
_DT = {torch.float16: MOE_F16, torch.bfloat16: MOE_BF16, torch.float32: MOE_F32}

EXPORTS = ["moe_last_error", "moe_last_ffn_kernels", "moe_device_info", "moe_abi_version", "moe_quantize_experts", "moe_gate_topk",
           "moe_permute_workspace_bytes", "moe_permute", "moe_grouped_ffn_wq_workspace_bytes",
           "moe_grouped_ffn_wq", "moe_combine", "moe_pack_fp16_experts", "moe_grouped_gemm_wq",
           "moe_grouped_ffn_wq_routed_supported", "moe_grouped_ffn_wq_routed",
           "moe_grouped_ffn_wq_gated_supported", "moe_grouped_ffn_wq_gated",
           "moe_grouped_ffn_wq_noalloc_max_bytes", "moe_grouped_ffn_wq_noalloc"]

LAYER_MAX_EXPERTS = 256   # experts of a whole layer call: moe_gate_topk's limit (moe_permute: 1024, the FFN: 4096)

_lib = None
ACTIVATIONS = {"relu": 0, "gelu": 1}     # MOE_ACT_RELU, MOE_ACT_GELU


class MoeError(RuntimeError):
    pass


def load():
    """Load libmoe_wq.so (once) and declare the signatures of include/moe_wq.h."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise MoeError("HIP library %s is missing: build it with "
                       "`python -m paper_2211_10017_amd.build` (no fallback exists)" % LIB_PATH)
    lib = ctypes.CDLL(LIB_PATH)
    vp, i, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
    lib.moe_last_error.restype = ctypes.c_char_p
    lib.moe_last_error.argtypes = []
    lib.moe_last_ffn_kernels.restype = ctypes.c_char_p
    lib.moe_last_ffn_kernels.argtypes = []
    lib.moe_device_info.restype = i
    lib.moe_device_info.argtypes = [ctypes.POINTER(i)] * 4
    lib.moe_abi_version.restype = i
    lib.moe_quantize_experts.restype = i
    lib.moe_quantize_experts.argtypes = [vp, i, i, i, i, i, vp, vp, vp, vp]
    lib.moe_gate_topk.restype = i
    lib.moe_gate_topk.argtypes = [vp, i, vp, vp, vp, i, i, i, i, i, vp, vp, vp]
    lib.moe_permute_workspace_bytes.restype = sz
    lib.moe_permute_workspace_bytes.argtypes = [i, i, i]
    lib.moe_permute.restype = i
    lib.moe_permute.argtypes = [vp, vp, i, i, i, i, i, vp, vp, vp, vp, vp, sz, vp]
    lib.moe_grouped_ffn_wq_workspace_bytes.restype = sz
    lib.moe_grouped_ffn_wq_workspace_bytes.argtypes = [i, i, i, i, i]
    lib.moe_grouped_ffn_wq.restype = i
    lib.moe_grouped_ffn_wq.argtypes = [vp, i, vp, i, i, i, i, i, i, i, i, vp, vp, vp, vp, vp, vp, vp, i, vp, sz, vp]
    lib.moe_grouped_ffn_wq_noalloc_max_bytes.restype = sz
    lib.moe_grouped_ffn_wq_noalloc_max_bytes.argtypes = []
    lib.moe_grouped_ffn_wq_noalloc.restype = i
    lib.moe_grouped_ffn_wq_noalloc.argtypes = [vp, i, vp, i, i, i, i, i, i, i, i, vp, vp, vp, vp, vp, vp, vp, i, vp]
    lib.moe_grouped_ffn_wq_routed_supported.restype = i
    lib.moe_grouped_ffn_wq_routed_supported.argtypes = [i, i, i, i, i, i, i, i]
    lib.moe_grouped_ffn_wq_routed.restype = i
    lib.moe_grouped_ffn_wq_routed.argtypes = [vp, i, vp, i, vp, vp, i, i, i, i, i, i, i, i, vp, vp, vp, vp, vp, vp, vp, i,
                                              vp, sz, vp]
    lib.moe_grouped_ffn_wq_gated_supported.restype = i
    lib.moe_grouped_ffn_wq_gated_supported.argtypes = [i, i, i, i, i, i, i, i]
    lib.moe_grouped_ffn_wq_gated.restype = i
    lib.moe_grouped_ffn_wq_gated.argtypes = [vp, i, vp, vp, i, i, i, i, i, i, i, i, vp, vp, vp, vp, vp, vp, vp, i, vp, vp, vp,
                                             vp, sz, vp]
    lib.moe_pack_fp16_experts.restype = i
    lib.moe_pack_fp16_experts.argtypes = [vp, i, i, i, vp, vp]
    lib.moe_grouped_gemm_wq.restype = i
    lib.moe_grouped_gemm_wq.argtypes = [vp, vp, i, i, i, i, i, i, i, vp, vp, vp, i, vp]
    lib.moe_combine.restype = i
    lib.moe_combine.argtypes = [vp, i, vp, vp, vp, i, i, i, vp, i, vp]
    _lib = lib
    return lib


def moe_device_info() -> dict:
    """Compute units, engine / memory clock (kHz) and memory bus width (bits) of the current device."""
    v = [ctypes.c_int(0) for _ in range(4)]
    _check(load().moe_device_info(*[ctypes.byref(x) for x in v]), "moe_device_info")
    return dict(zip(("compute_units", "engine_clock_khz", "memory_clock_khz", "memory_bus_bits"), (x.value for x in v)))


def _check(rc: int, what: str):
    if rc != 0:
        raise MoeError("%s failed (code %d): %s" % (what, rc, load().moe_last_error().decode()))


def _ptr(t, dtype=None, name="tensor"):
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise MoeError("%s must be a contiguous CUDA tensor" % name)
    if dtype is not None and t.dtype not in (dtype if isinstance(dtype, tuple) else (dtype,)):
        raise MoeError("%s has dtype %s, expected %s" % (name, t.dtype, dtype))
    return ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def moe_quantize_experts(w, bits: int, group_size: int = 0, want_canon: bool = True,
                         want_packed: bool = True):
    """w fp32 [E,K,N] -> (q_canon uint8/int8, scales fp16 [E,K/g,N], q_packed uint8)."""
    E, K, N = w.shape
    g = K if group_size in (0, K) else group_size
    dev = w.device
    nbytes = E * K * N * bits // 8
    q_canon = None
    if want_canon:
        q_canon = (torch.empty((E, K, N), dtype=torch.int8, device=dev) if bits == 8
                   else torch.empty((E, K, N // 2), dtype=torch.uint8, device=dev))
    scales = torch.empty((E, K // g, N), dtype=torch.float16, device=dev)
    q_packed = torch.empty(nbytes, dtype=torch.uint8, device=dev) if want_packed else None
    rc = load().moe_quantize_experts(_ptr(w, torch.float32, "w"), E, K, N, bits, group_size,
                                     _ptr(q_canon), _ptr(scales), _ptr(q_packed), _stream())
    _check(rc, "moe_quantize_experts")
    return q_canon, scales, q_packed


def moe_quantize_experts_into(w, bits, group_size, q_canon, scales, q_packed):
    """Same call writing into caller-provided slices (for expert-at-a-time quantisation)."""
    E, K, N = w.shape
    rc = load().moe_quantize_experts(_ptr(w, torch.float32, "w"), E, K, N, bits, group_size,
                                     _ptr(q_canon), _ptr(scales, torch.float16), _ptr(q_packed), _stream())
    _check(rc, "moe_quantize_experts")


def moe_gate_topk(x, wg, bias, k: int, renormalize: bool = True, out=None, finished=None):
    T, d = x.shape
    E = wg.shape[1]
    if wg.dtype != x.dtype or wg.shape[0] != d:
        raise MoeError("wg must be [d,E] in the dtype of x")
    if out is None:
        idx = torch.empty((T, k), dtype=torch.int32, device=x.device)
        scale = torch.empty((T, k), dtype=torch.float32, device=x.device)
    else:
        idx, scale = out
    rc = load().moe_gate_topk(_ptr(x, (torch.float16, torch.bfloat16), "x"), _DT[x.dtype], _ptr(wg),
                              _ptr(bias, torch.float32, "bias"), _ptr(finished, torch.uint8, "finished"),
                              T, d, E, k, int(renormalize),
                              _ptr(idx, torch.int32), _ptr(scale, torch.float32), _stream())
    _check(rc, "moe_gate_topk")
    return idx, scale


def moe_permute_workspace_bytes(T: int, k: int, E: int) -> int:
    return int(load().moe_permute_workspace_bytes(T, k, E))


def moe_permute(expert_idx, x, E: int, out=None, workspace=None):
    T, k = expert_idx.shape
    d = x.shape[1]
    R = T * k
    dev = x.device
    if out is None:
        x_perm = torch.empty((R, d), dtype=x.dtype, device=dev)
        perm_src = torch.empty(R, dtype=torch.int32, device=dev)
        inv_perm = torch.empty(R, dtype=torch.int32, device=dev)
        offsets = torch.empty(E + 1, dtype=torch.int32, device=dev)
    else:
        x_perm, perm_src, inv_perm, offsets = out
    if workspace is None:
        workspace = torch.empty(moe_permute_workspace_bytes(T, k, E), dtype=torch.uint8, device=dev)
    rc = load().moe_permute(_ptr(expert_idx, torch.int32, "expert_idx"), _ptr(x), _DT[x.dtype], T, k, E, d,
                            _ptr(x_perm), _ptr(perm_src, torch.int32), _ptr(inv_perm, torch.int32),
                            _ptr(offsets, torch.int32), _ptr(workspace), workspace.numel(), _stream())
    _check(rc, "moe_permute")
    return x_perm, perm_src, inv_perm, offsets


def moe_grouped_ffn_wq_workspace_bytes(R: int, d: int, F: int, E: int, act_dtype) -> int:
    return int(load().moe_grouped_ffn_wq_workspace_bytes(R, d, F, E, _DT[act_dtype]))


def moe_grouped_ffn_wq(x_perm, expert_offsets, E: int, d: int, F: int, bits: int, group_size: int,
                       w1_packed, s1, w2_packed, s2, b1=None, b2=None, y_dtype=None, y_perm=None,
                       workspace=None, max_rows_per_expert: int = 0, activation: str = "relu"):
    R = x_perm.shape[0]
    y_dtype = y_dtype or x_perm.dtype
    if y_perm is None:
        y_perm = torch.empty((R, d), dtype=y_dtype, device=x_perm.device)
    if workspace is None:
        workspace = torch.empty(moe_grouped_ffn_wq_workspace_bytes(R, d, F, E, x_perm.dtype),
                                dtype=torch.uint8, device=x_perm.device)
    rc = load().moe_grouped_ffn_wq(
        _ptr(x_perm, (torch.float16, torch.bfloat16), "x_perm"), _DT[x_perm.dtype],
        _ptr(expert_offsets, torch.int32, "expert_offsets"), R, E, max_rows_per_expert, d, F, bits, group_size,
        ACTIVATIONS[activation],
        _ptr(w1_packed, torch.uint8, "w1_packed"), _ptr(s1, torch.float16, "s1"), _ptr(b1, torch.float16, "b1"),
        _ptr(w2_packed, torch.uint8, "w2_packed"), _ptr(s2, torch.float16, "s2"), _ptr(b2, torch.float16, "b2"),
        _ptr(y_perm), _DT[y_perm.dtype], _ptr(workspace), workspace.numel(), _stream())
    _check(rc, "moe_grouped_ffn_wq")
    return y_perm


def moe_grouped_ffn_wq_noalloc(x_perm, expert_offsets, E: int, d: int, F: int, bits: int, group_size: int,
                               w1_packed, s1, w2_packed, s2, y_perm, b1=None, b2=None,
                               max_rows_per_expert: int = 0, activation: str = "relu"):
    """moe_grouped_ffn_wq without a workspace (scratch inside the library); y_perm is the caller's."""
    R = x_perm.shape[0]
    rc = load().moe_grouped_ffn_wq_noalloc(
        _ptr(x_perm, (torch.float16, torch.bfloat16), "x_perm"), _DT[x_perm.dtype],
        _ptr(expert_offsets, torch.int32, "expert_offsets"), R, E, max_rows_per_expert, d, F, bits, group_size,
        ACTIVATIONS[activation],
        _ptr(w1_packed, torch.uint8, "w1_packed"), _ptr(s1, torch.float16, "s1"), _ptr(b1, torch.float16, "b1"),
        _ptr(w2_packed, torch.uint8, "w2_packed"), _ptr(s2, torch.float16, "s2"), _ptr(b2, torch.float16, "b2"),
        _ptr(y_perm), _DT[y_perm.dtype], _stream())
    _check(rc, "moe_grouped_ffn_wq_noalloc")
    return y_perm


def moe_combine(y_perm, inv_perm, expert_scale, T: int, k: int, out_dtype=torch.float32, out=None,
                active_rows=None):
    """active_rows: a one-element int32 view (expert_offsets[E:E+1]) when rows may be pruned."""
    d = y_perm.shape[1]
    if out is None:
        out = torch.empty((T, d), dtype=out_dtype, device=y_perm.device)
    rc = load().moe_combine(_ptr(y_perm), _DT[y_perm.dtype], _ptr(inv_perm, torch.int32, "inv_perm"),
                            _ptr(expert_scale, torch.float32, "expert_scale"),
                            _ptr(active_rows, torch.int32, "active_rows"), T, k, d, _ptr(out),
                            _DT[out.dtype], _stream())
    _check(rc, "moe_combine")
    return out


def moe_pack_fp16_experts(w):
    """w fp32 [E,K,N] -> fp16 weights in the fragment layout (uint8, E*K*N*2 bytes)."""
    E, K, N = w.shape
    packed = torch.empty(E * K * N * 2, dtype=torch.uint8, device=w.device)
    rc = load().moe_pack_fp16_experts(_ptr(w, torch.float32, "w"), E, K, N, _ptr(packed), _stream())
    _check(rc, "moe_pack_fp16_experts")
    return packed


def moe_grouped_gemm_wq(x_perm, expert_offsets, E: int, K: int, N: int, bits: int, w_packed, scales=None,
                        native_convert: bool = False, y_dtype=None, y=None, max_rows_per_expert: int = 0):
    """One grouped GEMM of the decode-sized case (Table 1): y[r] = x_perm[r] @ deq(W[e])."""
    R = x_perm.shape[0]
    if y is None:
        y = torch.empty((R, N), dtype=y_dtype or x_perm.dtype, device=x_perm.device)
    rc = load().moe_grouped_gemm_wq(_ptr(x_perm, torch.float16, "x_perm"), _ptr(expert_offsets, torch.int32, "expert_offsets"),
                                    R, E, max_rows_per_expert, K, N, bits, int(native_convert),
                                    _ptr(w_packed, torch.uint8, "w_packed"), _ptr(scales, torch.float16, "scales"),
                                    _ptr(y), _DT[y.dtype], _stream())
    _check(rc, "moe_grouped_gemm_wq")
    return y


def moe_grouped_ffn_wq_routed_supported(R: int, E: int, max_rows_per_expert: int, d: int, F: int, bits: int,
                                        group_size: int, act_dtype) -> bool:
    return bool(load().moe_grouped_ffn_wq_routed_supported(R, E, max_rows_per_expert, d, F, bits, group_size,
                                                           _DT[act_dtype]))


def moe_grouped_ffn_wq_routed(x, perm_src, k: int, expert_offsets, E: int, d: int, F: int, bits: int, group_size: int,
                              w1_packed, s1, w2_packed, s2, b1=None, b2=None, expert_scale=None, out=None,
                              out_dtype=None, workspace=None, max_rows_per_expert: int = 0, activation: str = "relu"):
    """FFN with the gather (and, with expert_scale and k = 1, the combine) fused into the GEMMs."""
    R = perm_src.shape[0]
    T = x.shape[0]
    if out is None:
        out = torch.empty((T if expert_scale is not None else R, d), dtype=out_dtype or x.dtype, device=x.device)
    if workspace is None:
        workspace = torch.empty(moe_grouped_ffn_wq_workspace_bytes(R, d, F, E, x.dtype), dtype=torch.uint8, device=x.device)
    rc = load().moe_grouped_ffn_wq_routed(
        _ptr(x, torch.float16, "x"), _DT[x.dtype], _ptr(perm_src, torch.int32, "perm_src"), k,
        _ptr(expert_scale, torch.float32, "expert_scale"), _ptr(expert_offsets, torch.int32, "expert_offsets"), R, E,
        max_rows_per_expert, d, F, bits, group_size, ACTIVATIONS[activation], _ptr(w1_packed, torch.uint8, "w1_packed"),
        _ptr(s1, torch.float16, "s1"),
        _ptr(b1, torch.float16, "b1"), _ptr(w2_packed, torch.uint8, "w2_packed"), _ptr(s2, torch.float16, "s2"),
        _ptr(b2, torch.float16, "b2"), _ptr(out), _DT[out.dtype], _ptr(workspace), workspace.numel(), _stream())
    _check(rc, "moe_grouped_ffn_wq_routed")
    return out


def moe_grouped_ffn_wq_gated_supported(T: int, k: int, E: int, d: int, F: int, bits: int, group_size: int, act_dtype) -> int:
    """0: not taken; 1: permute + FFN; 2: expert_scale may be given as well (combine fused in)."""
    return int(load().moe_grouped_ffn_wq_gated_supported(T, k, E, d, F, bits, group_size, _DT[act_dtype]))


def moe_grouped_ffn_wq_gated(x, expert_idx, E: int, d: int, F: int, bits: int, group_size: int, w1_packed, s1, w2_packed,
                             s2, b1=None, b2=None, y_dtype=None, workspace=None, activation: str = "relu",
                             expert_scale=None):
    """Decode-sized batches: permute + FFN (+ combine when expert_scale is given) in one call.
    Returns (y_perm [R,d] or, with expert_scale, out [T,d] fp32, perm_src, inv_perm, expert_offsets)."""
    T, k = expert_idx.shape
    R = T * k
    dev = x.device
    if expert_scale is not None:
        y = torch.empty((T, d), dtype=torch.float32, device=dev)
    else:
        y = torch.empty((R, d), dtype=y_dtype or x.dtype, device=dev)
    perm_src = torch.empty(R, dtype=torch.int32, device=dev)
    inv_perm = torch.empty(R, dtype=torch.int32, device=dev)
    offsets = torch.empty(E + 1, dtype=torch.int32, device=dev)
    if workspace is None:
        workspace = torch.empty(moe_grouped_ffn_wq_workspace_bytes(R, d, F, E, x.dtype), dtype=torch.uint8, device=dev)
    rc = load().moe_grouped_ffn_wq_gated(
        _ptr(x, torch.float16, "x"), _DT[x.dtype], _ptr(expert_idx, torch.int32, "expert_idx"),
        _ptr(expert_scale, torch.float32, "expert_scale"), T, k, E, d, F, bits,
        group_size, ACTIVATIONS[activation], _ptr(w1_packed, torch.uint8, "w1_packed"), _ptr(s1, torch.float16, "s1"),
        _ptr(b1, torch.float16, "b1"), _ptr(w2_packed, torch.uint8, "w2_packed"), _ptr(s2, torch.float16, "s2"),
        _ptr(b2, torch.float16, "b2"), _ptr(y), _DT[y.dtype], _ptr(perm_src), _ptr(inv_perm), _ptr(offsets),
        _ptr(workspace), workspace.numel(), _stream())
    _check(rc, "moe_grouped_ffn_wq_gated")
    return y, perm_src, inv_perm, offsets
