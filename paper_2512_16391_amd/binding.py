"""Thin ctypes binding of libkascade.so: argument marshalling only.

Every function here has the name of the C entry point it calls (see
include/kascade.h) and does no arithmetic of the method: it builds the
descriptor from tensor shapes/strides, allocates outputs and the workspace as
torch tensors on the inputs' device, and passes raw device pointers plus the
current HIP stream.  There is no CPU fallback: if the library is not built, or
a tensor is not on the GPU, the call raises.
"""
import ctypes
import os
from typing import Optional

import torch

_PKG_DIR = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG_DIR, "libkascade.so")

KASCADE_OK = 0
KASCADE_F32, KASCADE_BF16, KASCADE_F16 = 0, 1, 2
KASCADE_OUT_DENSE, KASCADE_OUT_SPARSE = 0, 1
OP_DECODE_ANCHOR, OP_DECODE_REUSE, OP_PREFILL_ANCHOR, OP_PREFILL_REUSE, OP_DECODE_POOLED = 0, 1, 2, 3, 4
OP_PREFILL_ANCHOR_PRESOFTMAX = 5

EXPORTS = [
    "kascade_decode_anchor", "kascade_decode_reuse", "kascade_prefill_anchor", "kascade_prefill_reuse",
    "kascade_decode_reuse_static", "kascade_decode_reuse_static_capacity",
    "kascade_decode_anchor_shared", "kascade_prefill_anchor_shared",
    "kascade_decode_anchor_presoftmax", "kascade_prefill_anchor_presoftmax",
    "kascade_workspace_bytes", "kascade_status_string", "kascade_version",
    "kascade_decode_pooled", "kascade_topk_similarity", "kascade_select_anchor_layers",
    "kascade_head_similarity", "kascade_head_map", "kascade_layer_importance",
    "kascade_profile_enable", "kascade_profile_reset", "kascade_tuning_set", "kascade_tuning_get", "kascade_profile_kernels", "kascade_profile_read",
]


class KascadeDesc(ctypes.Structure):
    _fields_ = [
        ("batch", ctypes.c_int32), ("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32), ("dtype", ctypes.c_int32), ("softmax_scale", ctypes.c_float),
        ("q_stride", ctypes.c_int64 * 3), ("kv_stride", ctypes.c_int64 * 3), ("o_stride", ctypes.c_int64 * 3),
    ]


class KascadeError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} ({status})")


_lib = None


def load_library(path: Optional[str] = None):
    """Loads libkascade.so (built by build.py / __graft_entry__.build()); raises if absent."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    path = path or LIB_PATH
    if not os.path.exists(path):
        raise RuntimeError(f"{path} is not built: run `python -c 'import __graft_entry__ as g; g.build()'` "
                           "at the repository root (there is no fallback path)")
    lib = ctypes.CDLL(path)
    vp, i32, i64, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t
    dp = ctypes.POINTER(KascadeDesc)
    lib.kascade_decode_anchor.argtypes = [dp, vp, vp, vp, vp, vp, i32, i32, i32, i32, vp, vp, vp, sz, vp]
    lib.kascade_decode_anchor.restype = ctypes.c_int
    lib.kascade_decode_anchor_shared.argtypes = lib.kascade_decode_anchor.argtypes
    lib.kascade_decode_anchor_shared.restype = ctypes.c_int
    lib.kascade_decode_anchor_presoftmax.argtypes = lib.kascade_decode_anchor.argtypes
    lib.kascade_decode_anchor_presoftmax.restype = ctypes.c_int
    lib.kascade_decode_reuse.argtypes = [dp, vp, vp, vp, vp, vp, i32, vp, i32, vp, vp, vp, sz, vp]
    lib.kascade_decode_reuse.restype = ctypes.c_int
    lib.kascade_decode_reuse_static.argtypes = [dp, vp, vp, vp, vp, vp, i32, vp, i32, vp, vp, vp]
    lib.kascade_decode_reuse_static.restype = ctypes.c_int
    lib.kascade_decode_reuse_static_capacity.argtypes = []
    lib.kascade_decode_reuse_static_capacity.restype = sz
    lib.kascade_prefill_anchor.argtypes = [dp, vp, vp, vp, i32, i32, vp, vp, i64, i32, vp, vp, vp, sz, vp]
    lib.kascade_prefill_anchor.restype = ctypes.c_int
    lib.kascade_prefill_anchor_shared.argtypes = lib.kascade_prefill_anchor.argtypes
    lib.kascade_prefill_anchor_shared.restype = ctypes.c_int
    lib.kascade_prefill_anchor_presoftmax.argtypes = lib.kascade_prefill_anchor.argtypes
    lib.kascade_prefill_anchor_presoftmax.restype = ctypes.c_int
    lib.kascade_prefill_reuse.argtypes = [dp, vp, vp, vp, i32, i32, vp, vp, i64, vp, i32, vp, vp, vp, sz, vp]
    lib.kascade_prefill_reuse.restype = ctypes.c_int
    lib.kascade_decode_pooled.argtypes = [dp, vp, vp, vp, i32, vp, i64, vp, sz, vp]
    lib.kascade_decode_pooled.restype = ctypes.c_int
    lib.kascade_topk_similarity.argtypes = [i32, i32, vp, i64, vp, vp, i32, vp, i32, vp, vp, vp, vp, vp]
    lib.kascade_topk_similarity.restype = ctypes.c_int
    fpp = ctypes.POINTER(ctypes.c_float)
    lib.kascade_select_anchor_layers.argtypes = [fpp, fpp, i32, i32, ctypes.POINTER(i32),
                                                 ctypes.POINTER(ctypes.c_double)]
    lib.kascade_head_similarity.argtypes = [i32, i32, vp, i64, vp, vp, i32, vp, i32, vp, vp, vp]
    lib.kascade_head_similarity.restype = ctypes.c_int
    lib.kascade_head_map.argtypes = [i32, i32, i32, vp, vp, vp, vp]
    lib.kascade_head_map.restype = ctypes.c_int
    lib.kascade_layer_importance.argtypes = [vp, vp, i64, i32, i32, i64, i64, vp, vp]
    lib.kascade_layer_importance.restype = ctypes.c_int
    lib.kascade_select_anchor_layers.restype = ctypes.c_int
    lib.kascade_workspace_bytes.argtypes = [i32, dp, i64, i64, i32]
    lib.kascade_workspace_bytes.restype = sz
    lib.kascade_status_string.argtypes = [i32]
    lib.kascade_status_string.restype = ctypes.c_char_p
    lib.kascade_version.argtypes = []
    lib.kascade_version.restype = ctypes.c_char_p
    lib.kascade_profile_enable.argtypes = [i32]
    lib.kascade_profile_enable.restype = ctypes.c_int
    lib.kascade_tuning_set.argtypes = [i32, i32]
    lib.kascade_tuning_set.restype = ctypes.c_int
    lib.kascade_tuning_get.argtypes = [i32]
    lib.kascade_tuning_get.restype = i32
    lib.kascade_profile_reset.argtypes = []
    lib.kascade_profile_reset.restype = ctypes.c_int
    lib.kascade_profile_kernels.argtypes = []
    lib.kascade_profile_kernels.restype = i32
    lib.kascade_profile_read.argtypes = [i32, ctypes.POINTER(ctypes.c_char_p), ctypes.POINTER(ctypes.c_double),
                                         ctypes.POINTER(i64)]
    lib.kascade_profile_read.restype = ctypes.c_int
    _lib = lib
    return lib


def status_string(status: int) -> str:
    return load_library().kascade_status_string(int(status)).decode()


def version() -> str:
    return load_library().kascade_version().decode()


def kascade_profile_enable(on: bool) -> None:
    _check(load_library().kascade_profile_enable(1 if on else 0), "kascade_profile_enable")


TUNE_DECODE_FAMILY, TUNE_STREAM_CHUNK, TUNE_GATHER_CHUNK, TUNE_TOPK_PARTS = 0, 1, 2, 3
DECODE_FAMILY_AUTO, DECODE_FAMILY_VECTOR, DECODE_FAMILY_MATRIX = 0, 1, 2


def kascade_tuning_set(knob: int, value: int) -> None:
    _check(load_library().kascade_tuning_set(int(knob), int(value)), "kascade_tuning_set")


def kascade_tuning_get(knob: int) -> int:
    return int(load_library().kascade_tuning_get(int(knob)))


def kascade_profile_reset() -> None:
    _check(load_library().kascade_profile_reset(), "kascade_profile_reset")


def kascade_profile_read() -> dict:
    """{kernel name: (total_ms, launches)} for kernels launched since the last reset."""
    lib = load_library()
    res = {}
    for kid in range(lib.kascade_profile_kernels()):
        name, ms, n = ctypes.c_char_p(), ctypes.c_double(), ctypes.c_int64()
        _check(lib.kascade_profile_read(kid, ctypes.byref(name), ctypes.byref(ms), ctypes.byref(n)),
               "kascade_profile_read")
        if n.value:
            res[name.value.decode()] = (ms.value, n.value)
    return res


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return KASCADE_F32
    if t.dtype == torch.bfloat16:
        return KASCADE_BF16
    if t.dtype == torch.float16:
        return KASCADE_F16
    raise TypeError(f"unsupported dtype {t.dtype}")


def _need_gpu(*tensors):
    for t in tensors:
        if t is not None and not t.is_cuda:
            raise RuntimeError("kascade: tensors must live on the GPU (there is no CPU path)")


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr()) if t is not None else ctypes.c_void_p(0)


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def decode_desc(q, k_cache, out=None, softmax_scale=0.0, kv_layout="BHLD") -> KascadeDesc:
    """q [B,Hq,d]; k_cache [B,Hkv,L,d] ("BHLD") or [B,L,Hkv,d] ("BLHD")."""
    B, Hq, d = q.shape
    d_ = KascadeDesc()
    if kv_layout == "BHLD":
        Hkv = k_cache.shape[1]
        kvs = (k_cache.stride(0), k_cache.stride(1), k_cache.stride(2))
    elif kv_layout == "BLHD":
        Hkv = k_cache.shape[2]
        kvs = (k_cache.stride(0), k_cache.stride(2), k_cache.stride(1))
    else:
        raise ValueError(kv_layout)
    if q.stride(2) != 1 or k_cache.stride(3) != 1:
        raise ValueError("head dimension must be contiguous")
    d_.batch, d_.n_q_heads, d_.n_kv_heads, d_.head_dim = B, Hq, Hkv, d
    d_.dtype = _dtype_code(q)
    d_.softmax_scale = float(softmax_scale)
    d_.q_stride[:] = (q.stride(0), 0, q.stride(1))
    d_.kv_stride[:] = kvs
    o = out if out is not None else q
    d_.o_stride[:] = (o.stride(0), 0, o.stride(1))
    return d_


def prefill_desc(q, k, out=None, softmax_scale=0.0) -> KascadeDesc:
    """q [S,Hq,d]; k [Hkv,S,d] (any strides with contiguous head dimension)."""
    S, Hq, d = q.shape
    d_ = KascadeDesc()
    if q.stride(2) != 1 or k.stride(2) != 1:
        raise ValueError("head dimension must be contiguous")
    d_.batch, d_.n_q_heads, d_.n_kv_heads, d_.head_dim = 1, Hq, k.shape[0], d
    d_.dtype = _dtype_code(q)
    d_.softmax_scale = float(softmax_scale)
    d_.q_stride[:] = (0, q.stride(0), q.stride(1))
    d_.kv_stride[:] = (0, k.stride(0), k.stride(1))
    o = out if out is not None else q
    d_.o_stride[:] = (0, o.stride(0), o.stride(1))
    return d_


def kascade_workspace_bytes(op, desc, max_seqlen, k_or_idx_total, q_tile_tokens=0) -> int:
    return int(load_library().kascade_workspace_bytes(int(op), ctypes.byref(desc), int(max_seqlen),
                                                      int(k_or_idx_total), int(q_tile_tokens)))


def _workspace(op, desc, max_seqlen, k_or_total, T, device, workspace):
    need = kascade_workspace_bytes(op, desc, max_seqlen, k_or_total, T)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=device)
    return workspace, workspace.numel() * workspace.element_size()


def _check(st, where):
    if st != KASCADE_OK:
        raise KascadeError(st, where)


def kascade_decode_anchor(q, k_cache, v_cache, seqlens, k_per_seq, max_seqlen, k_max, recent_window=0,
                          out_mode=KASCADE_OUT_SPARSE, idx_out=None, out=None, workspace=None,
                          softmax_scale=0.0, kv_layout="BHLD"):
    """Returns (idx_out [B,Hkv,k_max] int32, out [B,Hq,d])."""
    _need_gpu(q, k_cache, v_cache, seqlens, k_per_seq, idx_out, out, workspace)
    lib = load_library()
    B, Hq, d = q.shape
    if out is None:
        out = torch.empty_like(q)
    desc = decode_desc(q, k_cache, out, softmax_scale, kv_layout)
    if idx_out is None:
        idx_out = torch.empty(B, desc.n_kv_heads, int(k_max), dtype=torch.int32, device=q.device)
    workspace, nbytes = _workspace(OP_DECODE_ANCHOR, desc, max_seqlen, k_max, 0, q.device, workspace)
    st = lib.kascade_decode_anchor(ctypes.byref(desc), _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(seqlens),
                                   _ptr(k_per_seq), int(max_seqlen), int(k_max), int(recent_window), int(out_mode),
                                   _ptr(idx_out), _ptr(out), _ptr(workspace), nbytes, _stream())
    _check(st, "kascade_decode_anchor")
    return idx_out, out


def kascade_decode_reuse(q, k_cache, v_cache, seqlens, k_per_seq, k_max, idx_in, head_map=None, out=None,
                         workspace=None, softmax_scale=0.0, kv_layout="BHLD"):
    """idx_in [B,Hkv_anchor,k_max] int32.  Returns out [B,Hq,d]."""
    _need_gpu(q, k_cache, v_cache, seqlens, k_per_seq, idx_in, head_map, out, workspace)
    lib = load_library()
    if out is None:
        out = torch.empty_like(q)
    desc = decode_desc(q, k_cache, out, softmax_scale, kv_layout)
    if idx_in.dtype != torch.int32 or not idx_in.is_contiguous() or idx_in.shape[2] != k_max:
        raise ValueError("idx_in must be a contiguous int32 [B, Hkv_anchor, k_max] tensor")
    workspace, nbytes = _workspace(OP_DECODE_REUSE, desc, 1, k_max, 0, q.device, workspace)
    st = lib.kascade_decode_reuse(ctypes.byref(desc), _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(seqlens),
                                  _ptr(k_per_seq), int(k_max), _ptr(idx_in), int(idx_in.shape[1]), _ptr(head_map),
                                  _ptr(out), _ptr(workspace), nbytes, _stream())
    _check(st, "kascade_decode_reuse")
    return out


def kascade_decode_reuse_static(q, k_cache, v_cache, seqlens, k_per_seq, k_max, idx_in, head_map=None, out=None,
                                softmax_scale=0.0, kv_layout="BHLD"):
    """kascade_decode_reuse without a workspace (the library's fixed scratch array).  Returns out [B,Hq,d]."""
    _need_gpu(q, k_cache, v_cache, seqlens, k_per_seq, idx_in, head_map, out)
    lib = load_library()
    if out is None:
        out = torch.empty_like(q)
    desc = decode_desc(q, k_cache, out, softmax_scale, kv_layout)
    if idx_in.dtype != torch.int32 or not idx_in.is_contiguous() or idx_in.shape[2] != k_max:
        raise ValueError("idx_in must be a contiguous int32 [B, Hkv_anchor, k_max] tensor")
    st = lib.kascade_decode_reuse_static(ctypes.byref(desc), _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(seqlens),
                                         _ptr(k_per_seq), int(k_max), _ptr(idx_in), int(idx_in.shape[1]), _ptr(head_map),
                                         _ptr(out), _stream())
    _check(st, "kascade_decode_reuse_static")
    return out


def kascade_decode_reuse_static_capacity() -> int:
    return int(load_library().kascade_decode_reuse_static_capacity())


def kascade_prefill_anchor(q, k, v, q_tile_tokens, k_per_tile, idx_offsets, idx_total,
                           out_mode=KASCADE_OUT_SPARSE, idx_out=None, out=None, workspace=None, softmax_scale=0.0):
    """q [S,Hq,d], k/v [Hkv,S,d].  Returns (idx_out [Hkv, idx_total] int32, out [S,Hq,d])."""
    _need_gpu(q, k, v, k_per_tile, idx_offsets, idx_out, out, workspace)
    lib = load_library()
    S = q.shape[0]
    if out is None:
        out = torch.empty_like(q)
    desc = prefill_desc(q, k, out, softmax_scale)
    if idx_out is None:
        idx_out = torch.empty(desc.n_kv_heads, max(int(idx_total), 1), dtype=torch.int32, device=q.device)
    workspace, nbytes = _workspace(OP_PREFILL_ANCHOR, desc, S, idx_total, q_tile_tokens, q.device, workspace)
    st = lib.kascade_prefill_anchor(ctypes.byref(desc), _ptr(q), _ptr(k), _ptr(v), int(S), int(q_tile_tokens),
                                    _ptr(k_per_tile), _ptr(idx_offsets), int(idx_total), int(out_mode),
                                    _ptr(idx_out), _ptr(out), _ptr(workspace), nbytes, _stream())
    _check(st, "kascade_prefill_anchor")
    return idx_out, out


def kascade_prefill_reuse(q, k, v, q_tile_tokens, k_per_tile, idx_offsets, idx_total, idx_in, head_map=None,
                          n_anchor_heads=None, out=None, workspace=None, softmax_scale=0.0):
    """idx_in [Hkv_anchor, idx_total] int32.  Returns out [S,Hq,d]."""
    _need_gpu(q, k, v, k_per_tile, idx_offsets, idx_in, head_map, out, workspace)
    lib = load_library()
    S = q.shape[0]
    if out is None:
        out = torch.empty_like(q)
    desc = prefill_desc(q, k, out, softmax_scale)
    if n_anchor_heads is None:
        n_anchor_heads = idx_in.shape[0]
    workspace, nbytes = _workspace(OP_PREFILL_REUSE, desc, S, idx_total, q_tile_tokens, q.device, workspace)
    st = lib.kascade_prefill_reuse(ctypes.byref(desc), _ptr(q), _ptr(k), _ptr(v), int(S), int(q_tile_tokens),
                                   _ptr(k_per_tile), _ptr(idx_offsets), int(idx_total), _ptr(idx_in),
                                   int(n_anchor_heads), _ptr(head_map), _ptr(out), _ptr(workspace), nbytes, _stream())
    _check(st, "kascade_prefill_reuse")
    return out


def kascade_decode_pooled(q, k_cache, seqlens, max_seqlen, pooled_out=None, workspace=None, softmax_scale=0.0,
                          kv_layout="BHLD"):
    """Returns pooled_out [B,Hkv,pitch] fp32 (pitch = max_seqlen rounded up to 4; columns past a
    sequence's length are left as they were)."""
    _need_gpu(q, k_cache, seqlens, pooled_out, workspace)
    lib = load_library()
    desc = decode_desc(q, k_cache, None, softmax_scale, kv_layout)
    if pooled_out is None:
        pooled_out = torch.zeros(q.shape[0], desc.n_kv_heads, (int(max_seqlen) + 3) // 4 * 4, dtype=torch.float32,
                                 device=q.device)
    if pooled_out.dtype != torch.float32 or not pooled_out.is_contiguous():
        raise ValueError("pooled_out must be a contiguous fp32 [B, Hkv, pitch] tensor")
    workspace, nbytes = _workspace(OP_DECODE_POOLED, desc, max_seqlen, 0, 0, q.device, workspace)
    st = lib.kascade_decode_pooled(ctypes.byref(desc), _ptr(q), _ptr(k_cache), _ptr(seqlens), int(max_seqlen),
                                   _ptr(pooled_out), int(pooled_out.shape[2]), _ptr(workspace), nbytes, _stream())
    _check(st, "kascade_decode_pooled")
    return pooled_out


def kascade_topk_similarity(pooled_b, seqlens, k_per_seq, idx_a, idx_b, head_map=None, sim_out=None, sim_min=None):
    """pooled_b [B,Hkv,pitch] fp32, idx_a [B,Ha,k_max], idx_b [B,Hkv,k_max] int32.
    Returns (sim_out [B,Hkv] fp32, sim_min): sim_min (one fp32, device) is lowered in place when given."""
    _need_gpu(pooled_b, seqlens, k_per_seq, idx_a, idx_b, head_map, sim_out, sim_min)
    B, Hkv, pitch = pooled_b.shape
    for t in (idx_a, idx_b):
        if t.dtype != torch.int32 or not t.is_contiguous() or t.shape[2] != idx_b.shape[2]:
            raise ValueError("index sets must be contiguous int32 [B, heads, k_max] tensors of one k_max")
    if pooled_b.dtype != torch.float32 or not pooled_b.is_contiguous():
        raise ValueError("pooled_b must be a contiguous fp32 [B, Hkv, pitch] tensor")
    if sim_out is None:
        sim_out = torch.empty(B, Hkv, dtype=torch.float32, device=pooled_b.device)
    st = load_library().kascade_topk_similarity(int(B), int(Hkv), _ptr(pooled_b), int(pitch), _ptr(seqlens),
                                                _ptr(k_per_seq), int(idx_b.shape[2]), _ptr(idx_a),
                                                int(idx_a.shape[1]), _ptr(head_map), _ptr(idx_b), _ptr(sim_out),
                                                _ptr(sim_min), _stream())
    _check(st, "kascade_topk_similarity")
    return sim_out, sim_min


def kascade_select_anchor_layers(similarity, n_anchors, layer_weights=None):
    """similarity: [L,L] array-like on the host (fp32); layer_weights [L] or None.
    Returns (anchors list, objective)."""
    import numpy as np
    S = np.ascontiguousarray(np.asarray(similarity, dtype=np.float32))
    if S.ndim != 2 or S.shape[0] != S.shape[1]:
        raise ValueError("similarity must be a square matrix")
    n = int(n_anchors)
    anchors = (ctypes.c_int32 * max(n, 1))()
    obj = ctypes.c_double()
    fpp = ctypes.POINTER(ctypes.c_float)
    w = None
    if layer_weights is not None:
        w = np.ascontiguousarray(np.asarray(layer_weights, dtype=np.float32))
        if w.shape != (S.shape[0],):
            raise ValueError("layer_weights must have one entry per layer")
    st = load_library().kascade_select_anchor_layers(S.ctypes.data_as(fpp), w.ctypes.data_as(fpp) if w is not None else None,
                                                     int(S.shape[0]), n, anchors, ctypes.byref(obj))
    _check(st, "kascade_select_anchor_layers")
    return list(anchors[:n]), obj.value


def kascade_head_similarity(pooled_b, seqlens, k_per_seq, idx_a, idx_b, sim_out=None):
    """Returns sim_out [B,Hkv,Ha] fp32: every anchor-layer head's set applied to every head of layer b."""
    _need_gpu(pooled_b, seqlens, k_per_seq, idx_a, idx_b, sim_out)
    B, Hkv, pitch = pooled_b.shape
    for t in (idx_a, idx_b):
        if t.dtype != torch.int32 or not t.is_contiguous() or t.shape[2] != idx_b.shape[2]:
            raise ValueError("index sets must be contiguous int32 [B, heads, k_max] tensors of one k_max")
    if pooled_b.dtype != torch.float32 or not pooled_b.is_contiguous():
        raise ValueError("pooled_b must be a contiguous fp32 [B, Hkv, pitch] tensor")
    Ha = idx_a.shape[1]
    if sim_out is None:
        sim_out = torch.empty(B, Hkv, Ha, dtype=torch.float32, device=pooled_b.device)
    st = load_library().kascade_head_similarity(int(B), int(Hkv), _ptr(pooled_b), int(pitch), _ptr(seqlens),
                                                _ptr(k_per_seq), int(idx_b.shape[2]), _ptr(idx_a), int(Ha),
                                                _ptr(idx_b), _ptr(sim_out), _stream())
    _check(st, "kascade_head_similarity")
    return sim_out


def kascade_head_map(sim):
    """sim [n_samples,Hkv,Ha] fp32 (device).  Returns (head_map [Hkv] int32, mean [Hkv,Ha] fp32)."""
    _need_gpu(sim)
    if sim.dtype != torch.float32 or not sim.is_contiguous() or sim.dim() != 3:
        raise ValueError("sim must be a contiguous fp32 [n_samples, Hkv, Ha] tensor")
    n, Hkv, Ha = sim.shape
    mean = torch.empty(Hkv, Ha, dtype=torch.float32, device=sim.device)
    head_map = torch.empty(Hkv, dtype=torch.int32, device=sim.device)
    _check(load_library().kascade_head_map(int(n), int(Hkv), int(Ha), _ptr(sim), _ptr(mean), _ptr(head_map), _stream()),
           "kascade_head_map")
    return head_map, mean


def kascade_layer_importance(x, y):
    """x, y [n_rows,n_cols] (fp32, bf16 or fp16, device, unit column stride).  Returns w [n_rows] fp32."""
    _need_gpu(x, y)
    if x.shape != y.shape or x.dim() != 2 or x.dtype != y.dtype or x.stride(1) != 1 or y.stride(1) != 1:
        raise ValueError("x and y must be 2-D tensors of one shape and dtype with contiguous rows")
    w = torch.empty(x.shape[0], dtype=torch.float32, device=x.device)
    st = load_library().kascade_layer_importance(_ptr(x), _ptr(y), int(x.shape[0]), int(x.shape[1]), _dtype_code(x),
                                                 int(x.stride(0)), int(y.stride(0)), _ptr(w), _stream())
    _check(st, "kascade_layer_importance")
    return w


def kascade_decode_anchor_shared(q, k_cache, v_cache, seqlens, k_per_seq, max_seqlen, k_max, recent_window=0,
                                 out_mode=KASCADE_OUT_SPARSE, idx_out=None, out=None, workspace=None,
                                 softmax_scale=0.0, kv_layout="BHLD"):
    """One index set per sequence for all heads.  Returns (idx_out [B,1,k_max] int32, out [B,Hq,d])."""
    _need_gpu(q, k_cache, v_cache, seqlens, k_per_seq, idx_out, out, workspace)
    lib = load_library()
    B = q.shape[0]
    if out is None:
        out = torch.empty_like(q)
    desc = decode_desc(q, k_cache, out, softmax_scale, kv_layout)
    if idx_out is None:
        idx_out = torch.empty(B, 1, int(k_max), dtype=torch.int32, device=q.device)
    workspace, nbytes = _workspace(OP_DECODE_ANCHOR, desc, max_seqlen, k_max, 0, q.device, workspace)
    st = lib.kascade_decode_anchor_shared(ctypes.byref(desc), _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(seqlens),
                                          _ptr(k_per_seq), int(max_seqlen), int(k_max), int(recent_window),
                                          int(out_mode), _ptr(idx_out), _ptr(out), _ptr(workspace), nbytes, _stream())
    _check(st, "kascade_decode_anchor_shared")
    return idx_out, out


def kascade_prefill_anchor_shared(q, k, v, q_tile_tokens, k_per_tile, idx_offsets, idx_total,
                                  out_mode=KASCADE_OUT_SPARSE, idx_out=None, out=None, workspace=None,
                                  softmax_scale=0.0):
    """One index set per tile for all heads.  Returns (idx_out [1, idx_total] int32, out [S,Hq,d])."""
    _need_gpu(q, k, v, k_per_tile, idx_offsets, idx_out, out, workspace)
    lib = load_library()
    S = q.shape[0]
    if out is None:
        out = torch.empty_like(q)
    desc = prefill_desc(q, k, out, softmax_scale)
    if idx_out is None:
        idx_out = torch.empty(1, max(int(idx_total), 1), dtype=torch.int32, device=q.device)
    workspace, nbytes = _workspace(OP_PREFILL_ANCHOR, desc, S, idx_total, q_tile_tokens, q.device, workspace)
    st = lib.kascade_prefill_anchor_shared(ctypes.byref(desc), _ptr(q), _ptr(k), _ptr(v), int(S), int(q_tile_tokens),
                                           _ptr(k_per_tile), _ptr(idx_offsets), int(idx_total), int(out_mode),
                                           _ptr(idx_out), _ptr(out), _ptr(workspace), nbytes, _stream())
    _check(st, "kascade_prefill_anchor_shared")
    return idx_out, out


def kascade_decode_anchor_presoftmax(q, k_cache, v_cache, seqlens, k_per_seq, max_seqlen, k_max, recent_window=0,
                                     out_mode=KASCADE_OUT_SPARSE, idx_out=None, out=None, workspace=None,
                                     softmax_scale=0.0, kv_layout="BHLD"):
    """Anchor call with Pre-Softmax pooling.  Returns (idx_out [B,Hkv,k_max] int32, out [B,Hq,d])."""
    _need_gpu(q, k_cache, v_cache, seqlens, k_per_seq, idx_out, out, workspace)
    lib = load_library()
    B = q.shape[0]
    if out is None:
        out = torch.empty_like(q)
    desc = decode_desc(q, k_cache, out, softmax_scale, kv_layout)
    if idx_out is None:
        idx_out = torch.empty(B, desc.n_kv_heads, int(k_max), dtype=torch.int32, device=q.device)
    workspace, nbytes = _workspace(OP_DECODE_ANCHOR, desc, max_seqlen, k_max, 0, q.device, workspace)
    st = lib.kascade_decode_anchor_presoftmax(ctypes.byref(desc), _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(seqlens),
                                              _ptr(k_per_seq), int(max_seqlen), int(k_max), int(recent_window),
                                              int(out_mode), _ptr(idx_out), _ptr(out), _ptr(workspace), nbytes, _stream())
    _check(st, "kascade_decode_anchor_presoftmax")
    return idx_out, out


def kascade_prefill_anchor_presoftmax(q, k, v, q_tile_tokens, k_per_tile, idx_offsets, idx_total,
                                      out_mode=KASCADE_OUT_SPARSE, idx_out=None, out=None, workspace=None,
                                      softmax_scale=0.0):
    """Prefill anchor call with Pre-Softmax pooling.  Returns (idx_out [Hkv, idx_total] int32, out [S,Hq,d])."""
    _need_gpu(q, k, v, k_per_tile, idx_offsets, idx_out, out, workspace)
    lib = load_library()
    S = q.shape[0]
    if out is None:
        out = torch.empty_like(q)
    desc = prefill_desc(q, k, out, softmax_scale)
    if idx_out is None:
        idx_out = torch.empty(desc.n_kv_heads, max(int(idx_total), 1), dtype=torch.int32, device=q.device)
    workspace, nbytes = _workspace(OP_PREFILL_ANCHOR_PRESOFTMAX, desc, S, idx_total, q_tile_tokens, q.device, workspace)
    st = lib.kascade_prefill_anchor_presoftmax(ctypes.byref(desc), _ptr(q), _ptr(k), _ptr(v), int(S), int(q_tile_tokens),
                                               _ptr(k_per_tile), _ptr(idx_offsets), int(idx_total), int(out_mode),
                                               _ptr(idx_out), _ptr(out), _ptr(workspace), nbytes, _stream())
    _check(st, "kascade_prefill_anchor_presoftmax")
    return idx_out, out
