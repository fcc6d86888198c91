"""Thin ctypes binding over libsvoo.so: same names as the C boundary (include/svoo.h), argument
marshalling only.  PyTorch provides device memory and the current stream; every step of the path
runs in the library's HIP kernels.  There is no fallback: a missing library raises."""
from __future__ import annotations

import ctypes
import math
import os
from typing import Dict, List, Optional, Sequence, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsvoo.so")

SVOO_BF16, SVOO_F32 = 0, 1
STATUS_OK = 0


class SvooError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {_lib().svoo_status_string(status).decode()} (status {status})")


class Shape(ctypes.Structure):
    _fields_ = [("bh", ctypes.c_int32), ("n", ctypes.c_int32), ("d", ctypes.c_int32),
                ("dtype", ctypes.c_int32), ("kq", ctypes.c_int32), ("kk", ctypes.c_int32)]


_LIB = None

_vp, _i32, _f32, _sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_float, ctypes.c_size_t
_SP = ctypes.POINTER(Shape)
_SIGNATURES = {
    "svoo_status_string": (ctypes.c_char_p, [ctypes.c_int]),
    "svoo_version": (_i32, []),
    "svoo_workspace_bytes": (_sz, [_SP]),
    "svoo_permute_workspace_bytes": (_sz, [_SP, _i32]),
    "svoo_cocluster": (ctypes.c_int, [_SP, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _vp, _vp, _vp, _vp, _vp, _vp, _vp,
                                      _vp, _sz, _vp]),
    "svoo_cocluster_sorted": (ctypes.c_int, [_SP, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _vp, _vp, _vp, _vp, _vp, _vp,
                                             _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
    "svoo_assign": (ctypes.c_int, [_SP, _vp, _vp, _i32, _vp, _i32, _vp, _vp, _sz, _vp]),
    "svoo_kmeans": (ctypes.c_int, [_SP, _vp, _i32, _vp, _vp, _i32, _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
    "svoo_permute": (ctypes.c_int, [_SP, _vp, _i32, _i32, ctypes.POINTER(_vp), ctypes.POINTER(_vp), _vp, _vp, _vp,
                                    _sz, _vp]),
    "svoo_gather": (ctypes.c_int, [_SP, _vp, _i32, ctypes.POINTER(_vp), ctypes.POINTER(_vp), _vp]),
    "svoo_unpermute": (ctypes.c_int, [_SP, _vp, _vp, _vp, _vp]),
    "svoo_block_mask": (ctypes.c_int, [_SP, _vp, _vp, _vp, _vp, _vp, _f32, _f32, _f32, _vp, _vp, _vp, _vp, _sz, _vp]),
    "svoo_block_sparse_attn": (ctypes.c_int, [_SP, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _f32, _vp, _vp, _vp, _sz, _vp]),
    "svoo_block_sparse_attn_static": (ctypes.c_int, [_SP, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _f32, _vp, _vp, _vp]),
    "svoo_block_sparse_attn_tokens": (ctypes.c_int, [_SP, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _f32, _vp, _vp, _vp,
                                                     _sz, _vp]),
    "svoo_attn": (ctypes.c_int, [_SP, _vp, _vp, _vp, _f32, _vp, _vp, _vp, _sz, _vp]),
    "svoo_row_recall": (ctypes.c_int, [_SP, _vp, _vp, _vp, _vp, _vp]),
    "svoo_attention_density": (ctypes.c_int, [_SP, _vp, _vp, _vp, _i32, _f32, _f32, _vp, _vp, _vp, _vp]),
    "svoo_microbench_mfma_bf16": (ctypes.c_int, [_i32, _i32, _i32, _vp, ctypes.POINTER(ctypes.c_double), _vp]),
    "svoo_microbench_copy": (ctypes.c_int, [_vp, _vp, _sz, _vp]),
    "svoo_microbench_attn_tile": (ctypes.c_int, [_i32, _i32, _vp, _vp, _vp]),
}
EXPORTS = tuple(_SIGNATURES)


def _lib():
    global _LIB
    if _LIB is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run `python -m paper_2603_18636_amd.build` first "
                               "(there is no fallback path)")
        lib = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(lib, name)
            fn.restype = res
            fn.argtypes = args
        _LIB = lib
    return _LIB


def version() -> int:
    return int(_lib().svoo_version())


def status_string(status: int) -> str:
    return _lib().svoo_status_string(status).decode()


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.bfloat16:
        return SVOO_BF16
    if t.dtype == torch.float32:
        return SVOO_F32
    raise TypeError(f"unsupported dtype {t.dtype}")


def make_shape(x: torch.Tensor, kq: int, kk: int) -> Shape:
    if x.dim() != 3:
        raise ValueError("expected [bh, n, d]")
    bh, n, d = x.shape
    return Shape(bh, n, d, _dtype_code(x), kq, kk)


def _check(t: Optional[torch.Tensor], dtype, shape, name: str):
    if t is None:
        return
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError(f"{name}: must be a contiguous device tensor")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"{name}: expected {dtype}, got {t.dtype}")
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name}: expected shape {tuple(shape)}, got {tuple(t.shape)}")


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def workspace_bytes(shape: Shape) -> int:
    return int(_lib().svoo_workspace_bytes(ctypes.byref(shape)))


_WS: Dict[Tuple[int, int], torch.Tensor] = {}


def workspace(shape: Shape, device, private: bool = False) -> torch.Tensor:
    """A uint8 device buffer large enough for any call with this shape.  By default it is ONE cached
    buffer per device, shared by every call made through this module: calls that may overlap on the GPU
    (different streams) race on it and must each bring a buffer of their own (``private=True``)."""
    need = workspace_bytes(shape)
    if need == 0:
        raise SvooError(1, "svoo_workspace_bytes")
    dev = torch.device(device)
    if private:
        buf = torch.empty(need + 256, dtype=torch.uint8, device=dev)
    else:
        key = (dev.index or 0, 0)
        buf = _WS.get(key)
        if buf is None or buf.numel() < need:
            buf = torch.empty(need + 256, dtype=torch.uint8, device=dev)
            _WS[key] = buf
    off = (-buf.data_ptr()) % 256
    return buf[off:off + need]


def _run(status: int, where: str):
    if status != STATUS_OK:
        raise SvooError(status, where)


def cocluster(q, k, init_q_idx=None, init_k_idx=None, iters=2, kq=None, kk=None, init_cq=None, init_ck=None,
              want_objective=False, ws=None):
    """svoo_cocluster.  Returns dict(labels_q, labels_k, cq, ck, counts_q, counts_k[, objective])."""
    bh, n, d = q.shape
    kq = kq or (init_q_idx.shape[1] if init_q_idx is not None else init_cq.shape[1])
    kk = kk or (init_k_idx.shape[1] if init_k_idx is not None else init_ck.shape[1])
    shape = make_shape(q, kq, kk)
    _check(q, None, (bh, n, d), "q")
    _check(k, q.dtype, (bh, n, d), "k")
    _check(init_q_idx, torch.int32, (bh, kq), "init_q_idx")
    _check(init_k_idx, torch.int32, (bh, kk), "init_k_idx")
    _check(init_cq, torch.float32, (bh, kq, d), "init_cq")
    _check(init_ck, torch.float32, (bh, kk, d), "init_ck")
    dev = q.device
    out = {
        "labels_q": torch.empty((bh, n), dtype=torch.int32, device=dev),
        "labels_k": torch.empty((bh, n), dtype=torch.int32, device=dev),
        "cq": torch.empty((bh, kq, d), dtype=torch.float32, device=dev),
        "ck": torch.empty((bh, kk, d), dtype=torch.float32, device=dev),
        "counts_q": torch.empty((bh, kq), dtype=torch.int32, device=dev),
        "counts_k": torch.empty((bh, kk), dtype=torch.int32, device=dev),
    }
    obj = torch.empty((bh, iters, 2), dtype=torch.float64, device=dev) if want_objective else None
    ws = workspace(shape, dev) if ws is None else ws
    st = _lib().svoo_cocluster(ctypes.byref(shape), _ptr(q), _ptr(k), _ptr(init_q_idx), _ptr(init_k_idx),
                               _ptr(init_cq), _ptr(init_ck), iters, _ptr(out["labels_q"]), _ptr(out["labels_k"]),
                               _ptr(out["cq"]), _ptr(out["ck"]), _ptr(out["counts_q"]), _ptr(out["counts_k"]),
                               _ptr(obj), _ptr(ws), ws.numel(), _stream())
    _run(st, "svoo_cocluster")
    if obj is not None:
        out["objective"] = obj
    return out


def kmeans(x, init_idx=None, iters=2, k=None, init_c=None, want_inertia=False, ws=None):
    """svoo_kmeans: independent Lloyd k-means of one tensor.  Returns dict(labels, c, counts[, inertia])."""
    bh, n, d = x.shape
    k = k or (init_idx.shape[1] if init_idx is not None else init_c.shape[1])
    shape = make_shape(x, k, k)
    _check(x, None, (bh, n, d), "x")
    _check(init_idx, torch.int32, (bh, k), "init_idx")
    _check(init_c, torch.float32, (bh, k, d), "init_c")
    dev = x.device
    out = {"labels": torch.empty((bh, n), dtype=torch.int32, device=dev),
           "c": torch.empty((bh, k, d), dtype=torch.float32, device=dev),
           "counts": torch.empty((bh, k), dtype=torch.int32, device=dev)}
    inertia = torch.empty((bh, iters), dtype=torch.float64, device=dev) if want_inertia else None
    ws = workspace(shape, dev) if ws is None else ws
    st = _lib().svoo_kmeans(ctypes.byref(shape), _ptr(x), k, _ptr(init_idx), _ptr(init_c), iters,
                            _ptr(out["labels"]), _ptr(out["c"]), _ptr(out["counts"]), _ptr(inertia), _ptr(ws),
                            ws.numel(), _stream())
    _run(st, "svoo_kmeans")
    if inertia is not None:
        out["inertia"] = inertia
    return out


def assign(x, c_own, c_opp, ws=None):
    """svoo_assign: labels [bh, n] of x against c_own through the affinity to c_opp."""
    bh, n, d = x.shape
    k_own, k_opp = c_own.shape[1], c_opp.shape[1]
    shape = make_shape(x, k_own, k_opp)
    _check(x, None, (bh, n, d), "x")
    _check(c_own, torch.float32, (bh, k_own, d), "c_own")
    _check(c_opp, torch.float32, (bh, k_opp, d), "c_opp")
    labels = torch.empty((bh, n), dtype=torch.int32, device=x.device)
    ws = workspace(shape, x.device) if ws is None else ws
    st = _lib().svoo_assign(ctypes.byref(shape), _ptr(x), _ptr(c_own), k_own, _ptr(c_opp), k_opp, _ptr(labels),
                            _ptr(ws), ws.numel(), _stream())
    _run(st, "svoo_assign")
    return labels


def permute(labels, n_clusters: int, tensors: Sequence[torch.Tensor], ws=None, outs=None):
    """svoo_permute.  Returns (perm, offsets, [sorted tensors])."""
    bh, n = labels.shape
    _check(labels, torch.int32, (bh, n), "labels")
    tensors = list(tensors)
    if tensors:
        d = tensors[0].shape[2]
        shape = make_shape(tensors[0], min(n_clusters, n), min(n_clusters, n))
        for i, t in enumerate(tensors):
            _check(t, tensors[0].dtype, (bh, n, d), f"src[{i}]")
    else:
        shape = Shape(bh, n, 64, SVOO_BF16, min(n_clusters, n), min(n_clusters, n))
    dev = labels.device
    perm = torch.empty((bh, n), dtype=torch.int32, device=dev)
    offsets = torch.empty((bh, n_clusters + 1), dtype=torch.int32, device=dev)
    outs = [torch.empty_like(t) for t in tensors] if outs is None else list(outs)
    nt = len(tensors)
    src = (ctypes.c_void_p * max(nt, 1))(*[t.data_ptr() for t in tensors])
    dst = (ctypes.c_void_p * max(nt, 1))(*[t.data_ptr() for t in outs])
    if ws is None:
        ws = workspace(shape, dev)
        need = int(_lib().svoo_permute_workspace_bytes(ctypes.byref(shape), n_clusters))   # more bins than tokens
        if ws.numel() < need:
            buf = torch.empty(need + 256, dtype=torch.uint8, device=dev)
            off = (-buf.data_ptr()) % 256
            ws = buf[off:off + need]
    st = _lib().svoo_permute(ctypes.byref(shape), _ptr(labels), n_clusters, nt, src, dst, _ptr(perm), _ptr(offsets),
                             _ptr(ws), ws.numel(), _stream())
    _run(st, "svoo_permute")
    return perm, offsets, outs


def gather(perm, tensors: Sequence[torch.Tensor], outs=None):
    """svoo_gather: outs[t][b, p] = tensors[t][b, perm[b, p]] with a permutation computed earlier."""
    tensors = list(tensors)
    bh, n, d = tensors[0].shape
    shape = make_shape(tensors[0], 1, 1)
    _check(perm, torch.int32, (bh, n), "perm")
    for i, t in enumerate(tensors):
        _check(t, tensors[0].dtype, (bh, n, d), f"src[{i}]")
    outs = [torch.empty_like(t) for t in tensors] if outs is None else list(outs)
    nt = len(tensors)
    src = (ctypes.c_void_p * nt)(*[t.data_ptr() for t in tensors])
    dst = (ctypes.c_void_p * nt)(*[t.data_ptr() for t in outs])
    _run(_lib().svoo_gather(ctypes.byref(shape), _ptr(perm), nt, src, dst, _stream()), "svoo_gather")
    return outs


def unpermute(src_sorted, perm, out=None):
    """svoo_unpermute: out[b, perm[b, p]] = src_sorted[b, p]."""
    bh, n, d = src_sorted.shape
    shape = make_shape(src_sorted, 1, 1)
    _check(src_sorted, None, (bh, n, d), "src_sorted")
    _check(perm, torch.int32, (bh, n), "perm")
    out = torch.empty_like(src_sorted) if out is None else out
    _check(out, src_sorted.dtype, (bh, n, d), "out")
    st = _lib().svoo_unpermute(ctypes.byref(shape), _ptr(src_sorted), _ptr(perm), _ptr(out), _stream())
    _run(st, "svoo_unpermute")
    return out


def block_mask(cq, ck, counts_q, counts_k, keep, tau: float, theta: float, scale: float, want_bitmap=True, ws=None):
    """svoo_block_mask.  Returns (block_count, block_list, bitmap or None)."""
    bh, kq, d = cq.shape
    kk = ck.shape[1]
    shape = Shape(bh, max(kq, kk), d, SVOO_F32, kq, kk)
    _check(cq, torch.float32, (bh, kq, d), "cq")
    _check(ck, torch.float32, (bh, kk, d), "ck")
    _check(counts_q, torch.int32, (bh, kq), "counts_q")
    _check(counts_k, torch.int32, (bh, kk), "counts_k")
    _check(keep, torch.float32, (bh,), "keep")
    dev = cq.device
    block_count = torch.empty((bh, kq), dtype=torch.int32, device=dev)
    block_list = torch.empty((bh, kq, kk), dtype=torch.int32, device=dev)
    bitmap = torch.empty((bh, kq, kk), dtype=torch.uint8, device=dev) if want_bitmap else None
    ws = workspace(shape, dev) if ws is None else ws
    st = _lib().svoo_block_mask(ctypes.byref(shape), _ptr(cq), _ptr(ck), _ptr(counts_q), _ptr(counts_k), _ptr(keep),
                                tau, theta, scale, _ptr(block_count), _ptr(block_list), _ptr(bitmap), _ptr(ws),
                                ws.numel(), _stream())
    _run(st, "svoo_block_mask")
    return block_count, block_list, bitmap


def block_sparse_attn(q_sorted, k_sorted, v_sorted, q_offsets, k_offsets, block_count, block_list, scale: float,
                      want_lse=False, out=None, ws=None):
    """svoo_block_sparse_attn.  Returns out_sorted (and lse if asked)."""
    bh, n, d = q_sorted.shape
    kq, kk = q_offsets.shape[1] - 1, k_offsets.shape[1] - 1
    shape = make_shape(q_sorted, kq, kk)
    for name, t in (("q_sorted", q_sorted), ("k_sorted", k_sorted), ("v_sorted", v_sorted)):
        _check(t, q_sorted.dtype, (bh, n, d), name)
    _check(q_offsets, torch.int32, (bh, kq + 1), "q_offsets")
    _check(k_offsets, torch.int32, (bh, kk + 1), "k_offsets")
    _check(block_count, torch.int32, (bh, kq), "block_count")
    _check(block_list, torch.int32, (bh, kq, kk), "block_list")
    out = torch.empty_like(q_sorted) if out is None else out
    _check(out, q_sorted.dtype, (bh, n, d), "out")
    lse = torch.empty((bh, n), dtype=torch.float32, device=q_sorted.device) if want_lse else None
    ws = workspace(shape, q_sorted.device) if ws is None else ws
    st = _lib().svoo_block_sparse_attn(ctypes.byref(shape), _ptr(q_sorted), _ptr(k_sorted), _ptr(v_sorted),
                                       _ptr(q_offsets), _ptr(k_offsets), _ptr(block_count), _ptr(block_list), scale,
                                       _ptr(out), _ptr(lse), _ptr(ws), ws.numel(), _stream())
    _run(st, "svoo_block_sparse_attn")
    return (out, lse) if want_lse else out


def block_sparse_attn_static(q_sorted, k_sorted, v_sorted, q_offsets, k_offsets, block_count, block_list, scale: float,
                             out, lse=None):
    """svoo_block_sparse_attn_static: the caller passes every buffer (also ``out`` and ``lse``); neither
    this wrapper nor the library allocates."""
    bh, n, d = q_sorted.shape
    kq, kk = q_offsets.shape[1] - 1, k_offsets.shape[1] - 1
    shape = make_shape(q_sorted, kq, kk)
    for name, t in (("q_sorted", q_sorted), ("k_sorted", k_sorted), ("v_sorted", v_sorted), ("out", out)):
        _check(t, q_sorted.dtype, (bh, n, d), name)
    _check(q_offsets, torch.int32, (bh, kq + 1), "q_offsets")
    _check(k_offsets, torch.int32, (bh, kk + 1), "k_offsets")
    _check(block_count, torch.int32, (bh, kq), "block_count")
    _check(block_list, torch.int32, (bh, kq, kk), "block_list")
    _check(lse, torch.float32, (bh, n), "lse")
    st = _lib().svoo_block_sparse_attn_static(ctypes.byref(shape), _ptr(q_sorted), _ptr(k_sorted), _ptr(v_sorted),
                                              _ptr(q_offsets), _ptr(k_offsets), _ptr(block_count), _ptr(block_list),
                                              scale, _ptr(out), _ptr(lse), _stream())
    _run(st, "svoo_block_sparse_attn_static")
    return out


def block_sparse_attn_tokens(q, q_perm, k_sorted, v_sorted, q_offsets, k_offsets, block_count, block_list, scale: float,
                             want_lse=False, out=None, ws=None):
    """svoo_block_sparse_attn_tokens: q and out in token order, moved through q_perm by the kernel.
    Returns out (and lse, in token order, if asked)."""
    bh, n, d = q.shape
    kq, kk = q_offsets.shape[1] - 1, k_offsets.shape[1] - 1
    shape = make_shape(q, kq, kk)
    for name, t in (("q", q), ("k_sorted", k_sorted), ("v_sorted", v_sorted)):
        _check(t, q.dtype, (bh, n, d), name)
    _check(q_perm, torch.int32, (bh, n), "q_perm")
    _check(q_offsets, torch.int32, (bh, kq + 1), "q_offsets")
    _check(k_offsets, torch.int32, (bh, kk + 1), "k_offsets")
    _check(block_count, torch.int32, (bh, kq), "block_count")
    _check(block_list, torch.int32, (bh, kq, kk), "block_list")
    out = torch.empty_like(q) if out is None else out
    _check(out, q.dtype, (bh, n, d), "out")
    lse = torch.empty((bh, n), dtype=torch.float32, device=q.device) if want_lse else None
    ws = workspace(shape, q.device) if ws is None else ws
    st = _lib().svoo_block_sparse_attn_tokens(ctypes.byref(shape), _ptr(q), _ptr(q_perm), _ptr(k_sorted), _ptr(v_sorted),
                                              _ptr(q_offsets), _ptr(k_offsets), _ptr(block_count), _ptr(block_list),
                                              scale, _ptr(out), _ptr(lse), _ptr(ws), ws.numel(), _stream())
    _run(st, "svoo_block_sparse_attn_tokens")
    return (out, lse) if want_lse else out


def attn(q, k, v, scale: float, want_lse=False, out=None, ws=None):
    """svoo_attn: dense softmax(scale * q k^T) v."""
    bh, n, d = q.shape
    shape = make_shape(q, 1, 1)
    for name, t in (("q", q), ("k", k), ("v", v)):
        _check(t, q.dtype, (bh, n, d), name)
    out = torch.empty_like(q) if out is None else out
    lse = torch.empty((bh, n), dtype=torch.float32, device=q.device) if want_lse else None
    ws = workspace(shape, q.device) if ws is None else ws
    st = _lib().svoo_attn(ctypes.byref(shape), _ptr(q), _ptr(k), _ptr(v), scale, _ptr(out), _ptr(lse), _ptr(ws),
                          ws.numel(), _stream())
    _run(st, "svoo_attn")
    return (out, lse) if want_lse else out


def attention_density(q, k, tau=0.95, scale=None, rows=None, want_passes=False):
    """svoo_attention_density.  Returns (prefix_len [bh, n_rows] int32, density [bh] float64[, passes [bh]])."""
    bh, n, d = q.shape
    _check(q, None, (bh, n, d), "q")
    _check(k, q.dtype, (bh, n, d), "k")
    n_rows = n if rows is None else rows.shape[0]
    _check(rows, torch.int32, (n_rows,), "rows")
    scale = ctypes.c_float(1.0 / math.sqrt(d)).value if scale is None else scale
    shape = make_shape(q, 1, 1)
    prefix_len = torch.empty((bh, n_rows), dtype=torch.int32, device=q.device)
    density = torch.empty((bh,), dtype=torch.float64, device=q.device)
    passes = torch.empty((bh,), dtype=torch.int32, device=q.device) if want_passes else None
    st = _lib().svoo_attention_density(ctypes.byref(shape), _ptr(q), _ptr(k), _ptr(rows), n_rows, tau, scale,
                                       _ptr(prefix_len), _ptr(density), _ptr(passes), _stream())
    _run(st, "svoo_attention_density")
    return (prefix_len, density, passes) if want_passes else (prefix_len, density)


def microbench_mfma_bf16(sink, iters, random_operands=True):
    """svoo_microbench_mfma_bf16 on sink.numel() / 256 workgroups.  Returns the launch's flop count."""
    _check(sink, torch.float32, None, "sink")
    flops = ctypes.c_double(0.0)
    st = _lib().svoo_microbench_mfma_bf16(sink.numel() // 256, iters, int(random_operands), _ptr(sink),
                                          ctypes.byref(flops), _stream())
    _run(st, "svoo_microbench_mfma_bf16")
    return flops.value


def microbench_attn_tile(parts: int, iters: int, src, sink):
    """svoo_microbench_attn_tile: the LDS traffic (and matrix instructions) of one attention tile step; the
    caller times the launch.  src: device tensor of at least 4 MiB + 64 KiB, sink: float32 [512 * 256]."""
    _check(sink, torch.float32, (512 * 256,), "sink")
    if src.numel() * src.element_size() < (4 << 20) + (64 << 10):
        raise ValueError("src too small")
    _run(_lib().svoo_microbench_attn_tile(parts, iters, _ptr(src), _ptr(sink), _stream()), "svoo_microbench_attn_tile")


def microbench_copy(src, dst):
    """svoo_microbench_copy of the whole of src into dst.  Returns the bytes moved (read + written)."""
    nbytes = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() != nbytes:
        raise ValueError("src and dst differ in size")
    st = _lib().svoo_microbench_copy(_ptr(src), _ptr(dst), nbytes, _stream())
    _run(st, "svoo_microbench_copy")
    return 2 * nbytes


class Layer:
    """Pre-allocated buffers for the five calls of one layer (what a benchmark or a DiT block keeps
    alive between diffusion steps).  ``run`` enqueues the whole online stage on the current stream.
    Layers share the device's cached workspace unless ``own_workspace`` is set: two layers whose calls
    may overlap on the GPU (different streams) each need their own."""

    def __init__(self, bh: int, n: int, d: int, dtype: torch.dtype, kq: int, kk: int, device="cuda:0",
                 own_workspace: bool = False):
        dev = torch.device(device)
        self.dev = dev
        self.kq, self.kk, self.d = kq, kk, d
        x = torch.empty((0,), dtype=dtype)
        self.shape = Shape(bh, n, d, _dtype_code(x), kq, kk)
        i32 = dict(dtype=torch.int32, device=dev)
        self.labels_q = torch.empty((bh, n), **i32)
        self.labels_k = torch.empty((bh, n), **i32)
        self.cq = torch.empty((bh, kq, d), dtype=torch.float32, device=dev)
        self.ck = torch.empty((bh, kk, d), dtype=torch.float32, device=dev)
        self.counts_q = torch.empty((bh, kq), **i32)
        self.counts_k = torch.empty((bh, kk), **i32)
        self.perm_q = torch.empty((bh, n), **i32)
        self.perm_k = torch.empty((bh, n), **i32)
        self.q_offsets = torch.empty((bh, kq + 1), **i32)
        self.k_offsets = torch.empty((bh, kk + 1), **i32)
        self.block_count = torch.empty((bh, kq), **i32)
        self.block_list = torch.empty((bh, kq, kk), **i32)
        self.bitmap = torch.empty((bh, kq, kk), dtype=torch.uint8, device=dev)
        self.q_sorted = torch.empty((bh, n, d), dtype=dtype, device=dev)
        self.k_sorted = torch.empty((bh, n, d), dtype=dtype, device=dev)
        self.v_sorted = torch.empty((bh, n, d), dtype=dtype, device=dev)
        self.o_sorted = torch.empty((bh, n, d), dtype=dtype, device=dev)
        self.out = torch.empty((bh, n, d), dtype=dtype, device=dev)
        self.ws = workspace(self.shape, dev, private=own_workspace)

    # the five calls, individually (the benchmark times them one by one and as a whole)
    def step_cocluster(self, q, k, init_q_idx, init_k_idx, iters):
        lib, s = _lib(), self.shape
        _run(lib.svoo_cocluster(ctypes.byref(s), _ptr(q), _ptr(k), _ptr(init_q_idx), _ptr(init_k_idx), None, None,
                                iters, _ptr(self.labels_q), _ptr(self.labels_k), _ptr(self.cq), _ptr(self.ck),
                                _ptr(self.counts_q), _ptr(self.counts_k), None, _ptr(self.ws), self.ws.numel(),
                                _stream()), "svoo_cocluster")

    def step_cocluster_sorted(self, q, k, init_q_idx, init_k_idx, iters):
        """Co-clustering that leaves perm_q / q_offsets / perm_k / k_offsets behind (no sorts in the permute)."""
        lib, s = _lib(), self.shape
        _run(lib.svoo_cocluster_sorted(ctypes.byref(s), _ptr(q), _ptr(k), _ptr(init_q_idx), _ptr(init_k_idx), None,
                                       None, iters, _ptr(self.labels_q), _ptr(self.labels_k), _ptr(self.cq),
                                       _ptr(self.ck), _ptr(self.counts_q), _ptr(self.counts_k), None,
                                       _ptr(self.perm_q), _ptr(self.q_offsets), _ptr(self.perm_k),
                                       _ptr(self.k_offsets), _ptr(self.ws), self.ws.numel(), _stream()),
             "svoo_cocluster_sorted")

    def step_kmeans(self, q, k, init_q_idx, init_k_idx, iters):
        """Independent partitioner (ablation "w/o On"): K-means of Q and of K, one after the other."""
        lib, s = _lib(), self.shape
        _run(lib.svoo_kmeans(ctypes.byref(s), _ptr(q), self.kq, _ptr(init_q_idx), None, iters, _ptr(self.labels_q),
                             _ptr(self.cq), _ptr(self.counts_q), None, _ptr(self.ws), self.ws.numel(), _stream()),
             "svoo_kmeans(q)")
        _run(lib.svoo_kmeans(ctypes.byref(s), _ptr(k), self.kk, _ptr(init_k_idx), None, iters, _ptr(self.labels_k),
                             _ptr(self.ck), _ptr(self.counts_k), None, _ptr(self.ws), self.ws.numel(), _stream()),
             "svoo_kmeans(k)")

    def step_permute(self, q, k, v):
        lib, s = _lib(), self.shape
        src = (ctypes.c_void_p * 1)(q.data_ptr())
        dst = (ctypes.c_void_p * 1)(self.q_sorted.data_ptr())
        _run(lib.svoo_permute(ctypes.byref(s), _ptr(self.labels_q), self.kq, 1, src, dst, _ptr(self.perm_q),
                              _ptr(self.q_offsets), _ptr(self.ws), self.ws.numel(), _stream()), "svoo_permute(q)")
        src = (ctypes.c_void_p * 2)(k.data_ptr(), v.data_ptr())
        dst = (ctypes.c_void_p * 2)(self.k_sorted.data_ptr(), self.v_sorted.data_ptr())
        _run(lib.svoo_permute(ctypes.byref(s), _ptr(self.labels_k), self.kk, 2, src, dst, _ptr(self.perm_k),
                              _ptr(self.k_offsets), _ptr(self.ws), self.ws.numel(), _stream()), "svoo_permute(kv)")

    def step_regather(self, q, k, v):
        """Move new Q, K, V into cluster order with the permutations of the last clustering."""
        lib, s = _lib(), self.shape
        src = (ctypes.c_void_p * 1)(q.data_ptr())
        dst = (ctypes.c_void_p * 1)(self.q_sorted.data_ptr())
        _run(lib.svoo_gather(ctypes.byref(s), _ptr(self.perm_q), 1, src, dst, _stream()), "svoo_gather(q)")
        src = (ctypes.c_void_p * 2)(k.data_ptr(), v.data_ptr())
        dst = (ctypes.c_void_p * 2)(self.k_sorted.data_ptr(), self.v_sorted.data_ptr())
        _run(lib.svoo_gather(ctypes.byref(s), _ptr(self.perm_k), 2, src, dst, _stream()), "svoo_gather(kv)")

    def step_regather_kv(self, k, v):
        lib, s = _lib(), self.shape
        src = (ctypes.c_void_p * 2)(k.data_ptr(), v.data_ptr())
        dst = (ctypes.c_void_p * 2)(self.k_sorted.data_ptr(), self.v_sorted.data_ptr())
        _run(lib.svoo_gather(ctypes.byref(s), _ptr(self.perm_k), 2, src, dst, _stream()), "svoo_gather(kv)")

    def run_reused(self, q, k, v, scale=None):
        """A step between two re-clusterings: labels, permutations and block lists are kept."""
        scale = 1.0 / math.sqrt(self.d) if scale is None else scale
        self.step_regather(q, k, v)
        self.step_attn(scale)
        self.step_unpermute()
        return self.out

    def step_block_mask(self, keep, tau, theta, scale):
        lib, s = _lib(), self.shape
        _run(lib.svoo_block_mask(ctypes.byref(s), _ptr(self.cq), _ptr(self.ck), _ptr(self.counts_q),
                                 _ptr(self.counts_k), _ptr(keep), tau, theta, scale, _ptr(self.block_count),
                                 _ptr(self.block_list), _ptr(self.bitmap), _ptr(self.ws), self.ws.numel(),
                                 _stream()), "svoo_block_mask")

    def step_attn(self, scale, lse=None):
        lib, s = _lib(), self.shape
        _run(lib.svoo_block_sparse_attn(ctypes.byref(s), _ptr(self.q_sorted), _ptr(self.k_sorted),
                                        _ptr(self.v_sorted), _ptr(self.q_offsets), _ptr(self.k_offsets),
                                        _ptr(self.block_count), _ptr(self.block_list), scale, _ptr(self.o_sorted),
                                        _ptr(lse), _ptr(self.ws), self.ws.numel(), _stream()), "svoo_block_sparse_attn")

    def step_permute_fused(self, k, v):
        """Sort both label arrays but move only K and V: the fused attention reads Q through perm_q."""
        lib, s = _lib(), self.shape
        _run(lib.svoo_permute(ctypes.byref(s), _ptr(self.labels_q), self.kq, 0, None, None, _ptr(self.perm_q),
                              _ptr(self.q_offsets), _ptr(self.ws), self.ws.numel(), _stream()), "svoo_permute(q)")
        src = (ctypes.c_void_p * 2)(k.data_ptr(), v.data_ptr())
        dst = (ctypes.c_void_p * 2)(self.k_sorted.data_ptr(), self.v_sorted.data_ptr())
        _run(lib.svoo_permute(ctypes.byref(s), _ptr(self.labels_k), self.kk, 2, src, dst, _ptr(self.perm_k),
                              _ptr(self.k_offsets), _ptr(self.ws), self.ws.numel(), _stream()), "svoo_permute(kv)")

    def step_attn_fused(self, q, scale, lse=None):
        """Attention with the Q gather and the output scatter folded in (token-order q in, ``out`` out)."""
        lib, s = _lib(), self.shape
        _run(lib.svoo_block_sparse_attn_tokens(ctypes.byref(s), _ptr(q), _ptr(self.perm_q), _ptr(self.k_sorted),
                                               _ptr(self.v_sorted), _ptr(self.q_offsets), _ptr(self.k_offsets),
                                               _ptr(self.block_count), _ptr(self.block_list), scale, _ptr(self.out),
                                               _ptr(lse), _ptr(self.ws), self.ws.numel(), _stream()),
             "svoo_block_sparse_attn_tokens")

    def run_fused(self, q, k, v, init_q_idx, init_k_idx, iters, keep, tau, theta, scale=None):
        """The layer in four calls: co-clustering, K/V permute, mask, attention with fused query-side moves."""
        scale = 1.0 / math.sqrt(self.d) if scale is None else scale
        self.step_cocluster_sorted(q, k, init_q_idx, init_k_idx, iters)
        self.step_regather_kv(k, v)
        self.step_block_mask(keep, tau, theta, scale)
        self.step_attn_fused(q, scale)
        return self.out

    def step_unpermute(self):
        lib, s = _lib(), self.shape
        _run(lib.svoo_unpermute(ctypes.byref(s), _ptr(self.o_sorted), _ptr(self.perm_q), _ptr(self.out), _stream()),
             "svoo_unpermute")

    def run(self, q, k, v, init_q_idx, init_k_idx, iters, keep, tau, theta, scale=None, partitioner="cocluster"):
        scale = 1.0 / math.sqrt(self.d) if scale is None else scale
        if partitioner == "cocluster":      # the layout comes with the clustering: gather only
            self.step_cocluster_sorted(q, k, init_q_idx, init_k_idx, iters)
            self.step_regather(q, k, v)
            self.step_block_mask(keep, tau, theta, scale)
            self.step_attn(scale)
            self.step_unpermute()
            return self.out
        elif partitioner == "kmeans":
            self.step_kmeans(q, k, init_q_idx, init_k_idx, iters)
        else:
            raise ValueError(partitioner)
        self.step_permute(q, k, v)
        self.step_block_mask(keep, tau, theta, scale)
        self.step_attn(scale)
        self.step_unpermute()
        return self.out

    def dense(self, q, k, v, scale=None, lse=None):
        scale = 1.0 / math.sqrt(self.d) if scale is None else scale
        lib, s = _lib(), self.shape
        _run(lib.svoo_attn(ctypes.byref(s), _ptr(q), _ptr(k), _ptr(v), scale, _ptr(self.out), _ptr(lse),
                           _ptr(self.ws), self.ws.numel(), _stream()), "svoo_attn")
        return self.out

    def row_recall(self, q, k, v, scale=None):
        """Diagnostic, not a step of the path: per token, the dense softmax mass that falls on the keys
        of its kept blocks, = exp(LSE over kept keys - LSE over all keys), from the two attention
        kernels' log-sum-exp outputs (svoo_row_recall) for the partition, permutation and block lists this object
        holds.  [bh, n] float32 in token order; its mean is the attention recall of the paper's
        clustering comparison.  Runs both attentions (overwrites ``out`` and ``o_sorted``)."""
        scale = 1.0 / math.sqrt(self.d) if scale is None else scale
        bh, n = self.labels_q.shape
        lse_s = torch.empty((bh, n), dtype=torch.float32, device=self.dev)
        lse_d = torch.empty((bh, n), dtype=torch.float32, device=self.dev)
        self.step_attn(scale, lse=lse_s)
        self.dense(q, k, v, scale, lse=lse_d)
        rec = torch.empty((bh, n), dtype=torch.float32, device=self.dev)
        _run(_lib().svoo_row_recall(ctypes.byref(self.shape), _ptr(lse_s), _ptr(lse_d), _ptr(self.perm_q), _ptr(rec),
                                    _stream()), "svoo_row_recall")
        return rec
