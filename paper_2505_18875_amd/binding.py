"""Thin ctypes binding of libsvg2_hip.so (include/svg2.h).

Argument marshalling only: tensors are torch CUDA(=HIP) tensors used as device
buffers, outputs and the workspace are allocated with torch, the current torch
stream is passed through, and every step of the path runs in the library's
kernels.  There is no fallback: if the library is missing or a call fails, an
exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from types import SimpleNamespace
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsvg2_hip.so")

SVG2_F32, SVG2_BF16 = 0, 1
SVG2_OK = 0
MAX_CLUSTERS = 4096

EXPORTS = (
    "svg2_last_error", "svg2_version",
    "svg2_kmeans_workspace_size", "svg2_kmeans",
    "svg2_permute_workspace_size", "svg2_permute", "svg2_permute_noalloc",
    "svg2_select_topp_workspace_size", "svg2_select_topp",
    "svg2_sparse_attn_workspace_size", "svg2_sparse_attn", "svg2_sparse_attn_gather_free",
    "svg2_forward_workspace_size", "svg2_forward",
    "svg2_forward_gather_free_workspace_size", "svg2_forward_gather_free",
    "svg2_quantize_fp8_workspace_size", "svg2_quantize_fp8", "svg2_sparse_attn_fp8",
    "svg2_forward_fp8_workspace_size", "svg2_forward_fp8",
    "svg2_attention_recall_workspace_size", "svg2_attention_recall",
    "svg2_kmeans_pp_init_workspace_size", "svg2_kmeans_pp_init",
    "svg2_profile_enable", "svg2_profile_read", "svg2_profile_read_kernels",
)
STAGES = ("kmeans", "permute", "select", "attn_plan", "attn")
KERNEL_CLASSES = ("kmeans_assign", "kmeans_settle", "kmeans_sort", "kmeans_segsum_full", "kmeans_segsum_delta",
                  "kmeans_finalize", "permute_sort", "permute_gather")


class Svg2Error(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__("svg2 error %d: %s" % (code, msg))
        self.code = code


class _ForwardAux(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in (
        "labels_q", "labels_k", "counts_q", "counts_k", "offsets_q", "offsets_k",
        "perm_q", "perm_k", "row_ptr", "col_idx", "density", "lse")]


_lib = None


def load_library() -> ctypes.CDLL:
    """Load the C-ABI library; raises if it has not been built (python -m paper_2505_18875_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                "%s not found: build it with `python paper_2505_18875_amd/build.py` "
                "(there is no CPU fallback)" % LIB_PATH)
        lib = ctypes.CDLL(LIB_PATH)
        lib.svg2_last_error.restype = ctypes.c_char_p
        lib.svg2_version.restype = ctypes.c_int
        for n in EXPORTS:
            if n.endswith("_workspace_size"):
                getattr(lib, n).restype = ctypes.c_size_t
        vp, i, f, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_float, ctypes.c_size_t
        lib.svg2_kmeans_workspace_size.argtypes = [i, i, i, i, i]
        lib.svg2_kmeans.argtypes = [vp, i, i, i, i, i, i, vp, vp, vp, vp, vp, vp, sz, vp]
        lib.svg2_permute_workspace_size.argtypes = [i, i, i]
        lib.svg2_permute.argtypes = [vp, i, i, i, vp, vp, vp, i, vp, vp, i, i, vp, sz, vp]
        lib.svg2_permute_noalloc.argtypes = [vp, i, i, i, vp, vp, vp, i, vp, vp, i, i, vp]
        lib.svg2_select_topp_workspace_size.argtypes = [i, i, i]
        lib.svg2_select_topp.argtypes = [vp, vp, vp, vp, i, i, i, i, f, vp, vp, vp, vp, vp, sz, vp]
        lib.svg2_sparse_attn_workspace_size.argtypes = [i, i, i, i, i, i]
        lib.svg2_sparse_attn.argtypes = [vp, vp, vp, i, i, i, i, i, i, vp, vp, vp, vp, vp, f, vp, vp, vp, sz, vp]
        lib.svg2_sparse_attn_gather_free.argtypes = [vp, vp, vp, i, i, i, i, i, i, vp, vp, vp, vp, vp, vp, f, vp, vp, vp,
                                                     sz, vp]
        lib.svg2_forward_workspace_size.argtypes = [i, i, i, i, i, i]
        lib.svg2_forward.argtypes = [vp, vp, vp, i, i, i, i, i, i, f, i, vp, vp, vp, vp, vp, sz, vp]
        lib.svg2_forward_gather_free_workspace_size.argtypes = [i, i, i, i, i, i]
        lib.svg2_forward_gather_free.argtypes = lib.svg2_forward.argtypes
        lib.svg2_quantize_fp8_workspace_size.argtypes = [i]
        lib.svg2_quantize_fp8.argtypes = [vp, i, i, i, i, vp, vp, vp, sz, vp]
        lib.svg2_sparse_attn_fp8.argtypes = [vp, vp, vp, vp, vp, vp, i, i, i, i, i, vp, vp, vp, vp, vp, vp, f, vp, vp,
                                             vp, sz, vp]
        lib.svg2_forward_fp8_workspace_size.argtypes = [i, i, i, i, i, i]
        lib.svg2_forward_fp8.argtypes = lib.svg2_forward.argtypes
        lib.svg2_attention_recall_workspace_size.argtypes = [i, i]
        lib.svg2_attention_recall.argtypes = [vp, vp, i, i, vp, vp, vp, sz, vp]
        lib.svg2_kmeans_pp_init_workspace_size.argtypes = [i, i, i]
        lib.svg2_kmeans_pp_init.argtypes = [vp, i, i, i, i, i, vp, vp, vp, vp, sz, vp]
        lib.svg2_profile_enable.argtypes = [i]
        lib.svg2_profile_read.argtypes = [vp, vp]
        lib.svg2_profile_read_kernels.argtypes = [vp, vp]
        _lib = lib
    return _lib


def _check(rc: int):
    if rc != SVG2_OK:
        raise Svg2Error(rc, load_library().svg2_last_error().decode())


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return SVG2_F32
    if t.dtype == torch.bfloat16:
        return SVG2_BF16
    raise TypeError("svg2 supports float32 and bfloat16 tensors, got %s" % t.dtype)


def _dev(t: Optional[torch.Tensor], dtype=None, name="tensor"):
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("%s must live on the GPU" % name)
    if not t.is_contiguous():
        raise ValueError("%s must be contiguous" % name)
    if dtype is not None and t.dtype != dtype:
        raise TypeError("%s must be %s, got %s" % (name, dtype, t.dtype))
    return ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _workspace(nbytes: int, device) -> torch.Tensor:
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


def svg2_kmeans(X, init_centroids, iters, *, centroids=None, want_objective=False, ws=None):
    """Section 4.1.  X [H,N,d]; init_centroids [H,C,d] fp32 -> centroids, labels, counts (, objective)."""
    lib = load_library()
    H, N, d = X.shape
    C = init_centroids.shape[1]
    dt = _dtype_code(X)
    dev = X.device
    centroids = torch.empty_like(init_centroids) if centroids is None else centroids
    labels = torch.empty((H, N), dtype=torch.int32, device=dev)
    counts = torch.empty((H, C), dtype=torch.int32, device=dev)
    objective = torch.empty((H, iters), dtype=torch.float32, device=dev) if want_objective else None
    need = lib.svg2_kmeans_workspace_size(dt, H, N, d, C)
    ws = _workspace(need, dev) if ws is None else ws
    _check(lib.svg2_kmeans(_dev(X, name="X"), dt, H, N, d, C, int(iters),
                           _dev(init_centroids, torch.float32, "init_centroids"),
                           _dev(centroids, torch.float32, "centroids"), _dev(labels), _dev(counts),
                           _dev(objective), _dev(ws), ws.numel(), _stream()))
    return SimpleNamespace(centroids=centroids, labels=labels, counts=counts, objective=objective)


def svg2_permute(labels, C, tensors=(), *, want_inverse=True, ws=None):
    """Section 4.1.  labels [H,N] int32 -> offsets, perm, inv_perm and the permuted copies of `tensors`."""
    lib = load_library()
    H, N = labels.shape
    dev = labels.device
    offsets = torch.empty((H, C + 1), dtype=torch.int32, device=dev)
    perm = torch.empty((H, N), dtype=torch.int32, device=dev)
    inv = torch.empty((H, N), dtype=torch.int32, device=dev) if want_inverse else None
    n = len(tensors)
    outs = [torch.empty_like(t) for t in tensors]
    dt, d = (SVG2_F32, 0)
    src = dst = None
    if n:
        dt, d = _dtype_code(tensors[0]), tensors[0].shape[-1]
        for t in tensors:
            if t.shape != (H, N, d) or _dtype_code(t) != dt:
                raise ValueError("tensors must all be [H,N,d] of one dtype")
            _dev(t, name="tensor")
        src = (ctypes.c_void_p * n)(*[t.data_ptr() for t in tensors])
        dst = (ctypes.c_void_p * n)(*[t.data_ptr() for t in outs])
    need = lib.svg2_permute_workspace_size(H, N, C)
    ws = _workspace(need, dev) if ws is None else ws
    _check(lib.svg2_permute(_dev(labels, torch.int32, "labels"), H, N, C, _dev(offsets), _dev(perm), _dev(inv),
                            n, src, dst, dt, d, _dev(ws), ws.numel(), _stream()))
    return SimpleNamespace(offsets=offsets, perm=perm, inv_perm=inv, tensors=outs)


def svg2_permute_noalloc(labels, C, offsets, perm, inv_perm=None, tensors=(), outs=()):
    """svg2_permute on the library's built-in scratch: every buffer is the caller's, nothing is allocated here
    or in the library.  labels [H,N] int32; offsets [H,C+1], perm [H,N], inv_perm [H,N] or None int32 outputs;
    outs[t] receives the permuted copy of tensors[t]."""
    lib = load_library()
    H, N = labels.shape
    n = len(tensors)
    if len(outs) != n:
        raise ValueError("one output per tensor")
    dt, d = (SVG2_F32, 0)
    src = dst = None
    if n:
        dt, d = _dtype_code(tensors[0]), tensors[0].shape[-1]
        for t, o in zip(tensors, outs):
            if t.shape != (H, N, d) or _dtype_code(t) != dt or o.shape != t.shape or o.dtype != t.dtype:
                raise ValueError("tensors and outs must all be [H,N,d] of one dtype")
            _dev(t, name="tensor")
            _dev(o, name="out")
        src = (ctypes.c_void_p * n)(*[t.data_ptr() for t in tensors])
        dst = (ctypes.c_void_p * n)(*[t.data_ptr() for t in outs])
    _check(lib.svg2_permute_noalloc(_dev(labels, torch.int32, "labels"), H, N, C, _dev(offsets, torch.int32, "offsets"),
                                    _dev(perm, torch.int32, "perm"), _dev(inv_perm, torch.int32, "inv_perm"),
                                    n, src, dst, dt, d, _stream()))


def svg2_select_topp(cq, ck, counts_q, counts_k, top_p, *, want_p_est=False, ws=None):
    """Section 4.2, Eq. 1-2 and the top-p rule -> CSR (row_ptr, col_idx), density (, p_est)."""
    lib = load_library()
    H, Cq, d = cq.shape
    Ck = ck.shape[1]
    dev = cq.device
    row_ptr = torch.empty((H, Cq + 1), dtype=torch.int32, device=dev)
    col_idx = torch.empty((H, Cq * Ck), dtype=torch.int32, device=dev)
    p_est = torch.empty((H, Cq, Ck), dtype=torch.float32, device=dev) if want_p_est else None
    density = torch.empty((H,), dtype=torch.float32, device=dev) if counts_q is not None else None
    need = lib.svg2_select_topp_workspace_size(H, Cq, Ck)
    ws = _workspace(need, dev) if ws is None else ws
    _check(lib.svg2_select_topp(_dev(cq, torch.float32, "cq"), _dev(ck, torch.float32, "ck"),
                                _dev(counts_q, torch.int32, "counts_q"), _dev(counts_k, torch.int32, "counts_k"),
                                H, Cq, Ck, d, float(top_p), _dev(row_ptr), _dev(col_idx), _dev(p_est),
                                _dev(density), _dev(ws), ws.numel(), _stream()))
    return SimpleNamespace(row_ptr=row_ptr, col_idx=col_idx, p_est=p_est, density=density)


def svg2_sparse_attn(Qp, Kp, Vp, offsets_q, offsets_k, row_ptr, col_idx, perm_q=None, *, scale=0.0,
                     want_lse=False, out=None, ws=None):
    """Section 4.3.  Permuted Q, K, V [H,N,d] + block list -> O [H,N,d] (original order if perm_q is given)."""
    lib = load_library()
    H, N, d = Qp.shape
    Cq, Ck = offsets_q.shape[1] - 1, offsets_k.shape[1] - 1
    dt = _dtype_code(Qp)
    dev = Qp.device
    if col_idx.numel() < H * Cq * Ck:
        raise ValueError("col_idx must have capacity H*Cq*Ck")
    O = torch.empty_like(Qp) if out is None else out
    lse = torch.empty((H, N), dtype=torch.float32, device=dev) if want_lse else None
    need = lib.svg2_sparse_attn_workspace_size(dt, H, N, d, Cq, Ck)
    ws = _workspace(need, dev) if ws is None else ws
    _check(lib.svg2_sparse_attn(_dev(Qp, name="Qp"), _dev(Kp, Qp.dtype, "Kp"), _dev(Vp, Qp.dtype, "Vp"), dt, H, N, d,
                                Cq, Ck, _dev(offsets_q, torch.int32, "offsets_q"),
                                _dev(offsets_k, torch.int32, "offsets_k"), _dev(row_ptr, torch.int32, "row_ptr"),
                                _dev(col_idx, torch.int32, "col_idx"), _dev(perm_q, torch.int32, "perm_q"),
                                float(scale), _dev(O, Qp.dtype, "O"), _dev(lse), _dev(ws), ws.numel(), _stream()))
    return SimpleNamespace(O=O, lse=lse)


def svg2_sparse_attn_gather_free(Q, K, V, offsets_q, offsets_k, row_ptr, col_idx, perm_q, perm_k, *, scale=0.0,
                                 want_lse=False, out=None, ws=None):
    """Section 4.3 with sparse loading: Q, K, V [H,N,d] in token order + both permutations + block list -> O."""
    lib = load_library()
    H, N, d = Q.shape
    Cq, Ck = offsets_q.shape[1] - 1, offsets_k.shape[1] - 1
    dt = _dtype_code(Q)
    dev = Q.device
    if col_idx.numel() < H * Cq * Ck:
        raise ValueError("col_idx must have capacity H*Cq*Ck")
    O = torch.empty_like(Q) if out is None else out
    lse = torch.empty((H, N), dtype=torch.float32, device=dev) if want_lse else None
    need = lib.svg2_sparse_attn_workspace_size(dt, H, N, d, Cq, Ck)
    ws = _workspace(need, dev) if ws is None else ws
    _check(lib.svg2_sparse_attn_gather_free(
        _dev(Q, name="Q"), _dev(K, Q.dtype, "K"), _dev(V, Q.dtype, "V"), dt, H, N, d, Cq, Ck,
        _dev(offsets_q, torch.int32, "offsets_q"), _dev(offsets_k, torch.int32, "offsets_k"),
        _dev(row_ptr, torch.int32, "row_ptr"), _dev(col_idx, torch.int32, "col_idx"),
        _dev(perm_q, torch.int32, "perm_q"), _dev(perm_k, torch.int32, "perm_k"), float(scale),
        _dev(O, Q.dtype, "O"), _dev(lse), _dev(ws), ws.numel(), _stream()))
    return SimpleNamespace(O=O, lse=lse)


def svg2_quantize_fp8(X, *, ws=None):
    """Table 1 (+ FP8): X [H,N,d] -> (X8 [H,N,d] uint8 E4M3 codes, scale [H] fp32), X ~ decode(X8) * scale[h]."""
    lib = load_library()
    H, N, d = X.shape
    dev = X.device
    X8 = torch.empty((H, N, d), dtype=torch.uint8, device=dev)
    scale = torch.empty((H,), dtype=torch.float32, device=dev)
    ws = _workspace(lib.svg2_quantize_fp8_workspace_size(H), dev) if ws is None else ws
    _check(lib.svg2_quantize_fp8(_dev(X, name="X"), _dtype_code(X), H, N, d, _dev(X8), _dev(scale), _dev(ws),
                                 ws.numel(), _stream()))
    return X8, scale


def svg2_sparse_attn_fp8(Q8, K8, V8, scale_q, scale_k, scale_v, offsets_q, offsets_k, row_ptr, col_idx,
                         perm_q=None, perm_k=None, *, scale=0.0, want_lse=False, out=None, ws=None):
    """Section 4.3 on E4M3 operands.  perm_k None: permuted copies; perm_k given: token order (gather-free)."""
    lib = load_library()
    H, N, d = Q8.shape
    Cq, Ck = offsets_q.shape[1] - 1, offsets_k.shape[1] - 1
    dev = Q8.device
    if col_idx.numel() < H * Cq * Ck:
        raise ValueError("col_idx must have capacity H*Cq*Ck")
    O = torch.empty((H, N, d), dtype=torch.bfloat16, device=dev) if out is None else out
    lse = torch.empty((H, N), dtype=torch.float32, device=dev) if want_lse else None
    need = lib.svg2_sparse_attn_workspace_size(SVG2_BF16, H, N, d, Cq, Ck)
    ws = _workspace(need, dev) if ws is None else ws
    _check(lib.svg2_sparse_attn_fp8(
        _dev(Q8, torch.uint8, "Q8"), _dev(K8, torch.uint8, "K8"), _dev(V8, torch.uint8, "V8"),
        _dev(scale_q, torch.float32, "scale_q"), _dev(scale_k, torch.float32, "scale_k"),
        _dev(scale_v, torch.float32, "scale_v"), H, N, d, Cq, Ck,
        _dev(offsets_q, torch.int32, "offsets_q"), _dev(offsets_k, torch.int32, "offsets_k"),
        _dev(row_ptr, torch.int32, "row_ptr"), _dev(col_idx, torch.int32, "col_idx"),
        _dev(perm_q, torch.int32, "perm_q"), _dev(perm_k, torch.int32, "perm_k"), float(scale),
        _dev(O, torch.bfloat16, "O"), _dev(lse), _dev(ws), ws.numel(), _stream()))
    return SimpleNamespace(O=O, lse=lse)


def svg2_forward_workspace_size(dtype_code, H, N, d, Cq, Ck, gather_free=False, fp8=False) -> int:
    lib = load_library()
    fn = (lib.svg2_forward_fp8_workspace_size if fp8 else
          lib.svg2_forward_gather_free_workspace_size if gather_free else lib.svg2_forward_workspace_size)
    return fn(dtype_code, H, N, d, Cq, Ck)


def svg2_forward_fp8(Q, K, V, cq_inout, ck_inout, top_p, iters, **kw):
    """svg2_forward with the attention step on E4M3 copies of Q, K, V (Table 1, + FP8)."""
    return svg2_forward(Q, K, V, cq_inout, ck_inout, top_p, iters, fp8=True, **kw)


def svg2_forward_gather_free(Q, K, V, cq_inout, ck_inout, top_p, iters, **kw):
    """svg2_forward without permuted copies of Q, K, V (Section 4.3, sparse loading)."""
    return svg2_forward(Q, K, V, cq_inout, ck_inout, top_p, iters, gather_free=True, **kw)


def svg2_forward(Q, K, V, cq_inout, ck_inout, top_p, iters, *, want_aux=False, out=None, ws=None,
                 gather_free=False, fp8=False):
    """Section 4, the whole layer.  cq_inout / ck_inout [H,C,d] fp32 are updated in place (centroid cache)."""
    lib = load_library()
    H, N, d = Q.shape
    Cq, Ck = cq_inout.shape[1], ck_inout.shape[1]
    dt = _dtype_code(Q)
    dev = Q.device
    O = torch.empty_like(Q) if out is None else out
    aux_t = None
    aux_p = None
    if want_aux:
        i32 = dict(dtype=torch.int32, device=dev)
        aux_t = SimpleNamespace(
            labels_q=torch.empty((H, N), **i32), labels_k=torch.empty((H, N), **i32),
            counts_q=torch.empty((H, Cq), **i32), counts_k=torch.empty((H, Ck), **i32),
            offsets_q=torch.empty((H, Cq + 1), **i32), offsets_k=torch.empty((H, Ck + 1), **i32),
            perm_q=torch.empty((H, N), **i32), perm_k=torch.empty((H, N), **i32),
            row_ptr=torch.empty((H, Cq + 1), **i32), col_idx=torch.empty((H, Cq * Ck), **i32),
            density=torch.empty((H,), dtype=torch.float32, device=dev),
            lse=torch.empty((H, N), dtype=torch.float32, device=dev))
        aux_s = _ForwardAux(**{n: getattr(aux_t, n).data_ptr() for n, _ in _ForwardAux._fields_})
        aux_p = ctypes.cast(ctypes.pointer(aux_s), ctypes.c_void_p)
    need = svg2_forward_workspace_size(dt, H, N, d, Cq, Ck, gather_free, fp8)
    ws = _workspace(need, dev) if ws is None else ws
    entry = lib.svg2_forward_fp8 if fp8 else lib.svg2_forward_gather_free if gather_free else lib.svg2_forward
    _check(entry(_dev(Q, name="Q"), _dev(K, Q.dtype, "K"), _dev(V, Q.dtype, "V"), dt, H, N, d, Cq, Ck,
                            float(top_p), int(iters), _dev(cq_inout, torch.float32, "cq_inout"),
                            _dev(ck_inout, torch.float32, "ck_inout"), _dev(O, Q.dtype, "O"), aux_p,
                            _dev(ws), ws.numel(), _stream()))
    return SimpleNamespace(O=O, aux=aux_t)


def svg2_attention_recall(lse_selected, lse_all, *, want_rows=True, ws=None):
    """Section 3.1.  lse of the selected keys and of all keys [H,N] fp32 -> recall per query (, mean per head)."""
    lib = load_library()
    H, N = lse_selected.shape
    dev = lse_selected.device
    rows = torch.empty((H, N), dtype=torch.float32, device=dev) if want_rows else None
    mean = torch.empty((H,), dtype=torch.float32, device=dev)
    need = lib.svg2_attention_recall_workspace_size(H, N)
    ws = _workspace(need, dev) if ws is None else ws
    _check(lib.svg2_attention_recall(_dev(lse_selected, torch.float32, "lse_selected"),
                                     _dev(lse_all, torch.float32, "lse_all"), H, N, _dev(rows), _dev(mean),
                                     _dev(ws), ws.numel(), _stream()))
    return SimpleNamespace(recall=rows, mean=mean)


def svg2_kmeans_pp_init(X, C, u, *, ws=None):
    """Sections 4.3 / 5.3: k-means++ seeding with the caller's uniform numbers u [H,C] fp64 -> centroids, picked."""
    lib = load_library()
    H, N, d = X.shape
    dev = X.device
    if u.shape != (H, C):
        raise ValueError("u must be [H,C]")
    centroids = torch.empty((H, C, d), dtype=torch.float32, device=dev)
    picked = torch.empty((H, C), dtype=torch.int32, device=dev)
    need = lib.svg2_kmeans_pp_init_workspace_size(H, N, C)
    ws = _workspace(need, dev) if ws is None else ws
    _check(lib.svg2_kmeans_pp_init(_dev(X, name="X"), _dtype_code(X), H, N, d, C, _dev(u, torch.float64, "u"),
                                   _dev(centroids), _dev(picked), _dev(ws), ws.numel(), _stream()))
    return SimpleNamespace(centroids=centroids, picked=picked)


def svg2_profile_enable(level) -> None:
    """0 / False: stop; 1 / True: record HIP events around the stages of svg2_forward; 2: also around every
    kernel launch of k-means and the permutation."""
    _check(load_library().svg2_profile_enable(int(level)))


def svg2_profile_read():
    """(dict stage -> summed milliseconds, number of recorded svg2_forward calls); clears the record."""
    ms = (ctypes.c_float * len(STAGES))()
    n = ctypes.c_int(0)
    _check(load_library().svg2_profile_read(ctypes.cast(ms, ctypes.c_void_p), ctypes.cast(ctypes.pointer(n), ctypes.c_void_p)))
    return {k: float(v) for k, v in zip(STAGES, ms)}, n.value


def svg2_profile_read_kernels():
    """dict kernel class -> (summed milliseconds, launches) of the spans recorded at profile level 2; clears them."""
    n = len(KERNEL_CLASSES)
    ms = (ctypes.c_float * n)()
    cnt = (ctypes.c_int * n)()
    _check(load_library().svg2_profile_read_kernels(ctypes.cast(ms, ctypes.c_void_p), ctypes.cast(cnt, ctypes.c_void_p)))
    return {k: (float(m), int(c)) for k, m, c in zip(KERNEL_CLASSES, ms, cnt)}
