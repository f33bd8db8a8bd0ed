"""ctypes front end of the CPU oracle (oracle/svg2_oracle.c).  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import
this module; the product package never does.  All functions work on ONE head;
callers loop over heads.  Arrays are numpy; floating results are float64.

`forward` strings the stages together in the order of the paper's Section 4:
k-means of Q and of K (4.1), the two permutations (4.1), centroid top-p
selection (4.2), block-sparse attention with the inverse query permutation
applied on output (4.3, 4.1).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from types import SimpleNamespace

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "svg2_oracle.c")
_LIB = os.path.join(_HERE, "libsvg2_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (OpenMP over independent rows)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-std=c11",
                               "-Wall", "-Wextra", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.svg2o_padding_waste.restype = ctypes.c_double
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def n_threads() -> int:
    """Threads the OpenMP regions will use (OMP_NUM_THREADS or the core count)."""
    v = os.environ.get("OMP_NUM_THREADS")
    if v:
        try:
            return max(1, int(v.split(",")[0]))
        except ValueError:
            pass
    return len(os.sched_getaffinity(0))


def dense_attention(Q, K, V, scale=None, want_lse=True):
    Q, K, V = _f32(Q), _f32(K), _f32(V)
    Nq, d = Q.shape
    Nk = K.shape[0]
    scale = 1.0 / np.sqrt(d) if scale is None else scale
    O = np.empty((Nq, d), dtype=np.float64)
    lse = np.empty(Nq, dtype=np.float64) if want_lse else None
    _load().svg2o_dense_attention(_p(Q), _p(K), _p(V), Nq, Nk, d, ctypes.c_double(scale), _p(O), _p(lse))
    return O, lse


def kmeans(X, init, iters, round_bf16):
    X = _f32(X)
    N, d = X.shape
    init = _f64(init)
    C = init.shape[0]
    cent = np.empty((C, d), dtype=np.float64)
    labels = np.empty(N, dtype=np.int32)
    counts = np.empty(C, dtype=np.int32)
    obj = np.empty(2 * iters, dtype=np.float64)
    _load().svg2o_kmeans(_p(X), N, d, C, int(iters), int(bool(round_bf16)), _p(init),
                         _p(cent), _p(labels), _p(counts), _p(obj))
    return SimpleNamespace(centroids=cent, labels=labels, counts=counts, objective=obj)


def top2_gap(X, centroids, round_bf16):
    X = _f32(X)
    N, d = X.shape
    c = _f64(centroids)
    gap = np.empty(N, dtype=np.float64)
    _load().svg2o_top2_gap(_p(X), N, d, c.shape[0], int(bool(round_bf16)), _p(c), _p(gap))
    return gap


def permute(labels, C):
    labels = _i32(labels)
    N = labels.shape[0]
    counts = np.empty(C, dtype=np.int32)
    offsets = np.empty(C + 1, dtype=np.int32)
    perm = np.empty(N, dtype=np.int32)
    inv = np.empty(N, dtype=np.int32)
    _load().svg2o_permute(_p(labels), N, C, _p(counts), _p(offsets), _p(perm), _p(inv))
    return SimpleNamespace(counts=counts, offsets=offsets, perm=perm, inv_perm=inv)


def gather_rows(X, perm):
    X = _f32(X)
    perm = _i32(perm)
    Xp = np.empty_like(X)
    _load().svg2o_gather_rows(_p(X), _p(perm), X.shape[0], X.shape[1], _p(Xp))
    return Xp


def select_topp(cq, ck, counts_q, counts_k, top_p):
    cq, ck = _f64(cq), _f64(ck)
    Cq, d = cq.shape
    Ck = ck.shape[0]
    counts_k = _i32(counts_k)
    counts_q = None if counts_q is None else _i32(counts_q)
    row_ptr = np.empty(Cq + 1, dtype=np.int32)
    col_idx = np.empty(Cq * Ck, dtype=np.int32)
    p_est = np.empty((Cq, Ck), dtype=np.float64)
    margin = np.empty(Cq, dtype=np.float64)
    dens = ctypes.c_double(0.0)
    _load().svg2o_select_topp(_p(cq), _p(ck), _p(counts_q), _p(counts_k), Cq, Ck, d,
                              ctypes.c_double(top_p), _p(row_ptr), _p(col_idx), _p(p_est),
                              _p(margin), ctypes.byref(dens))
    return SimpleNamespace(row_ptr=row_ptr, col_idx=col_idx[: row_ptr[-1]].copy(), p_est=p_est,
                           margin=margin, density=dens.value)


def sparse_attention(Qp, Kp, Vp, offsets_q, offsets_k, row_ptr, col_idx, perm_q=None,
                     scale=None, rows=None):
    """Returns (O, lse); with `rows` only those permuted rows are filled (others NaN)."""
    Qp, Kp, Vp = _f32(Qp), _f32(Kp), _f32(Vp)
    N, d = Qp.shape
    offsets_q, offsets_k = _i32(offsets_q), _i32(offsets_k)
    row_ptr, col_idx = _i32(row_ptr), _i32(col_idx)
    Cq, Ck = offsets_q.shape[0] - 1, offsets_k.shape[0] - 1
    scale = 1.0 / np.sqrt(d) if scale is None else scale
    O = np.full((N, d), np.nan, dtype=np.float64)
    lse = np.full(N, np.nan, dtype=np.float64)
    pq = None if perm_q is None else _i32(perm_q)
    rr = None if rows is None else _i32(rows)
    _load().svg2o_sparse_attention(_p(Qp), _p(Kp), _p(Vp), N, d, Cq, Ck, _p(offsets_q), _p(offsets_k),
                                   _p(row_ptr), _p(col_idx), _p(pq), ctypes.c_double(scale),
                                   _p(rr), 0 if rr is None else rr.shape[0], _p(O), _p(lse))
    return O, lse


def rounded_weights_budget(Qp, Kp, Vp, offsets_q, offsets_k, row_ptr, col_idx, perm_q=None, scale=None, rows=None,
                           tail_ratio=0.0, tail_abs=0.0):
    """Error budget of the block-sparse attention output when the probabilities are rounded before they multiply V
    and the row sum is taken over the rounded values.  Returns (dev1, dev2, tail1, tail2, tailw); the first four
    [N,d], tailw [N], float64, indexed like the attention output (NaN for rows not computed):
      dev1 = sum_j pi_j |v_jc - O_c|          |error| <= eps / (1 - eps) * dev1 for relative weight errors <= eps
      dev2 = sum_j pi_j^2 (v_jc - O_c)^2      error std = eps / sqrt(3) * sqrt(dev2) for independent uniform errors
      tail1, tail2, tailw: the same sums with a_j = min(pi_j, tail_abs * pi_max) in place of pi_j (tailw: of a_j
      alone) over the keys with pi_j < tail_ratio * pi_max, whose weights may carry an absolute error a_j."""
    Qp, Kp, Vp = _f32(Qp), _f32(Kp), _f32(Vp)
    N, d = Qp.shape
    offsets_q, offsets_k = _i32(offsets_q), _i32(offsets_k)
    row_ptr, col_idx = _i32(row_ptr), _i32(col_idx)
    Cq, Ck = offsets_q.shape[0] - 1, offsets_k.shape[0] - 1
    scale = 1.0 / np.sqrt(d) if scale is None else scale
    outs = [np.full((N, d), np.nan, dtype=np.float64) for _ in range(4)] + [np.full(N, np.nan, dtype=np.float64)]
    pq = None if perm_q is None else _i32(perm_q)
    rr = None if rows is None else _i32(rows)
    _load().svg2o_rounded_weights_budget(_p(Qp), _p(Kp), _p(Vp), N, d, Cq, Ck, _p(offsets_q), _p(offsets_k),
                                         _p(row_ptr), _p(col_idx), _p(pq), ctypes.c_double(scale),
                                         ctypes.c_double(tail_ratio), ctypes.c_double(tail_abs), _p(rr),
                                         0 if rr is None else rr.shape[0], *[_p(o) for o in outs])
    return tuple(outs)


def attention_recall(Q, K, labels_q, labels_k, Cq, Ck, row_ptr, col_idx, scale=None, rows=None):
    """Section 3.1: per query token, the true attention mass of the keys its cluster's selection computes.
    Q, K in original token order; with `rows` only those tokens are filled (others NaN)."""
    Q, K = _f32(Q), _f32(K)
    N, d = Q.shape
    lq, lk, rp, ci = _i32(labels_q), _i32(labels_k), _i32(row_ptr), _i32(col_idx)
    scale = 1.0 / np.sqrt(d) if scale is None else scale
    out = np.full(N, np.nan, dtype=np.float64)
    rr = None if rows is None else _i32(rows)
    _load().svg2o_attention_recall(_p(Q), _p(K), N, d, _p(lq), _p(lk), int(Cq), int(Ck), _p(rp), _p(ci),
                                   ctypes.c_double(scale), _p(rr), 0 if rr is None else rr.shape[0], _p(out))
    return out


def kmeans_pp(X, C, u):
    """k-means++ seeding with the uniform numbers u[C] given: (picked token indices [C], centres [C,d])."""
    X = _f32(X)
    N, d = X.shape
    u = _f64(u)
    assert u.shape == (C,)
    picked = np.empty(C, dtype=np.int32)
    _load().svg2o_kmeans_pp(_p(X), N, d, int(C), _p(u), _p(picked))
    return picked, X[picked].copy()


def round_e4m3(y):
    """Nearest OCP E4M3 value (ties to even, clamped to +-448) of each element of y."""
    lib = _load()
    lib.svg2o_round_e4m3.restype = ctypes.c_double
    y = np.asarray(y, dtype=np.float64)
    return np.array([lib.svg2o_round_e4m3(ctypes.c_double(v)) for v in y.ravel()]).reshape(y.shape)


def encode_e4m3(v):
    """8-bit codes of E4M3 values."""
    lib = _load()
    lib.svg2o_encode_e4m3.restype = ctypes.c_uint8
    v = np.asarray(v, dtype=np.float64)
    return np.array([lib.svg2o_encode_e4m3(ctypes.c_double(x)) for x in v.ravel()], dtype=np.uint8).reshape(v.shape)


def quantize_e4m3(X):
    """One head of one tensor: (codes uint8, decoded float32 = decode(codes), scale float32) with
    X ~ decoded * scale (per-head amax scaling, single-precision products)."""
    X = _f32(X)
    codes = np.empty(X.shape, dtype=np.uint8)
    dec = np.empty(X.shape, dtype=np.float32)
    sc = ctypes.c_float(0.0)
    _load().svg2o_quantize_e4m3(_p(X), ctypes.c_long(X.size), _p(codes), _p(dec), ctypes.byref(sc))
    return codes, dec, np.float32(sc.value)


def padding_waste(rows, cols, bm, bn) -> float:
    return float(_load().svg2o_padding_waste(int(rows), int(cols), int(bm), int(bn)))


def forward(Q, K, V, init_cq, init_ck, iters, top_p, round_bf16, rows=None):
    """The whole per-head path.  `rows` (permuted query rows) restricts the attention step."""
    kq = kmeans(Q, init_cq, iters, round_bf16)
    kk = kmeans(K, init_ck, iters, round_bf16)
    pq = permute(kq.labels, kq.centroids.shape[0])
    pk = permute(kk.labels, kk.centroids.shape[0])
    Qp, Kp, Vp = gather_rows(Q, pq.perm), gather_rows(K, pk.perm), gather_rows(V, pk.perm)
    sel = select_topp(kq.centroids, kk.centroids, kq.counts, kk.counts, top_p)
    O, lse = sparse_attention(Qp, Kp, Vp, pq.offsets, pk.offsets, sel.row_ptr, sel.col_idx,
                              perm_q=pq.perm, rows=rows)
    return SimpleNamespace(kq=kq, kk=kk, pq=pq, pk=pk, Qp=Qp, Kp=Kp, Vp=Vp, sel=sel, O=O, lse=lse,
                           density=sel.density)
