"""Helpers shared by the GPU parity tests: numpy <-> device tensors in the workload's storage type."""
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import torch

from paper_2505_18875_amd import workloads as wl


def to_dev(x: np.ndarray, dtype: str = "f32") -> torch.Tensor:
    """float32 numpy -> cuda tensor (bf16 workloads: values are bf16-representable, so the cast is exact)."""
    t = torch.from_numpy(np.ascontiguousarray(x))
    if t.dtype == torch.float32 and dtype == "bf16":
        return t.cuda().to(torch.bfloat16).contiguous()
    return t.cuda().contiguous()


def to_np(t: torch.Tensor) -> np.ndarray:
    if t.dtype == torch.bfloat16:
        return t.float().cpu().numpy()
    return t.cpu().numpy()


def head_inputs(w: wl.Workload, heads):
    """Q, K, V [len(heads),N,d] float32 numpy plus seeded initial centroids for both sides."""
    Q, K, V = wl.make_heads(w, heads)
    cq = np.stack([wl.init_centroids(w, h, Q[i], w.Cq, 0) for i, h in enumerate(heads)])
    ck = np.stack([wl.init_centroids(w, h, K[i], w.Ck, 1) for i, h in enumerate(heads)])
    return Q, K, V, cq, ck


def assert_label_disagreements_are_near_ties(svg2, oracle, X, X_dev, init, iters, bf16, gpu_labels, ref_labels):
    """The GPU's last assign step, judged on its own input: the centroids after iters - 1 GPU
    iterations (k-means on the GPU is reproducible bit for bit, so re-running it gives the state the
    last assign saw) go through ONE oracle assign step; wherever that disagrees with the GPU's labels
    the token must be a near-tie (relative gap of its two smallest squared distances < 1e-3).
    Against the oracle's own full run only the agreement rate is meaningful after several
    iterations: an early near-tie flip moves centroids a little and later labels follow.
    X [N,d] numpy, X_dev [1,N,d] device tensor of the same head, init [C,d] numpy."""
    if np.array_equal(gpu_labels, ref_labels):
        return 0
    if iters > 1:
        prev = svg2.svg2_kmeans(X_dev, torch.from_numpy(np.ascontiguousarray(init[None], dtype=np.float32)).cuda(),
                                iters - 1).centroids
        torch.cuda.synchronize()
        prev = prev[0].cpu().numpy()
    else:
        prev = np.asarray(init, dtype=np.float32)
    one = oracle.kmeans(X, prev, 1, bf16).labels
    bad = np.nonzero(gpu_labels != one)[0]
    if bad.size:
        gap = oracle.top2_gap(X[bad], prev, bf16)
        assert np.all(gap < 1e-3), "label disagreement away from a tie: gaps %s" % np.sort(gap)[-5:]
    assert bad.size <= 1e-3 * gpu_labels.size
    return int(bad.size)


def upload_heads(w, heads):
    """All requested heads of a bf16 workload as device tensors (Q, K, V) plus their seeded initial centroids."""
    H = len(heads)
    Q = torch.empty((H, w.N, w.d), dtype=torch.bfloat16, device="cuda")
    K, V = torch.empty_like(Q), torch.empty_like(Q)
    cq = torch.empty((H, w.Cq, w.d), dtype=torch.float32, device="cuda")
    ck = torch.empty((H, w.Ck, w.d), dtype=torch.float32, device="cuda")

    def gen(i):
        h = heads[i]
        q, k, v = wl.make_head(w, h)
        return i, q, k, v, wl.init_centroids(w, h, q, w.Cq, 0), wl.init_centroids(w, h, k, w.Ck, 1)

    with ThreadPoolExecutor(max_workers=8) as ex:
        for i, q, k, v, a, b in ex.map(gen, range(H)):
            Q[i], K[i], V[i] = to_dev(q, "bf16"), to_dev(k, "bf16"), to_dev(v, "bf16")
            cq[i], ck[i] = to_dev(a), to_dev(b)
    return Q, K, V, cq, ck
