"""Helpers shared by the GPU parity tests: numpy <-> device tensors in the workload's storage type."""
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
