"""The synthetic input generators: shapes, determinism, storage type."""
import numpy as np
import torch

from paper_2505_18875_amd import workloads as wl


def test_shapes_match_the_paper_sequence_lengths():
    # Section 5.1: 3600 tokens per frame, 21 frames (Wan2.1) and 33 frames (HunyuanVideo)
    assert wl.WORKLOADS["wan_like"].N == 21 * 3600 == 75600
    assert wl.WORKLOADS["hunyuan_like"].N == 33 * 3600 == 118800
    for w in wl.WORKLOADS.values():
        assert (w.Cq, w.Ck) in ((16, 32), (100, 500))


def test_heads_are_seeded_and_independent():
    w = wl.replace(wl.WORKLOADS["small"], grid=(4, 8, 8))
    a = wl.make_head(w, 3)
    b = wl.make_head(w, 3)
    c = wl.make_head(w, 4)
    for x, y in zip(a, b):
        np.testing.assert_array_equal(x, y)
    assert not np.array_equal(a[0], c[0])
    Q, K, V = wl.make_heads(w, [3, 4])
    np.testing.assert_array_equal(Q[0], a[0])
    np.testing.assert_array_equal(K[1], c[1])
    assert Q.shape == (2, w.N, w.d) and Q.dtype == np.float32


def test_bf16_workloads_are_exactly_representable():
    w = wl.replace(wl.WORKLOADS["small"], grid=(2, 8, 8))
    Q, K, V = wl.make_head(w, 0)
    for X in (Q, K, V):
        t = torch.from_numpy(X)
        assert torch.equal(t.to(torch.bfloat16).to(torch.float32), t)
        np.testing.assert_array_equal(wl.bf16_bits_to_f32(wl.bf16_bits(X)), X)
    # the rounding helper is round-to-nearest-even, like the library's
    x = np.random.default_rng(0).standard_normal(10000).astype(np.float32)
    np.testing.assert_array_equal(wl.round_to_bf16(x), torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy())


def test_component_maps():
    for name in ("tiny", "small", "hunyuan_like"):
        w = wl.WORKLOADS[name]
        comp = wl.component_map(w, 0)
        assert comp.shape == (w.N,) and comp.min() >= 0 and comp.max() < w.n_components
    w = wl.WORKLOADS["hunyuan_like"]
    sizes = np.sort(np.bincount(wl.component_map(w, 1), minlength=w.n_components))[::-1]
    assert sizes[0] > 50 * sizes[-1]            # rank^-1.1 skew
    assert sizes.sum() == w.N


def test_noise_tokens_and_initial_centroids():
    w = wl.replace(wl.WORKLOADS["wan_like"], grid=(2, 20, 20))
    Q, K, V = wl.make_head(w, 0)
    frac = np.mean(np.abs(Q).max(axis=1) <= np.sqrt(3.0) + 1e-2)
    assert 0.05 < frac < 0.2
    init = wl.init_centroids(w, 0, Q, 10, 0)
    assert init.shape == (10, w.d)
    assert len({tuple(r) for r in init}) == 10
    assert all(any(np.array_equal(r, q) for q in Q) for r in init[:2])
    D = wl.drift(w, 0, 1, Q, 0)
    assert 0.03 < np.std(D - Q) < 0.08
