"""GPU parity of the pieces around the layer path: attention recall (Section 3.1) and k-means++ seeding
(Sections 4.3 / 5.3), each against the CPU oracle on the same seeded inputs."""
import numpy as np
import pytest
import torch

from paper_2505_18875_amd import workloads as wl
from _util import head_inputs, to_dev, to_np

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def svg2():
    import paper_2505_18875_amd as pkg
    pkg.load_library()
    assert torch.cuda.is_available()
    return pkg


def _dense_lse(svg2, Q, K, V):
    H, N, _ = Q.shape
    one = torch.tensor([[0, N]] * H, dtype=torch.int32, device="cuda")
    rp = torch.tensor([[0, 1]] * H, dtype=torch.int32, device="cuda")
    ci = torch.zeros((H, 1), dtype=torch.int32, device="cuda")
    return svg2.svg2_sparse_attn(Q, K, V, one, one, rp, ci, None, want_lse=True).lse


@pytest.mark.parametrize("name,heads,top_p,sample", [("tiny", [0], 0.9, None), ("small", [2, 19], 0.9, 512),
                                                     ("small", [7], 0.5, 512)])
def test_attention_recall_matches_oracle(svg2, oracle, name, heads, top_p, sample):
    w = wl.replace(wl.WORKLOADS[name], top_p=top_p)
    Q, K, V, cq, ck = head_inputs(w, heads)
    Qd, Kd, Vd = (to_dev(x, w.dtype) for x in (Q, K, V))
    res = svg2.svg2_forward(Qd, Kd, Vd, to_dev(cq), to_dev(ck), w.top_p, w.iters, want_aux=True)
    lse_all = _dense_lse(svg2, Qd, Kd, Vd)
    rec = svg2.svg2_attention_recall(res.aux.lse, lse_all)
    torch.cuda.synchronize()
    a = res.aux
    for i, h in enumerate(heads):
        rows = None if sample is None else np.sort(
            np.random.default_rng(h).choice(w.N, sample, replace=False)).astype(np.int32)
        rp, ci = to_np(a.row_ptr[i]), to_np(a.col_idx[i])
        want = oracle.attention_recall(Q[i], K[i], to_np(a.labels_q[i]), to_np(a.labels_k[i]), w.Cq, w.Ck,
                                       rp, ci[: rp[-1]], rows=rows)
        chk = np.arange(w.N) if rows is None else rows
        got = to_np(rec.recall[i])
        # the two lse values are fp32 results of bf16 / fp32 attention passes: a few 1e-3 absolute on a ratio in [0,1]
        np.testing.assert_allclose(got[chk], want[chk], atol=4e-3, rtol=4e-3)
        np.testing.assert_allclose(float(rec.mean[i]), got.mean(), rtol=1e-5)
        assert got.min() >= 0.0 and got.max() <= 1.0 + 1e-3
    # everything selected: recall is exactly 1
    one = svg2.svg2_attention_recall(lse_all, lse_all)
    torch.cuda.synchronize()
    assert torch.all(one.recall == 1.0) and torch.all(one.mean == 1.0)


@pytest.mark.parametrize("name,heads,C", [("tiny", [0], 32), ("small", [0, 9, 23], 100), ("small", [4], 500)])
def test_kmeans_pp_matches_oracle(svg2, oracle, name, heads, C):
    w = wl.WORKLOADS[name]
    Q, K, V, _, _ = head_inputs(w, heads)
    u = np.random.default_rng(11).random((len(heads), C))
    res = svg2.svg2_kmeans_pp_init(to_dev(K, w.dtype), C, torch.from_numpy(u).cuda())
    torch.cuda.synchronize()
    for i in range(len(heads)):
        picked, centres = oracle.kmeans_pp(K[i], C, u[i])
        np.testing.assert_array_equal(to_np(res.picked[i]), picked)
        np.testing.assert_array_equal(to_np(res.centroids[i]), centres)


def test_kmeans_pp_degenerate_inputs(svg2, oracle):
    # all tokens identical: every D2 is zero and the draw falls back to token floor(u N); duplicates of one token
    X = np.ones((1, 300, 64), dtype=np.float32)
    u = np.array([[0.01, 0.5, 0.999, 0.25]])
    res = svg2.svg2_kmeans_pp_init(to_dev(X), 4, torch.from_numpy(u).cuda())
    torch.cuda.synchronize()
    np.testing.assert_array_equal(to_np(res.picked[0]), oracle.kmeans_pp(X[0], 4, u[0])[0])
    np.testing.assert_array_equal(to_np(res.picked[0]), [3, 150, 299, 75])
    # ragged N (not a multiple of the 1024-token block), two distinct values
    X = np.zeros((1, 1500, 128), dtype=np.float32)
    X[0, 1100:] = 2.0
    u = np.array([[0.0, 0.3, 0.9]])
    res = svg2.svg2_kmeans_pp_init(to_dev(X, "bf16"), 3, torch.from_numpy(u).cuda())
    torch.cuda.synchronize()
    np.testing.assert_array_equal(to_np(res.picked[0]), oracle.kmeans_pp(X[0], 3, u[0])[0])


def test_kmeans_pp_then_lloyd_lowers_the_objective(svg2):
    # seeding feeds svg2_kmeans: the objective after the first assign step is the k-means++ potential and it
    # does not grow over the iterations (Section 4.1 / 4.3)
    w = wl.WORKLOADS["small"]
    Q, K, V, _, _ = head_inputs(w, [1])
    Kd = to_dev(K, w.dtype)
    u = torch.from_numpy(np.random.default_rng(3).random((1, 50))).cuda()
    init = svg2.svg2_kmeans_pp_init(Kd, 50, u).centroids
    res = svg2.svg2_kmeans(Kd, init, 6, want_objective=True)
    torch.cuda.synchronize()
    obj = to_np(res.objective[0])
    assert np.all(np.diff(obj) <= 1e-4 * obj[0])
