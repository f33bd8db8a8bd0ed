"""The Small configuration in full: all 24 heads (H = 24, N = 16,384, d = 128, bf16, C_q = 100, C_k = 500, 10
k-means iterations, top-p 0.9) go through svg2_forward in one call, and EVERY head and EVERY query row is checked
against the CPU oracle, stage by stage -- labels, centroids, permutations, CSR lists, attention output, lse,
density.  The same for svg2_forward_fp8 (Table 1, "+ FP8"): identical selection, and every output element inside
the per-element budget of a weighted mean with E4M3-rounded probabilities."""
import numpy as np
import pytest
import torch

from paper_2505_18875_amd import workloads as wl
from _util import assert_fp8_attention_within_budget, check_layer_head, to_np, upload_heads

pytestmark = pytest.mark.gpu

GROUPS = [list(range(g, g + 4)) for g in range(0, 24, 4)]


@pytest.fixture(scope="module")
def svg2():
    import paper_2505_18875_amd as pkg
    pkg.load_library()
    assert torch.cuda.is_available()
    return pkg


@pytest.fixture(scope="module")
def layer(svg2):
    """Both layers (bf16 and E4M3 attention) of all 24 heads, computed once."""
    w = wl.WORKLOADS["small"]
    heads = list(range(w.H))
    Q, K, V, cq0, ck0 = upload_heads(w, heads)
    cq, ck = cq0.clone(), ck0.clone()
    res = svg2.svg2_forward(Q, K, V, cq, ck, w.top_p, w.iters, want_aux=True)
    cq8, ck8 = cq0.clone(), ck0.clone()
    res8 = svg2.svg2_forward_fp8(Q, K, V, cq8, ck8, w.top_p, w.iters, want_aux=True)
    torch.cuda.synchronize()
    return dict(w=w, Q=Q, K=K, V=V, cq0=cq0, ck0=ck0, cq=cq, ck=ck, res=res, cq8=cq8, ck8=ck8, res8=res8)


@pytest.mark.parametrize("group", GROUPS, ids=lambda g: "heads%d-%d" % (g[0], g[-1]))
def test_small_every_head_every_row_bf16(svg2, oracle, layer, group):
    L, w = layer, layer["w"]
    for h in group:
        q, k, v = to_np(L["Q"][h]), to_np(L["K"][h]), to_np(L["V"][h])
        m = check_layer_head(svg2, oracle, w, q, k, v, to_np(L["cq0"][h]), to_np(L["ck0"][h]), w.iters, w.top_p,
                             L["res"].aux, h, L["res"].O[h], L["cq"][h], L["ck"][h], L["Q"][h:h + 1], L["K"][h:h + 1],
                             n_rows=None, labels_exact=True)
        print("small head %2d: density %.3f  max|err| %.2e  mean|err| %.2e  rows inside the top-p margin %d"
              % (h, m["density"], m["err_max"], m["err_mean"], m["low_margin"]), flush=True)


@pytest.mark.parametrize("group", GROUPS, ids=lambda g: "heads%d-%d" % (g[0], g[-1]))
def test_small_every_head_every_row_fp8(svg2, oracle, layer, group):
    L, w = layer, layer["w"]
    a, a8 = L["res"].aux, L["res8"].aux
    # everything before the attention step reads the bf16 tensors: identical to the bf16 layer
    for n in ("labels_q", "labels_k", "counts_q", "counts_k", "offsets_q", "offsets_k", "perm_q", "perm_k", "row_ptr",
              "density"):
        assert torch.equal(getattr(a8, n), getattr(a, n)), n
    assert torch.equal(L["cq8"], L["cq"]) and torch.equal(L["ck8"], L["ck"])
    for h in group:
        q, k, v = to_np(L["Q"][h]), to_np(L["K"][h]), to_np(L["V"][h])
        (_, dq, sq), (_, dk, sk), (_, dv, sv) = (oracle.quantize_e4m3(x) for x in (q, k, v))
        rp, ci = to_np(a8.row_ptr[h]), to_np(a8.col_idx[h])
        m = assert_fp8_attention_within_budget(
            oracle, to_np(L["res8"].O[h]).astype(np.float64), to_np(a8.lse[h]).astype(np.float64), dq, dk, dv, sq, sk, sv,
            w.d, to_np(a8.perm_q[h]), to_np(a8.perm_k[h]), to_np(a8.offsets_q[h]), to_np(a8.offsets_k[h]), rp, ci,
            rows=None, what="small head %d" % h)
        print("small head %2d, E4M3: worst |err| / bound %.3f  max z %.2f  rms z %.3f  relative rms error %.4f"
              % (h, m["worst"], m["z_max"], m["z_rms"], m["rel_rms"]), flush=True)
