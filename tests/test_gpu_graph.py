"""The whole layer recorded into a HIP graph: the library enqueues kernels only (no allocation, no
memset or copy node, no host synchronisation, no grid size read back from the device), so a caller may
capture svg2_forward once and replay it.  Every replay is compared bit for bit with an eager call on the
same inputs, with eager work and synchronisations of the program between the replays, and the inputs
are changed in place between replays (the graph holds addresses, not values)."""
import numpy as np
import pytest
import torch

from paper_2505_18875_amd import workloads as wl
from _util import upload_heads

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def svg2():
    import paper_2505_18875_amd as pkg
    pkg.load_library()
    assert torch.cuda.is_available()
    return pkg


@pytest.mark.parametrize("mode", ["permute", "gather_free", "fp8"])
def test_forward_replays_from_a_graph(svg2, mode):
    w = wl.replace(wl.WORKLOADS["small"], H=2, Cq=24, Ck=60, iters=4)
    kw = dict(gather_free=(mode == "gather_free"), fp8=(mode == "fp8"))
    Q, K, V, cq0, ck0 = upload_heads(w, [0, 1])
    Q2, K2, V2, cq2, ck2 = upload_heads(w, [5, 7])
    need = svg2.svg2_forward_workspace_size(svg2.SVG2_BF16, w.H, w.N, w.d, w.Cq, w.Ck, kw["gather_free"], kw["fp8"])
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")

    def eager(q, k, v, a, b):
        cq, ck = a.clone(), b.clone()
        o = svg2.svg2_forward(q, k, v, cq, ck, w.top_p, w.iters, ws=ws, **kw).O
        torch.cuda.synchronize()
        return o.clone(), cq, ck

    ref1 = eager(Q, K, V, cq0, ck0)
    ref2 = eager(Q2, K2, V2, cq2, ck2)
    assert not torch.equal(ref1[0], ref2[0])

    # static buffers of the graph
    q, k, v = Q.clone(), K.clone(), V.clone()
    cq, ck = cq0.clone(), ck0.clone()
    out = torch.empty_like(q)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):               # one call outside the capture (function attributes, lazy loading)
        svg2.svg2_forward(q, k, v, cq, ck, w.top_p, w.iters, out=out, ws=ws, **kw)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        svg2.svg2_forward(q, k, v, cq, ck, w.top_p, w.iters, out=out, ws=ws, **kw)

    for rep in range(4):
        src, ref = ((Q, K, V, cq0, ck0), ref1) if rep % 2 == 0 else ((Q2, K2, V2, cq2, ck2), ref2)
        q.copy_(src[0]); k.copy_(src[1]); v.copy_(src[2]); cq.copy_(src[3]); ck.copy_(src[4])
        out.zero_()
        ws.random_(0, 256)                      # stale workspace contents must not matter
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, ref[0]), "replay %d differs from the eager result" % rep
        assert torch.equal(cq, ref[1]) and torch.equal(ck, ref[2])
        # eager work of the program between replays
        again = eager(*src)
        assert torch.equal(again[0], ref[0])
