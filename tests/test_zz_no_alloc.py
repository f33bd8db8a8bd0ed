"""svg2_permute_noalloc, the entry point for callers that cannot allocate (graph capture, serving loops): it runs
the counting sort of svg2_permute on a scratch array inside the library.  Called through the C ABI twice in a row,
the second time on a smaller input (the array still holds the first call's histograms), and compared bit for bit
with svg2_permute on a caller's workspace."""
import numpy as np
import pytest
import torch

from paper_2505_18875_amd import workloads as wl
from _util import to_dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def svg2():
    import paper_2505_18875_amd as pkg
    pkg.load_library()
    assert torch.cuda.is_available()
    return pkg


def _case(svg2, H, N, C, d, seed):
    r = np.random.default_rng(seed)
    labels = r.integers(0, C, size=(H, N)).astype(np.int32)
    if C > 4:
        labels[labels == 3] = 2                                 # an empty cluster
    X = wl.round_to_bf16(r.standard_normal((H, N, d)).astype(np.float32))
    Y = wl.round_to_bf16(r.standard_normal((H, N, d)).astype(np.float32))
    lab, Xd, Yd = to_dev(labels), to_dev(X, "bf16"), to_dev(Y, "bf16")
    ref = svg2.svg2_permute(lab, C, [Xd, Yd])
    i32 = dict(dtype=torch.int32, device="cuda")
    offsets, perm, inv = torch.full((H, C + 1), -1, **i32), torch.full((H, N), -1, **i32), torch.full((H, N), -1, **i32)
    Xo, Yo = torch.zeros_like(Xd), torch.zeros_like(Yd)
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    svg2.svg2_permute_noalloc(lab, C, offsets, perm, inv, [Xd, Yd], [Xo, Yo])
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before              # nothing came from torch's allocator either
    assert torch.equal(offsets, ref.offsets) and torch.equal(perm, ref.perm) and torch.equal(inv, ref.inv_perm)
    assert torch.equal(Xo, ref.tensors[0]) and torch.equal(Yo, ref.tensors[1])
    # index-only call, no inverse
    perm2 = torch.full((H, N), -1, **i32)
    svg2.svg2_permute_noalloc(lab, C, offsets, perm2)
    torch.cuda.synchronize()
    assert torch.equal(perm2, ref.perm)


def test_permute_noalloc_matches_permute_twice_in_a_row_second_call_smaller(svg2):
    _case(svg2, 3, 9000, 300, 128, 1)           # 3 x 9 chunks x 300 clusters of scratch
    _case(svg2, 2, 2500, 37, 64, 2)             # smaller: most of the array keeps the first call's contents
    _case(svg2, 1, 1, 1, 128, 3)


def test_permute_noalloc_rejects_what_exceeds_the_built_in_scratch(svg2):
    from paper_2505_18875_amd.binding import Svg2Error
    H, N, C = 40, 75600, 4096                   # 40 x 74 x 4096 x 4 bytes = 48 MB > 16 MiB
    lab = torch.zeros((H, N), dtype=torch.int32, device="cuda")
    offsets = torch.empty((H, C + 1), dtype=torch.int32, device="cuda")
    perm = torch.empty((H, N), dtype=torch.int32, device="cuda")
    with pytest.raises(Svg2Error, match="scratch") as e:
        svg2.svg2_permute_noalloc(lab, C, offsets, perm)
    assert e.value.code == 3
    # the Wan-like K side fits
    C = 500
    lab = torch.randint(0, C, (H, N), dtype=torch.int32, device="cuda")
    ref = svg2.svg2_permute(lab, C, [], want_inverse=False)
    offsets = torch.empty((H, C + 1), dtype=torch.int32, device="cuda")
    svg2.svg2_permute_noalloc(lab, C, offsets, perm)
    torch.cuda.synchronize()
    assert torch.equal(perm, ref.perm) and torch.equal(offsets, ref.offsets)
