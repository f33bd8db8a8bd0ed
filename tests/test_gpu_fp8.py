"""GPU parity of the FP8 (E4M3) attention path (Table 1, "+ FP8" rows) against the CPU oracle.

The quantiser is compared bit for bit (codes and scales).  The attention kernel is compared with
the oracle's block-sparse attention evaluated on the SAME quantised operands (decoded codes, scales
folded in), so what is left is the kernel's own arithmetic: fp32 scores and softmax, probabilities
rounded to E4M3 (3 mantissa bits: relative rounding error within 2^-4), fp32 accumulation, bf16
output.  Tolerances (derived from that, see _util.assert_fp8_attention_within_budget):
  * O:   EVERY checked element within the budget of a weighted mean whose weights carry a relative
         error of 2^-4 (an absolute one of 2^-16 of the row sum for the keys far below the row
         maximum), (2^-4 dev1 + 2^-16 tail1) / (1 - 2^-4 - 2^-16 keys) + 2^-8 |O_ref| + 1e-5, with
         dev1 = sum_j pi_j |v_jc - O_c| from the oracle; and within 10 standard deviations of what
         independent rounding errors give, rms of the normalised error at most 1.25;
  * lse: the row sum is the sum of the rounded probabilities, so |lse - ref| <= ln(1 + 2^-4) = 0.0606
         in the worst case, and far less on average (<= 0.01) unless a row's probabilities are all
         nearly equal (then they all round the same way).
"""
import numpy as np
import pytest
import torch

from paper_2505_18875_amd import workloads as wl
from _util import FP8_LSE_MAX as LSE_MAX, assert_fp8_attention_within_budget, head_inputs, to_dev, to_np

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def svg2():
    import paper_2505_18875_amd as pkg
    pkg.load_library()
    assert torch.cuda.is_available()
    return pkg


def _quantise_all(svg2, *tensors):
    out = [svg2.svg2_quantize_fp8(t) for t in tensors]
    torch.cuda.synchronize()
    return out


@pytest.mark.parametrize("name,heads", [("small", [0, 13]), ("tiny", [0])])
def test_quantize_fp8_matches_oracle_bit_for_bit(svg2, oracle, name, heads):
    w = wl.WORKLOADS[name]
    Q, K, V, _, _ = head_inputs(w, heads)
    for X in (Q, K, V):
        X8, scale = svg2.svg2_quantize_fp8(to_dev(X, w.dtype))
        torch.cuda.synchronize()
        for i in range(len(heads)):
            codes, _, sc = oracle.quantize_e4m3(X[i])
            assert float(scale[i]) == float(sc)
            np.testing.assert_array_equal(X8[i].cpu().numpy(), codes)


def test_quantize_fp8_ties_signs_zero_heads(svg2, oracle):
    # head 0: amax = 448, so the scaling is exact and every value is its own pre-rounding value: all E4M3 values,
    # all midpoints between neighbours (ties go to the even code), values next to the midpoints, both signs
    tab = np.unique(np.abs(oracle.round_e4m3(np.linspace(-448, 448, 20001))))
    mids = (tab[:-1] + tab[1:]) / 2
    vals = np.concatenate([tab, mids, np.nextafter(mids.astype(np.float32), np.float32(0)),
                           np.nextafter(mids.astype(np.float32), np.float32(1e9)), [448.0]])
    vals = np.concatenate([vals, -vals]).astype(np.float32)
    n = 64 * ((vals.size + 63) // 64)
    X = np.zeros((3, n // 64, 64), dtype=np.float32)
    X[0].reshape(-1)[: vals.size] = vals
    X[2] = np.random.default_rng(0).standard_normal((n // 64, 64)) * 1e-30      # tiny values: scale far from 1
    X8, scale = svg2.svg2_quantize_fp8(to_dev(X))                 # head 1 stays all zero: scale 1, codes 0
    torch.cuda.synchronize()
    for h in range(3):
        codes, _, sc = oracle.quantize_e4m3(X[h])
        assert float(scale[h]) == float(sc)
        np.testing.assert_array_equal(X8[h].cpu().numpy(), codes)
    assert float(scale[0]) == 1.0 and float(scale[1]) == 1.0 and not X8[1].any()


def _check_head(oracle, O, lse, Q, K, V, d, perm_q, perm_k, offsets_q, offsets_k, row_ptr, col_idx, rows=None,
                lse_mean=None, statistical=True, what=""):
    """One head of the kernel's output against the oracle on the decoded E4M3 operands, element by element."""
    (_, dq, sq), (_, dk, sk), (_, dv, sv) = (oracle.quantize_e4m3(x) for x in (Q, K, V))
    kw = dict(statistical=statistical)
    if lse_mean is not None:
        kw["lse_mean"] = lse_mean
    return assert_fp8_attention_within_budget(oracle, np.asarray(O, np.float64), np.asarray(lse, np.float64), dq, dk, dv,
                                              sq, sk, sv, d, perm_q, perm_k, offsets_q, offsets_k, row_ptr, col_idx,
                                              rows=rows, what=what, **kw)


def _check_aux_head(oracle, res_O, lse, Q, K, V, a, i, d, rows, what=""):
    return _check_head(oracle, to_np(res_O[i]), to_np(lse[i]), Q, K, V, d, to_np(a.perm_q[i]), to_np(a.perm_k[i]),
                       to_np(a.offsets_q[i]), to_np(a.offsets_k[i]), to_np(a.row_ptr[i]), to_np(a.col_idx[i]),
                       rows=rows, what=what)


@pytest.mark.parametrize("heads,top_p", [([2, 19], 0.9), ([7], 0.5)])
def test_sparse_attn_fp8_matches_oracle_on_the_quantised_operands(svg2, oracle, heads, top_p):
    w = wl.replace(wl.WORKLOADS["small"], top_p=top_p)
    Q, K, V, cq, ck = head_inputs(w, heads)
    Qd, Kd, Vd = (to_dev(x, w.dtype) for x in (Q, K, V))
    a = svg2.svg2_forward(Qd, Kd, Vd, to_dev(cq), to_dev(ck), w.top_p, w.iters, want_aux=True).aux
    (Q8, sq), (K8, sk), (V8, sv) = _quantise_all(svg2, Qd, Kd, Vd)
    res = svg2.svg2_sparse_attn_fp8(Q8, K8, V8, sq, sk, sv, a.offsets_q, a.offsets_k, a.row_ptr, a.col_idx,
                                    a.perm_q, a.perm_k, want_lse=True)
    torch.cuda.synchronize()
    for i, h in enumerate(heads):
        rows = np.sort(np.random.default_rng(h).choice(w.N, 512, replace=False)).astype(np.int32)
        _check_aux_head(oracle, res.O, res.lse, Q[i], K[i], V[i], a, i, w.d, rows, what="head %d" % h)
    # the operands as permuted copies (perm_k = None): same rows in the same order, same bits
    def gather(X8, perm):
        return torch.gather(X8, 1, perm.long()[:, :, None].expand(-1, -1, X8.shape[2])).contiguous()
    cp = svg2.svg2_sparse_attn_fp8(gather(Q8, a.perm_q), gather(K8, a.perm_k), gather(V8, a.perm_k), sq, sk, sv,
                                   a.offsets_q, a.offsets_k, a.row_ptr, a.col_idx, a.perm_q, None, want_lse=True)
    torch.cuda.synchronize()
    assert torch.equal(cp.O, res.O) and torch.equal(cp.lse, res.lse)


def test_sparse_attn_fp8_ragged_and_empty_clusters(svg2, oracle):
    r = np.random.default_rng(77)
    N, d, Cq, Ck = 1500, 128, 9, 40
    Q, K, V = (wl.round_to_bf16(r.standard_normal((N, d)).astype(np.float32)) for _ in range(3))
    V[:, 5] *= 30.0                                             # one wide channel sets the head's V scale
    V = wl.round_to_bf16(V)
    lq = r.integers(0, Cq, size=N).astype(np.int32)
    lq[lq == 4] = 5                                             # empty query cluster
    lq[:700] = 0                                                # one query cluster spanning several row tiles
    lk = r.integers(0, Ck, size=N).astype(np.int32)
    lk[lk == 7] = 8                                             # empty key cluster
    sel = [np.sort(r.choice(Ck, size=int(r.integers(1, Ck)), replace=False)) for _ in range(Cq)]
    sel[1] = np.array([7], dtype=np.int64)                      # only an empty key cluster: rows get O = 0
    sel[2] = np.zeros(0, dtype=np.int64)                        # nothing selected at all
    sel[3] = np.arange(Ck)                                      # everything
    sel[6] = np.array([int(np.argmin(np.bincount(lk, minlength=Ck) + 1000 * (np.bincount(lk, minlength=Ck) == 0)))])
    pq, pk = oracle.permute(lq, Cq), oracle.permute(lk, Ck)
    row_ptr = np.concatenate([[0], np.cumsum([len(s) for s in sel])]).astype(np.int32)
    col = np.zeros(Cq * Ck, dtype=np.int32)
    cat = np.concatenate(sel).astype(np.int32)
    col[: cat.size] = cat
    (Q8, sq), (K8, sk), (V8, sv) = _quantise_all(svg2, to_dev(Q[None], "bf16"), to_dev(K[None], "bf16"),
                                                 to_dev(V[None], "bf16"))
    res = svg2.svg2_sparse_attn_fp8(Q8, K8, V8, sq, sk, sv, to_dev(pq.offsets[None]), to_dev(pk.offsets[None]),
                                    to_dev(row_ptr[None]), to_dev(col[None]), to_dev(pq.perm[None]),
                                    to_dev(pk.perm[None]), want_lse=True)
    torch.cuda.synchronize()
    O, lse = to_np(res.O[0]).astype(np.float64), to_np(res.lse[0]).astype(np.float64)
    _check_head(oracle, O, lse, Q, K, V, d, pq.perm, pk.perm, pq.offsets, pk.offsets, row_ptr, col)
    for i in (1, 2):
        rows = np.nonzero(lq == i)[0]
        assert rows.size and np.all(O[rows] == 0.0) and np.all(np.isneginf(lse[rows]))


def test_sparse_attn_fp8_scores_that_climb_between_tiles(svg2, oracle):
    """Keys ordered so that every query's scores grow along the key sequence by more per 32-key block than the
    head-room the kernel leaves above its reference level: the level moves in nearly every block (within a tile
    too, which makes the kernel redo the tile's first block), the accumulators are rescaled by factors down to
    zero, and one key ends up with all the weight."""
    r = np.random.default_rng(29)
    N, d = 1600, 128
    u = r.standard_normal(d).astype(np.float32)
    u /= np.linalg.norm(u)
    Q = wl.round_to_bf16((4.0 * u[None] + 0.3 * r.standard_normal((N, d))).astype(np.float32) * 10.0)
    ramp = np.linspace(-12.0, 12.0, N).astype(np.float32)
    K = wl.round_to_bf16((ramp[:, None] * u[None] + 0.3 * r.standard_normal((N, d))).astype(np.float32) * 10.0)
    V = wl.round_to_bf16(r.standard_normal((N, d)).astype(np.float32))
    lq = (np.arange(N) % 4).astype(np.int32)
    lk = (np.arange(N) // 200).astype(np.int32)
    sel = [np.arange(8), np.array([0, 1, 2]), np.array([7]), np.array([3, 5])]
    pq, pk = oracle.permute(lq, 4), oracle.permute(lk, 8)
    row_ptr = np.concatenate([[0], np.cumsum([len(x) for x in sel])]).astype(np.int32)
    col = np.zeros(4 * 8, dtype=np.int32)
    cat = np.concatenate(sel).astype(np.int32)
    col[: cat.size] = cat
    (Q8, sq), (K8, sk), (V8, sv) = _quantise_all(svg2, to_dev(Q[None], "bf16"), to_dev(K[None], "bf16"),
                                                 to_dev(V[None], "bf16"))
    res = svg2.svg2_sparse_attn_fp8(Q8, K8, V8, sq, sk, sv, to_dev(pq.offsets[None]), to_dev(pk.offsets[None]),
                                    to_dev(row_ptr[None]), to_dev(col[None]), to_dev(pq.perm[None]),
                                    to_dev(pk.perm[None]), want_lse=True)
    torch.cuda.synchronize()
    O, lse = to_np(res.O[0]).astype(np.float64), to_np(res.lse[0]).astype(np.float64)
    # rows with a handful of keys that matter: the errors of a row are not independent, so no sigma-based check;
    # lse is compared at the size of the scores (hundreds), where 1e-3 relative is what fp32 scores allow
    _check_head(oracle, O, lse, Q, K, V, d, pq.perm, pk.perm, pq.offsets, pk.offsets, row_ptr, col, statistical=False,
                lse_mean=0.07)


def test_sparse_attn_fp8_thousands_of_short_key_clusters(svg2, oracle):
    """Key clusters of one or two rows: a 64-key tile crosses dozens of runs of the virtual key sequence, and the row
    look-up of a tile starts from the run the plan recorded for it."""
    r = np.random.default_rng(78)
    N, d, Cq, Ck = 4200, 128, 3, 2700
    Q, K, V = (wl.round_to_bf16(r.standard_normal((N, d)).astype(np.float32)) for _ in range(3))
    lq = r.integers(0, Cq, size=N).astype(np.int32)
    lk = r.integers(0, Ck, size=N).astype(np.int32)
    sel = [np.sort(r.choice(Ck, size=2600, replace=False)), np.sort(r.choice(Ck, size=1500, replace=False)),
           np.array([5, 900, 2699], dtype=np.int64)]
    pq, pk = oracle.permute(lq, Cq), oracle.permute(lk, Ck)
    row_ptr = np.concatenate([[0], np.cumsum([len(s) for s in sel])]).astype(np.int32)
    col = np.zeros(Cq * Ck, dtype=np.int32)
    cat = np.concatenate(sel).astype(np.int32)
    col[: cat.size] = cat
    (Q8, sq), (K8, sk), (V8, sv) = _quantise_all(svg2, to_dev(Q[None], "bf16"), to_dev(K[None], "bf16"),
                                                 to_dev(V[None], "bf16"))
    res = svg2.svg2_sparse_attn_fp8(Q8, K8, V8, sq, sk, sv, to_dev(pq.offsets[None]), to_dev(pk.offsets[None]),
                                    to_dev(row_ptr[None]), to_dev(col[None]), to_dev(pq.perm[None]),
                                    to_dev(pk.perm[None]), want_lse=True)
    torch.cuda.synchronize()
    O, lse = to_np(res.O[0]).astype(np.float64), to_np(res.lse[0]).astype(np.float64)
    # (a query cluster whose 3 key clusters are all empty has no keys: the check wants O = 0, lse = -inf there)
    _check_head(oracle, O, lse, Q, K, V, d, pq.perm, pk.perm, pq.offsets, pk.offsets, row_ptr, col)


def test_sparse_attn_fp8_dense_special_case_flat_and_peaked_rows(svg2, oracle):
    # one cluster on each side = dense attention.  Half of the queries are tiny (flat softmax over 3000 keys:
    # every probability is about 2^-11.5 of the sum and must not be flushed to zero), half are large (peaked).
    r = np.random.default_rng(6)
    N, d = 3000, 128
    Q, K, V = (r.standard_normal((N, d)).astype(np.float32) for _ in range(3))
    Q[: N // 2] *= 0.01
    Q[N // 2:] *= 3.0
    Q, K, V = wl.round_to_bf16(Q), wl.round_to_bf16(K), wl.round_to_bf16(V)
    (Q8, sq), (K8, sk), (V8, sv) = _quantise_all(svg2, to_dev(Q[None], "bf16"), to_dev(K[None], "bf16"),
                                                 to_dev(V[None], "bf16"))
    one = to_dev(np.array([[0, N]], dtype=np.int32))
    res = svg2.svg2_sparse_attn_fp8(Q8, K8, V8, sq, sk, sv, one, one, to_dev(np.array([[0, 1]], dtype=np.int32)),
                                    to_dev(np.zeros((1, 1), dtype=np.int32)), None, None, want_lse=True)
    torch.cuda.synchronize()
    O, lse = to_np(res.O[0]).astype(np.float64), to_np(res.lse[0]).astype(np.float64)
    ident = np.arange(N, dtype=np.int32)
    off = np.array([0, N], dtype=np.int32)
    rp1, ci1 = np.array([0, 1], dtype=np.int32), np.zeros(1, dtype=np.int32)
    # flat rows: all probabilities of a row are nearly the same number and round the same way, so the error of
    # the row sum does not average out -- only the worst-case bound holds for lse (the output is a ratio of two
    # sums with that common factor and keeps its accuracy)
    _check_head(oracle, O, lse, Q, K, V, d, ident, ident, off, off, rp1, ci1, rows=np.arange(N // 2, dtype=np.int32),
                lse_mean=LSE_MAX, statistical=False, what="flat rows")
    _check_head(oracle, O, lse, Q, K, V, d, ident, ident, off, off, rp1, ci1,
                rows=np.arange(N // 2, N, dtype=np.int32), what="peaked rows")


def test_forward_fp8_same_selection_as_forward_and_close_output(svg2, oracle):
    w = wl.WORKLOADS["small"]
    heads = [3, 11]
    Q, K, V, cq, ck = head_inputs(w, heads)
    Qd, Kd, Vd = (to_dev(x, w.dtype) for x in (Q, K, V))
    cq1, ck1, cq2, ck2 = to_dev(cq), to_dev(ck), to_dev(cq), to_dev(ck)
    ref = svg2.svg2_forward(Qd, Kd, Vd, cq1, ck1, w.top_p, w.iters, want_aux=True)
    res = svg2.svg2_forward_fp8(Qd, Kd, Vd, cq2, ck2, w.top_p, w.iters, want_aux=True)
    torch.cuda.synchronize()
    # everything before the attention step reads the bf16 tensors: identical
    for n in ("labels_q", "labels_k", "counts_q", "counts_k", "offsets_q", "offsets_k", "perm_q", "perm_k", "row_ptr",
              "density"):
        assert torch.equal(getattr(res.aux, n), getattr(ref.aux, n)), n
    assert torch.equal(cq1, cq2) and torch.equal(ck1, ck2)
    # the attention step equals the stand-alone entry points on the same operands
    (Q8, sq), (K8, sk), (V8, sv) = _quantise_all(svg2, Qd, Kd, Vd)
    a = res.aux
    alone = svg2.svg2_sparse_attn_fp8(Q8, K8, V8, sq, sk, sv, a.offsets_q, a.offsets_k, a.row_ptr, a.col_idx,
                                      a.perm_q, a.perm_k, want_lse=True)
    torch.cuda.synchronize()
    assert torch.equal(alone.O, res.O) and torch.equal(alone.lse, a.lse)
    # against the oracle on the quantised operands
    for i, h in enumerate(heads):
        rows = np.sort(np.random.default_rng(h).choice(w.N, 256, replace=False)).astype(np.int32)
        _check_aux_head(oracle, res.O, a.lse, Q[i], K[i], V[i], a, i, w.d, rows, what="head %d" % h)


def test_fp8_entry_points_reject_what_they_do_not_support(svg2):
    from paper_2505_18875_amd.binding import Svg2Error
    x64 = torch.zeros((1, 256, 64), dtype=torch.bfloat16, device="cuda")
    c64 = torch.zeros((1, 4, 64), dtype=torch.float32, device="cuda")
    with pytest.raises(Svg2Error, match="head dimension 128"):
        svg2.svg2_forward_fp8(x64, x64, x64, c64, c64.clone(), 0.9, 1)
    x32 = torch.zeros((1, 256, 128), dtype=torch.float32, device="cuda")
    c128 = torch.zeros((1, 4, 128), dtype=torch.float32, device="cuda")
    with pytest.raises(Svg2Error, match="SVG2_BF16"):
        svg2.svg2_forward_fp8(x32, x32, x32, c128, c128.clone(), 0.9, 1)


def test_sparse_attn_fp8_is_reproducible_run_to_run(svg2):
    # the kernel has no atomics and a fixed summation order: repeated launches must give the same bits
    # (a missing wait between a matrix instruction and a vector instruction shows up here as rare differences)
    w = wl.WORKLOADS["small"]
    heads = [0, 5]
    Q, K, V, cq, ck = head_inputs(w, heads)
    Qd, Kd, Vd = (to_dev(x, w.dtype) for x in (Q, K, V))
    a = svg2.svg2_forward(Qd, Kd, Vd, to_dev(cq), to_dev(ck), w.top_p, w.iters, want_aux=True).aux
    (Q8, sq), (K8, sk), (V8, sv) = _quantise_all(svg2, Qd, Kd, Vd)
    outs = []
    for _ in range(4):
        r = svg2.svg2_sparse_attn_fp8(Q8, K8, V8, sq, sk, sv, a.offsets_q, a.offsets_k, a.row_ptr, a.col_idx,
                                      a.perm_q, a.perm_k, want_lse=True)
        torch.cuda.synchronize()
        outs.append((r.O.clone(), r.lse.clone()))
    for O, lse in outs[1:]:
        assert torch.equal(O, outs[0][0]) and torch.equal(lse, outs[0][1])


def test_forward_fp8_wan_like_full_size(svg2, oracle):
    # the benchmark's shape and launch configuration (H = 40, N = 75,600): the whole layer once, then two heads against
    # the oracle on their quantised operands, on a seeded sample of query rows
    from _util import upload_heads
    w = wl.WORKLOADS["wan_like"]
    heads = list(range(w.H))
    Q, K, V, cq, ck = upload_heads(w, heads)
    cq2, ck2 = cq.clone(), ck.clone()
    ref = svg2.svg2_forward(Q, K, V, cq, ck, w.top_p, w.iters, want_aux=True)
    res = svg2.svg2_forward_fp8(Q, K, V, cq2, ck2, w.top_p, w.iters, want_aux=True)
    torch.cuda.synchronize()
    a = res.aux
    for n in ("labels_q", "labels_k", "perm_q", "perm_k", "row_ptr", "density"):
        assert torch.equal(getattr(a, n), getattr(ref.aux, n)), n
    assert bool(torch.isfinite(res.O.float()).all())
    for h in (0, 19, 39):
        q, k, v = to_np(Q[h]), to_np(K[h]), to_np(V[h])
        rows = np.sort(np.random.default_rng(h).choice(w.N, 192, replace=False)).astype(np.int32)
        m = _check_aux_head(oracle, res.O, a.lse, q, k, v, a, h, w.d, rows, what="wan-like head %d" % h)
        print("wan-like head %d, E4M3: worst |err| / bound %.3f  max z %.2f  rms z %.3f" % (
            h, m["worst"], m["z_max"], m["z_rms"]), flush=True)
    # against the bf16 layer on the same selection: the operands' rounding, a loose sanity bound
    d = (res.O.float() - ref.O.float())
    rel = (d.pow(2).sum((1, 2)) / ref.O.float().pow(2).sum((1, 2))).sqrt()
    assert float(rel.max()) < 0.3


@pytest.mark.parametrize("N", [1, 31, 40, 65, 129])
def test_sparse_attn_fp8_very_short_sequences(svg2, oracle, N):
    # fewer keys than one 64-key tile, one tile and a bit, a query tile and a bit: everything ragged
    r = np.random.default_rng(50 + N)
    d = 128
    Q, K, V = (wl.round_to_bf16(r.standard_normal((N, d)).astype(np.float32)) for _ in range(3))
    (Q8, sq), (K8, sk), (V8, sv) = _quantise_all(svg2, to_dev(Q[None], "bf16"), to_dev(K[None], "bf16"),
                                                 to_dev(V[None], "bf16"))
    one = to_dev(np.array([[0, N]], dtype=np.int32))
    res = svg2.svg2_sparse_attn_fp8(Q8, K8, V8, sq, sk, sv, one, one, to_dev(np.array([[0, 1]], dtype=np.int32)),
                                    to_dev(np.zeros((1, 1), dtype=np.int32)), None, None, want_lse=True)
    torch.cuda.synchronize()
    O, lse = to_np(res.O[0]).astype(np.float64), to_np(res.lse[0]).astype(np.float64)
    ident = np.arange(N, dtype=np.int32)
    off = np.array([0, N], dtype=np.int32)
    # with a handful of keys the rounding errors of a row do not average out: only the worst-case figures apply
    _check_head(oracle, O, lse, Q, K, V, d, ident, ident, off, off, np.array([0, 1], dtype=np.int32),
                np.zeros(1, dtype=np.int32), lse_mean=LSE_MAX, statistical=False)
