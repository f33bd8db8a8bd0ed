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


def bisector_case(d, C, N=24000, n_tie=2000):
    """Centroids and tokens for the near-tie test below: (X [N,d], cent [C,d], number of exact ties built)."""
    r = np.random.default_rng(4100 + d + C)
    cent = wl.round_to_bf16((3.0 * r.standard_normal((C, d))).astype(np.float32))
    # a quarter of the centroids get a twin that differs in ONE coordinate by two units in the last place, so that
    # the mid-point of the pair is a bf16 number: tokens there are exactly tied (the lower index has to win)
    order = r.permutation(C)
    twins = []
    for i in range(C // 4):
        j, t = sorted((int(order[2 * i]), int(order[2 * i + 1])))
        k = int(r.integers(0, d))
        bits = int(wl.bf16_bits(cent[j:j + 1, k])[0])
        tw = wl.bf16_bits_to_f32(np.array([bits + 2], dtype=np.uint16))[0]
        m = np.float32(0.5 * (float(cent[j, k]) + float(tw)))
        if np.isfinite(tw) and wl.round_to_bf16(np.array([m]))[0] == m and m != cent[j, k] and m != tw:
            cent[t] = cent[j]
            cent[t, k] = tw
            twins.append((j, t, k, m))
    a = r.integers(0, C, size=N)
    b = (a + 1 + r.integers(0, C - 1, size=N)) % C
    mid = 0.5 * (cent[a].astype(np.float64) + cent[b].astype(np.float64))
    delta = (cent[a] - cent[b]).astype(np.float64)
    X = wl.round_to_bf16(mid.astype(np.float32))
    # The rounding of X alone puts a token hundreds of rounding errors away from the hyperplane.  Walk it back: move
    # single coordinates to their neighbouring bf16 values until (x - mid).delta, the difference of the two scores,
    # is as close as it gets to a target drawn log-uniformly between 1e-6 and 1e-1 on either side.
    target = np.exp(r.uniform(np.log(1e-6), np.log(1e-1), size=N)) * r.choice([-1.0, 1.0], size=N)
    rows = np.arange(N)
    for _ in range(48):
        g = ((X.astype(np.float64) - mid) * delta).sum(axis=1)
        bits = wl.bf16_bits(X).astype(np.int64)
        best_err, best_k, best_v = np.abs(g - target), np.full(N, -1), np.zeros(N, dtype=np.float32)
        for db in (1, -1):
            nb = wl.bf16_bits_to_f32(np.clip(bits + db, 0, 0xFFFF).astype(np.uint16))
            ok = np.isfinite(nb) & ((bits & 0x7FFF) + db >= 0)
            err = np.abs(g[:, None] + (nb.astype(np.float64) - X) * delta - target[:, None])
            err[~ok] = np.inf
            k = err.argmin(axis=1)
            better = err[rows, k] < best_err
            best_err = np.where(better, err[rows, k], best_err)
            best_k = np.where(better, k, best_k)
            best_v = np.where(better, nb[rows, k], best_v)
        move = best_k >= 0
        if not move.any():
            break
        X[rows[move], best_k[move]] = best_v[move]
    # exact ties: the pair's mid-point in the coordinate where the twins differ, the centroid's own value plus some
    # noise (the same for both, so the tie stays exact) in eight others
    for i in range(n_tie if twins else 0):
        j, t, k, m = twins[int(r.integers(0, len(twins)))]
        x = cent[j].copy()
        other = r.choice(np.delete(np.arange(d), k), size=8, replace=False)
        x[other] = wl.round_to_bf16((x[other] + 0.5 * r.standard_normal(8)).astype(np.float32))
        x[k] = m
        X[i] = x
    return X, cent, (n_tie if twins else 0)


def csr_rows(row_ptr, col_idx):
    return [col_idx[row_ptr[i]:row_ptr[i + 1]] for i in range(len(row_ptr) - 1)]


def assert_csr_matches(sel, row_ptr, col_idx, what=""):
    """CSR lists of one head against the oracle's selection `sel` (computed from the same centroids and sizes).
    A row whose stopping decision has margin > 1e-5 must match exactly.  A row inside the margin (the accumulated
    mass is within fp32 rounding of p, or last kept and first dropped P' are nearly equal) may differ from the
    oracle's by the clusters at the stopping point only: at most two clusters, each with a P' within 1e-4
    (relative) of the oracle's last kept one or of p's crossing.  Returns (rows inside the margin, rows among them
    whose lists differ).  How many rows are inside the margin depends on p (at p = 0.99 the clusters at the stopping
    point carry ~1e-5 of the mass each, so most rows are); how many DIFFER is what the callers bound."""
    assert row_ptr[0] == 0
    low = ndiff = 0
    for i, (g, e) in enumerate(zip(csr_rows(row_ptr, col_idx), csr_rows(sel.row_ptr, sel.col_idx))):
        if sel.margin[i] > 1e-5:
            np.testing.assert_array_equal(g, e, err_msg="%s row %d" % (what, i))
            continue
        low += 1
        assert np.all(np.diff(g) > 0), (what, i)
        diff = sorted(set(g.tolist()) ^ set(e.tolist()))
        assert len(diff) <= 2, (what, i, diff)
        ndiff += bool(diff)
        if diff:
            # the clusters in dispute sit at the stopping point: their P' is the smallest kept or the largest dropped
            pe = sel.p_est[i]
            kept = pe[e]
            edge = kept.min() if kept.size else 0.0
            for j in diff:
                assert pe[j] <= edge * (1 + 1e-4) + 1e-12, (what, i, j, pe[j], edge)
                dropped = np.delete(pe, e)
                top_dropped = dropped.max() if dropped.size else 0.0
                assert pe[j] >= min(edge, top_dropped) * (1 - 1e-4) - 1e-12, (what, i, j, pe[j], edge, top_dropped)
    return low, ndiff


def assert_centroids_close(got, ref, same_members, what=""):
    """Centroids within 1e-3 relative (max-norm per centroid) on the clusters whose membership agrees."""
    if same_members.size == 0:
        return
    num = np.abs(got[same_members] - ref[same_members]).max(axis=1)
    den = np.maximum(np.abs(ref[same_members]).max(axis=1), 1e-6)
    assert np.all(num / den < 1e-3), "%s: centroid error %.3g" % (what, (num / den).max())


def same_member_clusters(got_labels, ref_labels, C):
    """Clusters that hold exactly the same tokens under both labelings."""
    if np.array_equal(got_labels, ref_labels):
        return np.arange(C)
    bad = got_labels != ref_labels
    touched = np.union1d(got_labels[bad], ref_labels[bad])
    return np.setdiff1d(np.arange(C), touched)


def check_layer_head(svg2, oracle, w, q, k, v, init_q, init_k, iters, top_p, aux, i, O_i, cq_out_i, ck_out_i, Qd, Kd,
                     n_rows=None, seed=0, compounded_min=0.999, tol=(2e-2, 1e-3), labels_exact=False, kmeans_ref=None):
    """One head of a svg2_forward result against the oracle, stage by stage.  q, k, v [N,d] numpy; init_* the
    centroids the call started from; aux / O_i / c*_out_i the GPU's results (index i of the batch); Qd, Kd the
    [1,N,d] device tensors of this head (for the near-tie check).  Downstream stages are judged on the GPU's own
    upstream results.  Returns a dict of what was measured."""
    bf16 = w.dtype == "bf16"
    out = {}
    kq, kk = kmeans_ref if kmeans_ref is not None else (oracle.kmeans(q, init_q, iters, bf16),
                                                         oracle.kmeans(k, init_k, iters, bf16))
    out["kmeans_ref"] = (kq, kk)
    lq, lk = to_np(aux.labels_q[i]), to_np(aux.labels_k[i])
    for side, got, ref, X, Xd, init, C, cen in (("q", lq, kq, q, Qd, init_q, w.Cq, cq_out_i),
                                                ("k", lk, kk, k, Kd, init_k, w.Ck, ck_out_i)):
        agree = float(np.mean(got == ref.labels))
        out["agree_" + side] = agree
        if labels_exact:
            assert agree == 1.0, (side, agree, int((got != ref.labels).sum()))
        assert agree >= compounded_min, (side, agree)
        assert_label_disagreements_are_near_ties(svg2, oracle, X, Xd, init, iters, bf16, got, ref.labels)
        # the layer's centroids (the cache handed to the next step) against the oracle's, where membership agrees
        assert_centroids_close(to_np(cen), ref.centroids, same_member_clusters(got, ref.labels, C), "centroids " + side)
    pq, pk = oracle.permute(lq, w.Cq), oracle.permute(lk, w.Ck)
    for name, ref in (("perm_q", pq.perm), ("perm_k", pk.perm), ("offsets_q", pq.offsets), ("offsets_k", pk.offsets),
                      ("counts_q", pq.counts), ("counts_k", pk.counts)):
        np.testing.assert_array_equal(to_np(getattr(aux, name)[i]), ref, err_msg=name)
    sel = oracle.select_topp(to_np(cq_out_i), to_np(ck_out_i), pq.counts, pk.counts, top_p)
    rp, ci = to_np(aux.row_ptr[i]), to_np(aux.col_idx[i])
    out["low_margin"], out["csr_rows_differing"] = assert_csr_matches(sel, rp, ci)
    assert out["csr_rows_differing"] <= max(2, w.Cq // 20)
    rows = None if n_rows is None else np.sort(
        np.random.default_rng(seed).choice(w.N, n_rows, replace=False)).astype(np.int32)
    O_ref, lse_ref = oracle.sparse_attention(q[pq.perm], k[pk.perm], v[pk.perm], pq.offsets, pk.offsets, rp,
                                             ci[: rp[-1]], perm_q=pq.perm, rows=rows)
    chk = np.arange(w.N) if rows is None else pq.perm[rows]
    err = np.abs(to_np(O_i)[chk] - O_ref[chk])
    out["err_max"], out["err_mean"] = float(err.max()), float(err.mean())
    assert err.max() <= tol[0] and err.mean() <= tol[1], (err.max(), err.mean())
    if aux.lse is not None:
        lse = to_np(aux.lse[i])[chk]
        fin = np.isfinite(lse_ref[chk])
        np.testing.assert_allclose(lse[fin], lse_ref[chk][fin], rtol=1e-3, atol=2e-3)
        assert np.all(np.isneginf(lse[~fin]))
    keys = np.array([pk.counts[c].sum() for c in csr_rows(rp, ci)])
    np.testing.assert_allclose(float(aux.density[i]), (pq.counts * keys).sum() / float(w.N) ** 2, rtol=1e-5)
    out["density"] = float(aux.density[i])
    return out


# ---- per-element bound for the E4M3 attention kernel -------------------------------------------------------------
# The kernel rounds every probability to E4M3 before it multiplies V and normalises by the sum of the rounded
# values.  Normal E4M3 numbers carry a relative error of at most 2^-4 (3 mantissa bits).  A probability is
# scaled so that the row maximum sits between 2^6 and 2^8, so only probabilities below 2^-12 of the row maximum can
# land in the subnormal range (below 2^-6 after scaling), where the error is absolute: at most 2^-10 after scaling,
# i.e. 2^-16 of the row's largest probability, and never more than the probability itself (flush to zero).  With
# dev1 / tail1 / tailw from the oracle's budget of a weighted mean with rounded weights (tail_ratio 2^-12,
# tail_abs 2^-16):
#     |O - O_ref| <= (2^-4 dev1 + tail1) / (1 - 2^-4 - tailw)  +  2^-8 |O_ref|  +  1e-5
# (the last two terms: bf16 storage of the output and fp32 arithmetic).  The spread expected for independent
# rounding errors, sigma = sqrt((2^-4)^2 dev2 / 3 + tail2 / 3 + (2^-9 O_ref)^2 / 3 + 1e-12), gives a second, much
# sharper check where a row has enough keys for the errors to average: no element further than FP8_Z_MAX sigma,
# rms of err / sigma at most FP8_Z_RMS (measured on the Small workload, all heads and rows: 3.6 and 0.65).
FP8_EPS, FP8_TAIL_ABS, FP8_TAIL_RATIO = 2.0 ** -4, 2.0 ** -16, 2.0 ** -12
FP8_Z_MAX, FP8_Z_RMS = 6.0, 0.9
FP8_LSE_MAX, FP8_LSE_MEAN = 0.0606 + 2e-3, 0.01


def assert_fp8_attention_within_budget(oracle, O, lse, dq, dk, dv, sq, sk, sv, d, pq, pk, offsets_q, offsets_k, rp, ci,
                                       rows=None, lse_mean=FP8_LSE_MEAN, statistical=True, what=""):
    """O [N,d], lse [N] (numpy, from the kernel) against the oracle on the SAME quantised operands.  dq, dk, dv
    decoded E4M3 values [N,d] in token order, sq, sk, sv their scales; pq, pk permutations; rows: sorted rows
    to check (None: all).  Every checked element must satisfy the bound above; statistical=False leaves the
    sigma-based check out (rows with a handful of keys, or rows whose probabilities are all nearly equal and
    round the same way: the errors of such a row are not independent)."""
    scale = float(sq) * float(sk) / np.sqrt(d)
    args = (dq[pq], dk[pk], dv[pk], offsets_q, offsets_k, rp, ci[: rp[-1]])
    O_ref, lse_ref = oracle.sparse_attention(*args, perm_q=pq, scale=scale, rows=rows)
    dev1, dev2, tail1, tail2, tailw = oracle.rounded_weights_budget(
        *args, perm_q=pq, scale=scale, rows=rows, tail_ratio=FP8_TAIL_RATIO, tail_abs=FP8_TAIL_ABS)
    tok = np.arange(O.shape[0]) if rows is None else pq[rows]
    fin = np.isfinite(lse_ref[tok])
    assert np.all(O[tok][~fin] == 0.0) and np.all(np.isneginf(lse[tok][~fin]))
    tok = tok[fin]
    if tok.size == 0:
        return {}
    sv = float(sv)
    O_ref, dev1, tail1 = O_ref[tok] * sv, dev1[tok] * sv, tail1[tok] * sv
    dev2, tail2 = dev2[tok] * sv * sv, tail2[tok] * sv * sv
    denom = 1.0 - FP8_EPS - tailw[tok]
    assert np.all(denom > 0.5), denom.min()
    err = O[tok] - O_ref
    bound = (FP8_EPS * dev1 + tail1) / denom[:, None] + 2.0 ** -8 * np.abs(O_ref) + 1e-5
    worst = np.abs(err) / bound
    assert worst.max() <= 1.0, "%s: element %s exceeds its bound by %.3f" % (
        what, np.unravel_index(worst.argmax(), worst.shape), worst.max())
    sigma = np.sqrt(FP8_EPS ** 2 * dev2 / 3 + tail2 / 3 + (2.0 ** -9 * O_ref) ** 2 / 3 + 1e-12)
    z = np.abs(err) / sigma
    z_rms = float(np.sqrt((z ** 2).mean()))
    if statistical:
        assert z.max() <= FP8_Z_MAX and z_rms <= FP8_Z_RMS, "%s: max z %.2f, rms z %.3f" % (what, z.max(), z_rms)
    dl = np.abs(lse[tok] - lse_ref[tok])
    assert dl.max() <= FP8_LSE_MAX and dl.mean() <= lse_mean, (what, dl.max(), dl.mean())
    return dict(worst=float(worst.max()), z_max=float(z.max()), z_rms=z_rms,
                rel_rms=float(np.sqrt((err ** 2).mean() / max((O_ref ** 2).mean(), 1e-30))))
