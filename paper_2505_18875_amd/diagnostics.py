#!/usr/bin/env python3
"""Diagnostics of the SVG2 layer path on one MI355X, as markdown tables (synthetic analogues of the paper's
figures; every number comes from the library's kernels through the C ABI):

  recall     attention recall and density against top-p                (Section 3.1, Fig. 3 / Section 5.5)
  clusters   attention-kernel efficiency against C_q and C_k           (Appendix D.1, Figs. 8-9)
  seeding    k-means from k-means++ seeding until the labels settle, against the warm start from the
             previous step's centroids                                 (Section 4.3 / 5.3, Fig. 5a)
  fp8        output error and speed of the E4M3 attention path against the bf16 path, both measured against
             the fp32 kernel on the same selection                     (Table 1, "+ FP8" rows)
  sequence   a denoising sequence: 10 steps, Q and K drifting by 0.05 N(0,1) per step, k-means warm-started
             from the previous step's centroids with 2 iterations, C_k in {500, 1000}, top-p from 0.5 to
             0.99: per-step layer time, density and attention recall      (Section 4.3, centroid cache)

Usage: python -m paper_2505_18875_amd.diagnostics {recall,clusters,seeding,fp8,sequence} [--workload wan_like] [--heads 8]
"""
from __future__ import annotations

import argparse
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

from paper_2505_18875_amd import workloads as wl  # noqa: E402


def _inputs(w, heads):
    import torch
    Q, K, V = wl.make_heads(w, heads)

    def up(a):
        t = torch.from_numpy(np.ascontiguousarray(a)).cuda()
        return t.to(torch.bfloat16).contiguous() if w.dtype == "bf16" else t
    return Q, K, V, up(Q), up(K), up(V)


def _init(w, heads, X, C, side):
    import torch
    return torch.from_numpy(np.stack([wl.init_centroids(w, h, X[i], C, side) for i, h in enumerate(heads)])).cuda()


def _timed(fn, runs=3):
    import torch
    fn()
    torch.cuda.synchronize()
    best = 1e30
    for _ in range(runs):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        out = fn()
        e1.record()
        torch.cuda.synchronize()
        best = min(best, e0.elapsed_time(e1))
    return best, out


def _dense_lse(svg2, Qd, Kd, Vd):
    import torch
    H, N, _ = Qd.shape
    one = torch.tensor([[0, N]] * H, dtype=torch.int32, device="cuda")
    rp = torch.tensor([[0, 1]] * H, dtype=torch.int32, device="cuda")
    ci = torch.zeros((H, 1), dtype=torch.int32, device="cuda")
    return svg2.svg2_sparse_attn(Qd, Kd, Vd, one, one, rp, ci, None, want_lse=True).lse


def _cluster(svg2, w, heads, Q, K, Qd, Kd, Vd, Cq, Ck, iters):
    kq = svg2.svg2_kmeans(Qd, _init(w, heads, Q, Cq, 0), iters)
    kk = svg2.svg2_kmeans(Kd, _init(w, heads, K, Ck, 1), iters)
    pq = svg2.svg2_permute(kq.labels, Cq, [Qd])
    pk = svg2.svg2_permute(kk.labels, Ck, [Kd, Vd])
    return kq, kk, pq, pk


def recall(args):
    import torch
    import paper_2505_18875_amd as svg2
    w = wl.WORKLOADS[args.workload]
    heads = list(range(args.heads))
    Q, K, V, Qd, Kd, Vd = _inputs(w, heads)
    kq, kk, pq, pk = _cluster(svg2, w, heads, Q, K, Qd, Kd, Vd, w.Cq, w.Ck, w.iters)
    lse_all = _dense_lse(svg2, Qd, Kd, Vd)
    flops = 4.0 * len(heads) * float(w.N) ** 2 * w.d
    print("Attention recall against top-p: %s, heads 0..%d, C_q=%d, C_k=%d, %d k-means iterations" %
          (w.name, args.heads - 1, w.Cq, w.Ck, w.iters))
    print("\n| top-p | density | mean recall | min head recall | attention ms | TFLOP/s on selected |\n|---|---|---|---|---|---|")
    for p in (0.5, 0.6, 0.7, 0.8, 0.9, 0.95, 0.99, 1.0):
        sel = svg2.svg2_select_topp(kq.centroids, kk.centroids, kq.counts, kk.counts, p)
        run = lambda: svg2.svg2_sparse_attn(pq.tensors[0], pk.tensors[0], pk.tensors[1], pq.offsets, pk.offsets,  # noqa: E731
                                            sel.row_ptr, sel.col_idx, pq.perm, want_lse=True)
        ms, out = _timed(run)
        rec = svg2.svg2_attention_recall(out.lse, lse_all, want_rows=False)
        torch.cuda.synchronize()
        dens = sel.density.double().mean().item()
        print("| %.2f | %.4f | %.4f | %.4f | %.2f | %.0f |" % (p, dens, rec.mean.double().mean().item(),
                                                               rec.mean.min().item(), ms, flops * dens / ms / 1e9))


def clusters(args):
    import torch
    import paper_2505_18875_amd as svg2
    w = wl.WORKLOADS[args.workload]
    heads = list(range(args.heads))
    Q, K, V, Qd, Kd, Vd = _inputs(w, heads)
    flops = 4.0 * len(heads) * float(w.N) ** 2 * w.d
    print("Attention kernel against the numbers of clusters: %s, heads 0..%d, top-p %.2f, %d k-means iterations" %
          (w.name, args.heads - 1, w.top_p, w.iters))
    print("\n| C_q | C_k | mean |Q_i| | mean |K_j| | density | attention ms | TFLOP/s on selected | k-means Q ms | k-means K ms | select ms |\n"
          "|---|---|---|---|---|---|---|---|---|---|")
    grid = [(100, 500), (50, 500), (200, 500), (400, 500), (100, 250), (100, 1000), (100, 2000), (100, 4000)]
    for Cq, Ck in grid:
        cq0, ck0 = _init(w, heads, Q, Cq, 0), _init(w, heads, K, Ck, 1)
        tq, kq = _timed(lambda: svg2.svg2_kmeans(Qd, cq0, w.iters), 1)
        tk, kk = _timed(lambda: svg2.svg2_kmeans(Kd, ck0, w.iters), 1)
        pq = svg2.svg2_permute(kq.labels, Cq, [Qd])
        pk = svg2.svg2_permute(kk.labels, Ck, [Kd, Vd])
        ts, sel = _timed(lambda: svg2.svg2_select_topp(kq.centroids, kk.centroids, kq.counts, kk.counts, w.top_p), 1)
        run = lambda: svg2.svg2_sparse_attn(pq.tensors[0], pk.tensors[0], pk.tensors[1], pq.offsets, pk.offsets,  # noqa: E731
                                            sel.row_ptr, sel.col_idx, pq.perm)
        ms, _ = _timed(run)
        torch.cuda.synchronize()
        dens = sel.density.double().mean().item()
        print("| %d | %d | %.0f | %.0f | %.4f | %.2f | %.0f | %.2f | %.2f | %.3f |" %
              (Cq, Ck, w.N / Cq, w.N / Ck, dens, ms, flops * dens / ms / 1e9, tq, tk, ts))
        del kq, kk, pq, pk, sel


def seeding(args):
    import torch
    import paper_2505_18875_amd as svg2
    w = wl.WORKLOADS[args.workload]
    heads = list(range(args.heads))
    Q, K, V, Qd, Kd, Vd = _inputs(w, heads)
    H = len(heads)
    print("k-means of the K tokens (C_k=%d): k-means++ seeding and Lloyd iterations until fewer than 0.1 %% of the "
          "labels change, against the warm start from the previous step's centroids: %s, heads 0..%d" %
          (w.Ck, w.name, args.heads - 1))
    u = torch.from_numpy(np.random.default_rng(w.seed).random((H, w.Ck))).cuda()
    t_seed, seed = _timed(lambda: svg2.svg2_kmeans_pp_init(Kd, w.Ck, u), 1)
    cent = seed.centroids.clone()
    labels = None
    t_iter, n_iter = 0.0, 0
    while n_iter < 300:
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        res = svg2.svg2_kmeans(Kd, cent, 1, centroids=cent)
        e1.record()
        torch.cuda.synchronize()
        t_iter += e0.elapsed_time(e1)
        n_iter += 1
        if labels is not None and (res.labels != labels).float().mean().item() < 1e-3:
            break
        labels = res.labels
    # next denoising step: K drifts, two warm-started iterations (Section 4.3)
    K2 = np.stack([wl.drift(w, h, 1, K[i], 1) for i, h in enumerate(heads)])
    K2d = torch.from_numpy(K2).cuda().to(Kd.dtype).contiguous()
    warm = cent.clone()
    t_warm, res_w = _timed(lambda: svg2.svg2_kmeans(K2d, warm.clone(), 2, want_objective=True), 3)
    # what the two warm iterations reach, against iterating the drifted tokens to the same stopping rule
    ref = svg2.svg2_kmeans(K2d, cent.clone(), 20, want_objective=True)
    torch.cuda.synchronize()
    o_w = res_w.objective[:, -1].double().mean().item()
    o_r = ref.objective[:, -1].double().mean().item()
    print("\n| | ms | note |\n|---|---|---|")
    print("| k-means++ seeding | %.1f | %d draws, each a pass over K in fp64 |" % (t_seed, w.Ck))
    print("| Lloyd iterations after seeding | %.1f | %d iterations until < 0.1 %% of the labels change |" % (t_iter, n_iter))
    print("| cold start, total | %.1f | |" % (t_seed + t_iter))
    print("| warm start, 2 iterations on the drifted tokens | %.2f | objective %.6g, 20 iterations reach %.6g (%.3f %% lower) |"
          % (t_warm, o_w, o_r, 100.0 * (o_w - o_r) / o_w))
    print("| ratio cold / warm | %.0fx | the paper reports up to 76x for its centroid cache |" % ((t_seed + t_iter) / t_warm))


def fp8(args):
    import torch
    import paper_2505_18875_amd as svg2
    w = wl.WORKLOADS[args.workload]
    if w.dtype != "bf16" or w.d != 128:
        raise SystemExit("the FP8 path needs a bf16 workload with head dimension 128")
    heads = list(range(args.heads))
    Q, K, V, Qd, Kd, Vd = _inputs(w, heads)
    kq = svg2.svg2_kmeans(Qd, _init(w, heads, Q, w.Cq, 0), w.iters)
    kk = svg2.svg2_kmeans(Kd, _init(w, heads, K, w.Ck, 1), w.iters)
    pq = svg2.svg2_permute(kq.labels, w.Cq)
    pk = svg2.svg2_permute(kk.labels, w.Ck)
    Qf, Kf, Vf = Qd.float(), Kd.float(), Vd.float()
    t_q, q8 = _timed(lambda: [svg2.svg2_quantize_fp8(t) for t in (Qd, Kd, Vd)])
    (Q8, sq), (K8, sk), (V8, sv) = q8
    flops = 4.0 * len(heads) * float(w.N) ** 2 * w.d
    print("E4M3 attention against bf16 attention, reference = the fp32 kernel on the same selection: %s, heads 0..%d"
          % (w.name, args.heads - 1))
    print("(quantising Q, K and V of these heads: %.3f ms)" % t_q)
    print("\n| top-p | density | bf16 rel. rms err | bf16 min cosine | fp8 rel. rms err | fp8 min cosine | bf16 ms | fp8 ms | "
          "fp8 TFLOP/s on selected | speed-up |\n|---|---|---|---|---|---|---|---|---|---|")

    def err(O, ref):
        O, ref = O.double(), ref.double()
        rel = ((O - ref).pow(2).sum((1, 2)) / ref.pow(2).sum((1, 2))).sqrt().mean().item()
        cos = torch.nn.functional.cosine_similarity(O, ref, dim=2).min().item()
        return rel, cos
    for p in (0.5, 0.9, 1.0):
        sel = svg2.svg2_select_topp(kq.centroids, kk.centroids, kq.counts, kk.counts, p)
        common = (pq.offsets, pk.offsets, sel.row_ptr, sel.col_idx, pq.perm, pk.perm)
        ref = svg2.svg2_sparse_attn_gather_free(Qf, Kf, Vf, *common).O
        t_b, ob = _timed(lambda: svg2.svg2_sparse_attn_gather_free(Qd, Kd, Vd, *common))
        t_8, o8 = _timed(lambda: svg2.svg2_sparse_attn_fp8(Q8, K8, V8, sq, sk, sv, *common))
        torch.cuda.synchronize()
        dens = sel.density.double().mean().item()
        eb, e8 = err(ob.O, ref), err(o8.O, ref)
        print("| %.2f | %.4f | %.4f | %.5f | %.4f | %.5f | %.2f | %.2f | %.0f | %.2fx |"
              % (p, dens, eb[0], eb[1], e8[0], e8[1], t_b, t_8, flops * dens / t_8 / 1e9, t_b / t_8))
        del ref, ob, o8


def sequence(args):
    import torch
    import paper_2505_18875_amd as svg2
    w = wl.WORKLOADS[args.workload]
    heads = list(range(args.heads))
    H, steps = len(heads), 10
    Q, K, V, Qd0, Kd0, Vd = _inputs(w, heads)
    flops = 4.0 * H * float(w.N) ** 2 * w.d
    print("Denoising sequence: %s, heads 0..%d, %d steps; step 0 runs %d k-means iterations from the seeded centroids, every "
          "later step drifts Q and K by 0.05 N(0,1) (drawn on the device, seeded) and runs 2 iterations from the previous "
          "step's centroids.  Times are means over steps 1..%d of svg2_forward on these %d heads; recall is measured at the "
          "last step (share of the true attention mass that the selected keys hold, mean over queries)."
          % (w.name, args.heads - 1, steps, w.iters, steps - 1, H))
    print("\n| C_k | top-p | density (steps 1..9) | step 0 ms | later steps ms | of which k-means | attention | TFLOP/s on selected | "
          "recall at step 9 | labels changed by the 2nd warm iteration |\n|---|---|---|---|---|---|---|---|---|---|")
    for Ck in (500, 1000):
        cq0 = _init(w, heads, Q, w.Cq, 0)
        ck0 = _init(w, heads, K, Ck, 1)
        ws = torch.empty(svg2.svg2_forward_workspace_size(svg2.SVG2_BF16, H, w.N, w.d, w.Cq, Ck, False, False),
                         dtype=torch.uint8, device="cuda")
        out = torch.empty_like(Qd0)
        for p in (0.5, 0.6, 0.7, 0.8, 0.9, 0.95, 0.99):
            g = torch.Generator(device="cuda")
            g.manual_seed(1000 + w.seed)
            Qd, Kd = Qd0.clone(), Kd0.clone()
            cq, ck = cq0.clone(), ck0.clone()
            t0 = t_rest = t_km = t_at = dens = 0.0
            for step in range(steps):
                if step:
                    Qd = (Qd.float() + 0.05 * torch.randn(Qd.shape, generator=g, device="cuda")).to(Qd.dtype)
                    Kd = (Kd.float() + 0.05 * torch.randn(Kd.shape, generator=g, device="cuda")).to(Kd.dtype)
                iters = w.iters if step == 0 else 2
                svg2.svg2_profile_enable(1)
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                res = svg2.svg2_forward(Qd, Kd, Vd, cq, ck, p, iters, want_aux=True, out=out, ws=ws)
                e1.record()
                torch.cuda.synchronize()
                st, _ = svg2.svg2_profile_read()
                svg2.svg2_profile_enable(0)
                ms = e0.elapsed_time(e1)
                if step == 0:
                    t0 = ms
                else:
                    t_rest += ms / (steps - 1)
                    t_km += (st["kmeans"]) / (steps - 1)
                    t_at += st["attn"] / (steps - 1)
                    dens += res.aux.density.double().mean().item() / (steps - 1)
            # last step: how far is the 2-iteration warm start from settled labels, and the recall of the selection
            one = svg2.svg2_kmeans(Kd, ck.clone(), 1)
            moved = (one.labels != res.aux.labels_k).float().mean().item()
            lse_all = _dense_lse(svg2, Qd, Kd, Vd)
            rec = svg2.svg2_attention_recall(res.aux.lse, lse_all, want_rows=False).mean.double().mean().item()
            torch.cuda.synchronize()
            print("| %d | %.2f | %.4f | %.2f | %.2f | %.2f | %.2f | %.0f | %.4f | %.2f %% |" %
                  (Ck, p, dens, t0, t_rest, t_km, t_at, flops * dens / t_at / 1e9, rec, 100.0 * moved))
            del lse_all, res, one


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("what", choices=("recall", "clusters", "seeding", "fp8", "sequence"))
    ap.add_argument("--workload", default="wan_like", choices=sorted(wl.WORKLOADS))
    ap.add_argument("--heads", type=int, default=8)
    args = ap.parse_args()
    import torch
    import paper_2505_18875_amd as svg2
    svg2.load_library()
    if not torch.cuda.is_available():
        raise RuntimeError("diagnostics need a GPU")
    {"recall": recall, "clusters": clusters, "seeding": seeding, "fp8": fp8, "sequence": sequence}[args.what](args)


if __name__ == "__main__":
    main()
