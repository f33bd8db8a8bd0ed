#!/usr/bin/env python3
"""Benchmark of the SVG2 sparse-attention layer path on one MI355X.

A step is one svg2_forward call (k-means of Q and K, both permutations, top-p
selection, block-sparse attention) over one synthetic Wan-like layer:
H = 40 heads, N = 75,600 tokens, d = 128, bf16, C_q = 100, C_k = 500,
10 k-means iterations from seeded initial centroids, top-p = 0.9.  Inputs are
resident in HBM before the timed region starts.

Prints ONE JSON line: whole-layer throughput as effective TFLOP/s
(4*H*N^2*d / layer time; ms per layer is `ms_per_step`), the roofline of the
dominant kernel (sparse attention, bf16 MFMA) measured with HIP events inside
the timed region, per-stage times, dense attention at the same shape, and the
CPU oracle timed on the host cores on a bounded sample (a baseline only).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time
from concurrent.futures import ProcessPoolExecutor

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

from paper_2505_18875_amd import workloads as wl  # noqa: E402

BF16_MFMA_PEAK_TFLOPS = 2500.0          # MI355X dense bf16 MFMA peak
FP8_MFMA_PEAK_TFLOPS = 5000.0           # MI355X dense fp8 MFMA peak
HBM_PEAK_GBPS = 8000.0                  # MI355X HBM3E peak
# Bytes per attention-kernel launch that leave the L2s towards the fabric (Infinity Cache / HBM) on the Wan-like
# layer at top-p 0.9, from two rocprofv3 --pmc runs (FETCH_SIZE x 2.0 + WRITE_SIZE x 1.0, factors from a 1 GiB copy
# in the same runs): profiles/wan_like_attention_hbm_traffic.md.  A constant from that profile, not measured by
# this script (counters need the profiler); other workloads report null.
ATTN_TRAFFIC_BYTES = {("wan_like", 0.9): (2.0 * 17221511.7 + 1030321.2) * 1024.0}
ATTN_TRAFFIC_SOURCE = ("fabric-side bytes (L2 misses, FETCH_SIZE / WRITE_SIZE), part of which the Infinity Cache serves; "
                       "constant from profiles/wan_like_attention_hbm_traffic.md, not measured in this run")


def _gen_head(args):
    name, h = args
    w = wl.WORKLOADS[name]
    Q, K, V = wl.make_head(w, h)
    cq = wl.init_centroids(w, h, Q, w.Cq, 0)
    ck = wl.init_centroids(w, h, K, w.Ck, 1)
    return h, wl.bf16_bits(Q), wl.bf16_bits(K), wl.bf16_bits(V), cq, ck


def start_generation(w):
    """Start worker processes that build the heads.  Called before anything touches the GPU."""
    workers = min(8, len(os.sched_getaffinity(0)))
    ex = ProcessPoolExecutor(max_workers=workers)
    futs = [ex.submit(_gen_head, (w.name, h)) for h in range(w.H)]
    return ex, futs


def upload_inputs(w, gen, log):
    """Collect the generated heads and upload them as bf16 device tensors."""
    import torch
    ex, futs = gen
    H, N, d = w.H, w.N, w.d
    Q = torch.empty((H, N, d), dtype=torch.bfloat16, device="cuda")
    K = torch.empty_like(Q)
    V = torch.empty_like(Q)
    cq = torch.empty((H, w.Cq, d), dtype=torch.float32, device="cuda")
    ck = torch.empty((H, w.Ck, d), dtype=torch.float32, device="cuda")
    t0 = time.time()
    for f in futs:
        h, qb, kb, vb, cqh, ckh = f.result()
        Q[h] = torch.from_numpy(qb.view(np.int16)).cuda().view(torch.bfloat16)
        K[h] = torch.from_numpy(kb.view(np.int16)).cuda().view(torch.bfloat16)
        V[h] = torch.from_numpy(vb.view(np.int16)).cuda().view(torch.bfloat16)
        cq[h] = torch.from_numpy(cqh).cuda()
        ck[h] = torch.from_numpy(ckh).cuda()
        if h % 10 == 9:
            log("generated %d/%d heads (%.0f s)" % (h + 1, H, time.time() - t0))
    ex.shutdown()
    torch.cuda.synchronize()
    return Q, K, V, cq, ck


def cpu_baseline(w, log, n_rows=None):
    """The CPU oracle, as it stands, on one head: k-means, permutation, selection in full and the
    attention step on a seeded sample of query rows (rows are independent, so the sample is exact)."""
    from oracle import svg2_oracle as orc
    h = 0
    n_rows = w.N if n_rows is None else n_rows
    Q, K, V = wl.make_head(w, h)
    cq = wl.init_centroids(w, h, Q, w.Cq, 0)
    ck = wl.init_centroids(w, h, K, w.Ck, 1)
    bf16 = w.dtype == "bf16"
    t0 = time.perf_counter()
    kq = orc.kmeans(Q, cq, w.iters, bf16)
    kk = orc.kmeans(K, ck, w.iters, bf16)
    pq = orc.permute(kq.labels, w.Cq)
    pk = orc.permute(kk.labels, w.Ck)
    Qp, Kp, Vp = orc.gather_rows(Q, pq.perm), orc.gather_rows(K, pk.perm), orc.gather_rows(V, pk.perm)
    sel = orc.select_topp(kq.centroids, kk.centroids, kq.counts, kk.counts, w.top_p)
    t1 = time.perf_counter()
    rows = np.sort(np.random.default_rng(w.seed).choice(w.N, n_rows, replace=False)).astype(np.int32)
    orc.sparse_attention(Qp, Kp, Vp, pq.offsets, pk.offsets, sel.row_ptr, sel.col_idx, perm_q=pq.perm, rows=rows)
    t2 = time.perf_counter()
    t_head = (t1 - t0) + (t2 - t1) * (w.N / n_rows)
    t_layer = t_head * w.H
    dense_flops = 4.0 * w.H * float(w.N) ** 2 * w.d
    log("cpu oracle: identify %.1f s, %d attention rows %.1f s, density %.3f" % (t1 - t0, n_rows, t2 - t1, sel.density))
    return {
        "value": dense_flops / t_layer / 1e12, "unit": "TFLOP/s (effective)", "cores": orc.n_threads(),
        "kind": "oracle",
        "sample": "head 0 of %d: k-means (%d iters, Q and K), permutation, top-p in full (%.1f s) + sparse "
                  "attention on %d of %d query rows (%.1f s); layer time extrapolated x N/rows x H = %.0f s"
                  % (w.H, w.iters, t1 - t0, n_rows, w.N, t2 - t1, t_layer),
        "measured_s": t2 - t0, "extrapolated_layer_s": t_layer,
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="wan_like", choices=sorted(wl.WORKLOADS))
    ap.add_argument("--top-p", type=float, default=None)
    ap.add_argument("--iters", type=int, default=None)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-dense", action="store_true")
    ap.add_argument("--gather-free", action="store_true",
                    help="time svg2_forward_gather_free (no permuted copies of Q, K, V) instead of svg2_forward")
    ap.add_argument("--fp8", action="store_true",
                    help="time svg2_forward_fp8 (attention step on E4M3 copies of Q, K, V; the paper's '+ FP8' variant) "
                         "-- a reduced-precision mode, reported beside the bf16 headline, never instead of it")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 1 GiB device copy (reference for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()

    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures ONE MI355X; the path shards by head with no exchange "
              "inside it, so --gpus %d is not run" % args.gpus, file=sys.stderr)
        sys.exit(2)

    def log(msg):
        print("[bench] " + msg, file=sys.stderr, flush=True)

    w = wl.WORKLOADS[args.workload]
    if args.top_p is not None:
        w = wl.replace(w, top_p=args.top_p)
    if args.iters is not None:
        w = wl.replace(w, iters=args.iters)
    if w.dtype != "bf16":
        raise SystemExit("bench.py times the bf16 workloads")
    H, N, d = w.H, w.N, w.d
    log("workload %s: H=%d N=%d d=%d Cq=%d Ck=%d iters=%d top_p=%g" % (w.name, H, N, d, w.Cq, w.Ck, w.iters, w.top_p))
    gen = start_generation(w)                 # worker processes start before the GPU is initialised

    import torch
    import paper_2505_18875_amd as svg2
    svg2.load_library()                       # fails loudly if the HIP library is not built
    if not torch.cuda.is_available():
        raise RuntimeError("bench.py needs a GPU")
    Q, K, V, cq0, ck0 = upload_inputs(w, gen, log)

    if args.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        log("copy calibration: one device copy of %d bytes" % src.numel())
        del src, dst

    total = args.warmup + args.steps
    # every step starts from the same seeded centroids: one in/out buffer pair per step, filled beforehand
    cqs = [cq0.clone() for _ in range(total + 1)]
    cks = [ck0.clone() for _ in range(total + 1)]
    O = torch.empty_like(Q)
    ws = torch.empty(svg2.svg2_forward_workspace_size(svg2.SVG2_BF16, H, N, d, w.Cq, w.Ck, args.gather_free, args.fp8),
                     dtype=torch.uint8, device="cuda")
    mode = "fp8 attention, gather-free" if args.fp8 else "gather-free" if args.gather_free else "physical permutation"
    log("workspace %.2f GB (%s)" % (ws.numel() / 1e9, mode))

    def step(i, aux=False):
        return svg2.svg2_forward(Q, K, V, cqs[i], cks[i], w.top_p, w.iters, out=O, ws=ws, want_aux=aux,
                                 gather_free=args.gather_free, fp8=args.fp8)

    r = step(total, aux=True)                 # an extra, untimed pass that also reports the density
    torch.cuda.synchronize()
    density = r.aux.density.double().cpu().numpy()
    log("density per head: mean %.4f min %.4f max %.4f" % (density.mean(), density.min(), density.max()))
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()

    svg2.svg2_profile_enable(1)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.warmup, total):
        step(i)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    svg2.svg2_profile_enable(0)
    stage_ms, n_calls = svg2.svg2_profile_read()
    assert n_calls == args.steps, (n_calls, args.steps)
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    stage_ms = {k: v / n_calls for k, v in stage_ms.items()}

    # a short second pass with an event pair around every kernel of k-means and of the permutation: which kernel
    # takes what (these events sit between kernels that otherwise run back to back, so this pass is not the timing)
    kernel_ms = {}
    if not args.fp8:
        n_kp = 3
        svg2.svg2_profile_enable(2)
        for i in range(n_kp):
            cqs[i].copy_(cq0)
            cks[i].copy_(ck0)
            step(i)
        torch.cuda.synchronize()
        svg2.svg2_profile_enable(0)
        svg2.svg2_profile_read()
        kernel_ms = {k: (ms / n_kp, cnt // n_kp) for k, (ms, cnt) in svg2.svg2_profile_read_kernels().items()}

    dense_flops = 4.0 * H * float(N) ** 2 * d
    sel_flops = dense_flops * float(density.mean())            # 4 d sum_sel |Q_i||K_j| over all heads
    attn_ms = stage_ms["attn"]
    achieved = sel_flops / (attn_ms * 1e-3) / 1e12
    peak = FP8_MFMA_PEAK_TFLOPS if args.fp8 else BF16_MFMA_PEAK_TFLOPS
    out = {
        "metric": "effective TFLOP/s of one SVG2 layer (kmeans+permute+topp+sparse-attn), 4*H*N^2*d / layer time, "
                  "at N=75,600, H=40; ms/layer is ms_per_step",
        "value": dense_flops / (ms_per_step * 1e-3) / 1e12, "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "fp8_e4m3 attention operands (fp32 softmax and accumulation), bf16 elsewhere" if args.fp8 else "bf16",
        "data": "synthetic",
        "config": {"workload": w.name, "H": H, "N": N, "d": d, "Cq": w.Cq, "Ck": w.Ck, "kmeans_iters": w.iters,
                   "top_p": w.top_p, "density": float(density.mean()),
                   "entry_point": "svg2_forward_fp8" if args.fp8 else
                                  "svg2_forward_gather_free" if args.gather_free else "svg2_forward"},
        "stages_ms": stage_ms,
        "roofline": {"kernel": "attn_fp8_kernel" if args.fp8 else "attn_bf16_kernel", "bound": "mfma",
                     "achieved": achieved, "peak": peak, "unit": "TFLOP/s", "frac": achieved / peak,
                     "traffic": None if args.fp8 or w.iters != wl.WORKLOADS[w.name].iters
                     else ATTN_TRAFFIC_BYTES.get((w.name, w.top_p)),
                     "traffic_source": ATTN_TRAFFIC_SOURCE,
                     "flops_per_launch": sel_flops, "ms_per_launch": attn_ms},
    }
    if kernel_ms:
        tensor_bytes = float(H) * N * d * 2                     # one [H,N,d] bf16 tensor
        rk = []

        def add(name, key, bound=None, flops=None, nbytes=None, note=None):
            ms, launches = kernel_ms[key]
            if launches == 0:
                return
            e = {"kernel": name, "launches_per_layer": launches, "ms_per_launch": ms / launches, "ms_per_layer": ms}
            t = ms / launches * 1e-3
            if flops is not None:
                e["tflops"] = flops / t / 1e12
            if nbytes is not None:
                e["gbps"] = nbytes / t / 1e9
            if bound == "mfma":
                e.update(bound="mfma", achieved=e["tflops"], peak=BF16_MFMA_PEAK_TFLOPS, unit="TFLOP/s",
                         frac=e["tflops"] / BF16_MFMA_PEAK_TFLOPS)
            elif bound == "hbm":
                e.update(bound="hbm", achieved=e["gbps"], peak=HBM_PEAK_GBPS, unit="GB/s", frac=e["gbps"] / HBM_PEAK_GBPS)
            if note:
                e["note"] = note
            rk.append(e)

        # a1: 2 N C d flops per head and side; both sides read their tokens once
        add("kmeans_assign_bf16_kernel (Q side C=%d and K side C=%d in one launch)" % (w.Cq, w.Ck), "kmeans_assign",
            bound="mfma", flops=2.0 * N * (w.Cq + w.Ck) * d * H, nbytes=2 * tensor_bytes,
            note="the K side is matrix-bound, the Q side memory-bound; gbps = Q and K read once")
        add("kmeans_settle_kernel (near-ties in double precision)", "kmeans_settle")
        add("permute_hist/scan/scatter_kernel inside k-means (Q and K)", "kmeans_sort")
        # a2: the first iteration sums every token (both sides read once), the others only the tokens that moved
        add("kmeans_segsum_kernel, all tokens (Q and K)", "kmeans_segsum_full", bound="hbm", nbytes=2 * tensor_bytes)
        add("kmeans_segsum_kernel, moved tokens only (Q and K)", "kmeans_segsum_delta")
        add("kmeans_finalize_kernel (Q and K)", "kmeans_finalize")
        add("permute_hist/scan/scatter_kernel (pi_q, pi_k)", "permute_sort")
        # a4: Q', K', V' = three tensors read and written once (two launches: Q, then K and V)
        if kernel_ms["permute_gather"][1]:
            ms, _ = kernel_ms["permute_gather"]
            rk.append({"kernel": "permute_gather_kernel (Q; K and V)", "launches_per_layer": 2, "ms_per_layer": ms,
                       "bound": "hbm", "achieved": 6 * tensor_bytes / (ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBPS,
                       "unit": "GB/s", "frac": 6 * tensor_bytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS})
        out["roofline_kernels"] = rk

    if not args.no_dense:
        # dense attention at the same shape: the same kernel with one query cluster, one key cluster, all selected
        one = torch.tensor([[0, N]] * H, dtype=torch.int32, device="cuda")
        rp = torch.tensor([[0, 1]] * H, dtype=torch.int32, device="cuda")
        ci = torch.zeros((H, 1), dtype=torch.int32, device="cuda")
        wsd = ws if not (args.gather_free or args.fp8) else None   # (those workspaces may be smaller than this call needs)
        svg2.svg2_sparse_attn(Q, K, V, one, one, rp, ci, None, out=O, ws=wsd)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        svg2.svg2_sparse_attn(Q, K, V, one, one, rp, ci, None, out=O, ws=wsd)
        e1.record()
        torch.cuda.synchronize()
        dense_ms = e0.elapsed_time(e1)
        out["dense"] = {"ms": dense_ms, "tflops": dense_flops / (dense_ms * 1e-3) / 1e12,
                        "speedup_of_sparse_layer": dense_ms / ms_per_step,
                        "density_bound_speedup": 1.0 / float(density.mean()),
                        "layer_ms_over_density_x_dense_ms": ms_per_step / (float(density.mean()) * dense_ms)}
        log("dense attention, same shape: %.1f ms" % dense_ms)

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, log)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
