#!/usr/bin/env python3
"""Benchmark of the LaRoSA decode hot path on one MI355X.

A step is one pass of the whole path -- pre-norm + rotation, Top-K, column-sparse q|k|v,
attention stand-in, Top-K, o + residual, pre-norm + rotation, Top-K, gate|up, SiLU*up, Top-K,
down + residual -- for one decoder layer and one batch of tokens, through larosa_layer_forward.
Consecutive steps use different weight sets (default 8, > 3 GB) so weight rows come from HBM
and not from the 256 MB memory-side cache.  Everything is resident in HBM before timing.

Prints ONE JSON line (metric: microseconds per decoder layer; lower is better) that also
carries the HBM roofline of the dominant kernel (the indexed row-streaming mat-vec), measured
with HIP events, and the CPU oracle timed on the host cores as a baseline.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0

# HBM bytes per launch of the dominant kernel come from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of
# this script scaled by a 1 GiB copy; the summaries under profiles/ carry the figure on a line
# "traffic_bytes_per_launch: <number>", which is read back here (the counters cannot be collected from
# inside an ordinary run).  Keyed by (config, batch, sparsity, form); other workloads have not been counted.
TRAFFIC_SUMMARIES = {
    (1, 1, 0.4, "shortcut"): "profiles/fused_topk_gemv_llama2_7b_layer_b1_s40_shortcut_form_hbm_traffic.txt",
    (1, 1, 0.4, "explicit"): "profiles/gemv_rows_llama2_7b_layer_b1_s40_hbm_traffic.txt",
}


def measured_traffic(key):
    """(bytes per launch, summary file) from the committed counter summary of this workload, or (None, None)."""
    rel = TRAFFIC_SUMMARIES.get(key)
    if rel is None:
        return None, None
    try:
        with open(os.path.join(ROOT, rel)) as f:
            for line in f:
                if line.startswith("traffic_bytes_per_launch:"):
                    return float(line.split(":", 1)[1].split()[0]), rel
    except OSError:
        pass
    return None, None

CONFIGS = {
    1: dict(shape="llama2-7b", workload="LLaMA2-7B-shaped decoder layer, fp16, batch 1, 40% sparsity, "
                                        "rotations Q_attn/Q_mlp from PCA of 4096 synthetic calibration tokens",
            n_cal=4096, latent="gauss"),
    2: dict(shape="llama3-8b", workload="LLaMA3-8B-shaped decoder layer (GQA), bf16", n_cal=4096, latent="gauss"),
    3: dict(shape="llama2-70b", workload="LLaMA2-70B-shaped decoder layer on one GPU, bf16", n_cal=8192,
            latent="t3"),
    4: dict(shape="llama2-7b", workload="32-layer LLaMA2-7B-shaped projection stack, fp16, per-layer rotations with a "
                                        "4096 x 4096 residual adapter between layers", n_cal=4096, latent="gauss",
            n_layers=32),
}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def offline_report(args, api, torch, shape, cfg, dev):
    """Matrix-core contractions of the offline part for one layer of the chosen shape: second
    moment of n_cal tokens, the four folds of the deployed form and the residual adapter.  Times are
    HIP-event averages; TFLOP/s counts 2 M N K once per product (the extra passes over the 16-bit
    terms of an fp32 rotation are overhead, not work), against the dense 16-bit MFMA peak."""
    td = torch.float16 if shape.dtype == "f16" else torch.bfloat16
    d, d_q, d_kv, d_ff, n = shape.d, shape.d_q, shape.d_kv, shape.d_ff, cfg["n_cal"]
    gen = torch.Generator(device=dev)
    gen.manual_seed(1299)

    def gauss(r, c, s=0.02):
        return (torch.randn(r, c, generator=gen, device=dev, dtype=torch.float32) * s).to(td)

    X = gauss(n, d, 1.0)
    def orthogonal():   # (--host-solver: the vendor's device QR does not survive hardware-counter collection)
        g = torch.randn(d, d, generator=gen, device=dev, dtype=torch.float32)
        return (torch.linalg.qr(g.cpu())[0].to(dev) if args.host_solver else torch.linalg.qr(g)[0]).contiguous()

    Q, Q2 = orthogonal(), orthogonal()
    sc = api.OfflineScratch(d, shape.dtype)
    C = torch.empty(d, d, dtype=torch.float32, device=dev)
    Wqkv, Wgu, Wo, Wdown = gauss(d, d_q + 2 * d_kv), gauss(d, 2 * d_ff), gauss(d_q, d), gauss(d_ff, d)
    outs = [torch.empty_like(w) for w in (Wqkv, Wgu, Wo, Wdown)]
    A = torch.empty(d, d, dtype=td, device=dev)
    jobs = [
        ("second_moment", lambda: api.second_moment(X, C, shape.dtype), 2.0 * n * d * d, 2.0 * n * d * d / 2),
        ("fold_input_qkv", lambda: api.fold_input(Q, Wqkv, outs[0], shape.dtype, sc), 2.0 * d * d * Wqkv.shape[1], None),
        ("fold_input_gate_up", lambda: api.fold_input(Q, Wgu, outs[1], shape.dtype, sc), 2.0 * d * d * Wgu.shape[1], None),
        ("fold_output_o", lambda: api.fold_output(Wo, Q, outs[2], shape.dtype, sc), 2.0 * d_q * d * d, None),
        ("fold_output_down", lambda: api.fold_output(Wdown, Q, outs[3], shape.dtype, sc), 2.0 * d_ff * d * d, None),
        ("residual_adapter", lambda: api.residual_adapter(Q, Q2, A, shape.dtype, sc), 2.0 * d * d * d, None),
    ]
    reps = max(3, min(args.steps, 20))
    rows, total_ms = {}, 0.0
    for name, fn, flops, _ in jobs:
        for _ in range(2):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / reps
        rows[name] = dict(ms=round(ms, 4), TFLOPs=round(flops / (ms * 1e-3) / 1e12, 1))
        total_ms += ms
    # vendor BLAS on the same second moment, for context (16-bit inputs, 16-bit output)
    for _ in range(2):
        torch.matmul(X.T, X)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        torch.matmul(X.T, X)
    e1.record()
    torch.cuda.synchronize()
    blas_ms = e0.elapsed_time(e1) / reps
    dom = "fold_input_gate_up"
    report = {
        "metric": "offline_contractions_ms_per_layer", "value": round(total_ms, 3), "unit": "ms", "n_gpus": 1,
        "steps": reps, "warmup": 2, "ms_per_step": round(total_ms, 3), "higher_is_better": False, "scaling": "weak",
        "vs_baseline": None, "dtype": shape.dtype, "data": "synthetic",
        "config": {"workload": f"offline contractions of one {shape.name} layer, {n} calibration tokens",
                   "shape": shape.name},
        "roofline": {"bound": "mfma", "achieved": rows[dom]["TFLOPs"], "peak": 2500.0, "unit": "TFLOP/s",
                     "frac": round(rows[dom]["TFLOPs"] / 2500.0, 4), "traffic": None,
                     "kernel": f"contraction_kernel ({dom}: Q^T W with Q in {2 if shape.dtype == 'f16' else 3} "
                               "16-bit terms; flops counted once)"},
        "cpu_baseline": None,
        "extra": {"per_call": rows, "blas_XtX_16bit_ms": round(blas_ms, 4),
                  "blas_XtX_TFLOPs": round(2.0 * n * d * d / (blas_ms * 1e-3) / 1e12, 1)},
    }
    print(json.dumps(report), flush=True)


def _graph_event_us(torch, fn, launches, reps):
    """Average microseconds per launch of fn's launches, replayed as one HIP graph."""
    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        fn()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    with torch.cuda.graph(g):
        fn()
    g.replay()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        g.replay()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e3 / (reps * launches)


def _heavy_tokens(torch, gen, B, d, td, dev):
    """Rotated-activation stand-in: Gaussian entries with an i^-0.6 envelope and 4 outlier channels."""
    env = torch.arange(1, d + 1, device=dev, dtype=torch.float32) ** -0.6
    h = torch.randn(B, d, generator=gen, device=dev, dtype=torch.float32) * env
    h[:, torch.randperm(d, generator=gen, device=dev)[:4]] *= 20.0
    return h.to(td).contiguous()


def w4_report(args, api, torch, shape, cfg, dev):
    """The four column-sparse projections of one layer (indices given) over 4-bit weights and over the
    16-bit weights they were quantised from, B = 1.  Bytes per launch: K (d_out / 2 + 2 ceil(d_out / 128))
    for codes and scales of the kept rows."""
    td = torch.float16 if shape.dtype == "f16" else torch.bfloat16
    d, d_q, d_kv, d_ff = shape.d, shape.d_q, shape.d_kv, shape.d_ff
    p, nsets = args.sparsity, max(1, args.nsets)
    gen = torch.Generator(device=dev)
    gen.manual_seed(1299)
    dims = [("qkv", d, d_q + 2 * d_kv), ("o", d_q, d), ("gu", d, 2 * d_ff), ("down", d_ff, d)]
    ws = api.workspace(1, max(d, d_ff), 2 * d_ff, max(d, d_ff))
    rows = {}
    tot16 = tot4 = bytes16 = bytes4 = 0.0
    reps = max(1, args.steps // nsets)
    for name, din, dout in dims:
        K = int(round((1 - p) * din))
        W16 = [(torch.randn(din, dout, generator=gen, device=dev, dtype=torch.float32) * 0.02).to(td)
               for _ in range(nsets)]
        W4 = [api.quantize_w4(w, shape.dtype) for w in W16]
        h = _heavy_tokens(torch, gen, 1, din, td, dev)
        idx = torch.empty(1, K, dtype=torch.int32, device=dev)
        api.topk(h, K, idx, shape.dtype)
        y = torch.zeros(1, dout, dtype=td, device=dev)

        def run16():
            for w in W16:
                api.sparse_gemv(w, h, idx, y, shape.dtype, ws)

        def run4():
            for wq, sc in W4:
                api.sparse_gemv_w4(wq, sc, h, idx, y, shape.dtype, ws)

        us16 = _graph_event_us(torch, run16, nsets, reps)
        us4 = _graph_event_us(torch, run4, nsets, reps)
        b16 = 2.0 * K * dout
        b4 = K * (dout / 2 + 2 * ((dout + 127) // 128))
        rows[name] = dict(K=K, d_out=dout, us_16bit=round(us16, 3), us_w4=round(us4, 3),
                          GBs_16bit=round(b16 / us16 / 1e3, 1), GBs_w4=round(b4 / us4 / 1e3, 1))
        tot16 += us16; tot4 += us4; bytes16 += b16; bytes4 += b4
        del W16, W4
    ach = bytes4 / 4 / (tot4 / 4) / 1e3
    report = {
        "metric": "us_per_layer_sparse_projections_w4", "value": round(tot4, 3), "unit": "us", "n_gpus": 1,
        "steps": reps * nsets, "warmup": 1, "ms_per_step": round(tot4 / 1e3, 6), "higher_is_better": False,
        "scaling": "weak", "vs_baseline": None, "dtype": shape.dtype, "data": "synthetic",
        "config": {"workload": f"four column-sparse projections of one {shape.name} layer over 4-bit weights, "
                               f"batch 1, sparsity {p}", "shape": shape.name, "weight_sets": nsets},
        "roofline": {"bound": "hbm", "achieved": round(ach, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(ach / HBM_PEAK_GBS, 4), "traffic": None,
                     "kernel": "gemv_rows_w4_kernel (codes + scales of the kept rows, average over the 4 launches)"},
        "cpu_baseline": None,
        "extra": {"per_projection": rows, "us_per_layer_16bit": round(tot16, 3),
                  "speedup_w4_vs_16bit": round(tot16 / tot4, 3),
                  "bytes_per_layer_w4": bytes4, "bytes_per_layer_16bit": bytes16},
    }
    print(json.dumps(report), flush=True)


def threshold_report(args, api, torch, shape, cfg, dev):
    """Sec. 4.1 on synthetic tokens: a cutoff calibrated offline for the target sparsity against Top-K
    at the same target, on a stream whose per-token scale drifts (log-normal, sigma 0.3).  For every
    token: kept count, and the time of the gate|up-shaped column-sparse projection with that count
    (eager launches, HIP events, median of 7 runs per token)."""
    import numpy as np
    td = torch.float16 if shape.dtype == "f16" else torch.bfloat16
    d, dout, p = shape.d, 2 * shape.d_ff, args.sparsity
    n_tok = max(16, min(args.steps, 512))
    gen = torch.Generator(device=dev)
    gen.manual_seed(1299)
    nsets = max(1, args.nsets)
    Ws = [(torch.randn(d, dout, generator=gen, device=dev, dtype=torch.float32) * 0.02).to(td) for _ in range(nsets)]
    ws = api.workspace(1, d, dout, d)
    cal = _heavy_tokens(torch, gen, 512, d, td, dev)
    eps = float(torch.quantile(cal.float().abs().flatten()[: 1 << 20], p))       # offline calibrated cutoff
    drift = torch.exp(0.3 * torch.randn(n_tok, generator=gen, device=dev))
    toks = (_heavy_tokens(torch, gen, n_tok, d, td, dev).float() * drift[:, None]).to(td).contiguous()
    K = int(round((1 - p) * d))
    y = torch.zeros(1, dout, dtype=td, device=dev)
    idx_t = torch.zeros(1, d, dtype=torch.int32, device=dev)
    cnt = torch.zeros(1, dtype=torch.int32, device=dev)
    idx_k = torch.zeros(1, K, dtype=torch.int32, device=dev)

    def timed(fn, rep=7):
        """Median of `rep` event-timed runs: the spread over tokens should show the kept count, not
        launch jitter."""
        ts = []
        for _ in range(rep):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            fn()
            e1.record()
            torch.cuda.synchronize()
            ts.append(e0.elapsed_time(e1) * 1e3)
        return sorted(ts)[rep // 2]

    t_thr, t_top, kept = [], [], []
    for rnd in range(2):                       # first round warms up
        t_thr.clear(); t_top.clear(); kept.clear()
        for i in range(n_tok if rnd else min(n_tok, 16)):
            h = toks[i:i + 1]
            W = Ws[i % nsets]
            api.threshold_select(h, eps, idx_t, cnt, shape.dtype)
            k_i = int(cnt.item())               # the projection's launch shape depends on the count
            kept.append(k_i)
            if k_i > 0:
                sel = idx_t[:, :k_i].contiguous()
                t_thr.append(timed(lambda: api.sparse_gemv(W, h, sel, y, shape.dtype, ws)))
            else:
                t_thr.append(0.0)

            def topk_path():
                api.topk(h, K, idx_k, shape.dtype)
                api.sparse_gemv(W, h, idx_k, y, shape.dtype, ws)
            t_top.append(timed(topk_path))

    def stats(v):
        a = np.asarray(v, np.float64)
        return dict(mean=round(float(a.mean()), 3), std=round(float(a.std()), 3), min=round(float(a.min()), 3),
                    p10=round(float(np.percentile(a, 10)), 3), p90=round(float(np.percentile(a, 90)), 3),
                    max=round(float(a.max()), 3))

    frac = np.asarray(kept) / d
    report = {
        "metric": "per_token_us_spread_threshold_vs_topk", "value": stats(t_thr)["std"], "unit": "us (std over tokens)",
        "n_gpus": 1, "steps": n_tok, "warmup": n_tok, "ms_per_step": round(float(np.mean(t_thr)) / 1e3, 6),
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": shape.dtype, "data": "synthetic",
        "config": {"workload": f"gate|up-shaped projection ({d} x {dout}) of {shape.name}, {n_tok} tokens with "
                               f"log-normal scale drift (sigma 0.3), target sparsity {p}", "shape": shape.name},
        "roofline": None, "cpu_baseline": None,
        "extra": {"threshold_eps": eps, "threshold_kept_fraction": stats(frac), "topk_kept_fraction": K / d,
                  "threshold_projection_us": stats(t_thr), "topk_select_plus_projection_us": stats(t_top),
                  "note": "threshold time excludes its select kernel and the count read-back; Top-K time includes "
                          "its select kernel"},
    }
    print(json.dumps(report), flush=True)


def stack_report(args, api, torch, shape, cfg, dev):
    """The whole projection stack of a 7B-shaped model for one decode step: n_layers layers with
    their own weights (13 GB in all) and their own rotation Q_l, every rotation absorbed; the
    residual adapter Q_l^T Q_{l+1} sits on the MLP shortcut (so it shares gate|up's launch at batch 1)
    and down carries Q_{l+1} on its output side.  Rotations are seeded orthogonal matrices, adapters
    are built with larosa_residual_adapter, folded weights of Gaussian weights are Gaussian and drawn
    directly.  One HIP graph holds the n_layers calls; the dense comparator runs the four dense
    projections of every layer over the same weights."""
    td = torch.float16 if shape.dtype == "f16" else torch.bfloat16
    d, d_q, d_kv, d_ff = shape.d, shape.d_q, shape.d_kv, shape.d_ff
    d_qkv = d_q + 2 * d_kv
    p, B, n_layers = args.sparsity, args.batch, cfg["n_layers"]
    from paper_2507_01299_amd import allocation, synth
    K1, K2, K3, K4 = allocation.kept_counts(d, d_q, d_ff, p, 1.0, 1.0)
    gen = torch.Generator(device=dev)
    gen.manual_seed(1299 * 1000 + 40)

    def gauss(r, c):
        return (torch.randn(r, c, generator=gen, device=dev, dtype=torch.float32) * 0.02).to(td)

    def basis():
        q, r = torch.linalg.qr(torch.randn(d, d, generator=gen, device=dev, dtype=torch.float32))
        return (q * torch.sign(torch.diagonal(r))[None, :]).contiguous()

    scratch = api.OfflineScratch(d, shape.dtype)
    Q_prev = basis()
    layers, weights = [], []
    for l in range(n_layers):
        Q_next = basis()
        A = torch.empty(d, d, dtype=td, device=dev)
        api.residual_adapter(Q_prev, Q_next, A, shape.dtype, scratch)
        w = dict(Wqkv=gauss(d, d_qkv), Wo=gauss(d_q, d), Wgu=gauss(d, 2 * d_ff), Wdown=gauss(d_ff, d), A=A)
        weights.append(w)
        layers.append(api.Layer(d, d_q, d_kv, d_ff, shape.head_dim, K1, K2, K3, K4, w["Wqkv"], w["Wo"], w["Wgu"],
                                w["Wdown"], shape.dtype, rms_eps=synth.RMS_EPS, shortcut_mlp=A))
        Q_prev = Q_next
    torch.cuda.synchronize()
    env = torch.arange(1, d + 1, device=dev, dtype=torch.float32) ** -0.8
    x0 = (torch.randn(B, d, generator=gen, device=dev, dtype=torch.float32) * env * 8.0).to(td).contiguous()
    bufs = [torch.zeros_like(x0), torch.zeros_like(x0)]
    ws = api.Workspace(layers[0].workspace_bytes(B))

    def stack():
        cur = x0
        for i, L in enumerate(layers):
            api.layer_forward(L, cur, bufs[i & 1], ws)
            cur = bufs[i & 1]

    reps = max(2, args.steps // n_layers)
    stack_us = _graph_event_us(torch, stack, 1, reps)
    assert bool(torch.isfinite(bufs[(n_layers - 1) & 1].float()).all())
    ys = dict(qkv=torch.zeros(B, d_qkv, dtype=td, device=dev), o=torch.zeros(B, d, dtype=td, device=dev),
              gu=torch.zeros(B, 2 * d_ff, dtype=td, device=dev), down=torch.zeros(B, d, dtype=td, device=dev))
    xin = dict(qkv=x0, o=gauss(B, d_q), gu=x0, down=gauss(B, d_ff))

    def dense_stack():
        for w in weights:
            api.dense_gemv(w["Wqkv"], xin["qkv"], ys["qkv"], shape.dtype, ws)
            api.dense_gemv(w["Wo"], xin["o"], ys["o"], shape.dtype, ws)
            api.dense_gemv(w["Wgu"], xin["gu"], ys["gu"], shape.dtype, ws)
            api.dense_gemv(w["Wdown"], xin["down"], ys["down"], shape.dtype, ws)

    dense_us = _graph_event_us(torch, dense_stack, 1, reps)
    lin_w = [[w["Wqkv"].T.contiguous(), w["Wo"].T.contiguous(), w["Wgu"].T.contiguous(), w["Wdown"].T.contiguous()]
             for w in weights[:8]]
    lin_x = [xin["qkv"], xin["o"], xin["gu"], xin["down"]]

    def blas8():
        for wset in lin_w:
            for w_, x_ in zip(wset, lin_x):
                torch.nn.functional.linear(x_, w_)

    blas_us = _graph_event_us(torch, blas8, 1, reps) * (n_layers / 8.0)
    sel = 2.0 * (K1 * d_qkv + K2 * d + K3 * 2 * d_ff + K4 * d) if B == 1 else None
    all_bytes = None if sel is None else sel + 2.0 * d * d
    report = {
        "metric": "us_per_token_projection_stack", "value": round(stack_us, 2), "unit": "us", "n_gpus": 1,
        "steps": reps, "warmup": 1, "ms_per_step": round(stack_us / 1e3, 5), "higher_is_better": False,
        "scaling": "weak", "vs_baseline": None, "dtype": shape.dtype, "data": "synthetic",
        "config": {"workload": f"{cfg['workload']}; batch {B}; sparsity {p}", "shape": shape.name, "batch": B,
                   "layers": n_layers, "K": [K1, K2, K3, K4], "launch": "one HIP graph of the whole stack"},
        "roofline": None if all_bytes is None else {
            "bound": "hbm", "achieved": round(all_bytes * n_layers / stack_us / 1e3, 1), "peak": HBM_PEAK_GBS,
            "unit": "GB/s", "frac": round(all_bytes * n_layers / stack_us / 1e3 / HBM_PEAK_GBS, 4), "traffic": None,
            "kernel": "whole stack: kept rows of the four projections + one adapter per layer over the stack time"},
        "cpu_baseline": None,
        "extra": {"us_per_layer": round(stack_us / n_layers, 2), "tokens_per_s": round(B * 1e6 / stack_us, 1),
                  "dense_gemv_stack_us": round(dense_us, 2), "blas_linear_stack_us": round(blas_us, 2),
                  "speedup_vs_own_dense": round(dense_us / stack_us, 3),
                  "speedup_vs_blas_dense": round(blas_us / stack_us, 3),
                  "weights_GB": round(n_layers * 2.0 * (d * d_qkv + d_q * d + d * 2 * d_ff + d_ff * d + d * d) / 1e9, 2)},
    }
    print(json.dumps(report), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=40)
    ap.add_argument("--config", type=int, default=1, choices=sorted(CONFIGS))
    ap.add_argument("--sparsity", type=float, default=0.4)
    ap.add_argument("--batch", type=int, default=1)
    ap.add_argument("--nsets", type=int, default=8)
    ap.add_argument("--replays", type=int, default=25,
                    help="timed replays of the graph of --steps steps (at least 25, and as many as about half a second takes); "
                         "the value is their median")
    ap.add_argument("--alpha", default="1.0,1.0", metavar="A1,A3",
                    help="sparsity coefficients of h1 and h3 (h2, h4 follow from the block constraints)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=15.0)
    ap.add_argument("--detail", default=None, help="also write the full report to this JSON file")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 1 GiB device copy (torch copy kernel) so that hardware counters "
                         "read under rocprofv3 can be scaled by a transfer of known size")
    ap.add_argument("--form", default="shortcut", choices=["shortcut", "explicit"],
                    help="how the layer's two rotations are executed: absorbed into the weights with a residual "
                         "adapter on each shortcut (the deployed block-level form, default), or as explicit "
                         "mat-vecs in front of q|k|v and gate|up")
    ap.add_argument("--offline", action="store_true",
                    help="time the offline contractions (second moment, folds, adapter) of the chosen "
                         "config's layer instead of the decode step; prints its own JSON line")
    ap.add_argument("--w4", action="store_true",
                    help="time the four column-sparse projections of the chosen layer over 4-bit weights "
                         "next to the 16-bit ones; prints its own JSON line")
    ap.add_argument("--threshold-comparator", action="store_true",
                    help="per-token time and kept-count spread of the magnitude-threshold sparsifier against "
                         "Top-K on a synthetic token stream with scale drift; prints its own JSON line")
    ap.add_argument("--host-solver", action="store_true",
                    help="run the eigen-solver of the weight preparation on the host (the device solver does not "
                         "run under hardware-counter collection)")
    ap.add_argument("--tune", action="append", default=[], metavar="KEY=VALUE",
                    help="larosa_set_tuning(KEY, VALUE) before anything is sized (experiments)")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this build runs on ONE GPU only (no sharding, no collectives); "
            f"--gpus {args.gpus} is not supported. Re-run with --gpus 1.")
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2507_01299_amd import api, offline, synth

    if not torch.cuda.is_available():
        log("bench.py: no GPU visible")
        sys.exit(2)
    api.lib()
    for kv in args.tune:
        k, v = kv.split("=")
        api.set_tuning(int(k), int(v))
    dev = torch.device("cuda:0")
    cfg = CONFIGS[args.config]
    shape = synth.SHAPES[cfg["shape"]]
    if args.offline:
        return offline_report(args, api, torch, shape, cfg, dev)
    if args.config == 4:
        return stack_report(args, api, torch, shape, cfg, dev)
    if args.w4:
        return w4_report(args, api, torch, shape, cfg, dev)
    if args.threshold_comparator:
        return threshold_report(args, api, torch, shape, cfg, dev)
    td = torch.float16 if shape.dtype == "f16" else torch.bfloat16
    p, B, nsets = args.sparsity, args.batch, max(1, args.nsets)
    d, d_q, d_kv, d_ff = shape.d, shape.d_q, shape.d_kv, shape.d_ff
    from paper_2507_01299_amd import allocation
    alpha1, alpha3 = (float(v) for v in args.alpha.split(","))
    K1, K2, K3, K4 = allocation.kept_counts(d, d_q, d_ff, p, alpha1, alpha3)
    d_qkv = d_q + 2 * d_kv

    # ---- weight set 0: the canonical synthetic layer (seeded numpy draws, PCA rotations)
    t0 = time.time()
    seed = synth.seed_for(args.config, 0)
    src = synth.activation_source(d, seed, latent=cfg["latent"])
    W = synth.layer_weights(shape, seed + 100)
    Xc = src.draw(cfg["n_cal"], seed + 1)
    # prepared through the library's own offline calls (second moments, folds and adapters on the matrix
    # cores; the eigen-solver in between is torch's, on the host for widths where the device solver is slow)
    Wdev = {k: torch.as_tensor(v).to(dev).to(td).contiguous() for k, v in W.items()}
    Xcd = torch.as_tensor(Xc).to(dev).to(td).contiguous()
    ops0 = offline.prepare_shortcut_layer(shape, Wdev, Xcd, rms_eps=synth.RMS_EPS,
                                          solver_device="cpu" if (d > 4096 or args.host_solver) else None)
    del W, Xc, Wdev, Xcd
    x = torch.as_tensor(src.draw(B, synth.seed_for(args.config, 5))).to(dev).to(td).contiguous()
    x_explicit = x
    shortcut_form = args.form == "shortcut"
    if shortcut_form:      # the stream arrives in the attention block's basis
        x = (x.double() @ ops0["Q_attn32"].double()).to(td).contiguous()
    log(f"canonical layer prepared in {time.time() - t0:.1f}s")

    # ---- further weight sets: the folded weight of a Gaussian W under an orthogonal Q is again
    # iid Gaussian, so W' ~ N(0, 0.02^2) is drawn directly on the device; rotations are copies.
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed + 7)

    def gauss(r, c):
        return (torch.randn(r, c, generator=gen, device=dev, dtype=torch.float32) * 0.02).to(td)

    if shortcut_form:
        ops0["Wo"], ops0["Wdown"] = ops0["Wo_out"], ops0["Wdown_out"]
    sets = [ops0]
    for _ in range(1, nsets):
        sets.append(dict(Wqkv=gauss(d, d_qkv), Wo=gauss(d_q, d), Wgu=gauss(d, 2 * d_ff), Wdown=gauss(d_ff, d),
                         Q_attn=ops0["Q_attn"].clone(), Q_mlp=ops0["Q_mlp"].clone(),
                         shortcut_attn=ops0["shortcut_attn"].clone(), shortcut_mlp=ops0["shortcut_mlp"].clone()))

    def make_layer(s, form_shortcut):
        if form_shortcut:
            return api.Layer(d, d_q, d_kv, d_ff, shape.head_dim, K1, K2, K3, K4, s["Wqkv"], s["Wo"], s["Wgu"],
                             s["Wdown"], shape.dtype, rms_eps=synth.RMS_EPS, shortcut_attn=s["shortcut_attn"],
                             shortcut_mlp=s["shortcut_mlp"])
        return api.Layer(d, d_q, d_kv, d_ff, shape.head_dim, K1, K2, K3, K4, s["Wqkv"], s["Wo"], s["Wgu"],
                         s["Wdown"], shape.dtype, Q_attn=s["Q_attn"], Q_mlp=s["Q_mlp"], rms_eps=synth.RMS_EPS)

    layers = [make_layer(s, shortcut_form) for s in sets]
    # the other form on the same weight sets (timing only: the weights are random either way)
    layers_other = [make_layer(s, not shortcut_form) for s in sets]
    ws = api.Workspace(max(layers[0].workspace_bytes(B), layers_other[0].workspace_bytes(B)))
    out = torch.zeros_like(x)
    trace = layers[0].trace_buffers(B)

    if args.copy_calibration:
        src_c = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(3)
        dst_c = torch.empty_like(src_c)
        for _ in range(3):
            dst_c.copy_(src_c)
        torch.cuda.synchronize()
        del src_c, dst_c

    # ---- eager timing: exactly `steps` steps, host launches one C-ABI call per step
    for i in range(args.warmup):
        api.layer_forward(layers[i % nsets], x, out, ws)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        api.layer_forward(layers[i % nsets], x, out, ws)
    torch.cuda.synchronize()
    eager_us = (time.perf_counter() - t0) / args.steps * 1e6

    # ---- graph timing: the same steps captured once per weight set into one HIP graph
    def capture(fn):
        g = torch.cuda.CUDAGraph()
        s = torch.cuda.Stream()
        s.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(s):
            fn()                      # warm-up on the side stream
        torch.cuda.current_stream().wait_stream(s)
        torch.cuda.synchronize()
        with torch.cuda.graph(g):
            fn()
        return g

    # The timed unit is ONE graph of exactly `steps` steps (step i uses weight set i mod nsets); it is replayed
    # `replays` times, every replay bracketed by HIP events on the launch stream, and the figure reported is the
    # median replay (p10 / p90 beside it).  One event record costs a few microseconds per replay, i.e. per
    # `steps` steps.
    K_steps = max(1, args.steps)
    replays = max(25, args.replays)

    def timed_steps():
        for i in range(K_steps):
            api.layer_forward(layers[i % nsets], x, out, ws)

    def replay_stats(g, n):
        evs = [torch.cuda.Event(enable_timing=True) for _ in range(n + 1)]
        g.replay()
        torch.cuda.synchronize()
        evs[0].record()
        for i in range(n):
            g.replay()
            evs[i + 1].record()
        torch.cuda.synchronize()
        per = sorted(evs[i].elapsed_time(evs[i + 1]) * 1e3 / K_steps for i in range(n))
        return dict(median=per[n // 2], p10=per[n // 10], p90=per[(n * 9) // 10], min=per[0], max=per[-1], n=n)

    g_layer = capture(timed_steps)
    for _ in range(max(1, -(-args.warmup // K_steps))):
        g_layer.replay()
    torch.cuda.synchronize()
    # enough replays that the timed region lasts about half a second (a short --steps would otherwise be over
    # in milliseconds and leave nothing for an outside observer of the GPU to corroborate)
    tp = time.perf_counter()
    g_layer.replay()
    torch.cuda.synchronize()
    pilot_s = max(time.perf_counter() - tp, 1e-6)
    replays = min(4000, max(replays, int(0.5 / pilot_s) + 1))
    t0 = time.perf_counter()
    st_graph = replay_stats(g_layer, replays)
    graph_wall_s = time.perf_counter() - t0
    graph_us = st_graph["median"]
    graph_steps = K_steps

    x_other = x_explicit if shortcut_form else (x.double() @ ops0["Q_attn32"].double()).to(td).contiguous()

    def other_steps():
        for i in range(K_steps):
            api.layer_forward(layers_other[i % nsets], x_other, out, ws)

    g_other = capture(other_steps)
    g_other.replay()
    other_us = replay_stats(g_other, max(25, args.replays))["median"]
    del g_other

    # ---- the dominant kernel alone: the four column-sparse projections of a layer on real
    # activations / index sets (taken from a traced run of set 0), HIP events on the launch stream
    api.layer_forward(layers[0], x, out, ws, trace)
    torch.cuda.synchronize()
    ys = dict(qkv=torch.zeros(B, d_qkv, dtype=td, device=dev), o=torch.zeros(B, d, dtype=td, device=dev),
              gu=torch.zeros(B, 2 * d_ff, dtype=td, device=dev), down=torch.zeros(B, d, dtype=td, device=dev))
    proj = [("Wqkv", "h1", "idx1", "qkv", K1, d_qkv), ("Wo", "h2", "idx2", "o", K2, d),
            ("Wgu", "h3", "idx3", "gu", K3, 2 * d_ff), ("Wdown", "h4", "idx4", "down", K4, d)]

    def event_time_us(fn, launches, reps):
        g = capture(fn)
        g.replay()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            g.replay()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / (reps * launches)

    def sparse_all():
        for s in sets:
            for wn, hn, inn, yn, K, dout in proj:
                api.sparse_gemv(s[wn], trace[hn], trace[inn], ys[yn], shape.dtype, ws)

    reps = max(3, min(64, args.steps // nsets))
    sparse_launch_us = event_time_us(sparse_all, 4 * nsets, reps)
    standalone_launch_us = sparse_launch_us
    stage_us = None
    if True:
        # The kernel that dominates the timed layer step is the projection with the Top-K fused in
        # (4 launches per step).  Time it inside larosa_layer_forward itself: the library records
        # caller-supplied HIP events at the stage boundaries of each (eagerly launched) step.
        n_ev = max(nsets, min(args.steps, 128))
        evs = [[torch.cuda.Event(enable_timing=True) for _ in range(8)] for _ in range(n_ev)]
        for es in evs:
            for e in es:
                e.record()              # creates the underlying hipEvent_t
        torch.cuda.synchronize()
        for i in range(nsets):
            api.layer_forward(layers[i % nsets], x, out, ws)
        for i in range(n_ev):
            api.layer_forward(layers[i % nsets], x, out, ws, stage_events=evs[i])
        torch.cuda.synchronize()
        names = ["h1_stage", "qkv", "o", "h3_stage", "gu", "down"]
        stage_us = {n: 0.0 for n in names}
        step_us = []
        for es in evs:
            for k, n in enumerate(names):
                stage_us[n] += es[k].elapsed_time(es[k + 1]) * 1e3 / n_ev
            step_us.append(es[0].elapsed_time(es[6]) * 1e3)
        step_us.sort()
        step_pct = {"p10": round(step_us[len(step_us) // 10], 2), "median": round(step_us[len(step_us) // 2], 2),
                    "p90": round(step_us[(len(step_us) * 9) // 10], 2), "n": len(step_us)}
        if B == 1:
            sparse_launch_us = (stage_us["qkv"] + stage_us["o"] + stage_us["gu"] + stage_us["down"]) / 4.0
        if B == 1 and shortcut_form:
            # In this form the step IS four launches of the fused kernel and nothing else, so the launch
            # time is the step time / 4, taken with HIP events around graph replays on the launch stream
            # (the per-stage events above each add the cost of an event record to their interval).
            sparse_launch_us = graph_us / 4.0
    # rows a launch has to read: the kept rows at batch 1, the union of the tokens' kept rows otherwise
    U = [int(torch.unique(trace[n]).numel()) for n in ("idx1", "idx2", "idx3", "idx4")]
    sel_bytes_layer = 2 * (U[0] * d_qkv + U[1] * d + U[2] * 2 * d_ff + U[3] * d)
    sel_bytes_launch = sel_bytes_layer / 4.0
    if B == 1 and shortcut_form:
        # two of the four launches also stream a d x d residual adapter each: bytes the kernel must move
        sel_bytes_launch = (sel_bytes_layer + 2 * 2 * d * d) / 4.0
    achieved_gbs = sel_bytes_launch / (sparse_launch_us * 1e-6) / 1e9

    per_proj = {}
    for wn, hn, inn, yn, K, dout in proj:
        def one(wn=wn, hn=hn, inn=inn, yn=yn):
            for s in sets:
                api.sparse_gemv(s[wn], trace[hn], trace[inn], ys[yn], shape.dtype, ws)
        us = event_time_us(one, nsets, reps)
        Un = U[[p_[3] for p_ in proj].index(yn)]
        per_proj[yn] = dict(us=round(us, 3), GBs=round(2 * Un * dout / (us * 1e-6) / 1e9, 1), K=K, rows_read=Un,
                            d_out=dout)

    # ---- dense comparators on the same GPU: the library's dense mat-vec over the same fused
    # weights (4 launches), and the vendor BLAS through torch (harness-side only)
    xin = dict(qkv=trace["h1"], o=trace["h2"], gu=trace["h3"], down=trace["h4"])

    def dense_all():
        for s in sets:
            for wn, hn, inn, yn, K, dout in proj:
                api.dense_gemv(s[wn], xin[yn], ys[yn], shape.dtype, ws)

    dense_layer_us = event_time_us(dense_all, nsets, reps)
    dense_bytes_layer = 2 * (d * d_qkv + d_q * d + d * 2 * d_ff + d_ff * d)
    lin_w = [[gauss(dout, din) for (din, dout) in ((d, d_qkv), (d_q, d), (d, 2 * d_ff), (d_ff, d))]
             for _ in range(nsets)]
    lin_x = [xin["qkv"], xin["o"], xin["gu"], xin["down"]]

    def blas_all():
        for wset in lin_w:
            for w_, x_ in zip(wset, lin_x):
                torch.nn.functional.linear(x_, w_)

    try:
        blas_layer_us = event_time_us(blas_all, nsets, reps)
    except Exception as e:  # vendor BLAS not capturable on this stack: time it eagerly
        log(f"BLAS graph capture failed ({e}); timing eagerly")
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        blas_all()
        e0.record()
        for _ in range(reps):
            blas_all()
        e1.record()
        torch.cuda.synchronize()
        blas_layer_us = e0.elapsed_time(e1) * 1e3 / (reps * nsets)
    del lin_w
    sparse_proj_layer_us = standalone_launch_us * 4      # the 4 projections with given indices, nothing else
    best_dense = min(dense_layer_us, blas_layer_us)

    # ---- CPU baseline: the fp64 oracle's layer on the host cores, bounded sample
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import larosa_oracle as O
        from threadpoolctl import threadpool_info

        def bits(t):
            return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)

        def vals(t):
            return O.decode16(bits(t), shape.dtype).astype(np.float32)

        s0 = sets[0]
        rot = (dict(shortcut_attn=vals(s0["shortcut_attn"]).astype(np.float64),
                    shortcut_mlp=vals(s0["shortcut_mlp"]).astype(np.float64)) if shortcut_form else
               dict(Q_attn=vals(s0["Q_attn"]).astype(np.float64), Q_mlp=vals(s0["Q_mlp"]).astype(np.float64)))
        OL = O.Layer(d, d_q, d_kv, d_ff, shape.head_dim, K1, K2, K3, K4, Wqkv=vals(s0["Wqkv"]), Wo=vals(s0["Wo"]),
                     Wgu=vals(s0["Wgu"]), Wdown=vals(s0["Wdown"]), rms_eps=synth.RMS_EPS, dtype=shape.dtype, **rot)
        xs = O.decode16(bits(x), shape.dtype)
        t0 = time.perf_counter()
        r = O.layer_forward(OL, xs[0])
        one = time.perf_counter() - t0
        n_tok = int(max(1, min(64, args.cpu_seconds / max(one, 1e-3))))
        t0 = time.perf_counter()
        for _ in range(n_tok):
            r = O.layer_forward(OL, xs[0])
        cpu_us = (time.perf_counter() - t0) / n_tok * 1e6
        threads = max([i.get("num_threads", 1) for i in threadpool_info()] or [1])
        # parity spot check of the timed configuration against the oracle (indices of the first Top-K)
        idx_equal = bool(np.array_equal(trace["idx1"][0].cpu().numpy(), O.topk_indices(bits(trace["h1"])[0], K1)))
        cpu = dict(value=round(cpu_us, 1), unit="us per decoder layer", cores=int(threads), kind="oracle",
                   sample=f"{n_tok} passes of the fp64 oracle layer_forward over one token of the same layer "
                          f"(numpy, {threads} BLAS threads, {os.cpu_count()} host cpus)",
                   idx1_matches_oracle=idx_equal)

    all_bytes_layer = sel_bytes_layer + 2 * 2 * d * d       # + the two d x d rotations / shortcut adapters
    traffic, traffic_src = (measured_traffic((args.config, B, p, args.form)) if args.alpha == "1.0,1.0" else (None, None))
    sel_GBs = sel_bytes_layer / (graph_us * 1e-6) / 1e9
    all_GBs = all_bytes_layer / (graph_us * 1e-6) / 1e9
    report = {
        "metric": "us_per_decoder_layer",
        "value": round(graph_us, 3),
        "unit": "us",
        "n_gpus": 1,
        "steps": graph_steps,
        "warmup": args.warmup,
        "ms_per_step": round(graph_us / 1e3, 6),
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": shape.dtype,
        "data": "synthetic",
        "config": {"workload": cfg["workload"] if args.config == 1 and p == 0.4 and B == 1 and args.alpha == "1.0,1.0"
                   else f"{cfg['workload']}; batch {B}; sparsity {p}; alpha1,alpha3 = {args.alpha}",
                   "form": ("rotations absorbed into the weights, residual adapters Q_attn^T Q_mlp and Q_mlp^T Q_attn "
                            "on the two shortcuts (each shares the launch of its block's first projection at batch 1)"
                            if shortcut_form else "explicit rotation mat-vecs in front of q|k|v and gate|up"),
                   "shape": shape.name, "batch": B, "sparsity": p, "K": [K1, K2, K3, K4], "union_rows": U,
                   "weight_sets": nsets,
                   "launch": f"one HIP graph of {K_steps} larosa_layer_forward steps (weight set i mod {nsets}), replayed "
                             f"{replays} times; value = median replay"},
        "roofline": {"bound": "hbm", "achieved": round(achieved_gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(achieved_gbs / HBM_PEAK_GBS, 4),
                     "traffic": traffic,
                     "traffic_source": (None if traffic_src is None else
                                        f"{traffic_src} (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this script, "
                                        "scaled by a 1 GiB copy; not collected in this run)"),
                     # the same step time against the two byte counts of the whole layer
                     "selected_row_bytes_per_layer": sel_bytes_layer,
                     "achieved_selected_rows": round(sel_GBs, 1), "frac_selected_rows": round(sel_GBs / HBM_PEAK_GBS, 4),
                     "achieved_all_bytes": round(all_GBs, 1), "frac_all_bytes": round(all_GBs / HBM_PEAK_GBS, 4),
                     "kernel": (("fused_topk_gemv_kernel: the 4 Top-K + column-sparse projections of a layer step "
                                 + ("(two of them carry a residual adapter in the same launch; its bytes are counted), "
                                    if shortcut_form else ", ")
                                 + (("timed by HIP events around graph replays of the step (= exactly these 4 launches)"
                                     if shape.d_ff <= 16384 else
                                     "timed by HIP events around graph replays of the step; the MLP vector is wider than "
                                     "16384, so its Top-K runs as a kernel of its own in front of the down projection "
                                     "(5 launches; the step time is still divided by the 4 projections)")
                                    if shortcut_form else "timed by HIP events recorded inside larosa_layer_forward"))
                                if B == 1 else
                                "skinny_mfma_kernel: the 4 batched projections of a layer (union of kept rows)"),
                     "bytes_per_launch": sel_bytes_launch, "us_per_launch": round(sparse_launch_us, 3)},
        "cpu_baseline": cpu,
        "extra": {
            "eager_us_per_layer": round(eager_us, 2),
            ("explicit_rotation_form_us_per_layer" if shortcut_form else "shortcut_form_us_per_layer"):
                round(other_us, 2),
            "graph_us_per_layer": round(graph_us, 2),
            "graph_replay_us_per_layer": {k: (round(v, 3) if k != "n" else v) for k, v in st_graph.items()},
            "graph_replays_wall_s": round(graph_wall_s, 3),
            "tokens_per_s_32_layers": round(1e6 / (graph_us * 32), 1),
            "selected_row_bytes_per_layer": sel_bytes_layer,
            "layer_GBs_on_selected_rows": round(sel_bytes_layer / (graph_us * 1e-6) / 1e9, 1),
            "layer_GBs_on_all_bytes": round(all_bytes_layer / (graph_us * 1e-6) / 1e9, 1),
            "sparse_projections_us_per_layer": round(sparse_proj_layer_us, 2),
            "stage_us_in_layer": None if stage_us is None else {k: round(v, 2) for k, v in stage_us.items()},
            "stage_us_note": "eager launches, each interval includes one HIP event record (an empty stage reads ~5 us)",
            "eager_step_us_percentiles": step_pct,      # per-step HIP events (first to last kernel of a step)
            "standalone_sparse_gemv_us_per_launch": round(standalone_launch_us, 3),
            "per_projection": per_proj,
            "dense_gemv_us_per_layer": round(dense_layer_us, 2),
            "dense_gemv_GBs": round(dense_bytes_layer / (dense_layer_us * 1e-6) / 1e9, 1),
            "blas_linear_us_per_layer": round(blas_layer_us, 2),
            "speedup_sparse_projections_vs_best_dense": round(best_dense / sparse_proj_layer_us, 3),
            "speedup_whole_layer_vs_best_dense_projections": round(best_dense / graph_us, 3),
        },
    }
    if args.detail:
        os.makedirs(os.path.dirname(os.path.abspath(args.detail)), exist_ok=True)
        with open(args.detail, "w") as f:
            json.dump(report, f, indent=1)
    print(json.dumps(report), flush=True)


if __name__ == "__main__":
    main()
