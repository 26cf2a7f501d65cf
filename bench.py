#!/usr/bin/env python3
"""Benchmark of the active-weight decode hot path on one MI355X.

A step is one batch-1 decode of one token through the whole 7B-shape stack (32 layers,
d_model 4096, FFN 11008, 32 heads, 512-token KV cache) at 50 % activation sparsity: four
selections and four gathered GEMVs per layer plus norm, rotary attention and SwiGLU glue,
replayed as one HIP graph.  Weights, caches and the input state are synthetic (seeded) and
already resident in HBM when the timed region starts.

Prints ONE JSON line: decode tokens/s (value), the active-weight GB/s it corresponds to,
the HBM roofline of the dominant kernel (the gate|up gathered GEMV) measured live with
events on the library's stream, and the CPU oracle timed on a bounded sample.
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

HBM_PEAK_GBPS = 8000.0          # MI355X published HBM3E bandwidth
# HBM bytes per launch of the dominant kernel (fused gate|up GEMV, 7B shape, 50 %).  Counters
# cannot be read from inside this process; the figure comes from the two rocprofv3 --pmc runs
# of this very command that profiles/gateup_7b_f16_sp50_pmc_traffic.md summarises (file, kernel
# name and launch shape are repeated in the output so that a stale figure shows):
# FETCH_SIZE KiB x fetch factor + WRITE_SIZE KiB x write factor, the factors being what the same
# counters read for a plain 256 MiB device copy of known size.
TRAFFIC = {("7b", "f16", 50): {"fetch_KiB": 44360.0, "fetch_factor": 2.000, "write_KiB": 409.8, "write_factor": 1.000,
                               "kernel": "gemv_f16_kernel<64, 8, 16, false, 5> grid 43x4",
                               "source": "profiles/gateup_7b_f16_sp50_pmc_traffic.md"}}


def keep_count(n: int, sp: int) -> int:
    return n - (sp * n) // 100


def gemv_bytes(k: int, out: int, residual: bool = False) -> int:
    """Algorithmic bytes of one gathered GEMV: k active rows of out fp16 weights, their
    (x, idx) pairs, and the fp16 result (plus the residual it adds)."""
    return k * (out * 2 + 6) + out * 2 + (out * 2 if residual else 0)


def union_bench(args, S, B, torch, np) -> int:
    """Small-batch decode GEMVs of one layer over the union of the tokens' active sets."""
    shape = S.MODEL_SHAPES[args.shape]
    Bt, sp = args.union, args.sparsity
    d, f, hd = shape.d_model, shape.d_ffn, shape.head_dim
    ops = [("qkv", d, shape.qkv_out), ("o", shape.n_heads * hd, d), ("gateup", d, 2 * f), ("down", f, d)]
    ctx = B.Context(0)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(0)
    mats, Xs, idxs = [], [], []
    for name, n_in, out in ops:
        W = (torch.randn((n_in, out), generator=gen, device="cuda", dtype=torch.float32) * 0.02).to(torch.float16)
        sc = S.channel_scales(0, n_in, shape.name, name)          # shared by the tokens of the batch
        X = np.stack([S.activation(0, sc, shape.name, name, b) for b in range(Bt)])
        Xd = torch.from_numpy(X).cuda()
        k = keep_count(n_in, sp)
        idx_b = torch.empty((Bt, k), dtype=torch.int32, device="cuda")
        torch.cuda.synchronize()
        for b in range(Bt):
            ctx.select_topk(Xd[b], k, idx_b[b])
        ctx.synchronize()
        mats.append(W); Xs.append(Xd); idxs.append(idx_b)

    def step():
        outs = []
        for W, Xd, idx_b in zip(mats, Xs, idxs):
            outs.append(ctx.sparse_gemv_union_f16(W, Xd, idx_b))
        return outs

    outs = step()
    ctx.synchronize()
    union_frac = [float(o[2].item()) / n_in for o, (_, n_in, _) in zip(outs, ops)]
    union_bytes = sum(int(o[2].item()) * out * 2 for o, (_, _, out) in zip(outs, ops))
    for _ in range(args.warmup):
        step()
    ctx.synchronize()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    ctx.synchronize()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    # the widest operator alone, with events
    W, Xd, idx_b = mats[2], Xs[2], idxs[2]
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(ctx.stream)
    for _ in range(20):
        ctx.sparse_gemv_union_f16(W, Xd, idx_b)
    e1.record(ctx.stream)
    ctx.synchronize()
    us = e0.elapsed_time(e1) * 1e3 / 20
    alg = int(outs[2][2].item()) * ops[2][2] * 2 + Bt * (ops[2][1] * 2 + ops[2][1] // 8) + Bt * ops[2][2] * 2
    achieved = alg / (us * 1e-6) / 1e9
    out = {
        "metric": "active-weight GB/s (% of HBM peak) + decode tokens/s, 7B-shape @50% sparsity",
        "value": round(Bt * args.steps / dt, 2), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(dt / args.steps * 1e3, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f16", "data": "synthetic",
        "config": {"workload": f"{args.shape}-shape layer, union small-batch GEMVs (qkv, o, gate|up, down), "
                               f"B={Bt} tokens, {sp}% sparsity per token, GEMVs only",
                   "B": Bt, "union_fraction_of_channels": [round(u, 4) for u in union_frac]},
        "union_weight_bytes_per_step": union_bytes,
        "union_weight_GBps": round(union_bytes * args.steps / dt / 1e9, 1),
        "roofline": {"bound": "hbm", "kernel": "union_scan_kernel + union_place_kernel + gemv_union_kernel (gate|up)",
                     "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": None,
                     "bytes_per_launch": alg, "us_per_launch": round(us, 3), "launches": 20},
        "cpu_baseline": None,
    }
    print(json.dumps(out))
    ctx.close()
    return 0


def batch_layer_bench(args, S, B, M, torch, np) -> int:
    """--batch-layer B: one whole decoder layer of --shape for B tokens decoded together
    (af_decode_layer_batch): per-token selection, union GEMVs, per-token attention; each token has
    its own KV cache and length."""
    shape = S.MODEL_SHAPES[args.shape]
    Bt, sp = args.batch_layer, args.sparsity
    widths = (shape.d_model, shape.n_heads * shape.head_dim, shape.d_model, shape.d_ffn)
    outs = (shape.qkv_out, shape.d_model, 2 * shape.d_ffn, shape.d_model)
    ks = tuple(keep_count(n, sp) for n in widths)
    kv_cap = args.kv_len + 16
    ctx = B.Context(0)
    w = S.device_layer_weights(0, shape, 0)
    lay = M.DeviceLayer(ctx, shape, w)
    del w
    cfg = M.layer_cfg(shape)
    sc = S.channel_scales(0, shape.d_model, shape.name)          # shared by the tokens of the batch
    H = torch.from_numpy(np.stack([S.activation(0, sc, "hidden", b) for b in range(Bt)])).cuda()
    Hout = torch.zeros_like(H)
    kv_lens = [max(1, args.kv_len - 37 * b) for b in range(Bt)]   # every token at its own length
    caches = [S.device_kv_cache(0, shape, b, kv_cap, kv_lens[b]) for b in range(Bt)]
    Ks, Vs = [c[0] for c in caches], [c[1] for c in caches]
    idx = [torch.zeros((Bt, n), dtype=torch.int32, device="cuda") for n in widths]
    cnt = [torch.zeros(Bt, dtype=torch.int32, device="cuda") for _ in widths]
    sets = B.IdxSets()
    for p in range(4):
        sets.idx[p] = idx[p].data_ptr()
        sets.count[p] = cnt[p].data_ptr()
    un = torch.zeros(4, dtype=torch.int32, device="cuda")
    sel = M.select_cfg(B.AF_SEL_TOPK, ks)
    torch.cuda.synchronize()
    run = lambda: ctx.decode_layer_batch(cfg, lay.struct(), H, Hout, Ks, Vs, kv_lens, kv_cap, kv_lens, sel, sets, un)
    run()
    ctx.synchronize()
    union_rows = [int(v) for v in un.cpu().numpy()]
    ctx.capture_begin()
    run()
    graph = ctx.capture_end()
    for _ in range(args.warmup):
        ctx.graph_launch(graph)
    ctx.synchronize()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        ctx.graph_launch(graph)
    ctx.synchronize()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ctx.graph_destroy(graph)
    # the same tokens one after the other through the single-token layer, for comparison
    one = M.DeviceStack(ctx, shape, [lay], [(Ks[0], Vs[0])], kv_cap)
    h1 = H[0].contiguous()
    one.layer(0, h1, one.hidden_out, kv_lens[0], kv_lens[0], sel)
    ctx.synchronize()
    ctx.capture_begin()
    one.layer(0, h1, one.hidden_out, kv_lens[0], kv_lens[0], sel)
    g1 = ctx.capture_end()
    for _ in range(5):
        ctx.graph_launch(g1)
    ctx.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        ctx.graph_launch(g1)
    ctx.synchronize()
    dt1 = time.perf_counter() - t0
    ctx.graph_destroy(g1)
    union_bytes = sum(r * o * 2 for r, o in zip(union_rows, outs))
    ms = dt / args.steps * 1e3
    out = {
        "metric": "active-weight GB/s (% of HBM peak) + decode tokens/s, 7B-shape @50% sparsity",
        "value": round(Bt * args.steps / dt, 2), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f16", "data": "synthetic",
        "config": {"workload": f"{args.shape}-shape decoder layer, B={Bt} tokens decoded together "
                               f"(af_decode_layer_batch: per-token top-k at {sp}% sparsity, union GEMVs, "
                               f"per-token attention over own KV caches of {kv_lens} tokens)",
                   "B": Bt, "k": list(ks), "graph": True,
                   "union_fraction_of_channels": [round(r / n, 4) for r, n in zip(union_rows, widths)]},
        "union_weight_bytes_per_step": union_bytes,
        "union_weight_GBps": round(union_bytes / (ms * 1e-3) / 1e9, 1),
        "union_weight_frac_of_hbm_peak": round(union_bytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
        "single_token_layer_ms": round(dt1 / args.steps * 1e3, 4),
        "speedup_over_token_by_token": round(Bt * dt1 / dt, 2),
        "roofline": None, "cpu_baseline": None,
    }
    print(json.dumps(out))
    ctx.close()
    return 0


def config0_bench(args, S, B, torch, np) -> int:
    """--config0: one 2048x2048 fp16 layer, top-k 50 % (k = 1024), selection fused into the GEMV.
    4 MB of active weights fit every cache, so the launch is timed cold (rotating through 160
    distinct matrices, 1.3 GB) and warm (one matrix) separately; only cold counts against HBM."""
    n = out = 2048
    k = keep_count(n, 50)
    ctx = B.Context(0)
    x = torch.from_numpy(S.activation(0, S.channel_scales(0, n, "config0"), "config0", 0)).cuda()
    gen = torch.Generator(device="cuda"); gen.manual_seed(0)
    mats = [(torch.randn((n, out), generator=gen, device="cuda") * 0.02).to(torch.float16) for _ in range(160)]
    y = torch.empty(out, dtype=torch.float16, device="cuda")
    idx = torch.empty(n, dtype=torch.int32, device="cuda"); cnt = torch.empty(1, dtype=torch.int32, device="cuda")
    torch.cuda.synchronize()
    call = lambda W: ctx.select_gemv_f16(W, x, sel_mode=B.AF_SEL_TOPK, k=k, idx_out=idx, count_out=cnt, y=y)

    def timed(seq, reps):
        for W in seq[:8]:
            call(W)
        ctx.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(ctx.stream)
        for _ in range(reps):
            for W in seq:
                call(W)
        e1.record(ctx.stream)
        ctx.synchronize()
        return e0.elapsed_time(e1) * 1e3 / (reps * len(seq))

    cold_us = timed(mats, max(1, args.steps // 40))
    warm_us = timed(mats[:1] * 40, max(1, args.steps // 10))
    alg = gemv_bytes(k, out) + n * 2
    out_j = {
        "metric": "active-weight GB/s (% of HBM peak) + decode tokens/s, 7B-shape @50% sparsity",
        "value": round(1e6 / cold_us, 1), "unit": "launches/s", "n_gpus": 1, "steps": args.steps, "warmup": 8,
        "ms_per_step": round(cold_us * 1e-3, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16", "data": "synthetic",
        "config": {"workload": "config 0: one 2048x2048 fp16 layer, top-k 50 % fused into the GEMV, batch 1"},
        "cold_us_per_launch": round(cold_us, 3), "warm_us_per_launch": round(warm_us, 3),
        "roofline": {"bound": "hbm", "kernel": "gemv_f16_kernel<16, 8, 16> (top-k + gathered GEMV, cold matrices)",
                     "achieved": round(alg / (cold_us * 1e-6) / 1e9, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(alg / (cold_us * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4), "traffic": None,
                     "bytes_per_launch": alg, "us_per_launch": round(cold_us, 3)},
        "cpu_baseline": None,
    }
    print(json.dumps(out_j))
    ctx.close()
    return 0


def moe_bench(args, S, B, M, torch, np) -> int:
    """--shape mixtral: decoder blocks with a mixture-of-experts feed-forward half (8 experts,
    top-2).  Like the paper's technique evaluation it runs a slice of the model (8 layers by
    default); tokens/s is the rate of that slice."""
    shape = S.MODEL_SHAPES[args.shape]
    L = args.layers or 8
    sp, top = args.sparsity, 2
    kv_len, kv_cap = args.kv_len, args.kv_len + 16
    d, f = shape.d_model, shape.d_ffn
    widths = (d, shape.n_heads * shape.head_dim, d, f)
    ks = tuple(keep_count(n, sp) for n in widths)
    kind = {"f16": B.AF_W_F16, "q4": B.AF_W_Q4G32, "q4cl": B.AF_W_Q4CL}[args.weights]
    ctx = B.Context(0)
    t_build = time.time()
    layers, kv = [], []
    for l in range(L):
        w = S.device_moe_layer_weights(0, shape, l)
        layers.append(M.DeviceMoeLayer(ctx, shape, w, top, kind))
        kv.append(S.device_kv_cache(0, shape, l, kv_cap, kv_len))
        del w
    hin = torch.from_numpy(S.activation(0, S.channel_scales(0, d, shape.name), "hidden", 0)).cuda()
    bufs = [torch.zeros_like(hin), torch.zeros_like(hin)]
    torch.cuda.synchronize()
    t_build = time.time() - t_build
    sel_topk = M.select_cfg(B.AF_SEL_TOPK, ks)
    sels = [sel_topk] * L
    keep_frac = None
    if args.select == "threshold":
        # calibration as in the dense-FFN stack: pool the operator inputs of a top-k run over
        # --calib-tokens tokens; the down point pools the inputs of all chosen experts
        hists = [[ctx.calib_hist() for _ in range(4)] for _ in range(L)]
        torch.cuda.synchronize()
        scales = S.channel_scales(0, d, shape.name)
        taps = ((0, d), (2, widths[1]), (4, d), (6, top * f))
        for tok in range(1, args.calib_tokens + 1):
            cur = torch.from_numpy(S.activation(0, scales, "hidden", tok)).cuda()
            torch.cuda.synchronize()
            for l in range(L):
                layers[l].run(cur, bufs[l & 1], kv[l][0], kv[l][1], kv_len, kv_cap, kv_len, sel_topk)
                ctx.synchronize()
                for p_, (tap, n_) in enumerate(taps):
                    ctx.calib_accumulate(ctx.layer_tap(tap, n_), hists[l][p_])
                cur = bufs[l & 1]
            ctx.synchronize()
        t_dev = [[ctx.calib_thresholds(hists[l][p_], [sp]) for p_ in range(4)] for l in range(L)]
        ctx.synchronize()
        thr = [[float(t_dev[l][p_].item()) for p_ in range(4)] for l in range(L)]
        cur = hin
        kept = []
        for l in range(L):   # kept fractions on the bench token (sets written)
            layers[l].run(cur, bufs[l & 1], kv[l][0], kv[l][1], kv_len, kv_cap, kv_len,
                          M.select_cfg(B.AF_SEL_THRESHOLD, t=thr[l]))
            ctx.synchronize()
            c = [int(layers[l].count[p_].item()) for p_ in range(3 + top)]
            kept.append([c[0], c[1], c[2], sum(c[3:]) / top])
            cur = bufs[l & 1]
        keep_frac = [round(sum(k_[p_] for k_ in kept) / (L * widths[p_]), 4) for p_ in range(4)]
        sels = [M.select_cfg(B.AF_SEL_THRESHOLD, t=thr[l], flags=B.AF_SEL_SKIP_SETS) for l in range(L)]

    def run():
        cur = hin
        for l in range(L):
            layers[l].run(cur, bufs[l & 1], kv[l][0], kv[l][1], kv_len, kv_cap, kv_len, sels[l])
            cur = bufs[l & 1]

    run()
    ctx.synchronize()
    experts = [layers[l].experts.cpu().tolist() for l in range(L)]
    ctx.capture_begin()
    run()
    graph = ctx.capture_end()
    for _ in range(args.warmup):
        ctx.graph_launch(graph)
    ctx.synchronize()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        ctx.graph_launch(graph)
    ctx.synchronize()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    tok_s = args.steps / dt
    outs = (shape.qkv_out, d, top * 2 * f, d)
    mult = (1, 1, 1, top)                                   # the down projection runs once per slot
    bpw = 2.0 if kind == B.AF_W_F16 else 0.5
    rows = ks if keep_frac is None else [keep_frac[p] * widths[p] for p in range(4)]   # mean active channels
    per_layer = sum(mult[p] * rows[p] * outs[p] for p in range(4)) * bpw
    if kind == B.AF_W_Q4G32:
        per_layer += sum(mult[p] * (widths[p] // 32) * outs[p] for p in range(4)) * 2
    elif kind == B.AF_W_Q4CL:
        per_layer += sum(mult[p] * rows[p] * (outs[p] // 32) for p in range(4)) * 2
    active_bytes = per_layer * L
    sel_note = "" if keep_frac is None else f", threshold selection calibrated on {args.calib_tokens} tokens (no index lists)"

    roofline = None
    if kind != B.AF_W_F16:
        out = {
            "metric": "active-weight GB/s (% of HBM peak) + decode tokens/s, 7B-shape @50% sparsity",
            "value": round(tok_s, 2), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
            "ms_per_step": round(dt / args.steps * 1e3, 4), "higher_is_better": True, "scaling": "weak",
            "vs_baseline": None, "dtype": "int4", "data": "synthetic",
            "config": {"workload": f"{args.shape}-shape mixture-of-experts blocks ({shape.n_experts} experts, top-{top}), "
                                   f"{L} layers, batch-1 decode, {args.weights} weights, {sp}% sparsity at "
                                   f"qkv/o/gate-up/down, {kv_len}-token KV cache{sel_note}", "layers": L, "d_model": d,
                       "d_ffn": f, "k": list(ks), "graph": True, "experts_chosen_layer0": experts[0],
                       "kept_fraction_by_point": keep_frac},
            "active_weight_bytes_per_token": int(active_bytes),
            "active_weight_GBps": round(active_bytes * tok_s / 1e9, 1),
            "active_weight_frac_of_hbm_peak": round(active_bytes * tok_s / 1e9 / HBM_PEAK_GBPS, 4),
            "ms_per_layer": round(dt / args.steps * 1e3 / L, 4), "build_s": round(t_build, 1),
            "roofline": None, "cpu_baseline": None,
        }
        print(json.dumps(out))
        ctx.graph_destroy(graph)
        ctx.close()
        return 0

    # dominant kernel: gate|up of the two chosen experts in one launch (rmsnorm + top-k + GEMV
    # over device-selected matrices), rotating through the layers' expert banks
    h2 = torch.from_numpy(S.activation(0, S.channel_scales(0, d, "roof"), "roof", 0)).cuda()
    y2 = torch.empty(top * 2 * f, dtype=torch.float16, device="cuda")
    x2 = torch.empty(d, dtype=torch.float16, device="cuda")
    idx2 = torch.empty(d, dtype=torch.int32, device="cuda"); cnt2 = torch.empty(1, dtype=torch.int32, device="cuda")
    pairs = [torch.tensor([(2 * i) % shape.n_experts, (2 * i + 1) % shape.n_experts], dtype=torch.int32, device="cuda")
             for i in range(4)]
    torch.cuda.synchronize()

    def gateup(l, i):
        lay = layers[l]
        ctx.select_gemv_experts_f16(lay.Wgateup, pairs[i % 4], top, h2, producer=B.AF_PRO_RMSNORM,
                                    gain=lay.g_ffn, eps=1e-5, sel_mode=B.AF_SEL_TOPK, k=ks[2], x_out=x2,
                                    idx_out=idx2, count_out=cnt2, y=y2)

    for l in range(L):
        gateup(l, l)
    ctx.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    reps = 4
    e0.record(ctx.stream)
    for r in range(reps):
        for l in range(L):
            gateup(l, r)
    e1.record(ctx.stream)
    ctx.synchronize()
    us = e0.elapsed_time(e1) * 1e3 / (reps * L)
    alg = ks[2] * (top * 2 * f * 2 + 6) + top * 2 * f * 2 + 2 * d * 2
    achieved = alg / (us * 1e-6) / 1e9
    out = {
        "metric": "active-weight GB/s (% of HBM peak) + decode tokens/s, 7B-shape @50% sparsity",
        "value": round(tok_s, 2), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(dt / args.steps * 1e3, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f16", "data": "synthetic",
        "config": {"workload": f"{args.shape}-shape mixture-of-experts blocks ({shape.n_experts} experts, top-{top}), "
                               f"{L} layers, batch-1 decode, f16 weights, {sp}% sparsity at qkv/o/gate-up/down, "
                               f"{kv_len}-token KV cache{sel_note}", "layers": L, "d_model": d, "d_ffn": f, "k": list(ks),
                   "graph": True, "experts_chosen_layer0": experts[0], "kept_fraction_by_point": keep_frac},
        "active_weight_bytes_per_token": int(active_bytes),
        "active_weight_GBps": round(active_bytes * tok_s / 1e9, 1),
        "active_weight_frac_of_hbm_peak": round(active_bytes * tok_s / 1e9 / HBM_PEAK_GBPS, 4),
        "ms_per_layer": round(dt / args.steps * 1e3 / L, 4),
        "build_s": round(t_build, 1),
        "roofline": {"bound": "hbm", "kernel": "gemv_f16_kernel<64, 8, 16> (gate|up of both chosen experts: rmsnorm + top-k + gathered GEMV)",
                     "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": None, "bytes_per_launch": alg,
                     "us_per_launch": round(us, 3), "launches": reps * L},
        "cpu_baseline": None,
    }
    print(json.dumps(out))
    ctx.graph_destroy(graph)
    ctx.close()
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--shape", default="7b")
    ap.add_argument("--layers", type=int, default=0, help="0 = all layers of the shape")
    ap.add_argument("--sparsity", type=int, default=50)
    ap.add_argument("--weights", default="f16", choices=["f16", "q4", "q4cl"],
                    help="q4: 4-bit, groups of 32 input channels; q4cl: 4-bit, groups inside a channel's row")
    ap.add_argument("--group", type=int, default=1, help="cross-layer reuse group (1 = none)")
    ap.add_argument("--reuse-points", type=lambda s: int(s, 0), default=0b1111)
    ap.add_argument("--select", default="topk", choices=["topk", "threshold"],
                    help="threshold: per-operator thresholds calibrated for --sparsity on "
                         "--calib-tokens synthetic tokens, selection fused into the GEMVs")
    ap.add_argument("--calib-tokens", type=int, default=8)
    ap.add_argument("--lfu-tokens", type=int, default=0, metavar="T",
                    help="also decode T synthetic tokens (untimed) and feed the index sets of layer 0 and "
                         "the middle layer to the weight-cache simulator at cache fractions 25/50/75 %%")
    ap.add_argument("--kv-len", type=int, default=512)
    ap.add_argument("--overlap", action="store_true",
                    help="with --group > 1: report the overlap of the reused sets with each layer's own selection")
    ap.add_argument("--union", type=int, default=0, metavar="B",
                    help="small-batch union GEMV over the four operators of one layer of --shape (e.g. 70b) with B tokens")
    ap.add_argument("--batch-layer", type=int, default=0, metavar="B",
                    help="one whole decoder layer of --shape for B tokens decoded together (af_decode_layer_batch)")
    ap.add_argument("--config0", action="store_true",
                    help="the single 2048x2048 layer of BASELINE config 0, cold and warm")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="also run three plain 256 MiB device copies (float4 per lane), the known-size "
                         "reference the FETCH_SIZE / WRITE_SIZE counters are scaled by")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-threshold-leg", action="store_true",
                    help="skip the second measurement (threshold form of the selection) of a top-k run")
    ap.add_argument("--no-graph", action="store_true")
    ap.add_argument("--layer-kernel", action="store_true",
                    help="one launch per layer (AF_OPT_LAYER_KERNEL) instead of one per operator")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (no sharding, no collectives); "
              "run with --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import synth_inputs as S
    from paper_2504_08378_amd import binding as B
    from paper_2504_08378_amd import model as M

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        return 2

    if args.config0:
        return config0_bench(args, S, B, torch, np)
    if args.union:
        return union_bench(args, S, B, torch, np)
    if args.batch_layer:
        return batch_layer_bench(args, S, B, M, torch, np)
    if S.MODEL_SHAPES[args.shape].n_experts:
        return moe_bench(args, S, B, M, torch, np)
    if args.overlap and args.select != "topk":
        print("bench.py: --overlap compares top-k sets; use it with --select topk", file=sys.stderr)
        return 2

    base = S.MODEL_SHAPES[args.shape]
    L = args.layers or base.n_layers
    shape = base
    sp = args.sparsity
    kind = {"f16": B.AF_W_F16, "q4": B.AF_W_Q4G32, "q4cl": B.AF_W_Q4CL}[args.weights]
    kv_len, kv_cap = args.kv_len, args.kv_len + 16
    widths = (shape.d_model, shape.n_heads * shape.head_dim, shape.d_model, shape.d_ffn)
    ks = tuple(keep_count(n, sp) for n in widths)

    ctx = B.Context(0)
    if args.layer_kernel:
        ctx.set_option(B.AF_OPT_LAYER_KERNEL, 1)
    t_build = time.time()
    layers, kv, host_layer0 = [], [], None
    for l in range(L):
        w = S.device_layer_weights(0, shape, l)
        if l == 0 and not args.no_cpu_baseline:
            host_layer0 = {k: v.cpu().numpy() for k, v in w.items()}
        layers.append(M.DeviceLayer(ctx, shape, w, kind))
        kv.append(S.device_kv_cache(0, shape, l, kv_cap, kv_len))
        del w
    st = M.DeviceStack(ctx, shape, layers, kv, kv_cap, kind)
    h_host = S.activation(0, S.channel_scales(0, shape.d_model, shape.name), "hidden", 0)
    hin = torch.from_numpy(h_host).cuda()
    torch.cuda.synchronize()
    t_build = time.time() - t_build

    if args.pmc_calibration:
        ca = torch.zeros(64 * 1024 * 1024, dtype=torch.float32, device="cuda")
        cb = torch.empty_like(ca)
        for _ in range(3):
            cb.copy_(ca)
        torch.cuda.synchronize()
        del ca, cb

    sel = M.select_cfg(B.AF_SEL_TOPK, ks)
    keep_frac = None
    def threshold_selection():
        # Calibration (untimed): decode --calib-tokens synthetic tokens layer by layer with
        # top-k selection at the target sparsity, pooling the magnitudes of every operator's
        # input; the thresholds of one operator come from its pooled histogram.
        sel_k = M.select_cfg(B.AF_SEL_TOPK, ks)
        hists = [[ctx.calib_hist() for _ in range(4)] for _ in range(L)]
        torch.cuda.synchronize()
        scales = S.channel_scales(0, shape.d_model, shape.name)
        bufs = [torch.zeros_like(hin), torch.zeros_like(hin)]
        for tok in range(1, args.calib_tokens + 1):
            cur = torch.from_numpy(S.activation(0, scales, "hidden", tok)).cuda()
            torch.cuda.synchronize()
            for l in range(L):
                st.layer(l, cur, bufs[l & 1], kv_len, kv_len, sel_k)
                ctx.calib_accumulate_layer(st.cfg, hists[l])
                cur = bufs[l & 1]
            ctx.synchronize()
        t_dev = [[ctx.calib_thresholds(hists[l][p], [sp]) for p in range(4)] for l in range(L)]
        ctx.synchronize()            # the library's stream, not torch's: .item() would not wait for it
        thr = [[float(t_dev[l][p].item()) for p in range(4)] for l in range(L)]
        # kept fraction on the bench token (eager, sets written), then the timed configuration
        sel_sets = [M.select_cfg(B.AF_SEL_THRESHOLD, t=thr[l]) for l in range(L)]
        st.run(hin, kv_len, kv_len, sel_sets, group=args.group, reuse_points=args.reuse_points)
        ctx.synchronize()
        src_of = lambda l, p: l - l % args.group if (args.group > 1 and args.reuse_points >> p & 1) else l
        kept_ = [[int(st.sets[src_of(l, p)].count[p].item()) for p in range(4)] for l in range(L)]
        keep_frac_ = [round(sum(kept_[l][p] for l in range(L)) / (L * widths[p]), 4) for p in range(4)]
        sel_ = [M.select_cfg(B.AF_SEL_THRESHOLD, t=thr[l], flags=B.AF_SEL_SKIP_SETS) for l in range(L)]
        return sel_, keep_frac_, kept_, thr

    def weight_bytes(rows_):
        """Active weight bytes of one token (the four operators of every layer)."""
        bpw_ = 2.0 if kind == B.AF_W_F16 else 0.5
        outs_ = (shape.qkv_out, shape.d_model, 2 * shape.d_ffn, shape.d_model)
        ab = sum(rows_[l][p] * outs_[p] for l in range(L) for p in range(4)) * bpw_
        if kind == B.AF_W_Q4G32:   # every scale row is touched at these sparsities
            ab += L * sum(widths[p] // 32 * outs_[p] for p in range(4)) * 2
        elif kind == B.AF_W_Q4CL:  # a channel's scales travel with its nibbles
            ab += sum(rows_[l][p] * (outs_[p] // 32) * 2 for l in range(L) for p in range(4))
        return ab

    if args.select == "threshold":
        sel, keep_frac, kept, thr = threshold_selection()
    run = lambda: st.run(hin, kv_len, kv_len, sel, group=args.group, reuse_points=args.reuse_points)
    run()
    ctx.synchronize()
    graph = None
    if not args.no_graph:
        ctx.capture_begin()
        run()
        graph = ctx.capture_end()
        step = lambda: ctx.graph_launch(graph)
    else:
        step = run

    for _ in range(args.warmup):
        step()
    ctx.synchronize()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    ctx.synchronize()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3
    tok_s = args.steps / dt

    # ---- spread of the step time: one event pair per step on the library's stream ----------
    n_ev = max(20, min(args.steps, 400))
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(n_ev + 1)]
    evs[0].record(ctx.stream)
    for i in range(n_ev):
        step()
        evs[i + 1].record(ctx.stream)
    ctx.synchronize()
    per_step = sorted(evs[i].elapsed_time(evs[i + 1]) for i in range(n_ev))
    pct = lambda q: per_step[min(n_ev - 1, int(q * n_ev))]
    step_ms = {"n": n_ev, "median": round(pct(0.5), 4), "p10": round(pct(0.1), 4), "p90": round(pct(0.9), 4),
               "min": round(per_step[0], 4), "max": round(per_step[-1], 4),
               "note": "event pair per step; the events add a little to each step"}

    rows = [list(ks)] * L if keep_frac is None else kept     # active channels per layer and point
    active_bytes = weight_bytes(rows)

    # ---- every operator of the step, in place: device time stamps written by the kernels ---
    per_op = None
    khz = ctx.wall_clock_khz()
    if graph is not None and khz > 0 and args.group == 1:
        n_ops = 5 * L
        stamps = torch.empty((n_ops, 2), dtype=torch.int64, device="cuda")
        torch.cuda.synchronize()
        ctx.profile_set(stamps)
        ctx.capture_begin()
        run()
        graph_prof = ctx.capture_end()
        ctx.profile_set(None)
        samples = []
        for _ in range(12):
            stamps[:, 0] = torch.iinfo(torch.int64).max
            stamps[:, 1] = 0
            torch.cuda.synchronize()
            ctx.graph_launch(graph_prof)
            ctx.synchronize()
            samples.append(stamps.cpu().numpy().astype(np.int64))
        ctx.graph_destroy(graph_prof)
        samples = np.stack(samples[2:])                     # [rep, launch, 2]
        tick_us = 1e3 / khz
        busy = (samples[:, :, 1] - samples[:, :, 0]) * tick_us                      # entry -> exit
        nxt = np.concatenate([samples[:, 1:, 0], samples[:, -1:, 1]], axis=1)
        pitch = (nxt - samples[:, :, 0]) * tick_us                                  # entry -> next entry
        names = ("qkv", "attention", "o", "gate|up", "down")
        if keep_frac is None:
            rows_l = [list(ks)] * L
        else:
            rows_l = kept
        kvb = 2 * (kv_len + 1) * shape.n_kv_heads * shape.head_dim * 2             # K and V read by attention
        d_, f_ = shape.d_model, shape.d_ffn

        def op_bytes(l, o):
            r4 = rows_l[l]
            if kind != B.AF_W_F16:
                wb = lambda k_, n_in, out_: k_ * (out_ // 2 + 6) + out_ * 2 + (
                    (n_in // 32) * out_ * 2 if kind == B.AF_W_Q4G32 else k_ * (out_ // 32) * 2)
            else:
                wb = lambda k_, n_in, out_: k_ * (out_ * 2 + 6) + out_ * 2
            if o == 0:
                return wb(r4[0], d_, shape.qkv_out) + 2 * d_ * 2
            if o == 1:
                return kvb + shape.qkv_out * 2 + widths[1] * 2
            if o == 2:
                return wb(r4[1], widths[1], d_) + d_ * 2
            if o == 3:
                return wb(r4[2], d_, 2 * f_) + 2 * d_ * 2
            return wb(r4[3], f_, d_) + d_ * 2 + 2 * f_ * 2
        per_op = []
        for o, nm in enumerate(names):
            sel_ = np.arange(o, n_ops, 5)
            us_busy = float(np.median(busy[:, sel_].mean(axis=1)))
            us_pitch = float(np.median(pitch[:, sel_].mean(axis=1)))
            byts = float(np.mean([op_bytes(l, o) for l in range(L)]))
            per_op.append({"op": nm, "us": round(us_busy, 2), "us_to_next_start": round(us_pitch, 2),
                           "bytes": int(byts), "GBps": round(byts / max(us_pitch, 1e-9) / 1e3, 1),
                           "frac_of_hbm_peak": round(byts / max(us_pitch, 1e-9) / 1e3 / HBM_PEAK_GBPS, 4)})
        per_op_sum_us = round(sum(p_["us_to_next_start"] for p_ in per_op) * L, 1)

    # ---- roofline of the dominant kernel ------------------------------------------------
    # The gate|up operator as it runs inside the step: one launch that builds
    # rmsnorm(h_mid), selects the top-k channels and streams their weight rows.  Timed alone
    # with one launch per layer, rotating through all layers' matrices (far more than the
    # 256 MB last-level cache), bracketed by events on the library's stream.
    h2 = torch.from_numpy(S.activation(0, S.channel_scales(0, shape.d_model, "roof"), "roof", 0)).cuda()
    idx2 = torch.empty(shape.d_model, dtype=torch.int32, device="cuda")
    cnt2 = torch.empty(1, dtype=torch.int32, device="cuda")
    x2 = torch.empty(shape.d_model, dtype=torch.float16, device="cuda")
    y2 = torch.empty(2 * shape.d_ffn, dtype=torch.float16, device="cuda")
    torch.cuda.synchronize()

    def gateup(l):
        lay = st.layers[l]
        if kind == B.AF_W_F16 and keep_frac is not None:
            ctx.select_gemv_f16(lay.Wgateup, h2, producer=B.AF_PRO_RMSNORM, gain=lay.g_ffn, eps=1e-5,
                                sel_mode=B.AF_SEL_THRESHOLD, t=t2, x_out=x2, y=y2)
        elif kind == B.AF_W_F16:
            ctx.select_gemv_f16(lay.Wgateup, h2, producer=B.AF_PRO_RMSNORM, gain=lay.g_ffn, eps=1e-5,
                                sel_mode=B.AF_SEL_TOPK, k=ks[2], x_out=x2, idx_out=idx2,
                                count_out=cnt2, y=y2)
        elif kind == B.AF_W_Q4CL:
            ctx.sparse_gemv_q4_cl(lay.Wgateup, lay.Sgateup, h2, st.sets[0].idx[2], nidx=ks[2], y=y2)
        else:
            ctx.sparse_gemv_q4(lay.Wgateup, lay.Sgateup, h2, st.sets[0].idx[2], nidx=ks[2], y=y2)

    rows2 = ks[2]
    if keep_frac is not None and kind == B.AF_W_F16:
        # the roofline vector is not a hidden state of the stack: give it its own threshold,
        # and count the rows that threshold really keeps
        hx = ctx.calib_hist()
        torch.cuda.synchronize()
        ctx.select_gemv_f16(st.layers[0].Wgateup, h2, producer=B.AF_PRO_RMSNORM, gain=st.layers[0].g_ffn,
                            eps=1e-5, sel_mode=B.AF_SEL_DENSE, x_out=x2, y=y2)
        ctx.calib_accumulate(x2, hx)
        t2_dev = ctx.calib_thresholds(hx, [sp])
        ctx.synchronize()
        t2 = float(t2_dev.item())
        _, c2 = ctx.select_threshold(x2, t2)
        ctx.synchronize()
        rows2 = int(c2.item())
    reps = max(1, 256 // L)
    for l in range(L):
        gateup(l)
    ctx.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(ctx.stream)
    for _ in range(reps):
        for l in range(L):
            gateup(l)
    e1.record(ctx.stream)
    ctx.synchronize()
    launches = reps * L
    us_per_launch = e0.elapsed_time(e1) * 1e3 / launches
    if kind == B.AF_W_F16:
        # k rows of weights with their (x, idx) pairs, the result, plus the norm's input and gain
        alg = gemv_bytes(rows2, 2 * shape.d_ffn) + 2 * shape.d_model * 2
        kname = "gemv_f16_kernel<64, 8, 16> (gate|up: rmsnorm + top-k + gathered GEMV)"
        if keep_frac is not None:
            alg -= rows2 * 4     # no index list travels through memory
            kname = "gemv_f16_kernel (gate|up: rmsnorm + per-range threshold + gathered GEMV)"
    elif kind == B.AF_W_Q4CL:
        alg = ks[2] * (shape.d_ffn + 2 * shape.d_ffn // 16 + 6) + 2 * shape.d_ffn * 2
        kname = "gemv_q4_kernel, channel-local scales (gate|up, index set given)"
    else:
        alg = ks[2] * (shape.d_ffn + 6) + (shape.d_model // 32) * 2 * shape.d_ffn * 2 + 2 * shape.d_ffn * 2
        kname = "gemv_q4_kernel (gate|up, index set given)"
    achieved = alg / (us_per_launch * 1e-6) / 1e9
    roofline = {"bound": "hbm", "kernel": kname,
                "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBPS, 4),
                "traffic": None,
                "bytes_per_launch": alg, "us_per_launch": round(us_per_launch, 3), "launches": launches}

    tr_ = TRAFFIC.get((args.shape, args.weights, sp))
    if tr_ is not None and L == base.n_layers and args.group == 1 and keep_frac is None:
        roofline["traffic"] = int((tr_["fetch_KiB"] * tr_["fetch_factor"] + tr_["write_KiB"] * tr_["write_factor"]) * 1024)
        roofline["traffic_source"] = {k_: tr_[k_] for k_ in ("source", "kernel", "fetch_KiB", "fetch_factor",
                                                             "write_KiB", "write_factor")}
        roofline["traffic_over_algorithmic"] = round(roofline["traffic"] / alg, 4)

    # ---- the box's plain streaming-read rate (what an ideal reader of these bytes gets) ----
    probe = torch.zeros(4 << 30, dtype=torch.uint8, device="cuda")
    sink = ctx.probe_sink()
    torch.cuda.synchronize()
    stream_gbps = 0.0
    for wgs in (4, 8, 16, 32):                      # the best launch shape of the plain reader
        ctx.probe_stream_read(probe, sink, wgs)
        e0.record(ctx.stream)
        for _ in range(4):
            ctx.probe_stream_read(probe, sink, wgs)
        e1.record(ctx.stream)
        ctx.synchronize()
        stream_gbps = max(stream_gbps, 4 * probe.numel() / (e0.elapsed_time(e1) * 1e-3) / 1e9)
    best_shape = "256 threads, 8 loads in flight (af_probe_stream_read)"
    variants = {}
    for threads in (256, 1024):                     # other shapes of the plain reader
        for in_flight in (4, 8, 16):
            for nt in (False, True):
                if nt and in_flight == 4:
                    continue
                for wgs in ((4, 8, 16, 32) if threads == 256 else (1, 2, 4, 8)):
                    ctx.probe_stream_read_variant(probe, sink, wgs, threads, in_flight, nt)
                    e0.record(ctx.stream)
                    for _ in range(3):
                        ctx.probe_stream_read_variant(probe, sink, wgs, threads, in_flight, nt)
                    e1.record(ctx.stream)
                    ctx.synchronize()
                    g_ = 3 * probe.numel() / (e0.elapsed_time(e1) * 1e-3) / 1e9
                    key = f"{threads}thr_u{in_flight}{'_nt' if nt else ''}"
                    variants[key] = max(variants.get(key, 0.0), round(g_, 1))
                    if g_ > stream_gbps:
                        stream_gbps = g_
                        best_shape = f"{threads} threads, {in_flight} loads in flight, " \
                                     f"{'non-temporal, ' if nt else ''}{wgs} workgroups per compute unit"
    del probe
    roofline["measured_stream_read_variants_GBps"] = variants
    roofline["measured_stream_read_shape"] = best_shape
    roofline["measured_stream_read_GBps"] = round(stream_gbps, 1)
    roofline["frac_of_measured_stream_read"] = round(achieved / stream_gbps, 4)

    # ---- the same stack with the threshold form of the selection (Section 6: thresholds
    # preloaded per operator), reported beside the top-k headline -------------------------
    thr_form = None
    if args.select == "topk" and not args.no_threshold_leg and graph is not None and args.group == 1:
        sel_t, kf_t, kept_t, _ = threshold_selection()
        run_t = lambda: st.run(hin, kv_len, kv_len, sel_t)
        run_t()
        ctx.synchronize()
        ctx.capture_begin()
        run_t()
        g_t = ctx.capture_end()
        for _ in range(args.warmup):
            ctx.graph_launch(g_t)
        ctx.synchronize()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            ctx.graph_launch(g_t)
        ctx.synchronize()
        torch.cuda.synchronize()
        dt_t = time.perf_counter() - t0
        ctx.graph_destroy(g_t)
        ab_t = weight_bytes(kept_t)
        thr_form = {"value": round(args.steps / dt_t, 2), "unit": "tokens/s",
                    "ms_per_step": round(dt_t / args.steps * 1e3, 4),
                    "kept_fraction_by_point": kf_t, "calib_tokens": args.calib_tokens,
                    "active_weight_bytes_per_token": int(ab_t),
                    "active_weight_GBps": round(ab_t / (dt_t / args.steps) / 1e9, 1),
                    "active_weight_frac_of_hbm_peak": round(ab_t / (dt_t / args.steps) / 1e9 / HBM_PEAK_GBPS, 4),
                    "note": "same stack, same token; per-operator thresholds calibrated for the target "
                            "sparsity, compared inside the GEMV launches (no index lists); "
                            "bench.py --select threshold makes this the timed configuration"}

    # ---- CPU oracle on a bounded sample ------------------------------------------------
    cpu = None
    if host_layer0 is not None:
        from oracle import activeflow_oracle as O          # cpu_baseline leg only
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
        except Exception:
            cores = os.cpu_count()
        ocfg = O.LayerCfg(shape.d_model, shape.n_heads, shape.n_kv_heads, shape.head_dim, shape.d_ffn)
        K0, V0 = [t.cpu().numpy() for t in kv[0]]
        wq = host_layer0
        if kind == B.AF_W_Q4G32:
            wq = {k: (O.quantize_q4_g32(v) if k.startswith("W") else v) for k, v in host_layer0.items()}
        elif kind == B.AF_W_Q4CL:
            wq = {k: (O.quantize_q4_cl(v) if k.startswith("W") else v) for k, v in host_layer0.items()}
        oq4 = {B.AF_W_F16: False, B.AF_W_Q4G32: True, B.AF_W_Q4CL: "cl"}[kind]
        n_done, t_cpu, h = 0, 0.0, h_host
        tr = None
        osel = O.SelectCfg(O.SEL_TOPK, ks) if keep_frac is None else O.SelectCfg(O.SEL_THRESHOLD, t=tuple(thr[0]))
        while n_done < 40 and t_cpu < 12.0:
            t1 = time.perf_counter()
            tr = O.decode_layer(ocfg, wq, h, K0.copy(), V0.copy(), kv_len, kv_len,
                                osel, weights_q4=oq4)
            t_cpu += time.perf_counter() - t1
            n_done += 1
            if n_done == 1:
                first = tr
        cpu_tok_s = 1.0 / (t_cpu / n_done * L)
        # a second CPU figure, so that the speed-up is not only "GPU against a dense CPU loop":
        # the four gathered products of the layer (active columns only, fp32 BLAS) in plain NumPy
        gathered = None
        if kind == B.AF_W_F16 and first is not None:
            mats = [np.concatenate([host_layer0["Wq"], host_layer0["Wk"], host_layer0["Wv"]]), host_layer0["Wo"],
                    np.concatenate([host_layer0["Wgate"], host_layer0["Wup"]]), host_layer0["Wdown"]]
            # input-channel-major like the GPU's layout, so that an active channel is one contiguous row
            mats = [np.ascontiguousarray(m_.astype(np.float32).T) for m_ in mats]
            xs_ = [np.asarray(v_, dtype=np.float32) for v_ in first.x]
            t_g, n_g = 0.0, 0
            while n_g < 40 and t_g < 4.0:
                t1 = time.perf_counter()
                for m_, x_, i_ in zip(mats, xs_, first.idx):
                    _ = x_[i_] @ m_[i_]
                t_g += time.perf_counter() - t1
                n_g += 1
            gathered = {"value": round(1.0 / (t_g / n_g * L), 3), "unit": "tokens/s",
                        "what": "the four gathered fp32 products x[idx] @ Wt[idx] (input-channel-major Wt) of "
                                f"layer 0 in NumPy ({n_g}x, {t_g:.1f} s), scaled to {L} layers; linear operators only"}
            del mats
        cpu = {"value": round(cpu_tok_s, 4), "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
               "sample": f"layer 0 of the stack decoded {n_done}x by the fp64 NumPy oracle "
                         f"({t_cpu:.1f} s), scaled to {L} layers"}
        # correctness of the timed buffers: layer 0 of the GPU stack against the oracle
        sel0 = M.select_cfg(B.AF_SEL_TOPK, ks) if keep_frac is None else M.select_cfg(B.AF_SEL_THRESHOLD, t=thr[0])
        st.layer(0, hin, st.hidden_out, kv_len, kv_len, sel0)
        ctx.synchronize()
        got0 = st.sets[0].fetch(0, len(first.idx[0]))
        if not np.array_equal(got0, first.idx[0]):
            print("bench.py: WARNING layer-0 qkv index set differs from the oracle", file=sys.stderr)
        st.sets[0].load(first.idx)
        sel0.reuse_mask = 0b1111
        st.layer(0, hin, st.hidden_out, kv_len, kv_len, sel0)
        ctx.synchronize()
        err = O.rel_err(st.hidden_out.cpu().numpy(), first.hidden, 1.0)   # chained stages: rms floor
        cpu["gpu_vs_oracle_rel_err_layer0"] = float(f"{err:.3e}")
        if gathered is not None:
            cpu["gathered_columns_numpy"] = gathered
        if err > 2e-3:
            print(f"bench.py: WARNING layer-0 output differs from the oracle: {err}", file=sys.stderr)

    overlap = None
    if args.group > 1 and args.overlap:
        # eager, untimed: every layer with taps; followers carry the leader's sets, and the set
        # their own input would have selected is computed next to it for comparison
        tap_of = (0, 2, 4, 6)
        sums = [[0.0, 0] for _ in range(4)]
        per_layer = []
        cur = hin.clone()
        nxt = torch.zeros_like(cur)
        for l in range(L):
            lead = l - l % args.group
            follower = l != lead
            mask = args.reuse_points if follower else 0
            if follower:
                for p in range(4):
                    if mask >> p & 1:
                        st.sets[l].idx[p].copy_(st.sets[lead].idx[p])
                torch.cuda.synchronize()
            st.layer(l, cur, nxt, kv_len, kv_len, M.select_cfg(B.AF_SEL_TOPK, ks, reuse_mask=mask))
            ctx.synchronize()
            row = [None] * 4
            if follower:
                for p in range(4):
                    if not (mask >> p & 1):
                        continue
                    x = ctx.layer_tap(tap_of[p], widths[p])
                    own = ctx.select_topk(x, ks[p])
                    ctx.synchronize()
                    inter = torch.isin(st.sets[l].idx[p][: ks[p]], own).sum().item()
                    row[p] = inter / ks[p]
                    sums[p][0] += row[p]
                    sums[p][1] += 1
            per_layer.append(row)
            cur, nxt = nxt, cur
        overlap = {"points": ["qkv", "o", "gateup", "down"],
                   "mean": [round(a / n, 4) if n else None for a, n in sums],
                   "layer1": per_layer[1] if L > 1 else None,
                   "last_follower": per_layer[L - 1] if (L - 1) % args.group else per_layer[L - 2]}

    lfu = None
    if args.lfu_tokens > 0 and args.select == "topk":
        # Section 4.2 on the index streams of the hot path: per tensor, an LFU cache of a fraction
        # of its channels; hit ratio = needed channels found cached, averaged over the tokens after
        # the first (the cache starts with the lowest-numbered channels, an arbitrary content)
        watch = sorted({0, L // 2})
        fracs = (0.25, 0.5, 0.75)
        caches = {(l, p, fr): B.LfuCache(widths[p], int(widths[p] * fr), list(range(int(widths[p] * fr))))
                  for l in watch for p in range(4) for fr in fracs}
        hit = {k: [0, 0] for k in caches}
        scales = S.channel_scales(0, shape.d_model, shape.name)
        t_sim, n_sim = 0.0, 0
        for tok in range(1, args.lfu_tokens + 1):
            cur = torch.from_numpy(S.activation(0, scales, "hidden", tok)).cuda()
            torch.cuda.synchronize()
            st.run(cur, kv_len, kv_len, M.select_cfg(B.AF_SEL_TOPK, ks))
            ctx.synchronize()
            for l in watch:
                for p in range(4):
                    idx = st.sets[l].fetch(p, ks[p]).tolist()
                    for fr in fracs:
                        t1 = time.perf_counter()
                        h, ld, _ = caches[(l, p, fr)].step(idx)
                        t_sim += time.perf_counter() - t1
                        n_sim += 1
                        if tok > 1:
                            hit[(l, p, fr)][0] += h
                            hit[(l, p, fr)][1] += h + ld
        lfu = {"tokens": args.lfu_tokens, "points": ["qkv", "o", "gateup", "down"],
               "hit_ratio": {f"layer{l}@{int(fr * 100)}%": [round(hit[(l, p, fr)][0] / max(1, hit[(l, p, fr)][1]), 4)
                                                            for p in range(4)] for l in watch for fr in fracs},
               "keep_fraction": round(1 - sp / 100, 2),
               "simulator_us_per_step": round(t_sim / max(1, n_sim) * 1e6, 1)}

    wl = f"{args.shape}-shape decoder stack, {L} layers, batch-1 decode, {args.weights} weights, " \
         f"{sp}% sparsity at qkv/o/gate-up/down, {kv_len}-token KV cache"
    if keep_frac is not None:
        wl += f", threshold selection calibrated on {args.calib_tokens} tokens (no index lists)"
    if args.group > 1:
        wl += f", index reuse in groups of {args.group} (points mask {args.reuse_points:#06b})"
    clocks = None
    under_profiler = any(k.startswith(("ROCPROF", "ROCP_")) for k in os.environ) or \
        "rocprof" in os.environ.get("LD_PRELOAD", "")
    try:   # best effort; a child process, never an exec from this one; not under a profiler,
        # whose preloaded library has the child start with the GPU already initialised
        if under_profiler:
            raise RuntimeError("skipped under a profiler")
        import subprocess
        smi = subprocess.run(["rocm-smi", "--showclocks"], capture_output=True, text=True, timeout=20).stdout
        clocks = {ln.split(":")[1].strip().split()[0]: ln.split("(")[-1].rstrip(")\n ")
                  for ln in smi.splitlines() if "clock level" in ln and ("sclk" in ln or "mclk" in ln or "fclk" in ln)}
    except Exception:
        pass
    out = {
        "metric": "active-weight GB/s (% of HBM peak) + decode tokens/s, 7B-shape @50% sparsity",
        "value": round(tok_s, 2), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f16" if kind == B.AF_W_F16 else "int4",
        "data": "synthetic",
        "config": {"workload": wl, "layers": L, "d_model": shape.d_model, "d_ffn": shape.d_ffn,
                   "k": list(ks), "graph": graph is not None},
        "active_weight_bytes_per_token": int(active_bytes),
        "active_weight_GBps": round(active_bytes * tok_s / 1e9, 1),
        "active_weight_frac_of_hbm_peak": round(active_bytes * tok_s / 1e9 / HBM_PEAK_GBPS, 4),
        "build_s": round(t_build, 1),
        "step_ms": step_ms,
        "roofline": roofline,
        "cpu_baseline": cpu,
    }
    if clocks:
        out["clocks_after_run"] = clocks
    if per_op is not None:
        out["per_op"] = per_op
        out["per_op_note"] = ("mean over the layers of one graph replay, median over 10 replays; us = first "
                              "workgroup entry to last workgroup exit by the device wall clock, "
                              "us_to_next_start = entry to the next kernel's entry (sums to the step: "
                              f"{per_op_sum_us} us); bytes = algorithmic bytes of the operator (attention: "
                              "the KV rows it reads); fractions use us_to_next_start")
    if keep_frac is not None:
        out["config"]["kept_fraction_by_point"] = keep_frac
    if thr_form is not None:
        out["threshold_form"] = thr_form
    if lfu is not None:
        out["lfu_cache"] = lfu
    if overlap is not None:
        out["overlap_reused_vs_own"] = overlap
    print(json.dumps(out))
    if graph is not None:
        ctx.graph_destroy(graph)
    ctx.close()
    return 0


if __name__ == "__main__":
    sys.exit(main())
