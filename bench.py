#!/usr/bin/env python3
"""Benchmark of the MoE FFN layer with dynamic expert duplication on one MI355X.

One "step" is one pass of the whole path over one batch of seeded synthetic input
that is already resident in HBM: route -> histogram -> duplication plan -> permute
-> grouped SwiGLU FFN -> combine.  Prints one JSON line:
  value      = tokens/s of the whole layer (T / time per step)
  roofline   = the dominant kernel (the gate/up + SwiGLU grouped GEMM) against the
               MI355X dense bf16 MFMA peak, its duration measured with HIP events on
               the launch stream inside the timed region
  cpu_baseline = the CPU oracle timed on a bounded sample of the same workload
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA peak
PEAK_F32_TFLOPS = 157.3     # MI355X fp32 vector peak
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E

# Bytes moved between the L2s and memory by one launch of the gate/up product, from hardware
# counters (rocprofv3 --pmc FETCH_SIZE, then WRITE_SIZE, each scaled by what the same counter
# reads for the library's plain copy kernel).  The figures come from the profile named in
# `profile`, not from this run, and belong to one version of the kernel source: they are
# reported only while its digest still matches and no tuning option is forced.
KERNEL_SOURCE = os.path.join(os.path.dirname(os.path.abspath(__file__)), "paper_2506_07366_amd", "csrc",
                             "grouped_ffn.hip")
TRAFFIC = {
    "cfg2_mixtral_dist": {"source_sha256": "740699f2e08462455696c06cccf4e9c8c48cd40a0bbfb49dd36673e836e30972",
                          "fetch_bytes": 5228558792, "write_bytes": 235022779,
                          "profile": "profiles/gemm1_cfg2_mixtral_traffic_counters.md"},
}


def measured_traffic(config_name):
    """(bytes per launch, profile it comes from) or (None, None)."""
    import hashlib
    rec = TRAFFIC.get(config_name)
    if not rec or not rec["source_sha256"] or not os.path.exists(KERNEL_SOURCE):
        return None, None
    with open(KERNEL_SOURCE, "rb") as f:
        if hashlib.sha256(f.read()).hexdigest() != rec["source_sha256"]:
            return None, None
    return rec["fetch_bytes"] + rec["write_bytes"], rec["profile"]


def describe(cfg):
    mode = {0: "no prediction", 1: "distribution-only", 2: "token-to-expert"}[cfg.mode]
    return (f"{cfg.name}: T={cfg.T} d={cfg.d} ffn={cfg.ffn} E={cfg.E} top-{cfg.k} {cfg.dtype} {cfg.act} FFN "
            f"G={cfg.G}x{cfg.S} slots, {mode} plan")


def cpu_baseline(cfg, case_inputs, max_rows=16384):
    """Time the oracle on the host: integer stages in full, the fp64 FFN + combine on
    whole segments holding at most ``max_rows`` rows, scaled linearly to all rows."""
    import oracle
    logits, x, Ws, hist_pred, pred_idx, wl = case_inputs
    t0 = time.perf_counter()
    idx, w = oracle.route_topk(logits, cfg.k)
    hist = oracle.histogram(idx, cfg.E)
    hp = oracle.histogram(pred_idx, cfg.E) if cfg.mode == 2 else (hist_pred if cfg.mode == 1 else hist)
    plan = oracle.plan_duplicates(cfg.mode, hp, cfg.E, cfg.G, cfg.S, cfg.cmax)
    perm = oracle.permute(cfg.mode, x, idx, pred_idx, hist, hp, plan.slot_expert, plan.slot_quota,
                          cfg.E, cfg.G, cfg.S)
    t_int = time.perf_counter() - t0
    so = perm["seg_offsets"]
    sizes = np.diff(so)
    order = [s for s in np.argsort(sizes, kind="stable") if sizes[s] > 0]
    chosen, rows = [], 0
    for s in order:                       # smallest non-empty segments first
        if chosen and rows + sizes[s] > max_rows:
            break
        chosen.append(int(s))
        rows += int(sizes[s])
    t0 = time.perf_counter()
    for s in chosen:
        e = int(plan.slot_expert[s])
        if cfg.act == "relu":
            y = oracle.ffn.ffn_rows_relu(perm["x_perm"][so[s]:so[s + 1]], wl.from_storage(Ws[0][e], cfg.dtype),
                                         wl.from_storage(Ws[2][e], cfg.dtype))
        else:
            y = oracle.ffn_rows(perm["x_perm"][so[s]:so[s + 1]], wl.from_storage(Ws[0][e], cfg.dtype),
                                wl.from_storage(Ws[1][e], cfg.dtype), wl.from_storage(Ws[2][e], cfg.dtype))
    t_ffn = time.perf_counter() - t0
    # combine on the same number of rows
    nt = max(1, rows // cfg.k)
    yy = np.zeros((nt * cfg.k, cfg.d))
    t0 = time.perf_counter()
    oracle.combine(yy, np.arange(nt * cfg.k), w[:nt], nt, cfg.k)
    t_comb = time.perf_counter() - t0
    scale = cfg.A / max(rows, 1)
    total = t_int + (t_ffn + t_comb) * scale
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    return {
        "value": cfg.T / total, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
        "sample": (f"integer stages in full ({t_int:.2f} s); fp64 FFN + combine on {len(chosen)} whole segments = "
                   f"{rows} of {cfg.A} rows ({t_ffn + t_comb:.2f} s)"
                   + ("" if rows >= cfg.A else ", scaled linearly in rows (extrapolated)")),
    }


def dense_context(cfg):
    """The dense problem behind the gate/up product, [A, d] x [d, 2*ffn] with every row on one
    expert, run two ways over about a second each (the shader clock settles only after some
    hundred milliseconds of load): this library's grouped GEMM on one segment (SwiGLU epilogue,
    timed with the library's own events) and the vendor library's plain GEMM (torch.matmul ->
    hipBLASLt, bf16 output of twice the width, no epilogue).  Random operands."""
    import torch
    from paper_2506_07366_amd import binding as B
    A, d, ffn = cfg.A, cfg.d, cfg.ffn
    g = torch.Generator(device="cuda")
    g.manual_seed(1234)
    mk = lambda *shape, scale=1.0: (torch.randn(shape, device="cuda", generator=g) * scale).to(torch.bfloat16)
    x = mk(A, d)
    W1, W3, W2 = mk(1, d, ffn, scale=0.02), mk(1, d, ffn, scale=0.02), mk(1, ffn, d, scale=0.02)
    packed = B.moe_pack_weights(W1, W3, W2)
    seg = torch.tensor([0, A], dtype=torch.int32, device="cuda")
    slot = torch.tensor([0], dtype=torch.int32, device="cuda")
    ws = torch.empty(B.moe_grouped_ffn_workspace_bytes(A, d, ffn, 1, 1), dtype=torch.uint8, device="cuda")
    y = torch.empty_like(x)
    flop = 4.0 * A * d * ffn
    reps = max(20, int(1.0 / (flop / 1.2e15)))          # about a second at 1.2 PFLOP/s
    run = lambda: B.moe_grouped_ffn(x, seg, slot, packed, 1, ffn, workspace=ws, out=y)
    for _ in range(reps // 2):
        run()
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(20)]
    for q in evs:
        for e in q:
            e.record()   # torch creates the underlying event at the first record
    for q in evs:
        B.moe_grouped_ffn_time_next_call(q)
        run()
    torch.cuda.synchronize()
    own_ms = float(np.mean([q[0].elapsed_time(q[1]) for q in evs]))
    w = torch.cat([W1[0], W3[0]], dim=1).t().contiguous()   # [2*ffn, d], K-contiguous like the packed weights
    c = torch.empty((A, 2 * ffn), dtype=torch.bfloat16, device="cuda")
    for _ in range(reps // 2):
        torch.matmul(x, w.t(), out=c)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps // 2):
        torch.matmul(x, w.t(), out=c)
    e1.record()
    torch.cuda.synchronize()
    ven_ms = e0.elapsed_time(e1) / (reps // 2)
    return {"shape": [A, 2 * ffn, d],
            "grouped_gemm_one_segment": {"avg_ms": own_ms, "frac": flop / (own_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS},
            "vendor_plain_gemm": {"avg_ms": ven_ms, "frac": flop / (ven_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS}}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", default="cfg2_mixtral_dist")
    ap.add_argument("--tokens", type=int, default=0,
                    help="run the config's shape at another batch size (the tables of batch sizes in DESIGN.md); "
                         "the config's own size when 0")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--stages", action="store_true", help="also print per-stage timings to stderr")
    ap.add_argument("--fused-gather", action="store_true",
                    help="time the variant that gathers token rows inside the first FFN product (no x_perm) "
                         "as the main path; by default it is timed as an extra")
    ap.add_argument("--headline-only", action="store_true",
                    help="stop after the timed steps: no per-stage, per-rank, traffic, predictor or sweep extras "
                         "(every kernel launch of the run then belongs to a whole-layer step)")
    ap.add_argument("--dense-context", action="store_true",
                    help="also time the gate/up product with all A rows on one expert (one segment) and the vendor "
                         "library's plain GEMM of the same size (torch.matmul), each over about a second: context for "
                         "the roofline figure, not part of the step")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also launch the library's plain copy kernel on 256 MiB buffers (three launches), so that a "
                         "hardware-counter run of this command holds a kernel of known traffic to scale by")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this library runs on one GPU only (the G expert-parallel ranks are emulated as "
              "partitions of one device); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2506_07366_amd import binding as B
    from paper_2506_07366_amd import workloads as wl
    from paper_2506_07366_amd.layer import MoELayer, to_device

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    B.load_library()   # fails loudly if the HIP library is missing

    cfg = wl.CONFIGS[args.config]
    if args.tokens > 0 and args.tokens != cfg.T:
        cfg = cfg.replace(T=args.tokens, name=f"{cfg.name}@T={args.tokens}")   # (no stored counter figures for it)
    torch.cuda.set_device(0)
    if args.copy_calibration:
        # fp32 "packing" is three launches of copy_u4_kernel, each reading and writing E*d*ffn*4 bytes
        w = torch.ones((1, 8192, 8192), dtype=torch.float32, device="cuda")
        w2 = torch.ones((1, 8192, 8192), dtype=torch.float32, device="cuda")
        B.moe_pack_weights(w, w, w2)
        torch.cuda.synchronize()
        del w, w2
    logits_h = wl.gen_logits(cfg)
    x_h = wl.gen_x(cfg)
    Ws = wl.gen_weights_storage(cfg, threads=16)
    logits = torch.from_numpy(logits_h).cuda()
    x = to_device(wl.to_storage(x_h, cfg.dtype), cfg.dtype)
    layer = MoELayer(cfg, fused_gather=args.fused_gather)
    layer.set_weights(*[to_device(w, cfg.dtype) for w in Ws])

    # predictions are inputs of the step: drawn on the host from the routing result
    # of an untimed pass
    layer.route(logits)
    layer.histogram()
    torch.cuda.synchronize()
    hist_true = layer.hist.cpu().numpy()
    hist_pred_h = wl.gen_pred_hist(cfg, hist_true) if cfg.mode == 1 else None
    pred_idx_h = wl.gen_pred_idx(cfg, layer.topk_idx.cpu().numpy()) if cfg.mode == 2 else None
    hist_pred = None if hist_pred_h is None else torch.from_numpy(hist_pred_h).cuda()
    pred_idx = None if pred_idx_h is None else torch.from_numpy(pred_idx_h).cuda()

    # digests of the generated inputs (the arrays as they go to the device), so that a results line
    # names exactly the data it was measured on
    import hashlib

    def digest(a):
        return None if a is None else hashlib.sha256(np.ascontiguousarray(a).tobytes()).hexdigest()[:16]

    input_digests = {"logits": digest(logits_h), "x": digest(wl.to_storage(x_h, cfg.dtype)),
                     "W1": digest(Ws[0]), "W3": digest(Ws[1]), "W2": digest(Ws[2]),
                     "hist_pred": digest(hist_pred_h), "pred_idx": digest(pred_idx_h)}

    def step():
        return layer.step(logits, x, hist_pred=hist_pred, pred_idx=pred_idx)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    # events for the dominant kernel, recorded by the library on the launch stream
    bf16 = cfg.dtype == "bf16"
    evs = []
    if bf16:
        for _ in range(args.steps):
            quad = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
            for e in quad:
                e.record()      # creates the underlying hipEvent
            evs.append(quad)
        torch.cuda.synchronize()

    t0 = time.perf_counter()
    for i in range(args.steps):
        if bf16:
            B.moe_grouped_ffn_time_next_call(evs[i])
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    tokens_per_s = cfg.T / (ms_per_step * 1e-3)

    flops1 = (2.0 if cfg.act == "relu" else 4.0) * cfg.A * cfg.d * cfg.ffn   # gate + up products (ReLU form: one)
    flops2 = 2.0 * cfg.A * cfg.d * cfg.ffn      # down product
    traffic, traffic_source = measured_traffic(cfg.name)
    if bf16:
        g1_ms = float(np.mean([q[0].elapsed_time(q[1]) for q in evs]))
        g2_ms = float(np.mean([q[2].elapsed_time(q[3]) for q in evs]))
        achieved = flops1 / (g1_ms * 1e-3) / 1e12
        roofline = {"bound": "mfma", "kernel": ("grouped_gemm_bf16_kernel<relu> (first product)" if cfg.act == "relu"
                                                else "grouped_gemm_bf16_kernel<swiglu> (gate/up product)"),
                    "achieved": achieved, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                    "frac": achieved / PEAK_BF16_TFLOPS, "traffic": traffic, "traffic_source": traffic_source,
                    "avg_ms": g1_ms,
                    "down_product": {"avg_ms": g2_ms, "achieved": flops2 / (g2_ms * 1e-3) / 1e12,
                                     "frac": flops2 / (g2_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS},
                    "ffn_frac_of_peak": (flops1 + flops2) / ((g1_ms + g2_ms) * 1e-3) / 1e12 / PEAK_BF16_TFLOPS}
        # A batch of a few rows per segment (decode) streams weights: the ceiling of its FFN is
        # HBM bandwidth, and the bytes are those of the experts that got at least one row (each
        # expert's three matrices are read once, however many replicas serve it), plus the rows
        # in and out and the hidden activations written and read.
        if cfg.A < 64 * cfg.nseg:
            so = layer.perm["seg_offsets"].cpu().numpy()
            se = layer.slot_expert.cpu().numpy()
            touched = sorted({int(e) for s_, e in enumerate(se) if e >= 0 and so[s_ + 1] > so[s_]})
            n_mat = 2 if cfg.act == "relu" else 3
            bytes_ffn = (n_mat * cfg.d * cfg.ffn * 2 * len(touched) + 2 * cfg.A * cfg.d * 2
                         + 2 * cfg.A * cfg.ffn * 2)
            ach = bytes_ffn / ((g1_ms + g2_ms) * 1e-3) / 1e9
            roofline = {"bound": "hbm", "kernel": "grouped_gemm_bf16_kernel, both products (weight streaming)",
                        "achieved": ach, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": ach / PEAK_HBM_GBS,
                        "traffic": None, "traffic_source": None, "avg_ms": g1_ms + g2_ms,
                        "experts_touched": len(touched), "algorithmic_bytes": bytes_ffn,
                        "mfma_frac_of_peak": (flops1 + flops2) / ((g1_ms + g2_ms) * 1e-3) / 1e12 / PEAK_BF16_TFLOPS}
    else:
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.steps):
            layer.ffn()
        e1.record()
        torch.cuda.synchronize()
        f_ms = e0.elapsed_time(e1) / args.steps
        achieved = (flops1 + flops2) / (f_ms * 1e-3) / 1e12
        roofline = {"bound": "alu", "kernel": "grouped_gemm_f32_kernel (both products)", "achieved": achieved,
                    "peak": PEAK_F32_TFLOPS, "unit": "TFLOP/s", "frac": achieved / PEAK_F32_TFLOPS,
                    "traffic": None, "avg_ms": f_ms}

    result = {
        "metric": "MoE-layer tokens/s (route+plan+permute+FFN+combine); FFN MFMA % of peak",
        "value": tokens_per_s, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": describe(cfg), "T": cfg.T, "A": cfg.A, "mode": cfg.mode, "seed": cfg.seed,
                   "input_sha256": input_digests,
                   "row_gather": "fused into the first FFN product" if args.fused_gather else "x_perm copy (six-call path)"},
        "roofline": roofline,
    }
    if args.headline_only:
        # whole-layer launches only: what a profiler run of this command sees is the timed path
        if not args.no_cpu_baseline:
            result["cpu_baseline"] = cpu_baseline(cfg, (logits_h, x_h, Ws, hist_pred_h, pred_idx_h, wl))
        print(json.dumps(result))
        return

    # per-stage timings (outside the timed region)
    stage_ms = {}
    b = 2 if bf16 else 4

    stage_min_ms = {}

    def time_stage(name, fn, reps=20):
        """Median (and minimum) over ``reps`` single runs, each between its own pair of events
        on the launch stream, after 5 untimed runs."""
        for _ in range(5):
            fn()
        pairs = []
        for _ in range(reps):
            s, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            s.record()
            fn()
            e.record()
            pairs.append((s, e))
        torch.cuda.synchronize()
        ts = [s.elapsed_time(e) for s, e in pairs]
        stage_ms[name] = float(np.median(ts))
        stage_min_ms[name] = float(min(ts))

    time_stage("route", lambda: layer.route(logits))
    time_stage("histogram", layer.histogram)
    time_stage("plan", lambda: layer.plan(cfg.mode, hist_pred, pred_idx))
    time_stage("permute", lambda: layer.permute(cfg.mode, x, pred_idx))
    time_stage("ffn", layer.ffn)
    time_stage("combine", layer.combine)
    bytes_permute = cfg.T * cfg.d * b + cfg.A * cfg.d * b + 16 * cfg.A
    bytes_combine = cfg.A * cfg.d * b + 12 * cfg.A + cfg.T * cfg.d * b
    hbm = {
        "permute_GBs": bytes_permute / (stage_ms["permute"] * 1e-3) / 1e9,
        "combine_GBs": bytes_combine / (stage_ms["combine"] * 1e-3) / 1e9,
    }
    hbm["permute_frac"] = hbm["permute_GBs"] / PEAK_HBM_GBS
    hbm["combine_frac"] = hbm["combine_GBs"] / PEAK_HBM_GBS
    # routing and histogram: algorithmic bytes (logits in, indices and weights out; indices in)
    # over the call's time.  At the workload's own size both are a few microseconds of traffic
    # behind a launch, so the same calls are also timed on 2^20 tokens of the same E and k,
    # where they can show what bandwidth they reach.
    bytes_route = 4 * cfg.T * cfg.E + 8 * cfg.A
    bytes_hist = 4 * cfg.A
    hbm["route_GBs"] = bytes_route / (stage_ms["route"] * 1e-3) / 1e9
    hbm["route_frac"] = hbm["route_GBs"] / PEAK_HBM_GBS
    hbm["histogram_GBs"] = bytes_hist / (stage_ms["histogram"] * 1e-3) / 1e9
    hbm["histogram_frac"] = hbm["histogram_GBs"] / PEAK_HBM_GBS
    T_big = 1 << 20
    lg_big = torch.randn((T_big, cfg.E), device="cuda")
    idx_big = torch.empty((T_big, cfg.k), dtype=torch.int32, device="cuda")
    w_big = torch.empty((T_big, cfg.k), dtype=torch.float32, device="cuda")
    hist_big = torch.empty(cfg.E, dtype=torch.int32, device="cuda")
    time_stage("route_big", lambda: B.moe_route_topk(lg_big, cfg.k, out=(idx_big, w_big)))
    time_stage("hist_big", lambda: B.moe_histogram(idx_big, cfg.E, out=hist_big))
    rb, hb = stage_ms.pop("route_big"), stage_ms.pop("hist_big")
    stage_min_ms.pop("route_big")
    stage_min_ms.pop("hist_big")
    hbm["large_T"] = {"T": T_big, "E": cfg.E, "k": cfg.k,
                      "route_ms": rb, "route_GBs": (4 * T_big * cfg.E + 8 * T_big * cfg.k) / (rb * 1e-3) / 1e9,
                      "histogram_ms": hb, "histogram_GBs": 4 * T_big * cfg.k / (hb * 1e-3) / 1e9}
    hbm["large_T"]["route_frac"] = hbm["large_T"]["route_GBs"] / PEAK_HBM_GBS
    hbm["large_T"]["histogram_frac"] = hbm["large_T"]["histogram_GBs"] / PEAK_HBM_GBS
    del lg_big, idx_big, w_big, hist_big

    # the same two stages with cold caches: a 1 GiB fill between runs pushes the operands out of
    # the L2s and the 256 MB memory-side cache (median of 7 single runs)
    evict = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")

    def time_cold(fn, reps=7):
        ts = []
        for _ in range(reps):
            evict.fill_(1)
            s_, e_ = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            s_.record()
            fn()
            e_.record()
            torch.cuda.synchronize()
            ts.append(s_.elapsed_time(e_))
        return float(np.median(ts))

    cold_p = time_cold(lambda: layer.permute(cfg.mode, x, pred_idx))
    layer.ffn()     # y_perm of this permutation, then evicted before every combine
    cold_c = time_cold(layer.combine)
    del evict
    hbm["cold"] = {"permute_ms": cold_p, "permute_GBs": bytes_permute / (cold_p * 1e-3) / 1e9,
                   "combine_ms": cold_c, "combine_GBs": bytes_combine / (cold_c * 1e-3) / 1e9}
    report = layer.load_report()
    # prediction error of this batch's inputs, to be read against the paper's Table 1:
    # Distribution-Only: mean_e |p_hat_e - p_e| * E on the histograms; Token-to-Expert:
    # share of (token, expert) assignments the predicted rows miss
    if cfg.mode == 1:
        ht, hpn = hist_true.astype(np.float64), hist_pred_h.astype(np.float64)
        report["prediction_error"] = float(np.mean(np.abs(hpn / hpn.sum() - ht / ht.sum())) * cfg.E)
    elif cfg.mode == 2:
        ti = layer.topk_idx.cpu().numpy()
        hit = (ti[:, :, None] == pred_idx_h[:, None, :]).any(axis=2)
        report["prediction_error"] = float(1.0 - hit.mean())

    # each virtual rank's share of the FFN alone (its S slots), with and without the
    # duplication plan: the bottleneck rank is what expert parallelism would wait for
    def rank_ffn_ms(lay, reps=3):
        out = []
        for g in range(cfg.G):
            s_, e_ = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            lay.ffn(g * cfg.S, (g + 1) * cfg.S)
            s_.record()
            for _ in range(reps):
                lay.ffn(g * cfg.S, (g + 1) * cfg.S)
            e_.record()
            torch.cuda.synchronize()
            out.append(s_.elapsed_time(e_) / reps)
        return out

    ranks = {"mode": cfg.mode, "ffn_ms": rank_ffn_ms(layer)}
    ranks["makespan_ms"] = max(ranks["ffn_ms"])
    if cfg.mode != 0:
        home = MoELayer(cfg, fused_gather=args.fused_gather)
        home.packed = layer.packed
        home.step(logits, x, mode=0)
        torch.cuda.synchronize()
        t_home = rank_ffn_ms(home)
        ranks["no_duplication"] = {"ffn_ms": t_home, "makespan_ms": max(t_home),
                                   "rank_load": home.load_report()["rank_load"]}
        del home

    # rows that would cross the emulated ranks at dispatch and combine (one extra C-ABI call,
    # outside the timed region), with its own kernel time
    comm = layer.comm_report(cfg.mode, pred_idx)
    time_stage("comm_matrix", lambda: B.moe_comm_matrix(cfg.mode, layer.topk_idx, pred_idx if cfg.mode == 2 else None,
                                                        layer.perm["row_of_assign"], layer.perm["seg_offsets"],
                                                        cfg.G, cfg.S))
    comm["kernel_ms"] = stage_ms.pop("comm_matrix")
    stage_min_ms.pop("comm_matrix")

    # Distribution-Only predictor over a stream of batches with one fixed expert popularity:
    # the running estimate n_i/N predicts each batch before it is seen; the plan is rebuilt
    # every F batches and reused in between (placement frequency)
    def predictor_stream(n_batches=16, every=(1, 4, 16)):
        E, G, S = cfg.E, cfg.G, cfg.S
        batches = []
        for bi in range(n_batches):
            lg = torch.from_numpy(wl.gen_logits_batch(cfg, bi)).cuda()
            idx_b, _ = B.moe_route_topk(lg, cfg.k)
            batches.append((idx_b, B.moe_histogram(idx_b, E)))
        out = {"batches": n_batches, "imbalance_mean": {}}

        def imbalance(mode, idx_b, hist_b, hp, se, sq):
            perm = B.moe_permute(mode, None, idx_b, None, hist_b, hp, se, sq, E, G, S)
            return float(perm["rank_load"].max().item()) * G / cfg.A

        se0, sq0, _, _ = B.moe_plan_duplicates(0, batches[0][1], G, S, cfg.cmax)
        out["imbalance_mean"]["no_duplication"] = float(np.mean(
            [imbalance(0, i_, h_, h_, se0, sq0) for i_, h_ in batches[1:]]))
        errs, skews = [], []
        for F in every:
            counts = torch.zeros(E, dtype=torch.int64, device="cuda")
            vals = []
            for bi, (idx_b, hist_b) in enumerate(batches):
                if bi > 0:      # batch 0 only trains the estimate
                    if (bi - 1) % F == 0:
                        hp = B.moe_predictor_predict(counts, cfg.A)
                        se, sq, _, _ = B.moe_plan_duplicates(1, hp, G, S, cfg.cmax)
                    vals.append(imbalance(1, idx_b, hist_b, hp, se, sq))
                    if F == 1:
                        ht = hist_b.cpu().numpy().astype(np.float64)
                        hpn = hp.cpu().numpy().astype(np.float64)
                        errs.append(float(np.mean(np.abs(hpn / hpn.sum() - ht / ht.sum())) * E))
                        skews.append(float(ht.max() * E / ht.sum()))
                B.moe_predictor_update(hist_b, counts)
            out["imbalance_mean"][f"replan_every_{F}"] = float(np.mean(vals))
        out["error_rate_mean"] = float(np.mean(errs))
        out["skewness_mean"] = float(np.mean(skews))
        counts = torch.zeros(E, dtype=torch.int64, device="cuda")
        B.moe_predictor_update(batches[0][1], counts)
        hp = torch.empty(E, dtype=torch.int32, device="cuda")
        time_stage("predict", lambda: B.moe_predictor_predict(counts, cfg.A, out=hp), reps=20)
        time_stage("update", lambda: B.moe_predictor_update(batches[0][1], counts), reps=20)
        out["predict_ms"] = stage_ms.pop("predict")
        out["update_ms"] = stage_ms.pop("update")
        stage_min_ms.pop("predict")
        stage_min_ms.pop("update")
        return out

    stream = predictor_stream()

    # copies-per-expert cap and slot-count sweep: the imbalance the plan alone reaches on this
    # batch's true histogram (max planned rank load / mean), one planner call each
    def plan_sweep():
        H = -(-cfg.E // cfg.G)
        rows = []
        for S_ in sorted({H, H + 1, H + 2, min(H + 4, 16), cfg.S}):
            if S_ < H or S_ > 16:
                continue
            for cm in sorted({1, 2, 4, cfg.G}):
                if cm > cfg.G:
                    continue
                _, _, rl, it = B.moe_plan_duplicates(1, layer.hist, cfg.G, S_, cm)
                rows.append({"S": S_, "c_max": cm, "imbalance": float(rl.max().item()) * cfg.G / cfg.A,
                             "iters": int(it.item())})
        return rows

    sweep = plan_sweep()

    # the variants with the boundary copies folded into the FFN, timed the same way (extras, not
    # the headline; built for the SwiGLU form): rows gathered inside the first product, and on
    # top of that the gate weights applied by the second product with a plain sum in the combine
    fused = {}
    if cfg.act != "relu":
        for key, kw in (("fused_gather_path", dict(fused_gather=True)),
                        ("fused_gather_and_weights_path", dict(fused_weights=True))):
            if key == "fused_gather_path" and args.fused_gather:
                key, kw = "six_call_path", dict()
            other = MoELayer(cfg, **kw)
            other.packed = layer.packed
            for _ in range(max(1, args.warmup)):
                other.step(logits, x, hist_pred=hist_pred, pred_idx=pred_idx)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(args.steps):
                other.step(logits, x, hist_pred=hist_pred, pred_idx=pred_idx)
            torch.cuda.synchronize()
            other_ms = (time.perf_counter() - t0) * 1e3 / args.steps
            fused[key] = {"ms_per_step": other_ms, "value": cfg.T / (other_ms * 1e-3), "unit": "tokens/s"}
            del other

    # the same six calls replayed from a HIP graph (one capture, then replays timed like the steps
    # above): what the launch gaps between the small kernels cost
    graph = layer.capture(logits, x, hist_pred=hist_pred, pred_idx=pred_idx)
    for _ in range(max(1, args.warmup)):
        graph.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        graph.replay()
    torch.cuda.synchronize()
    g_ms = (time.perf_counter() - t0) * 1e3 / args.steps
    fused["hip_graph_replay"] = {"ms_per_step": g_ms, "value": cfg.T / (g_ms * 1e-3), "unit": "tokens/s"}
    del graph

    dense = None
    if args.dense_context and bf16 and cfg.act != "relu":
        dense = dense_context(cfg)

    result.update({
        "dense_context": dense,
        "stage_ms": stage_ms, "stage_min_ms": stage_min_ms, "hbm_stages": hbm, "load": report, "ranks": ranks, "comm": comm,
        "predictor_stream": stream, "plan_sweep": sweep,
    })
    result.update(fused)
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(cfg, (logits_h, x_h, Ws, hist_pred_h, pred_idx_h, wl))
    if args.stages:
        print(json.dumps(stage_ms, indent=1), file=sys.stderr)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
