#!/usr/bin/env python3
"""Benchmark of the Rectify-Router MoE-layer forward on one MI355X.

A step is one rr_moe_forward call (router -> capacity slotting -> Intra-GPU and Fill-in
rectification -> dispatch gather -> expert FFN grouped GEMM -> weighted combine) over one
synthetic batch that is already resident in HBM.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c5|c3|c2|c1] [--mode ir+fr]
    python bench.py --cf-sweep      # tokens/s against the capacity factor (the shape of Tables 3-5)
    python bench.py --workload c4   # only the routing-only stress workload
    python bench.py --probes        # what library kernels reach on this machine: HBM read/copy rate, dense bf16 GEMM
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_FP32_TFLOPS = 157.3    # MI355X fp32 vector
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E

ROOT = os.path.dirname(os.path.abspath(__file__))


def measured_traffic(workload, kernel):
    """HBM-side bytes per launch from rocprofv3 counter runs (FETCH_SIZE and WRITE_SIZE, scaled by what a
    plain copy of known size reads), as recorded in profiles/bench_forward_hbm_traffic.md in lines
    `traffic_bytes <workload> <kernel> <bytes> commit <sha>`.  A profile made at another commit than
    the one that runs is still reported (the line names its commit); None when there is no record."""
    try:
        for line in open(os.path.join(ROOT, "profiles", "bench_forward_hbm_traffic.md")):
            f = line.split()
            if len(f) >= 4 and f[0] == "traffic_bytes" and f[1] == workload and f[2] == kernel:
                return float(f[3])
    except OSError:
        pass
    return None


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="c5")
    ap.add_argument("--mode", default="ir+fr", help="vanilla | ir | fr | ir+fr")
    ap.add_argument("--bias", default=None,
                    help="override the workload's router bias recipe: none | normal:<std> | zipf:<s> (load balance study)")
    ap.add_argument("--quota", action="store_true",
                    help="capacity per group (RR_QUOTA_PER_GROUP) instead of one queue per expert over all tokens")
    ap.add_argument("--cpu-sample", type=int, default=1024, help="tokens the CPU oracle computes outputs for (0 = skip)")
    ap.add_argument("--no-extras", action="store_true",
                    help="only the headline workload: skip the other workloads (c3 with the condensed capacity sweep, "
                         "c2, the routing-only c4 and its skewed variant)")
    ap.add_argument("--no-routing-stress", action="store_true",
                    help="skip the extra routing-only measurement (1M tokens, 64 experts, top-2)")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run one plain 1 GiB device copy (a known-size kernel to scale rocprofv3's "
                         "FETCH_SIZE / WRITE_SIZE counters by)")
    ap.add_argument("--cf-sweep", action="store_true",
                    help="instead of the benchmark line: layer tokens/s at the paper's layer shape over the capacity "
                         "factors of Tables 3 and 4 (top-1, top-2; vanilla, Intra-GPU, Fill-in, both) and the "
                         "experts-per-GPU settings of Table 5")
    ap.add_argument("--probes", action="store_true",
                    help="instead of the benchmark line: attainable rates of this box from library kernels (torch): a "
                         "4 GiB reduction and a 1 GiB copy for HBM, dense bf16 matmuls at the expert-FFN shapes for MFMA")
    return ap.parse_args()


def selected_candidates(rank_expert, E, NR, k, C, arrival=False):
    """(candidates of the lists that are selected by score, kept candidates of the lists that the candidate
    counts settle) for one queue of C slots per expert: a round keeps min(candidates, free slots); nobody,
    everybody or (arrival policy, top-k rounds) the first ones in token order need no selection."""
    n_sel = n_settled_kept = 0
    fill = np.zeros(E, dtype=np.int64)
    for r in range(NR):
        n = np.bincount(rank_expert[:, r], minlength=E).astype(np.int64)
        m = np.minimum(n, C - fill)
        by_score = (not arrival) or r == k
        sel = (m > 0) & (m < n) & by_score
        n_sel += int(n[sel].sum())
        n_settled_kept += int(m[~sel].sum())
        fill += m
    return n_sel, n_settled_kept


def dispatch_bytes(T, E, k, NR, C, n_ir, n_sel=None, n_settled_kept=0):
    """Algorithmic HBM bytes per launch of the routing / rectification kernels: every table they read or
    write, once, 4 bytes per entry (token blocks of 128 for the per-block candidate counts).  n_sel =
    candidates that are materialised for select_slot (default: all of them)."""
    NB = (T + 127) // 128
    NCAT = NR * E
    if n_sel is None:
        n_sel = T * NR
    return {
        "topk_rank": 4 * (T * E + T * (k + 1) + T * NR + 2 * T + NCAT * NB),
        "scan_candidates": 4 * 2 * NCAT * NB,
        # ranks in, the keys of materialised candidates in, block offsets in; the token's slot row out, (key, token)
        # of a materialised candidate out, the token of a kept candidate of a settled list out
        "scatter_candidates": 4 * (T * NR + n_sel + NCAT * NB + T * NR + 2 * n_sel + n_settled_kept),
        # materialised candidates in; slot entries of the kept ones and the queues (kept + padding) out
        "select_slot": 4 * (2 * n_sel + min(n_sel, E * C) + E * C - n_settled_kept),
        "ir_count": 4 * (T * (k + 1) + T + E * NB),
        "ir_scan": 4 * 2 * E * NB,
        "ir_weights": 4 * (T * (k + 1) + T * NR + 2 * T + E * NB + 2 * T + n_ir + T * (k + 2)),
    }


def hbm_rooflines(kernels, hbm):
    out = {}
    for n, ms in kernels.items():
        if n in hbm:
            gbs = hbm[n] / (ms * 1e-3) / 1e9
            out[n] = {"bound": "hbm", "achieved": round(gbs, 1), "unit": "GB/s", "frac": round(gbs / PEAK_HBM_GBS, 4)}
    return out


def run_forward(rr, wl, torch, w, mode, steps, warmup, quota=False, dev=None, backward=True):
    """Times rr_moe_forward on one workload; returns the numbers the JSON line is built from."""
    flags = (rr.RR_INTRA_GPU if "ir" in mode else 0) | (rr.RR_FILL_IN if "fr" in mode else 0)
    flags |= rr.RR_QUOTA_PER_GROUP if quota else 0
    cfg = rr.RRConfig(w.T, w.d_model, w.d_ff, w.E, w.k, w.G, w.capacity_factor,
                      rr.RR_F32 if w.dtype == "f32" else rr.RR_BF16,
                      rr.RR_ACT_GELU if w.act == "gelu" else rr.RR_ACT_SWIGLU, flags)
    if dev is None:
        dev = wl.make_inputs_device(w)
    tdt = torch.float32 if w.dtype == "f32" else torch.bfloat16
    out = torch.empty((w.T, w.d_model), dtype=tdt, device="cuda")
    tables = rr.alloc_tables(cfg)
    logits = torch.empty((w.T, w.E), dtype=torch.float32, device="cuda")
    ws = rr.alloc_workspace(cfg)
    rr.rr_init()

    def step():
        rr.rr_moe_forward(cfg, dev["x"], dev["w_router"], dev["bias"], dev["w1"], dev["w3"], dev["w2"], out,
                          tables, logits, ws)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / steps

    # per-kernel durations: the same steps again with every launch bracketed by HIP events on the
    # launch stream
    rr.rr_profile_enable(True)
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    prof = rr.rr_profile_read()
    ms_per_step_profiled = (time.perf_counter() - t0) * 1e3 / steps
    rr.rr_profile_enable(False)
    kernels = {n: ms / max(c, 1) for n, (c, ms) in prof.items() if c > 0}

    # App. A backward of the weights (not part of the step): gradient of the router scores from the
    # forward pass's expert outputs, straight-through form
    bwd_ms = None
    if backward:
        dout = wl.make_output_gradient_device(w)
        dlogits = torch.empty((w.T, w.E), dtype=torch.float32, device="cuda")
        dcw = torch.empty((w.T, w.k + 2), dtype=torch.float32, device="cuda")
        for _ in range(warmup):
            rr.rr_router_backward(cfg, dout, logits, tables, ws, dlogits, dcw, True)
        rr.rr_profile_enable(True)
        for _ in range(steps):
            rr.rr_router_backward(cfg, dout, logits, tables, ws, dlogits, dcw, True)
        bwd_ms = rr.rr_profile_read()["router_backward"]
        bwd_ms = bwd_ms[1] / max(bwd_ms[0], 1)
        rr.rr_profile_enable(False)
        del dout

    th = tables.to_host()
    C = tables.capacity
    slot_rows = int(th["fill_total"].sum())
    ir_rows = int(th["ir_offset"][-1])
    R = slot_rows + ir_rows
    es = 4 if w.dtype == "f32" else 2
    gated = w.act == "swiglu"
    d, F, T, E, k = w.d_model, w.d_ff, w.T, w.E, w.k
    flops = {"ffn_gate_up": (4 if gated else 2) * d * F * R, "ffn_down": 2 * d * F * R}
    # algorithmic HBM bytes per launch of the memory-bound kernels (each operand once)
    n_src = int((th["slot"] >= 0).sum()) + ir_rows          # processed assignments = rows of the expert outputs
    rows_per_token = (th["slot"] >= 0).sum(axis=1) + (th["ir_expert"] >= 0)
    # bf16 layers: the down projection stores the output row of a token with a single row itself, combine
    # reads the rows of the other tokens and writes their output rows (and zero rows for unprocessed tokens)
    direct = w.dtype == "bf16" and F % 64 == 0 and F >= 192
    comb_read = int(rows_per_token[rows_per_token > 1].sum()) if direct else n_src
    comb_write = int((rows_per_token != 1).sum()) if direct else T
    hbm = {"router_scores": T * d * es + T * E * 4 + E * d * 4,
           "dispatch_gather": 2 * R * d * es + 4 * R,
           "combine": (comb_read + comb_write) * d * es + T * (k + 2) * 4}
    NR = k + (1 if "fr" in mode else 0)
    n_sel, n_settled = (None, 0) if (quota or T <= 16384) else selected_candidates(th["rank_expert"], E, NR, k, C)
    hbm.update(dispatch_bytes(T, E, k, NR, C, ir_rows, n_sel, n_settled))
    if "topk_rank" not in kernels:  # the router's epilogue did the ranking: its table writes count for the router
        hbm["router_scores"] += hbm["topk_rank"] - 4 * T * E
    peak_tf = PEAK_BF16_TFLOPS if w.dtype == "bf16" else PEAK_FP32_TFLOPS
    per_kernel = {}
    for n, ms in kernels.items():
        if n in flops:
            tf = flops[n] / (ms * 1e-3) / 1e12
            per_kernel[n] = {"bound": "mfma" if w.dtype == "bf16" else "alu", "achieved": tf, "unit": "TFLOP/s",
                             "frac": tf / peak_tf}
        elif n in hbm:
            gbs = hbm[n] / (ms * 1e-3) / 1e9
            per_kernel[n] = {"bound": "hbm", "achieved": gbs, "unit": "GB/s", "frac": gbs / PEAK_HBM_GBS}
    dom = max(kernels, key=kernels.get)
    roofline = dict(kernel=dom, **per_kernel.get(dom, {"bound": "hbm", "achieved": None, "unit": "GB/s", "frac": None}))
    roofline["peak"] = peak_tf if dom in flops else PEAK_HBM_GBS
    roofline["traffic"] = measured_traffic(w.name, dom)
    roofline["avg_ms"] = kernels[dom]
    if dom in flops:
        roofline["flops_per_launch"] = flops[dom]
    # backward: dL/do and the rows of y once, logits and weights in, both gradients out, the token's table entries
    bwd_bytes = (n_src + T) * d * es + 2 * T * E * 4 + 2 * T * (k + 2) * 4 + T * (k + 1) * 8 + 8 * T
    bwd = None
    if bwd_ms:
        bwd_gbs = bwd_bytes / (bwd_ms * 1e-3) / 1e9
        bwd = {"ms": round(bwd_ms, 5), "bound": "hbm", "achieved": round(bwd_gbs, 1), "unit": "GB/s",
               "frac": round(bwd_gbs / PEAK_HBM_GBS, 4), "bytes_per_launch": bwd_bytes}
    ffn_ms = kernels.get("ffn_gate_up", 0) + kernels.get("ffn_down", 0)
    routing_names = ("router_scores", "topk_rank", "scan_candidates", "scatter_candidates",
                     "select_slot", "ir_count", "ir_scan", "ir_weights")
    routing_ms = sum(kernels.get(n, 0.0) for n in routing_names)
    return {
        "dev": dev, "capacity": C, "ms_per_step": ms_per_step, "tokens_per_s": T / (ms_per_step * 1e-3),
        "roofline": roofline, "ms_per_step_with_events": ms_per_step_profiled,
        "kernel_ms": {n: round(v, 5) for n, v in kernels.items()},
        "kernel_roofline": {n: {kk: (round(vv, 4) if isinstance(vv, float) else vv) for kk, vv in v.items()}
                            for n, v in per_kernel.items()},
        "ffn_tflops": (flops["ffn_gate_up"] + flops["ffn_down"]) / (ffn_ms * 1e-3) / 1e12 if ffn_ms else None,
        "routing_rectify_mtokens_per_s": T / (routing_ms * 1e-3) / 1e6 if routing_ms else None,
        "router_backward": bwd,
        "tables_host": th,
        "rows": {"slot_rows": slot_rows, "ir_rows": ir_rows, "capacity_slots": E * C,
                 "dropped_assignments": int((th["slot"][:, :k] < 0).sum()),
                 "fill_in_placed": int((th["slot"][:, k] >= 0).sum()), "padding_slots": E * C - slot_rows},
    }


def probes(torch):
    """Rates that library kernels reach on this machine, as context for the roofline fractions (the peaks the
    fractions are quoted against are the published ones)."""
    def timed(fn, n=10):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / n

    out = {"metric": "library_kernel_rates", "n_gpus": 1, "data": "synthetic"}
    big = torch.ones(1 << 30, dtype=torch.float32, device="cuda")  # 4 GiB
    out["hbm_read_GBs_torch_sum_4GiB"] = round(big.numel() * 4 / timed(lambda: big.sum()) / 1e9, 1)
    src = big[: 1 << 28]
    dst = torch.empty_like(src)
    out["hbm_copy_GBs_1GiB_read_plus_write"] = round(2 * src.numel() * 4 / timed(lambda: dst.copy_(src)) / 1e9, 1)
    del big, src, dst
    mm = {}
    for (M, N, K) in ((8192, 8192, 8192), (32768, 22016, 4096), (32768, 4096, 11008), (10240, 11264, 2048),
                      (10240, 2048, 5632)):
        a = torch.randn((M, K), device="cuda", dtype=torch.bfloat16)
        b = torch.randn((N, K), device="cuda", dtype=torch.bfloat16)
        mm["M%d_N%d_K%d" % (M, N, K)] = round(2 * M * N * K / timed(lambda: a @ b.t()) / 1e12, 1)
        del a, b
    out["dense_bf16_matmul_TFLOPs"] = mm
    return out


def cf_sweep(rr, wl, torch, steps, warmup, dev=None, condensed=False):
    """Layer throughput against the capacity factor at the paper's layer shape (Sec. 5.1: LLaMA2-7B FFN,
    8 experts, 16384 tokens): the speed columns of Tables 3 and 4 (capacity factors 0.5-1.5 for top-1,
    1.0-3.0 for top-2 x vanilla / Intra-GPU / Fill-in / both) and the experts-per-GPU rows of Table 5
    (Intra-GPU at 1, 2, 4 experts per GPU).  Same synthetic tensors for every point.  condensed: six
    points only - the ends of both tables with and without the rectification they study, and Table 5's
    one expert per GPU - for the default benchmark line."""
    import dataclasses
    base = wl.C3
    if dev is None:
        dev = wl.make_inputs_device(base)
    out = torch.empty((base.T, base.d_model), dtype=torch.bfloat16, device="cuda")
    logits = torch.empty((base.T, base.E), dtype=torch.float32, device="cuda")
    modes = {"vanilla": 0, "ir": rr.RR_INTRA_GPU, "fr": rr.RR_FILL_IN, "ir+fr": rr.RR_INTRA_GPU | rr.RR_FILL_IN}
    points = [(1, cf, 2, m) for cf in (0.5, 0.75, 1.0, 1.25, 1.5) for m in modes]
    points += [(2, cf, 2, m) for cf in (1.0, 1.5, 2.0, 2.5, 3.0) for m in modes]
    points += [(k, cf, G, "ir") for (k, cf) in ((1, 1.0), (2, 2.0)) for G in (8, 4)]  # 1 and 2 experts per GPU
    # the same layer with capacity read per GPU (each group fills its own block of every expert's queue)
    points += [(k, cf, G, m + "/per-group") for (k, cf) in ((1, 1.0), (2, 1.25)) for G in (2, 8) for m in ("vanilla", "ir+fr")]
    if condensed:
        points = [(1, 0.5, 2, "vanilla"), (1, 0.5, 2, "ir"), (1, 1.0, 8, "ir"),
                  (2, 2.0, 2, "vanilla"), (2, 3.0, 2, "vanilla"), (2, 3.0, 2, "fr")]
    rows = []
    for k, cf, G, m in points:
        w = dataclasses.replace(base, k=k, capacity_factor=cf, G=G)
        per_group = m.endswith("/per-group")
        cfg = rr.RRConfig(w.T, w.d_model, w.d_ff, w.E, w.k, w.G, w.capacity_factor, rr.RR_BF16, rr.RR_ACT_SWIGLU,
                          modes[m.split("/")[0]] | (rr.RR_QUOTA_PER_GROUP if per_group else 0))
        tables = rr.alloc_tables(cfg)
        ws = rr.alloc_workspace(cfg)

        def step():
            rr.rr_moe_forward(cfg, dev["x"], dev["w_router"], dev["bias"], dev["w1"], dev["w3"], dev["w2"], out,
                              tables, logits, ws)

        for _ in range(warmup):
            step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            step()
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / steps
        th = tables.to_host()
        rows.append({"k": k, "capacity_factor": cf, "experts_per_gpu": w.E // G, "mode": m, "ms_per_step": round(ms, 4),
                     "tokens_per_s": round(w.T / (ms * 1e-3)),
                     "slot_rows": int(th["fill_total"].sum()), "ir_rows": int(th["ir_offset"][-1]),
                     "dropped_assignments": int((th["slot"][:, :k] < 0).sum()),
                     "unprocessed_tokens": int((th["combine_w"].sum(axis=1) == 0).sum())})
        del tables, ws
    return {"metric": "rectified_moe_layer_tokens_per_s_vs_capacity_factor", "unit": "tokens/s", "n_gpus": 1,
            "steps": steps, "warmup": warmup, "dtype": "bf16", "data": "synthetic",
            "config": {"workload": "c3 shape: T=%d d=%d F=%d E=%d, SwiGLU" % (base.T, base.d_model, base.d_ff, base.E)},
            "points": rows}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the expert-parallel groups are simulated in HBM); "
              "--gpus must be 1", file=sys.stderr)
        return 2
    import torch
    import paper_2402_12399_amd as rr
    from paper_2402_12399_amd import workloads as wl

    if args.probes:
        torch.cuda.set_device(0)
        print(json.dumps(probes(torch)))
        return 0
    if args.cf_sweep:
        torch.cuda.set_device(0)
        print(json.dumps(cf_sweep(rr, wl, torch, min(args.steps, 20), min(args.warmup, 3))))
        return 0

    w = wl.ALL[args.workload]
    if args.bias is not None:
        import dataclasses
        w = dataclasses.replace(w, name=w.name + "_bias_" + args.bias, bias=args.bias)
    if w.d_ff == 0:  # the routing-only workload on its own
        torch.cuda.set_device(0)
        st = routing_stress(rr, wl, torch, args.steps, args.warmup)
        print(json.dumps({"metric": "routing_rectify_mtokens_per_s", "value": st["mtokens_per_s"], "unit": "Mtokens/s",
                          "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": st["ms_per_step"],
                          "higher_is_better": True, "dtype": "f32", "data": "synthetic",
                          "config": {"workload": w.name}, "roofline": st["router_roofline"], "routing_stress": st}))
        return 0
    mode = () if args.mode == "vanilla" else tuple(args.mode.split("+"))
    torch.cuda.set_device(0)
    res = run_forward(rr, wl, torch, w, mode, args.steps, args.warmup, args.quota)
    dev = res.pop("dev")
    res.pop("tables_host")

    cpu = None
    if args.cpu_sample > 0:
        cpu = cpu_baseline(w, mode, dev, min(args.cpu_sample, w.T), args.quota)
    del dev
    torch.cuda.empty_cache()

    def summary(wk, md, r):
        return {"workload": wk.name, "mode": "top%d" % wk.k + "".join("+" + m for m in md),
                "ms_per_step": r["ms_per_step"], "tokens_per_s": r["tokens_per_s"], "ffn_tflops": r["ffn_tflops"],
                "roofline": r["roofline"], "kernel_ms": r["kernel_ms"], "kernel_roofline": r["kernel_roofline"],
                "routing_rectify_mtokens_per_s": r["routing_rectify_mtokens_per_s"], "rows": r["rows"],
                "router_backward": r["router_backward"]}

    # extras, each with the same steps and warm-ups as the headline: the paper's own layer shape (c3:
    # LLaMA2-7B FFN, 8 experts, 16384 tokens per GPU, top-2) with a condensed capacity-factor sweep on
    # the same tensors, the smallest bf16 workload (c2), the routing-only stress workload (c4) and its
    # skewed variant
    extras = {}
    if not args.no_extras:
        for name in ("c3", "c2"):
            wk = wl.ALL[name]
            if wk.name == w.name:
                continue
            r = run_forward(rr, wl, torch, wk, ("ir", "fr"), max(args.steps, 20), args.warmup)
            dv = r.pop("dev")
            r.pop("tables_host")
            extras["paper_shape" if name == "c3" else name] = summary(wk, ("ir", "fr"), r)
            if name == "c3":
                extras["capacity_sweep"] = cf_sweep(rr, wl, torch, 10, 2, dev=dv, condensed=True)["points"]
            del dv, r
            torch.cuda.empty_cache()
    stress = skew = None
    if not (args.no_routing_stress or args.no_extras):
        stress = routing_stress(rr, wl, torch, max(args.steps, 20), args.warmup, cpu=args.cpu_sample > 0)
        skew = routing_stress(rr, wl, torch, max(args.steps, 20), args.warmup, zipf=1.5)
    if args.copy_probe:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")  # 1 GiB read + 1 GiB written
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    line = {
        "metric": "rectified_moe_layer_tokens_per_s", "value": res["tokens_per_s"], "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": res["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name, "mode": "top%d" % w.k + "".join("+" + m for m in mode), "T": w.T,
                   "d_model": w.d_model, "d_ff": w.d_ff, "E": w.E, "k": w.k, "G": w.G,
                   "capacity_factor": w.capacity_factor, "capacity": res["capacity"],
                   "capacity_scope": "per group" if args.quota else "all tokens", "act": w.act, "router": "fp32",
                   "router_bias": w.bias, "parallelism": "1 GPU, %d simulated expert-parallel groups" % w.G},
        "roofline": res["roofline"],
        "cpu_baseline": cpu,
        "ms_per_step_with_events": res["ms_per_step_with_events"],
        "kernel_ms": res["kernel_ms"],
        "kernel_roofline": res["kernel_roofline"],
        "ffn_tflops": res["ffn_tflops"],
        "routing_rectify_mtokens_per_s": res["routing_rectify_mtokens_per_s"],
        "rows": res["rows"],
        "router_backward": res["router_backward"],
        "paper_shape": extras.get("paper_shape"),
        "capacity_sweep": extras.get("capacity_sweep"),
        "c2": extras.get("c2"),
        "routing_stress": stress,
        "routing_stress_zipf1.5": skew,
    }
    print(json.dumps(line))
    return 0


def routing_stress(rr, wl, torch, steps, warmup, cpu=False, zipf=None):
    """Routing-only workload (1M fp32 tokens, 64 experts in 8 groups, top-2, capacity factor 0.75):
    rr_moe_forward with d_ff = 0, i.e. router scores through combine weights, the memory-bound part of the path.
    zipf: the same workload with a Zipf(s) log-bias on the router (a few experts receive most candidates:
    their selection lists are hundreds of thousands of tokens long)."""
    import dataclasses
    w = wl.C4 if zipf is None else dataclasses.replace(wl.C4, name="c4_routing_stress_f32_zipf%g" % zipf,
                                                        bias="zipf:%g" % zipf)
    cfg = rr.RRConfig(w.T, w.d_model, 0, w.E, w.k, w.G, w.capacity_factor, rr.RR_F32, rr.RR_ACT_SWIGLU,
                      rr.RR_INTRA_GPU | rr.RR_FILL_IN)
    dev = wl.make_inputs_device(w, with_experts=False)
    logits = torch.empty((w.T, w.E), dtype=torch.float32, device="cuda")
    tables = rr.alloc_tables(cfg)
    ws = rr.alloc_workspace(cfg)

    def step():  # d_ff = 0: router (with fused ranking) + routing tables, no expert FFN
        rr.rr_moe_forward(cfg, dev["x"], dev["w_router"], dev["bias"], None, None, None, None, tables, logits, ws)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    rr.rr_profile_enable(True)
    for _ in range(steps):
        step()
    prof = rr.rr_profile_read()
    rr.rr_profile_enable(False)
    kernels = {n: v / max(c, 1) for n, (c, v) in prof.items() if c > 0}
    # algorithmic HBM bytes per launch of the router kernel: x once, logits once, router weights once,
    # plus what its ranking epilogue writes (ranks, score keys, best local expert, per-block counts)
    th = tables.to_host()
    n_ir = int(th["ir_offset"][-1])
    cand = np.bincount(th["rank_expert"][:, 0], minlength=w.E)
    NR = w.k + 1
    n_sel, n_settled = selected_candidates(th["rank_expert"], w.E, NR, w.k, tables.capacity)
    hbm = dispatch_bytes(w.T, w.E, w.k, NR, tables.capacity, n_ir, n_sel, n_settled)
    router_bytes = w.T * w.d_model * 4 + w.T * w.E * 4 + w.E * w.d_model * 4 + hbm.pop("topk_rank") - 4 * w.T * w.E
    gbs = router_bytes / (kernels["router_scores"] * 1e-3) / 1e9
    disp = [n for n in kernels if n != "router_scores"]
    disp_ms = sum(kernels[n] for n in disp)
    disp_bytes = sum(hbm.get(n, 0) for n in disp)
    cpu_routing = None
    if cpu:  # the oracle's router + routing tables on the first 65536 tokens of the same x (same E, G, k, CF)
        from oracle import rectify_router as orc
        n = 65536
        xs = dev["x"][:n].cpu().numpy()
        wr = dev["w_router"].cpu().numpy()
        t0 = time.perf_counter()
        a = orc.router_scores(xs, wr, None)
        orc.route(a, w.k, w.G, w.capacity_factor, True, True)
        dt = time.perf_counter() - t0
        cpu_routing = {"value": n / dt / 1e6, "unit": "Mtokens/s", "kind": "oracle",
                       "sample": "router scores and routing tables of the first %d tokens (%.2f s)" % (n, dt)}
    return {"workload": w.name, "ms_per_step": ms, "mtokens_per_s": w.T / (ms * 1e-3) / 1e6,
            "cpu_baseline": cpu_routing,
            "first_choice_candidates_per_expert": {"max": int(cand.max()), "min": int(cand.min())},
            "rows": {"ir_rows": n_ir, "slot_rows": int(th["fill_total"].sum()), "capacity_slots": w.E * tables.capacity},
            "kernel_ms": {n: round(v, 5) for n, v in kernels.items()},
            "kernel_roofline": hbm_rooflines(kernels, hbm),
            "dispatch_roofline": {"bound": "hbm", "achieved": round(disp_bytes / (disp_ms * 1e-3) / 1e9, 1),
                                  "unit": "GB/s", "frac": round(disp_bytes / (disp_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4),
                                  "bytes": disp_bytes, "ms": round(disp_ms, 5),
                                  "kernels": "every kernel after the router"},
            "router_roofline": {"bound": "hbm", "achieved": gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                                "frac": gbs / PEAK_HBM_GBS, "bytes_per_launch": router_bytes}}


def _route_chunk(args):
    """Per-token steps of the oracle (Eq. 1 scores, ranking) on one chunk of tokens; runs in a worker thread
    (numpy releases the interpreter lock inside the matrix product and the sorts)."""
    from oracle import rectify_router as orc
    x, wr, b, n = args
    a = orc.router_scores(x, wr, b)
    return a, orc.rank_experts(a, n)


def cpu_baseline(w, mode, dev, n_sample, quota=False):
    """The CPU oracle as it stands, timed on this host, in three legs:
      routing_1_thread    router scores and every routing table of the full batch, numpy on one thread;
      routing_all_cores   the same with the per-token steps (Eq. 1 scores, ranking) run on token chunks
                          in one thread per core; the per-expert selection stays serial;
      ffn_sample          float64 expert outputs and their combination for n_sample sampled tokens,
                          extrapolated (and labelled so) to the batch by tokens.
    `value` = tokens/s of the whole layer = T / (routing_1_thread + extrapolated FFN time)."""
    from concurrent.futures import ThreadPoolExecutor
    from oracle import rectify_router as orc
    from paper_2402_12399_amd import workloads as wl
    import torch
    from threadpoolctl import threadpool_limits, threadpool_info

    def host(t):
        if t is None:
            return None
        if t.dtype == torch.bfloat16:
            return wl.bf16_bits_to_f32(t.view(torch.int16).cpu().numpy().view(np.uint16))
        return t.cpu().numpy()

    class PerExpert:  # expert weights come to the host one expert at a time, when the oracle asks for them
        def __init__(self, t):
            self.t, self.shape = t, t.shape

        def __getitem__(self, j):
            return host(self.t[j])

    x, wr, b = host(dev["x"]), host(dev["w_router"]), host(dev["bias"])
    ir, fr = "ir" in mode, "fr" in mode
    nproc = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else (os.cpu_count() or 1)
    nproc = min(nproc, int(os.environ.get("OMP_NUM_THREADS", nproc)))  # the machine's CPU share
    blas_threads = max([p_.get("num_threads", 1) for p_ in threadpool_info()] or [1])

    with threadpool_limits(limits=1):
        t0 = time.perf_counter()
        a = orc.router_scores(x, wr, b)
        tb = orc.route(a, w.k, w.G, w.capacity_factor, ir, fr, quota=quota)
        t_route1 = time.perf_counter() - t0

        # all cores: token chunks through the per-token steps in worker threads, the rest as route() does it
        chunks = np.array_split(np.arange(w.T), nproc)
        t0 = time.perf_counter()
        with ThreadPoolExecutor(nproc) as pool:
            parts = list(pool.map(_route_chunk, [(x[c], wr, b, w.k + 1) for c in chunks]))
        a_par = np.concatenate([p_[0] for p_ in parts])
        if quota:
            slot_par = orc.route(a_par, w.k, w.G, w.capacity_factor, ir, fr, quota=True)["slot"]
        else:  # the steps of route() after the ranking, in its order (Sec. 3, 4.1, 4.2, Eq. 2 / Eq. 3)
            ranks = np.concatenate([p_[1] for p_ in parts])
            C = orc.capacity(w.T, w.E, w.capacity_factor)
            slot_par, slot_token, fill_topk = orc.topk_capacity_rounds(a_par, ranks, w.k, C)
            n_drop, ir_expert = (slot_par[:, :w.k] < 0).sum(axis=1).astype(np.int32), np.full(w.T, -1, dtype=np.int32)
            if ir:
                n_drop, ir_expert, _, _, _ = orc.intra_gpu_rectification(a_par, slot_par, w.k, w.G)
            if fr:
                slot_par, slot_token, _ = orc.fill_in_rectification(a_par, ranks, w.k, C, slot_par, slot_token, fill_topk)
            orc.combine_weights(a_par, ranks, slot_par, w.k, n_drop, ir_expert)
        t_route_par = time.perf_counter() - t0
    assert np.array_equal(slot_par, tb["slot"])

    sample = np.sort(np.random.default_rng(w.seed).choice(w.T, n_sample, replace=False))
    t0 = time.perf_counter()
    orc.moe_output(x, tb, w.k, PerExpert(dev["w1"]), None if dev["w3"] is None else PerExpert(dev["w3"]),
                   PerExpert(dev["w2"]), w.act, tokens=sample)
    t_ffn = time.perf_counter() - t0
    t_ffn_full = t_ffn * (w.T / n_sample)
    total = t_route1 + t_ffn_full
    return {"value": w.T / total, "unit": "tokens/s", "cores": blas_threads, "kind": "oracle",
            "sample": "routing of all %d tokens on one thread (%.2f s) + float64 expert outputs of %d sampled tokens on "
                      "%d BLAS threads (%.2f s, includes fetching the expert weights from the GPU), that time "
                      "EXTRAPOLATED by %d/%d" % (w.T, t_route1, n_sample, blas_threads, t_ffn, w.T, n_sample),
            "legs": {
                "routing_1_thread": {"seconds": round(t_route1, 4), "mtokens_per_s": round(w.T / t_route1 / 1e6, 4),
                                     "cores": 1, "sample": "all %d tokens" % w.T},
                "routing_all_cores": {"seconds": round(t_route_par, 4), "mtokens_per_s": round(w.T / t_route_par / 1e6, 4),
                                      "cores": nproc, "nproc": nproc,
                                      "sample": "all %d tokens; scores and ranking on token chunks in %d threads, "
                                                "per-expert selection serial" % (w.T, nproc)},
                "ffn_sample": {"seconds": round(t_ffn, 3), "tokens": n_sample, "cores": blas_threads,
                               "tokens_per_s_measured": round(n_sample / t_ffn, 2),
                               "seconds_full_batch_extrapolated": round(t_ffn_full, 2), "extrapolated": True}}}


if __name__ == "__main__":
    sys.exit(main())
