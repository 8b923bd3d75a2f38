#!/usr/bin/env python3
"""Benchmark of the SparseMoE expert hot path on one MI355X.

A "step" is one pass of the whole path over one synthetic batch: route,
permute, grouped GEMM forward, combine, combine backward, grouped GEMM backward
(dgrad + wgrad), permute backward (--graph replays them as one HIP graph).
Inputs are resident in HBM before the timed region.  Prints ONE JSON line: whole-path tokens/s, the roofline of the kernel
that takes the most time (measured with HIP events on the launch stream), a
per-kernel table, and the CPU oracle timed on a bounded sample of the workload.
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

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA peak
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E peak


def kernel_work(cfg, R):
    """Algorithmic work of ONE launch of each kernel: ('mfma', flop) or ('hbm', bytes).

    GEMM flop count uses the rows actually routed (no credit for tile padding).
    Row movers count compulsory bytes: every source row read once and every
    destination row written once, bf16.
    """
    T, d, f, k = cfg.T, cfg.d, cfg.f, cfg.k
    rdf = float(R) * d * f
    row = 2.0 * d
    return {
        "gemm_gate_up": ("mfma", 4 * rdf),
        "gemm_down": ("mfma", 2 * rdf),
        "gemm_dgrad_h": ("mfma", 2 * rdf),
        "gemm_dgrad_x": ("mfma", 4 * rdf),
        "gemm_wgrad_down": ("mfma", 2 * rdf),
        "gemm_wgrad_gate_up": ("mfma", 4 * rdf),
        "gemm_dgrad_h+wgrad_down": ("mfma", 4 * rdf),          # two independent products in one launch
        "gemm_wgrad_gate_up+dgrad_x": ("mfma", 8 * rdf),       # three
        "permute_rows": ("hbm", row * (T + R)),
        "combine": ("hbm", row * (R + T)),
        "combine_bwd": ("hbm", row * (T + R) + row * R),
        "permute_bwd": ("hbm", row * (R + T)),
        "route": ("hbm", 4.0 * T * cfg.E + 8.0 * T * k),
        "route_count": ("hbm", 4.0 * T * cfg.E + 8.0 * T * k),   # routing with the per-chunk expert counts as a by-product
        "permute_count": ("hbm", 4.0 * T * k),
        "permute_scan": ("hbm", 0.0),
        "permute_place": ("hbm", 12.0 * T * k),
        "dgate_finish": ("hbm", 4.0 * R * (f // 64) + 8.0 * T * k),
    }


def measured_traffic(workload, kernel):
    """HBM bytes per launch of `kernel` (fetch + write) from the committed rocprofv3 counter summary, and the
    file it came from; (None, None) when there is no summary for this workload.  The figure is NOT measured in
    this run: counters need a run of their own under rocprofv3."""
    rel = os.path.join("profiles", f"{workload}_hbm_traffic.txt")
    try:
        for line in open(os.path.join(ROOT, rel)):
            p = line.split()
            if len(p) == 3 and p[0] == kernel:
                return float(p[1]) + float(p[2]), rel
    except OSError:
        pass
    return None, None


def gemm_algorithmic_bytes(cfg, R, kernel):
    """Compulsory bf16 traffic of a grouped-GEMM launch (every operand read once, every result written once) in
    the launch configuration bench.py times by default (rows gathered, gate weights folded into h)."""
    Rd, Rf, Td = 2.0 * R * cfg.d, 2.0 * R * cfg.f, 2.0 * cfg.T * cfg.d
    W1 = 2.0 * cfg.n_local * cfg.d * cfg.f
    return {
        "gemm_gate_up": Td + 2 * W1 + 3 * Rf,                       # x, Wg, Wu -> g, u, h
        "gemm_down": Rf + W1 + Rd,                                  # h, Wd -> yp
        "gemm_dgrad_h+wgrad_down": (Td + W1 + 2 * Rf + 2 * Rf) + (Td + Rf + W1),   # dout, Wd, g, u -> dg, du ; dout, hw -> dWd
        "gemm_wgrad_gate_up+dgrad_x": (2 * Rf + Td + 2 * W1) + (2 * Rf + 2 * W1 + Rd),   # dg, du, x -> dWg, dWu ; dg, du, Wg, Wu -> dxp
    }.get(kernel)


def cpu_baseline(cfg, inp, sample_tokens):
    """The oracle, as it stands (NumPy fp64), on the first `sample_tokens` tokens of the batch."""
    import numpy as np
    from oracle import moe_oracle as O
    sub = {k: (v[:sample_tokens] if k in ("x", "dout", "logits") else v) for k, v in inp.items()}
    t0 = time.perf_counter()
    r = O.layer_fwd_bwd(sub, cfg.k, cfg.e_begin, cfg.n_local, cfg.renormalize)
    dt = time.perf_counter() - t0
    cores = len(os.sched_getaffinity(0))
    R = int(r["expert_offsets"][-1])
    return {
        "value": sample_tokens / dt, "unit": "tokens/s", "cores": cores, "kind": "oracle",
        "sample": f"first {sample_tokens} of {cfg.T} tokens, all {cfg.n_local} experts, full fwd+bwd in fp64 NumPy "
                  f"({R} routed rows, {dt:.2f} s incl. bf16 decode)",
        "gemm_gflops": 18.0 * R * cfg.d * cfg.f / dt / 1e9,
    }, r


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="olmoe", help="olmoe (headline) | fine | ep_share | tiny | skew | olmoe_fur | mula100b_ep12 | mula220b_ep12")
    ap.add_argument("--cpu-sample-tokens", type=int, default=8192,
                    help="tokens of the batch the CPU oracle is timed on (about 10-30 s of host work)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle leg")
    ap.add_argument("--materialize-xp", action="store_true",
                    help="gather the routed rows into xp with a kernel of its own (permute_rows) instead of letting "
                         "the gate/up product and the two weight gradients read x through row_token")
    ap.add_argument("--no-fold", action="store_true",
                    help="keep the gate weights in the combine (Stage 5 and its backward as kernels of their own) "
                         "instead of folding them into h, which takes dgate out of the backward product of the "
                         "down projection and needs no backward pass over the [R, d] rows")
    ap.add_argument("--graph", action="store_true",
                    help="time the step as one HIP graph replay instead of a dozen stream launches "
                         "(measured: no faster, the launches already queue ahead of the GPU)")
    ap.add_argument("--rotate", type=int, default=3,
                    help="buffer sets (each larger than the 256 MB last-level cache share a kernel could keep) the "
                         "HBM-bound row movers are rotated through for the cold-cache figure `gbs_cold`; 0 = skip")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 256 MiB device copy (reference dispatch for scaling rocprofv3 "
                         "FETCH_SIZE / WRITE_SIZE readings)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no collectives, no sharding); --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2604_00785_amd import binding as B
    from paper_2604_00785_amd import workloads as W

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    B.load(build_if_missing=True)
    cfg = W.CONFIGS[args.workload]
    dev = "cuda:0"
    inp = W.make_inputs(cfg)

    def up(bits):
        return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(dev).view(torch.bfloat16)

    x, dout = up(inp["x"]), up(inp["dout"])
    Wg, Wu, Wd = up(inp["Wg"]), up(inp["Wu"]), up(inp["Wd"])
    logits = torch.from_numpy(inp["logits"]).to(dev)
    fold = not args.no_fold and not args.materialize_xp and cfg.T * cfg.d * 2 <= 0xFFFFFFFF
    buf = B.MoELayerBuffers(cfg.T, cfg.d, cfg.E, cfg.k, cfg.f, cfg.e_begin, cfg.n_local, cfg.renormalize, dev,
                            gather=not args.materialize_xp, fold=fold)

    def eager_step():
        buf.run_fwd_bwd(x, logits, dout, Wg, Wu, Wd)

    if args.graph:   # the same launches, recorded once into a HIP graph and replayed
        graph = buf.capture_fwd_bwd(x, logits, dout, Wg, Wu, Wd)
        step = graph.replay
    else:
        step = eager_step

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    R = int(buf.expert_offsets[-1].item())
    if args.calibrate_copy:
        src = torch.empty(256 * 1024 * 1024, dtype=torch.uint8, device=dev).random_(0, 255)
        dst = torch.empty_like(src)
        dst.copy_(src)          # reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
        del src, dst

    # ---- timed region: exactly K steps ------------------------------------------
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed / args.steps * 1e3
    tokens_per_s = cfg.T * args.steps / elapsed

    # ---- the same K steps again with every launch bracketed by HIP events ---------
    B.moe_prof_enable(True)
    for _ in range(args.steps):
        eager_step()
    torch.cuda.synchronize()
    prof = B.moe_prof_read()
    B.moe_prof_enable(False)

    work = kernel_work(cfg, R)
    kernels = {}
    for name, total_ms, launches in prof:
        avg_ms = total_ms / max(launches, 1)
        kind, amount = work.get(name, ("hbm", 0.0))
        ent = {"avg_us": round(avg_ms * 1e3, 2), "launches_per_step": launches // args.steps, "bound": kind}
        if kind == "mfma":
            ent["tflops"] = round(amount / (avg_ms * 1e-3) / 1e12, 1)
            ent["frac"] = round(ent["tflops"] / PEAK_BF16_TFLOPS, 4)
        else:
            ent["gbs"] = round(amount / (avg_ms * 1e-3) / 1e9, 1)
            ent["frac"] = round(ent["gbs"] / PEAK_HBM_GBS, 4)
        kernels[name] = ent
    dom = max(kernels, key=lambda n: kernels[n]["avg_us"] * kernels[n]["launches_per_step"])
    dk = kernels[dom]
    if dk["bound"] == "mfma":
        roofline = {"kernel": dom, "bound": "mfma", "achieved": dk["tflops"], "peak": PEAK_BF16_TFLOPS,
                    "unit": "TFLOP/s", "frac": dk["frac"], "traffic": None}
    else:
        roofline = {"kernel": dom, "bound": "hbm", "achieved": dk["gbs"], "peak": PEAK_HBM_GBS, "unit": "GB/s",
                    "frac": dk["frac"], "traffic": None}
    traffic, traffic_file = measured_traffic(cfg.name, dom)
    roofline["traffic"] = traffic
    alg = gemm_algorithmic_bytes(cfg, R, dom) if fold else None
    roofline["traffic_source"] = (None if traffic is None else
                                  f"{traffic_file}: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE summary committed with the repository, "
                                  "NOT measured in this run (it may predate the library this run loaded)")
    if traffic is not None and alg:
        roofline["algorithmic_bytes"] = alg
        roofline["traffic_over_algorithmic"] = round(traffic / alg, 3)
    gemm_us = sum(v["avg_us"] * v["launches_per_step"] for n, v in kernels.items() if n.startswith("gemm_"))
    gemm_tflops = 18.0 * R * cfg.d * cfg.f / (gemm_us * 1e-6) / 1e12 if gemm_us > 0 else 0.0

    line = {
        "metric": "MoE layer fwd+bwd tokens/s (grouped-GEMM TFLOP/s and % of bf16 MFMA peak alongside), 1 GPU",
        "value": round(tokens_per_s, 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: T={cfg.T} d={cfg.d} E={cfg.E} (local {cfg.n_local}) k={cfg.k} f={cfg.f}",
                   "routed_rows": R, "renormalize": cfg.renormalize,
                   "launch": "hip graph replay" if args.graph else "stream launches",
                   "gate_weights": "folded into h (dgate from the backward product of the down projection)" if fold
                                   else "applied by the combine (combine backward as a kernel of its own)",
                   "row_gather": "own kernel (xp materialised)" if args.materialize_xp
                                 else "folded into the loads of the gate/up product and of two weight gradients"},
        "grouped_gemm": {"tflops": round(gemm_tflops, 1), "frac_of_bf16_peak": round(gemm_tflops / PEAK_BF16_TFLOPS, 4),
                         "flop_per_step": 18.0 * R * cfg.d * cfg.f, "us_per_step": round(gemm_us, 1)},
        "roofline": roofline,
        "kernels": kernels,
    }
    # ---- cold-cache rate of the HBM-bound row movers: each kernel alone, its large operand rotated through
    #      `--rotate` buffer sets so that no launch finds its rows in the 256 MB last-level cache
    if args.rotate >= 2:
        nset = args.rotate
        rows = [torch.randn(R, cfg.d, device=dev, dtype=torch.bfloat16) for _ in range(nset)]
        outs = [torch.empty(cfg.T, cfg.d, device=dev, dtype=torch.bfloat16) for _ in range(nset)]
        reps = max(4 * nset, 12)
        cold_calls = {"combine" if fold else "permute_bwd": lambda i: B.moe_unpermute_sum(rows[i], buf.slot_row, outs[i])}
        if fold:
            cold_calls["permute_bwd"] = lambda i: B.moe_permute_bwd(rows[i], buf.slot_row, outs[i])
        else:
            cold_calls["combine"] = lambda i: B.moe_unpermute_combine(rows[i], buf.slot_row, buf.topk_w, outs[i])
            dyps = [torch.empty_like(r) for r in rows[:2]]
            cold_calls["combine_bwd"] = lambda i: B.moe_unpermute_combine_bwd(outs[i], rows[i], buf.slot_row, buf.topk_w,
                                                                              dyps[i % 2], buf.dgate)
        for name, call in cold_calls.items():
            for i in range(nset):
                call(i)
            torch.cuda.synchronize()
            B.moe_prof_enable(True)
            for i in range(reps):
                call(i % nset)
            torch.cuda.synchronize()
            tot = [(ms, c) for n, ms, c in B.moe_prof_read()]
            B.moe_prof_enable(False)
            ms = sum(t for t, _ in tot) / max(sum(c for _, c in tot), 1)
            if name in kernels and ms > 0:
                amount = work[name][1]
                kernels[name]["cold_us"] = round(ms * 1e3, 2)
                kernels[name]["gbs_cold"] = round(amount / (ms * 1e-3) / 1e9, 1)
                kernels[name]["frac_cold"] = round(kernels[name]["gbs_cold"] / PEAK_HBM_GBS, 4)
        # what a kernel that only reads gets from the same rotating buffers: the memory system's practical rate
        sink = torch.empty(2048 * 256, dtype=torch.int32, device=dev)
        for i in range(nset):
            B.moe_prof_stream_read(rows[i], sink, 2048)
        torch.cuda.synchronize()
        B.moe_prof_enable(True)
        for i in range(reps):
            B.moe_prof_stream_read(rows[i % nset], sink, 2048)
        torch.cuda.synchronize()
        sr = [(ms, c) for n, ms, c in B.moe_prof_read()]
        B.moe_prof_enable(False)
        sr_ms = sum(t for t, _ in sr) / max(sum(c for _, c in sr), 1)
        stream_gbs = rows[0].numel() * 2 / (sr_ms * 1e-3) / 1e9 if sr_ms > 0 else None
        line["cold_cache"] = {"buffer_sets": nset, "bytes_per_set": rows[0].numel() * 2,
                              "stream_read_gbs_cold": None if stream_gbs is None else round(stream_gbs, 1),
                              "note": "gbs_cold / frac_cold in `kernels`: the kernel alone, its [R, d] operand rotated through "
                                      "this many buffer sets, so every launch reads its rows from HBM; `gbs` is the rate "
                                      "inside the step, where part of the rows may still lie in the last-level cache; "
                                      "stream_read_gbs_cold: a kernel that only reads (16-byte loads, contiguous) over the same "
                                      "rotating buffers, i.e. what this memory system delivers at best"}
        del rows, outs
    # ---- the router and the backward of Stage 1 (they make the layer a drop-in block): timed apart, not in `value`
    if "Wr" in inp:
        Wr = torch.from_numpy(inp["Wr"]).to(dev)
        lg = torch.empty_like(logits)
        dl = torch.empty_like(logits)
        dWr = torch.empty_like(Wr)
        rws = torch.zeros(max(B.moe_router_bwd_workspace_bytes(cfg.T, cfg.d, cfg.E), 256), dtype=torch.uint8, device=dev)

        def router_pass():
            B.moe_router_fwd(x, Wr, lg)
            B.moe_route_bwd(lg, buf.topk_idx, buf.dgate, cfg.renormalize, dl)
            B.moe_router_bwd(x, Wr, dl, buf.dx, dWr, rws)

        for _ in range(3):
            router_pass()
        torch.cuda.synchronize()
        B.moe_prof_enable(True)
        for _ in range(args.steps):
            router_pass()
        torch.cuda.synchronize()
        rp = {n: round(ms / max(c, 1) * 1e3, 2) for n, ms, c in B.moe_prof_read()}
        B.moe_prof_enable(False)
        # the whole drop-in block (router in front, its backward behind), timed like `value`
        for _ in range(3):
            buf.run_block_fwd_bwd(x, Wr, dout, Wg, Wu, Wd)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            buf.run_block_fwd_bwd(x, Wr, dout, Wg, Wu, Wd)
        torch.cuda.synchronize()
        block_ms = (time.perf_counter() - t0) / args.steps * 1e3
        line["router_path"] = {"kernels_us": rp, "us_per_step": round(sum(rp.values()), 1),
                               "block_ms_per_step": round(block_ms, 4),
                               "block_tokens_per_s": round(cfg.T / (block_ms * 1e-3), 1),
                               "flop_per_step": 6.0 * cfg.T * cfg.E * cfg.d,
                               "note": "router Linear layer, gradient of softmax/top-k/renormalisation, router weight "
                                       "and input gradients, timed apart; block_* = the whole drop-in block "
                                       "(router + expert path + router backward) timed like `value`; "
                                       "neither is part of `value`"}
    # ---- what the matrix pipe sustains for operand values like this workload's (the clock follows the
    #      power draw, which follows the data): pure MFMA on register-resident fragments, no memory traffic
    wgs = torch.cuda.get_device_properties(0).multi_processor_count
    gen = torch.Generator(device=dev).manual_seed(1)
    fa = torch.randn(wgs * 512, 32, device=dev, generator=gen).to(torch.bfloat16)                # activations ~ N(0,1)
    fb = (torch.randn(wgs * 512, 16, device=dev, generator=gen) * 0.02).to(torch.bfloat16)       # weights ~ N(0,0.02)
    B.moe_prof_mfma_ceiling(fa, fb, 2000)   # warm-up
    tf_data, ghz_data = B.moe_prof_mfma_ceiling(fa, fb, 40000)
    tf_zero, ghz_zero = B.moe_prof_mfma_ceiling(torch.zeros_like(fa), torch.zeros_like(fb), 40000)
    line["mfma_ceiling"] = {
        "workload_like_operands": {"tflops": round(tf_data, 1), "clock_ghz": round(ghz_data, 3)},
        "zero_operands": {"tflops": round(tf_zero, 1), "clock_ghz": round(ghz_zero, 3)},
        "grouped_gemm_frac_of_workload_like": round(gemm_tflops / tf_data, 4) if tf_data > 0 else None,
        "note": "v_mfma_f32_16x16x32_bf16 only (the form the grouped GEMM uses), operands in registers, 8 waves per CU, measured in this run; "
                "`roofline.peak` stays the published 2500 TFLOP/s"}
    if not args.no_cpu:
        n = min(args.cpu_sample_tokens, cfg.T)
        cb, _ = cpu_baseline(cfg, inp, n)
        cb["value"] = round(cb["value"], 2)
        cb["gemm_gflops"] = round(cb["gemm_gflops"], 1)
        line["cpu_baseline"] = cb
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
