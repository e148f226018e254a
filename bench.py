#!/usr/bin/env python3
"""Benchmark of the chunk-plan executor on one MI355X.

A step is one pass of the whole hot path (every region of every layer, segment by segment)
over one batch of synthetic input that is already resident in HBM.  Prints ONE JSON line:
tokens/s at the workload's activation budget, the chunked / unchunked peak activation bytes,
the roofline fraction of the dominant kernel class (timed with HIP events on the execute
stream), and the fp64 CPU oracle timed on the host cores on a bounded sample.
"""
from __future__ import annotations

import argparse
import dataclasses
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK = {"mfma_bf16": 2.5e15, "hbm": 8.0e12, "fp32_vector": 157.3e12}


def plan_regions(B, c_qkv, c_attn, c_ffn):
    return [(B.AC_REGION_QKV, B.AC_DIM_SEQ, c_qkv), (B.AC_REGION_ATTENTION, B.AC_DIM_SEQ, c_attn),
            (B.AC_REGION_FFN, B.AC_DIM_SEQ, c_ffn)]


def time_plan(B, torch, plan, dx, y, ws, steps, warmup):
    for _ in range(warmup):
        plan.ac_execute(dx, y, ws)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    peak = 0
    for _ in range(steps):
        peak = plan.ac_execute(dx, y, ws)
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / steps, peak


def profile_plan(plan, dx, y, ws, steps):
    plan.ac_plan_set_profiling(True)
    for _ in range(steps):
        plan.ac_execute(dx, y, ws)
    stats = plan.ac_plan_read_profile()
    plan.ac_plan_set_profiling(False)
    return stats


def cpu_baseline(cfg, x, layers):
    """The oracle as it stands, one layer over all tokens, on the host cores."""
    from oracle import transformer as O
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [os.cpu_count()])
    except Exception:
        cores = os.cpu_count()
    t0 = time.perf_counter()
    O.transformer_stack(x, layers[:1], cfg.heads, cfg.causal, cfg.activation, cfg.ln_eps, cfg.batch,
                        query_block=1024)
    dt = time.perf_counter() - t0
    return {"value": cfg.tokens / (dt * cfg.layers), "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"layer 1 of {cfg.layers} over all {cfg.tokens} tokens in fp64 ({dt:.1f} s), "
                      f"scaled by 1/{cfg.layers} layers"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="C2", choices=["C1", "C2", "C3", "C5"])
    ap.add_argument("--chunk", type=int, nargs=3, default=None, metavar=("QKV", "ATTN", "FFN"),
                    help="rows per segment for the three regions (default: the workload's plan)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--sweep", action="store_true", help="also time a sweep of chunk lengths")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2401_10652_amd import binding as B
    from paper_2401_10652_amd import inputs as I

    B.lib()
    torch.cuda.set_device(0)
    cfg = I.CONFIGS[args.config]
    x, layers = I.transformer_inputs(cfg)
    dx = B.to_device(x, cfg.dtype)
    dw = [B.to_device(w[n], cfg.dtype) for w in layers for n in I.TRANSFORMER_LAYER_TENSORS]
    y = torch.empty_like(dx)

    if args.chunk:
        regs, budget = plan_regions(B, *args.chunk), 0
    elif cfg.chunk_len:
        regs, budget = plan_regions(B, cfg.chunk_len, cfg.chunk_len, cfg.chunk_len), 0
    else:
        regs, budget = plan_regions(B, 0, 0, 0), cfg.act_budget
    desc = B.transformer_desc(cfg)
    plan = B.Plan(desc, regs, budget)
    info = plan.ac_plan_query()
    plan.ac_plan_bind_weights(dw)
    plan1 = B.Plan(desc, plan_regions(B, cfg.seq, cfg.seq, cfg.seq), 0)
    info1 = plan1.ac_plan_query()
    plan1.ac_plan_bind_weights(dw)
    ws = B.empty_workspace(max(info.workspace_bytes, info1.workspace_bytes))

    sec, peak = time_plan(B, torch, plan, dx, y, ws, args.steps, args.warmup)
    sec1, peak1 = time_plan(B, torch, plan1, dx, y, ws, args.steps, args.warmup)
    stats = profile_plan(plan, dx, y, ws, args.steps)

    tokens = cfg.tokens
    classes = {}
    for s in stats:
        per = s["total_ms"] / s["launches"]
        bound = "mfma" if s["name"] in ("gemm", "attention", "trimul") else "hbm"
        if bound == "mfma":
            ach, pk, unit = s["flops"] / (s["total_ms"] * 1e-3) / 1e12, PEAK["mfma_bf16"] / 1e12, "TFLOP/s"
            if cfg.dtype == "f32":
                pk = PEAK["fp32_vector"] / 1e12
        else:
            ach, pk, unit = s["bytes"] / (s["total_ms"] * 1e-3) / 1e9, PEAK["hbm"] / 1e9, "GB/s"
        classes[s["name"]] = {"bound": bound, "achieved": round(ach, 2), "peak": pk, "unit": unit,
                              "frac": round(ach / pk, 4), "launches_per_step": s["launches"] // args.steps,
                              "avg_launch_us": round(per * 1e3, 2),
                              "ms_per_step": round(s["total_ms"] / args.steps, 4)}
    dom = max(classes, key=lambda k: classes[k]["ms_per_step"])
    roof = dict(classes[dom])
    roof.update({"kernel": dom, "traffic": None})

    out = {
        "metric": "tokens/s at fixed activation budget",
        "value": round(tokens / sec, 1), "unit": "tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(sec * 1e3, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {
            "workload": cfg.name, "layers": cfg.layers, "seq": cfg.seq, "d_model": cfg.d_model,
            "heads": cfg.heads, "d_ffn": cfg.d_ffn, "causal": cfg.causal,
            "act_budget_bytes": budget,
            "chunk_len": {"qkv": info.regions[0].chunk_len, "attention": info.regions[1].chunk_len,
                          "ffn": info.regions[2].chunk_len},
            "n_segments": {"qkv": info.regions[0].n_segments, "attention": info.regions[1].n_segments,
                           "ffn": info.regions[2].n_segments},
        },
        "roofline": roof,
        "kernels": classes,
        "mfma_frac_whole_step": round(info.flops_per_execute / sec / PEAK["mfma_bf16"], 4),
        "unchunked": {"tokens_per_s": round(tokens / sec1, 1), "ms_per_step": round(sec1 * 1e3, 4),
                      "throughput_loss": round(1.0 - sec1 / sec, 4)},
        "peak_activation_bytes": {
            "chunked_measured": peak, "unchunked_measured": peak1,
            "chunked_paper_model": info.peak_bytes_model, "unchunked_paper_model": info.peak_bytes_model_unchunked,
            "ratio_vs_unchunked_paper_model": round(peak / info.peak_bytes_model_unchunked, 4),
            "ratio_model_vs_model": round(info.peak_bytes_model / info.peak_bytes_model_unchunked, 4),
            "ratio_vs_unchunked_measured": round(peak / peak1, 4),
        },
    }
    if args.sweep:
        sweep = []
        c = cfg.seq
        while c >= 128:
            ps = B.Plan(desc, plan_regions(B, c, c, c), 0)
            ps.ac_plan_bind_weights(dw)
            inf = ps.ac_plan_query()
            s_, pk_ = time_plan(B, torch, ps, dx, y, ws, max(3, args.steps // 2), 1)
            sweep.append({"chunk_len": c, "tokens_per_s": round(tokens / s_, 1), "peak_bytes": pk_,
                          "paper_model_bytes": inf.peak_bytes_model})
            ps.close()
            c //= 2
        out["sweep"] = sweep
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, x, layers)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
