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


def plan_regions(B, c_qkv, c_attn, c_ffn, c_out=None):
    """The four regions of a transformer layer; the output projection follows the attention's
    chunk length unless one is given."""
    return [(B.AC_REGION_QKV, B.AC_DIM_SEQ, c_qkv), (B.AC_REGION_ATTENTION, B.AC_DIM_SEQ, c_attn),
            (B.AC_REGION_OUT_PROJ, B.AC_DIM_SEQ, c_attn if c_out is None else c_out),
            (B.AC_REGION_FFN, B.AC_DIM_SEQ, c_ffn)]


PAIR_DIM = "row"     # --pair-dim: the chunk dimension of the pair-stack regions


def pair_regions(B, c):
    def dim(k):
        if PAIR_DIM == "natural":   # rows, except the ending node's attention, whose problems are columns
            return B.AC_DIM_COL if k == B.AC_REGION_TRIATT_END else B.AC_DIM_ROW
        return B.AC_DIM_COL if PAIR_DIM == "col" else B.AC_DIM_ROW
    return [(k, dim(k), c) for k in range(B.AC_REGION_TRIMUL_OUT, B.AC_REGION_PAIR_TRANSITION + 1)]


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


def cpu_baseline_pair(cfg, z, w):
    """The oracle as it stands on a bounded sample: 8 output rows of each of the five modules."""
    import numpy as np
    from oracle import pairstack as P
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [os.cpu_count()])
    except Exception:
        cores = os.cpu_count()
    rows = np.arange(0, cfg.n_res, cfg.n_res // 8)[:8]
    t0 = time.perf_counter()
    for name in P.PAIR_MODULES:
        P.pair_module(name, z, w, cfg.heads, cfg.activation, cfg.ln_eps, rows=rows)
    dt = time.perf_counter() - t0
    return {"value": len(rows) * cfg.n_res / dt, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"{len(rows)} of {cfg.n_res} output rows of each of the 5 modules in fp64 ({dt:.1f} s); the "
                      "whole-tensor projections every row needs are part of the sample, so this overstates "
                      "the per-row cost of a full run"}


def cpu_baseline_res(cfg, x, layers):
    """The oracle as it stands on a bounded sample: the first layer on the first two images (residual blocks only),
    or on all of them (residual + attention block, which the oracle finishes in seconds)."""
    from oracle import unet as U
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [os.cpu_count()])
    except Exception:
        cores = os.cpu_count()
    n = cfg.batch if cfg.heads > 0 else min(2, cfg.batch)     # a few seconds either way
    t0 = time.perf_counter()
    h = U.res_block(x, layers[0]["temb"], layers[0], cfg.groups, cfg.eps, images=list(range(n)))
    if cfg.heads > 0:
        ctx = layers[0].get("context")
        U.attn_block(h, layers[0], cfg.groups, cfg.heads, cfg.eps, context=None if ctx is None else ctx[:n], gated=cfg.gated)
    dt = time.perf_counter() - t0
    what = "residual + attention block" if cfg.heads > 0 else "block"
    return {"value": n * cfg.height * cfg.width / (dt * cfg.layers), "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"{what} 1 of {cfg.layers} on {n} of {cfg.batch} images in fp64 ({dt:.1f} s), scaled to {cfg.layers} layers"}


def cpu_baseline_rows(cfg, x, layers, cores):
    """The oracle as it stands on a bounded sample of a long sequence: the keys and values of every
    token of layer 1 (which any row needs) and 64 blocks of 16 query rows spread evenly over the
    sequence, through attention, output projection and feed-forward; scaled to all rows and layers."""
    from oracle import transformer as O
    S = cfg.seq
    t0 = time.perf_counter()
    O.transformer_block_row_blocks(x, layers[0], cfg.heads, cfg.causal, [], cfg.activation, cfg.ln_eps)
    t_kv = time.perf_counter() - t0
    n_blocks = 64          # about ten seconds of oracle time on the machine's host cores
    blocks = [(r, r + 16) for r in range(S // (2 * n_blocks), S, S // n_blocks)][:n_blocks]
    n_rows = sum(b - a for a, b in blocks)
    t0 = time.perf_counter()
    O.transformer_block_row_blocks(x, layers[0], cfg.heads, cfg.causal, blocks, cfg.activation, cfg.ln_eps)
    t_rows = max(time.perf_counter() - t0 - t_kv, 1e-9)
    per_layer = t_kv + t_rows * S / n_rows
    return {"value": S / (per_layer * cfg.layers), "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"layer 1 of {cfg.layers} in fp64: LayerNorm + key/value projection of all {S} tokens "
                      f"({t_kv:.1f} s) and {n_rows} query rows in {len(blocks)} blocks spread over the sequence through "
                      f"attention, output projection and feed-forward ({t_rows:.1f} s); scaled to {S} rows "
                      f"and {cfg.layers} layers"}


def cpu_baseline(cfg, x, layers):
    """The oracle as it stands on the host cores: whole layers where a layer takes seconds, else a
    row sample."""
    from oracle import transformer as O
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [os.cpu_count()])
    except Exception:
        cores = os.cpu_count()
    if cfg.seq > 16384:
        return cpu_baseline_rows(cfg, x, layers, cores)
    t0 = time.perf_counter()
    n = min(2, cfg.layers)
    O.transformer_stack(x, layers[:n], cfg.heads, cfg.causal, cfg.activation, cfg.ln_eps, cfg.batch,
                        query_block=1024)
    dt = time.perf_counter() - t0
    return {"value": cfg.tokens * n / (dt * cfg.layers), "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"layers 1-{n} of {cfg.layers} over all {cfg.tokens} tokens in fp64 ({dt:.1f} s), "
                      f"scaled to {cfg.layers} layers"}


BALANCE = PEAK["mfma_bf16"] / PEAK["hbm"]     # 312.5 flop per byte: below it a bf16 kernel is HBM-bound


def class_entry(s, steps, dtype):
    """Roofline entry of a kernel class from its event-timed launches.  The bound follows the
    arithmetic intensity of the class (algorithmic flops / algorithmic bytes against the machine
    balance), not its name: a contraction over few rows that re-reads a large operand is HBM-bound."""
    sec = s["total_ms"] * 1e-3
    contraction = s["name"] in ("gemm", "attention", "trimul")
    intensity = s["flops"] / s["bytes"] if s["bytes"] else float("inf")
    if contraction and dtype == "bf16" and intensity >= BALANCE:
        bound, ach, pk, unit = "mfma", s["flops"] / sec / 1e12, PEAK["mfma_bf16"] / 1e12, "TFLOP/s"
    elif contraction and dtype == "f32" and intensity >= PEAK["fp32_vector"] / PEAK["hbm"]:
        bound, ach, pk, unit = "alu", s["flops"] / sec / 1e12, PEAK["fp32_vector"] / 1e12, "TFLOP/s"
    else:
        bound, ach, pk, unit = "hbm", s["bytes"] / sec / 1e9, PEAK["hbm"] / 1e9, "GB/s"
    entry = {"bound": bound, "achieved": round(ach, 2), "peak": pk, "unit": unit, "frac": round(ach / pk, 4),
             "launches_per_step": s["launches"] // steps, "avg_launch_us": round(s["total_ms"] / s["launches"] * 1e3, 2),
             "ms_per_step": round(s["total_ms"] / steps, 4), "flop_per_byte": round(intensity, 1)}
    if contraction and bound == "hbm":
        entry["tflops"] = round(s["flops"] / sec / 1e12, 2)
    return entry


KERNEL_SOURCES = {"gemm": ["linear.hip", "common.h"], "trimul": ["linear.hip", "common.h"],
                  "attention": ["attention.hip", "common.h"], "layernorm": ["rowwise.hip", "common.h"],
                  "elementwise": ["rowwise.hip", "common.h"]}


def source_digest(kernel_class):
    """sha256 over the sources of a kernel class: counters taken from an older kernel do not count."""
    import hashlib
    h = hashlib.sha256()
    for name in KERNEL_SOURCES[kernel_class]:
        with open(os.path.join(ROOT, "paper_2401_10652_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def recorded_traffic(workload, kernel_class):
    """HBM bytes per launch from the committed rocprofv3 --pmc summary (FETCH_SIZE / WRITE_SIZE, each
    scaled by what the same counter reads for a plain copy of known size), or None if there is no
    summary for this workload and kernel class or the kernel's sources changed since it was taken."""
    path = os.path.join(ROOT, "profiles", f"traffic_{workload}.json")
    if not os.path.exists(path):
        return None
    with open(path) as f:
        rec = json.load(f)
    k = rec.get("kernels", {}).get(kernel_class)
    if not k or k.get("sources_sha256") != source_digest(kernel_class):
        return None
    return round((k["fetch_kib_per_launch"] * rec["fetch_scale"] + k["write_kib_per_launch"] * rec["write_scale"]) * 1024)


def copy_calibration(B, torch, steps):
    """A plain copy kernel of known size, for scaling the FETCH_SIZE / WRITE_SIZE counters."""
    n_rows, n_cols = 32768, 4096   # 256 MiB of bf16 read, 256 MiB written
    x = torch.zeros((n_rows, n_cols), dtype=torch.bfloat16, device="cuda")
    y = torch.empty_like(x)
    for _ in range(steps):
        B.ac_op_bias_act(x, None, y, B.AC_ACT_NONE)
    torch.cuda.synchronize()
    print(json.dumps({"copy_calibration": True, "kernel": "bias_act_vec", "launches": steps,
                      "bytes_read_per_launch": n_rows * n_cols * 2, "bytes_written_per_launch": n_rows * n_cols * 2}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="C5", choices=["C1", "C2", "C3", "C4", "C5", "U1", "U2"],
                    help="workload (default: C5, the largest that one GPU holds; beside the five: U1, UNet residual blocks; "
                         "U2, a residual block followed by an attention block)")
    ap.add_argument("--chunk", type=int, nargs=3, default=None, metavar=("QKV", "ATTN", "FFN"),
                    help="rows per segment for the three regions (default: the workload's plan)")
    ap.add_argument("--in-flight", type=int, default=1, choices=[1, 2],
                    help="segments of a region in flight at once (2: two streams, two per-segment workspaces)")
    ap.add_argument("--pair-dim", default="row", choices=["row", "col", "natural"],
                    help="pair stack: chunk along rows (the workload's plan) or columns of z")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--sequential-only", action="store_true",
                    help="skip the extra two-segments-in-flight timing (its overlapping kernels would "
                         "distort per-kernel durations in a profiler trace)")
    ap.add_argument("--sweep", action="store_true", help="also time a sweep of chunk lengths")
    ap.add_argument("--budget-on", default="executor", choices=["executor", "paper-model"],
                    help="what the workload's activation budget bounds in the headline plan: the bytes the "
                         "executor really holds, or also the paper-style bytes of the unfused graph")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run a plain 256 MiB copy kernel --steps times (for scaling rocprofv3 byte counters)")
    args = ap.parse_args()
    global PAIR_DIM
    PAIR_DIM = args.pair_dim
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2401_10652_amd import binding as B
    from paper_2401_10652_amd import inputs as I

    from paper_2401_10652_amd.build import ensure_built
    ensure_built()      # loads what is built; compiles only when nothing is
    B.lib()
    torch.cuda.set_device(0)
    if args.copy_calibration:
        copy_calibration(B, torch, args.steps)
        return
    cfg = I.CONFIGS[args.config]
    is_pair = isinstance(cfg, I.PairConfig)
    lanes_flag = B.AC_FLAG_TWO_SEGMENTS_IN_FLIGHT if args.in_flight == 2 else 0
    pm_flag = B.AC_FLAG_BUDGET_PAPER_MODEL
    is_res = isinstance(cfg, I.ResStackConfig)
    if is_res:
        x, layers = I.res_stack_inputs(cfg)
        names = I.RES_BLOCK_TENSORS + I.attn_block_tensors(cfg)
        flat = lambda t: t.reshape(t.shape[0], -1) if t.ndim == 4 else t.reshape(-1, t.shape[-1]) if t.ndim == 3 else t
        dw = [B.to_device(flat(w[n]), cfg.dtype) for w in layers for n in names]
        make_desc = lambda flags: B.res_stack_desc(cfg, flags=flags)
        res_regions = lambda c: [(k, B.AC_DIM_BATCH, c) for k in ((B.AC_REGION_RES_BLOCK, B.AC_REGION_UNET_ATTN) if cfg.heads > 0
                                                                  else (B.AC_REGION_RES_BLOCK,))]
        regs, budget = res_regions(args.chunk[0] if args.chunk else cfg.chunk_len), 0
        regs1 = res_regions(cfg.batch)
    elif is_pair:
        x, layers = I.pair_inputs(cfg)
        dw = [B.to_device(layers[n], cfg.dtype) for n, _ in I.pair_tensor_shapes(cfg)]
        make_desc = lambda flags: B.pair_desc(cfg, flags=flags)
        regs, budget = pair_regions(B, args.chunk[0] if args.chunk else cfg.chunk_len), 0
        regs1 = pair_regions(B, cfg.n_res)
    else:
        x, layers = I.transformer_inputs(cfg)
        dw = [B.to_device(w[n], cfg.dtype) for w in layers for n in I.TRANSFORMER_LAYER_TENSORS]
        make_desc = lambda flags: B.transformer_desc(cfg, flags=flags)
        if args.chunk:
            regs, budget = plan_regions(B, *args.chunk), 0
        elif cfg.chunk_len:
            regs, budget = plan_regions(B, cfg.chunk_len, cfg.chunk_len, cfg.chunk_len), 0
        else:
            regs, budget = plan_regions(B, 0, 0, 0, 0), cfg.act_budget
        regs1 = plan_regions(B, cfg.seq, cfg.seq, cfg.seq)
    desc = make_desc(lanes_flag | (pm_flag if budget and args.budget_on == "paper-model" else 0))
    dx = B.to_device(x, cfg.dtype)
    y = torch.empty_like(dx)
    plan = B.Plan(desc, regs, budget)
    info = plan.ac_plan_query()
    plan.ac_plan_bind_weights(dw)
    plan1 = B.Plan(make_desc(lanes_flag), regs1, 0)
    info1 = plan1.ac_plan_query()
    plan1.ac_plan_bind_weights(dw)
    ws = B.empty_workspace(max(info.workspace_bytes, info1.workspace_bytes))

    sec, peak = time_plan(B, torch, plan, dx, y, ws, args.steps, args.warmup)
    sec1, peak1 = time_plan(B, torch, plan1, dx, y, ws, args.steps, args.warmup)
    stats = profile_plan(plan, dx, y, ws, args.steps)

    tokens = cfg.tokens
    classes = {s["name"]: class_entry(s, args.steps, cfg.dtype) for s in stats}
    dom = max(classes, key=lambda k: classes[k]["ms_per_step"])
    s_dom = next(s for s in stats if s["name"] == dom)
    roof = dict(classes[dom])
    roof.update({"kernel": dom, "traffic": recorded_traffic(cfg.name, dom),
                 "algorithmic_per_launch": round((s_dom["bytes"] if roof["bound"] == "hbm" else s_dom["flops"]) / s_dom["launches"])})

    def chunk_lens(inf):
        return {"chunk_len": [inf.regions[i].chunk_len for i in range(inf.n_regions)],
                "n_segments": [inf.regions[i].n_segments for i in range(inf.n_regions)]}

    out = {
        "metric": "tokens/s at fixed activation budget",
        "value": round(tokens / sec, 1), "unit": "tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(sec * 1e3, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": dict(
            {"workload": cfg.name, "act_budget_bytes": budget,
             "budget_bounds": ("executor bytes" if args.budget_on == "executor" else "executor and paper-model bytes") if budget else None,
             "segments_in_flight": args.in_flight, **chunk_lens(info),
             **({"chunk_dim": args.pair_dim} if is_pair else {})},
            **({"layers": cfg.layers, "batch": cfg.batch, "height": cfg.height, "width": cfg.width, "channels": cfg.channels,
                "groups": cfg.groups, "heads": cfg.heads, "d_ffn": cfg.d_ffn, "context_tokens": cfg.context_tokens,
                "context_dim": cfg.context_dim, "gated_ffn": cfg.gated, "tokens": "pixels (batch * height * width)"} if is_res else
               {"n_res": cfg.n_res, "c_z": cfg.c_z, "c_hidden": cfg.c_hidden, "heads": cfg.heads,
                "head_dim": cfg.head_dim, "tokens": "pair positions (n_res^2)"} if is_pair else
               {"layers": cfg.layers, "seq": cfg.seq, "d_model": cfg.d_model, "heads": cfg.heads,
                "d_ffn": cfg.d_ffn, "causal": cfg.causal})),
        "roofline": roof,
        "kernels": classes,
        "mfma_frac_whole_step": round(info.flops_per_execute / sec / PEAK["mfma_bf16"], 4),
        "one_segment_per_region": {"tokens_per_s": round(tokens / sec1, 1), "ms_per_step": round(sec1 * 1e3, 4),
                                   "throughput_loss_of_the_plan": round(1.0 - sec1 / sec, 4)},
        # like-for-like ratios only: this executor chunked vs this executor with one segment per
        # region (measured), and the paper-style model of an unfused graph chunked vs unchunked
        "peak_activation_bytes": {
            "chunked_measured": peak, "one_segment_measured": peak1,
            "ratio_measured": round(peak / peak1, 4),
            "paper_model_chunked": info.peak_bytes_model, "paper_model_one_segment": info.peak_bytes_model_unchunked,
            "ratio_paper_model": round(info.peak_bytes_model / info.peak_bytes_model_unchunked, 4),
        },
    }
    extras = not args.sequential_only

    def timed_variant(flags, rg, bud, steps=None):
        p_ = B.Plan(make_desc(flags), rg, bud)
        i_ = p_.ac_plan_query()
        p_.ac_plan_bind_weights(dw)
        w_ = ws if i_.workspace_bytes <= ws.numel() else B.empty_workspace(i_.workspace_bytes)
        s_, pk_ = time_plan(B, torch, p_, dx, y, w_, steps or args.steps, args.warmup)
        entry = {"ms_per_step": round(s_ * 1e3, 4), "tokens_per_s": round(tokens / s_, 1),
                 "throughput_loss": round(1.0 - sec1 / s_, 4), "peak_bytes_measured": pk_,
                 "peak_ratio_vs_one_segment": round(pk_ / peak1, 4), **chunk_lens(i_)}
        p_.close()
        return entry

    if extras and budget and args.budget_on == "executor":
        # The same budget read as a planner of the paper would read it: a bound on the bytes of the
        # unfused graph (scores and probabilities of a segment stored), section 3.2 / 3.4.
        out["budget_on_paper_model_bytes"] = timed_variant(lanes_flag | pm_flag, regs, budget)
        # A budget that does bind on the executor's own bytes: 0.8 of what one segment per region needs.
        tight = int(0.8 * peak1)
        try:
            out["tight_budget_on_executor_bytes"] = dict(timed_variant(lanes_flag, regs, tight), act_budget_bytes=tight)
        except B.AcError as err:
            out["tight_budget_on_executor_bytes"] = {"act_budget_bytes": tight, "error": str(err)}
    if extras and args.in_flight == 1:
        # the same plan with two segments of a region in flight on two streams (an executor option
        # on top of the strictly sequential schedule timed above)
        out["two_segments_in_flight"] = timed_variant(desc.flags | B.AC_FLAG_TWO_SEGMENTS_IN_FLIGHT, regs, budget)
    if extras and is_pair and args.pair_dim == "row":
        # The workload fixes row chunks.  The ending node's attention has one problem per COLUMN, so a row
        # chunk gives each problem 64 queries and reads every key and value of the tensor per segment; the
        # same module chunked along columns (legal by section 3.3, and the dimension the stride term of
        # section 3.4 prefers) is the starting node's form on a gathered segment.  Reported beside the plan.
        natural = [(k, B.AC_DIM_COL if k == B.AC_REGION_TRIATT_END else d, c) for (k, d, c) in regs]
        out["ending_node_chunked_along_columns"] = timed_variant(desc.flags, natural, budget)
        out["ending_node_chunked_along_columns"]["two_segments_in_flight_ms_per_step"] = timed_variant(
            desc.flags | B.AC_FLAG_TWO_SEGMENTS_IN_FLIGHT, natural, budget)["ms_per_step"]
    if extras and not is_res and not (is_pair and args.pair_dim != "row"):
        # The standalone row passes (bias + activation, residual add, LayerNorm), which the fused
        # plan folds into GEMM epilogues, timed with HIP events in a plan that runs them unfused.
        pu = B.Plan(make_desc(B.AC_FLAG_UNFUSED_ELEMENTWISE), regs, 0 if is_pair else budget)
        iu = pu.ac_plan_query()
        pu.ac_plan_bind_weights(dw)
        wu = ws if iu.workspace_bytes <= ws.numel() else B.empty_workspace(iu.workspace_bytes)
        for _ in range(2):
            pu.ac_execute(dx, y, wu)
        su = profile_plan(pu, dx, y, wu, max(3, args.steps // 4))
        out["standalone_row_passes"] = {s_["name"]: class_entry(s_, max(3, args.steps // 4), cfg.dtype)
                                        for s_ in su if s_["name"] in ("elementwise", "layernorm")}
        pu.close()
        del wu
    if extras and not is_pair and not is_res:
        # The same two plans with the attention core run as an unfused graph would (scores and
        # probabilities stored in the workspace): here the workspace really holds the intermediate
        # activations the paper's equations count, so the memory ratio of chunking is measured.
        sflags = B.AC_FLAG_MATERIALIZED_SCORES | (pm_flag if budget else 0)
        stored = {}
        for label, rg, bud in (("chunked", regs, budget), ("one_segment", regs1, 0)):
            p3 = B.Plan(make_desc(sflags if bud else B.AC_FLAG_MATERIALIZED_SCORES), rg, bud)
            i3 = p3.ac_plan_query()
            entry = {"peak_bytes_planned": int(i3.peak_bytes_planned), **chunk_lens(i3)}
            if i3.workspace_bytes <= 48 << 30:      # the whole score tensor of a long sequence may not fit
                p3.ac_plan_bind_weights(dw)
                ws3 = B.empty_workspace(i3.workspace_bytes)
                s3, pk3 = time_plan(B, torch, p3, dx, y, ws3, max(3, args.steps // 4), 1)
                entry.update({"ms_per_step": round(s3 * 1e3, 4), "tokens_per_s": round(tokens / s3, 1),
                              "peak_bytes_measured": pk3})
                del ws3
            stored[label] = entry
            p3.close()
        stored["peak_ratio_chunked_vs_one_segment"] = round(
            stored["chunked"]["peak_bytes_planned"] / stored["one_segment"]["peak_bytes_planned"], 4)
        if "ms_per_step" in stored["chunked"] and "ms_per_step" in stored["one_segment"]:
            stored["throughput_loss"] = round(1.0 - stored["one_segment"]["ms_per_step"] / stored["chunked"]["ms_per_step"], 4)
        out["stored_scores"] = stored
        if budget:
            # The planning passes on the unfused graph of the same stack at the same budget (host
            # code: estimate, search around the peak, select, repeated), and the stored-scores
            # executor run with the chunks they choose.
            from paper_2401_10652_amd import graphs as PG
            spec, names = PG.transformer_stack_graph(cfg.batch, cfg.seq, cfg.d_model, cfg.heads, cfg.d_ffn, cfg.layers)
            nodes = B.graph_nodes(spec)
            e = 2 if cfg.dtype == "bf16" else 4
            _, whole, _ = B.ac_graph_estimate(nodes, e)
            t0 = time.perf_counter()
            chunks, planned = B.ac_graph_plan(nodes, e, budget, 12, (1.0, 0.0, 0.0, 0.0), beam=2, max_out=4 * cfg.layers)
            plan_ms = (time.perf_counter() - t0) * 1e3
            settings = PG.executor_regions(chunks, names)
            p4 = B.Plan(make_desc(B.AC_FLAG_MATERIALIZED_SCORES), settings, 0)
            i4 = p4.ac_plan_query()
            entry = {"graph_nodes": len(spec), "estimate_unchunked_bytes": whole, "estimate_planned_bytes": planned,
                     "planning_ms": round(plan_ms, 3), "chunks": len(chunks), "window": 12, "beam": 2,
                     "weights": [1.0, 0.0, 0.0, 0.0], "executor_regions": [list(s) for s in settings],
                     "executor_peak_bytes_planned": int(i4.peak_bytes_planned)}
            if i4.workspace_bytes <= 48 << 30:
                p4.ac_plan_bind_weights(dw)
                ws4 = B.empty_workspace(i4.workspace_bytes)
                s4, pk4 = time_plan(B, torch, p4, dx, y, ws4, max(3, args.steps // 4), 1)
                entry.update({"ms_per_step": round(s4 * 1e3, 4), "executor_peak_bytes_measured": pk4})
                del ws4
            p4.close()
            out["planned_on_the_graph"] = entry
    if args.sweep:
        sweep = []
        c = cfg.batch if is_res else cfg.n_res if is_pair else cfg.seq
        while c >= (1 if is_res else 8 if is_pair else 128):
            ps = B.Plan(desc, res_regions(c) if is_res else pair_regions(B, c) if is_pair else plan_regions(B, c, c, c), 0)
            ps.ac_plan_bind_weights(dw)
            inf = ps.ac_plan_query()
            if inf.workspace_bytes > ws.numel():
                ws = B.empty_workspace(inf.workspace_bytes)
            s_, pk_ = time_plan(B, torch, ps, dx, y, ws, max(3, args.steps // 2), 1)
            sweep.append({"chunk_len": c, "tokens_per_s": round(tokens / s_, 1), "peak_bytes": pk_,
                          "paper_model_bytes": inf.peak_bytes_model})
            ps.close()
            c //= 2
        out["sweep"] = sweep
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline_res(cfg, x, layers) if is_res else cpu_baseline_pair(cfg, x, layers) if is_pair else cpu_baseline(cfg, x, layers)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
