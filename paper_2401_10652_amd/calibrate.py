"""Fits the four weights of the selection cost L (AutoChunk section 3.4) to this GPU.

The paper tunes alpha, beta, gamma, lambda and prints no values.  This tool measures what L is
meant to predict, the speed a chunk costs: for a few transformer shapes it runs the executor with
one region kind at a time cut into SEGMENTS segments along the sequence (and the batch, where
there is one), takes loss = t_chunked / t_whole - 1, reads the four terms N_node, N_flop,
N_density, N_stride of the matching region of the stack's graph from ac_graph_chunk_cost, and
solves the least-squares problem loss ~ L.  It prints one JSON object: the weights, the fit's
R^2, the rank correlation of L with the measured losses, and every sample.

    python -m paper_2401_10652_amd.calibrate [--segments 4] [--steps 10]
"""
from __future__ import annotations

import argparse
import json
import time

import numpy as np

from . import binding as B
from . import graphs as G
from . import inputs as I

# (region kind, first node, last node) of one layer of transformer_stack_graph
KIND_SPANS = ((B.AC_REGION_QKV, "u", "qkv"), (B.AC_REGION_ATTENTION, "scores", "ctx"),
              (B.AC_REGION_OUT_PROJ, "o", "h"), (B.AC_REGION_FFN, "u2", "y"))
SHAPES = (  # name, layers, batch, seq, d_model, heads, d_ffn, causal
    ("gpt_s8192_d1024", 2, 1, 8192, 1024, 16, 4096, True),
    ("vit_s4096_d768", 2, 1, 4096, 768, 12, 3072, False),
    ("gpt_b4_s2048_d1024", 2, 4, 2048, 1024, 16, 4096, True),
    ("gpt_b2_s4096_d2048", 1, 2, 4096, 2048, 16, 8192, True),
)


def time_plan(torch, plan, x, y, ws, steps, repeats=3):
    """Best of `repeats` timings of `steps` executes (the first launches after a pause run at lower clocks)."""
    best = None
    for _ in range(repeats):
        for _ in range(3):
            plan.ac_execute(x, y, ws)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            plan.ac_execute(x, y, ws)
        torch.cuda.synchronize()
        t = (time.perf_counter() - t0) / steps
        best = t if best is None else min(best, t)
    return best


def terms(nodes, start, end, dim):
    """(N_node, N_flop, N_density, N_stride) of a region: L with one unit weight at a time."""
    return [B.ac_graph_chunk_cost(nodes, start, end, dim, [float(i == j) for j in range(4)]) for i in range(4)]


def ranks(v):
    order = np.argsort(v)
    r = np.empty(len(v))
    r[order] = np.arange(len(v))
    return r


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--segments", type=int, default=4)
    ap.add_argument("--steps", type=int, default=10)
    args = ap.parse_args()
    import torch
    B.lib()
    torch.cuda.set_device(0)
    samples = []
    for name, layers, batch, seq, d, heads, f, causal in SHAPES:
        cfg = I.TransformerConfig(name, 90, layers, seq, d, heads, f, causal, "bf16", 0.02, batch=batch)
        x, lw = I.transformer_inputs(cfg)
        dw = [B.to_device(w[n], cfg.dtype) for w in lw for n in I.TRANSFORMER_LAYER_TENSORS]
        dx = B.to_device(x, cfg.dtype)
        y = torch.empty_like(dx)
        desc = B.transformer_desc(cfg)
        spec, names = G.transformer_stack_graph(batch, seq, d, heads, f, layers)
        nodes = B.graph_nodes(spec)
        whole = B.Plan(desc, [], 0)
        whole.ac_plan_bind_weights(dw)
        ws = B.empty_workspace(whole.ac_plan_query().workspace_bytes)
        t_whole = time_plan(torch, whole, dx, y, ws, args.steps)
        first_sample = len(samples)
        for kind, first, last in KIND_SPANS:
            for dim_name, dim, graph_dim, extent in (("seq", B.AC_DIM_SEQ, 1, seq), ("batch", B.AC_DIM_BATCH, 0, batch)):
                if extent < args.segments:
                    continue
                plan = B.Plan(desc, [(kind, dim, -(-extent // args.segments))], 0)
                plan.ac_plan_bind_weights(dw)
                ws = B.empty_workspace(plan.ac_plan_query().workspace_bytes)
                t = time_plan(torch, plan, dx, y, ws, args.steps)
                plan.close()
                samples.append({"shape": name, "kind": kind, "dim": dim_name,
                                "terms": terms(nodes, names[first], names[last], graph_dim),
                                "ms_chunked": t * 1e3})
        # the unchunked plan once more, after everything else: the better of the two is the reference
        ws = B.empty_workspace(whole.ac_plan_query().workspace_bytes)
        t_whole = min(t_whole, time_plan(torch, whole, dx, y, ws, args.steps))
        whole.close()
        del ws
        for s in samples[first_sample:]:
            s["ms_whole"] = t_whole * 1e3
            s["loss"] = s["ms_chunked"] / s["ms_whole"] - 1.0
    a = np.array([s["terms"] for s in samples], dtype=np.float64)
    b = np.array([s["loss"] for s in samples], dtype=np.float64)
    scale = np.abs(a).max(axis=0)                    # columns differ by ten orders of magnitude
    w_scaled, *_ = np.linalg.lstsq(a / scale, b, rcond=None)
    weights = w_scaled / scale
    fit = a @ weights
    r2 = 1.0 - float(((b - fit) ** 2).sum() / ((b - b.mean()) ** 2).sum())
    rho = float(np.corrcoef(ranks(fit), ranks(b))[0, 1])
    for s, v in zip(samples, fit):
        s["L"] = float(v)
    print(json.dumps({"segments": args.segments, "weights": {"alpha": weights[0], "beta": weights[1], "gamma": weights[2],
                                                           "lambda": weights[3]},
                      "r2": r2, "rank_correlation": rho, "samples": samples}))


if __name__ == "__main__":
    main()
