"""GPU parity of whole chunk plans against the unchunked fp64 oracle, through the C-ABI."""
import numpy as np
import pytest

from oracle import transformer as O
from paper_2401_10652_amd import inputs as I
from util import TOL, check, host, rel_err

pytestmark = pytest.mark.gpu

CANARY = 0x5A


@pytest.fixture(scope="module")
def B():
    from paper_2401_10652_amd import binding
    binding.lib()
    return binding


def regions(B, c_qkv, c_attn, c_ffn, dim=None, c_out=None):
    dim = B.AC_DIM_SEQ if dim is None else dim
    return [(B.AC_REGION_QKV, dim, c_qkv), (B.AC_REGION_ATTENTION, dim, c_attn),
            (B.AC_REGION_OUT_PROJ, dim, c_attn if c_out is None else c_out), (B.AC_REGION_FFN, dim, c_ffn)]


class Runner:
    """Uploads one workload, runs plans on it; every buffer is a torch tensor."""

    def __init__(self, B, cfg, bias_std=0.0, ln_jitter=0.0):
        import torch
        self.B, self.cfg = B, cfg
        self.x, self.layers = I.transformer_inputs(cfg, bias_std=bias_std, ln_jitter=ln_jitter)
        self.dx = B.to_device(self.x, cfg.dtype)
        self.dw = [B.to_device(w[name], cfg.dtype) for w in self.layers for name in I.TRANSFORMER_LAYER_TENSORS]
        self.torch = torch

    def run(self, regs, budget=0, flags=0, slack=4096):
        B, torch = self.B, self.torch
        p = B.Plan(B.transformer_desc(self.cfg, flags=flags), regs, budget)
        info = p.ac_plan_query()
        assert p.weight_names() == [f"L{l}.{n}" for l in range(self.cfg.layers) for n in I.TRANSFORMER_LAYER_TENSORS]
        p.ac_plan_bind_weights(self.dw)
        need = int(info.workspace_bytes)
        ws = torch.full((need + slack,), CANARY, dtype=torch.uint8, device="cuda")
        y = torch.full_like(self.dx, float("nan"))
        peak = p.ac_execute(self.dx, y, ws[:need])
        torch.cuda.synchronize()
        # nothing beyond the declared workspace was touched, and the input is intact
        assert bool((ws[need:] == CANARY).all())
        assert torch.equal(self.dx, B.to_device(self.x, self.cfg.dtype))
        assert peak == info.peak_bytes_planned
        p.close()
        return y, info

    def oracle(self, query_block=None):
        c = self.cfg
        return O.transformer_stack(self.x, self.layers, c.heads, c.causal, c.activation, c.ln_eps, c.batch,
                                   query_block=query_block)


def test_c1_block_fp32_chunked_and_unchunked(B):
    r = Runner(B, I.C1)
    ref = r.oracle()
    y4, info4 = r.run(regions(B, 64, 64, 64))
    y1, info1 = r.run(regions(B, 256, 256, 256))
    assert [x.n_segments for x in info4.regions[:4]] == [4, 4, 4, 4]
    check(host(y4), ref, "f32")
    check(host(y1), ref, "f32")
    assert info4.peak_bytes_planned < info1.peak_bytes_planned
    assert info4.peak_bytes_unchunked_planned == info1.peak_bytes_planned


def test_fp32_every_epilogue_and_ragged_lengths(B):
    cfg = I.TransformerConfig("t32", 31, 2, 200, 64, 4, 160, True, "f32", None, activation="gelu_tanh")
    r = Runner(B, cfg, bias_std=0.3, ln_jitter=0.2)
    ref = r.oracle()
    outs = []
    for c in ((200, 200, 200), (64, 64, 64), (33, 77, 50), (1, 200, 7)):
        y, _ = r.run(regions(B, *c))
        check(host(y), ref, "f32", what=str(c), depth=2)
        outs.append(y)
    yu, _ = r.run(regions(B, 64, 64, 64), flags=B.AC_FLAG_UNFUSED_ELEMENTWISE)
    check(host(yu), ref, "f32", depth=2)


@pytest.mark.parametrize("causal,heads,act", [(True, 4, "gelu_erf"), (False, 8, "relu"), (False, 2, "gelu_tanh")])
def test_bf16_stack_chunked_equals_oracle(B, causal, heads, act):
    import torch
    cfg = I.TransformerConfig("t16", 32, 2, 640, 256, heads, 1024, causal, "bf16", 0.05, activation=act)
    r = Runner(B, cfg, bias_std=0.05, ln_jitter=0.1)
    ref = r.oracle()
    outs = []
    for c in ((640, 640, 640), (128, 128, 128), (256, 384, 512), (200, 136, 72), (640, 8, 640)):
        y, info = r.run(regions(B, *c, c_out=c[0]))
        check(host(y), ref, "bf16", what=str(c), depth=2)
        outs.append(y)
    # the K loop and the key-tile order do not depend on the segment a row falls in:
    # every chunk length gives bit-identical output
    for y in outs[1:]:
        assert torch.equal(y, outs[0])
    yu, _ = r.run(regions(B, 128, 128, 128), flags=B.AC_FLAG_UNFUSED_ELEMENTWISE)
    check(host(yu), ref, "bf16", depth=2)


def test_batch_and_batch_chunks(B):
    import torch
    cfg = I.TransformerConfig("tb", 33, 1, 136, 128, 2, 256, True, "bf16", 0.05, batch=3)
    r = Runner(B, cfg, bias_std=0.05, ln_jitter=0.1)
    ref = r.oracle()
    ys, _ = r.run(regions(B, 64, 64, 64))
    yb, info = r.run(regions(B, 2, 1, 3, dim=B.AC_DIM_BATCH))
    assert [x.n_segments for x in info.regions[:4]] == [2, 3, 3, 1]
    check(host(ys), ref, "bf16")
    check(host(yb), ref, "bf16")
    assert torch.equal(ys, yb)
    cfg32 = I.TransformerConfig("tb32", 34, 1, 50, 32, 2, 64, False, "f32", None, batch=2)
    r32 = Runner(B, cfg32, bias_std=0.2)
    y, _ = r32.run(regions(B, 1, 2, 1, dim=B.AC_DIM_BATCH))
    check(host(y), r32.oracle(), "f32")


def test_feature_chunks(B):
    """Section 3.3 leaves two feature dims legal: the attention core in runs of whole heads and the
    output projection in blocks of output columns.  Both span all rows.  Fused, neither region holds a
    tensor per segment, so the segments share one launch; with stored scores a head chunk divides the
    stored score and probability tensors, and the unfused output projection holds its block only."""
    import torch
    cfg = I.TransformerConfig("tfeat", 37, 2, 200, 128, 4, 256, True, "bf16", 0.05, batch=2)
    r = Runner(B, cfg, bias_std=0.05, ln_jitter=0.1)
    ref = r.oracle()
    F, S_ = B.AC_DIM_FEATURE, B.AC_DIM_SEQ
    plan = lambda c_att, c_out: [(B.AC_REGION_QKV, S_, 64), (B.AC_REGION_ATTENTION, F, c_att),
                                 (B.AC_REGION_OUT_PROJ, F, c_out), (B.AC_REGION_FFN, S_, 64)]
    y0, _ = r.run(regions(B, 64, 64, 64))
    yf, info = r.run(plan(64, 48))
    assert [x.n_segments for x in info.regions[1:3]] == [2, 3] and [x.launches for x in info.regions[1:3]] == [1, 1]
    assert torch.equal(yf, y0)
    check(host(yf), ref, "bf16", depth=2)
    # stored scores: one head at a time
    st = B.AC_FLAG_MATERIALIZED_SCORES
    ys, i_whole = r.run(regions(B, 200, 200, 200), flags=st)
    yh, i_heads = r.run(plan(32, 128), flags=st)
    assert i_heads.regions[1].n_segments == 4 and i_heads.regions[1].launches == 4
    assert torch.equal(yh, ys)
    check(host(yh), ref, "bf16", depth=2)
    al = lambda n: (n + 255) // 256 * 256
    scores = lambda batch, heads: 2 * al(batch * heads * cfg.seq * cfg.seq * 2)     # scores + probabilities, bf16
    # a sequence segment is one batch element with all its heads, a head segment all batch elements with one head
    assert i_whole.workspace_bytes - i_heads.workspace_bytes == scores(1, 4) - scores(cfg.batch, 1)
    # unfused output projection, one block of 32 columns at a time
    un = B.AC_FLAG_UNFUSED_ELEMENTWISE
    yu0, _ = r.run(regions(B, 64, 64, 64), flags=un)
    yu, i_un = r.run(plan(128, 32), flags=un)
    assert i_un.regions[2].launches == 4
    assert torch.equal(yu, yu0)
    check(host(yu), ref, "bf16", depth=2)


def test_budget_sized_plan_runs(B):
    cfg = I.TransformerConfig("tbud", 35, 1, 1024, 256, 4, 1024, True, "bf16", 0.05)
    r = Runner(B, cfg)
    ref = r.oracle()
    # the budget bounds what the executor holds: the feed-forward region (hidden tensor) and the
    # attention core (fp32 partial results of its key splits) have to be cut
    budget = 9 << 19
    y, info = r.run(regions(B, 0, 0, 0), budget=budget)
    assert [x.n_segments for x in info.regions[:4]] == [1, 2, 1, 2] and info.regions[3].chunk_len == 512
    assert info.regions[1].launches == 1       # the attention's two segments share a launch with capped key splits
    assert info.peak_bytes_planned <= budget < info.peak_bytes_unchunked_planned
    check(host(y), ref, "bf16")
    # ... and, on request, the paper-style bytes of the unfused graph as well: the attention core is cut
    budget = 6 << 20
    y, info = r.run(regions(B, 0, 0, 0), budget=budget, flags=B.AC_FLAG_BUDGET_PAPER_MODEL)
    assert info.regions[1].n_segments > 1 and info.peak_bytes_model <= budget and info.peak_bytes_planned <= budget
    check(host(y), ref, "bf16")


def test_profiling_reports_kernel_classes(B):
    import torch
    cfg = I.TransformerConfig("tprof", 36, 2, 256, 128, 2, 512, False, "bf16", 0.05)
    r = Runner(B, cfg)
    p = B.Plan(B.transformer_desc(cfg), regions(B, 128, 128, 128))
    info = p.ac_plan_query()
    p.ac_plan_bind_weights(r.dw)
    ws = B.empty_workspace(info.workspace_bytes)
    y = torch.empty_like(r.dx)
    p.ac_plan_set_profiling(True)
    p.ac_execute(r.dx, y, ws)
    stats = {s["name"]: s for s in p.ac_plan_read_profile()}
    assert set(stats) == {"gemm", "attention", "layernorm"}
    # per layer: the two segments of the feed-forward region run 2 GEMMs each; those of the
    # other three regions hold no tensor of their own and share one launch (LayerNorm + GEMM, attention, GEMM)
    assert stats["gemm"]["launches"] == 2 * (1 + 1 + 2 * 2) and stats["attention"]["launches"] == 2
    assert [x.n_segments for x in info.regions[:4]] == [2, 2, 2, 2]
    assert [x.launches for x in info.regions[:4]] == [1, 1, 1, 2]
    assert stats["layernorm"]["launches"] == 2 * 2      # both LayerNorms of a layer run over all rows at once
    total = sum(s["flops"] for s in stats.values())
    assert abs(total - info.flops_per_execute) <= 1e-9 * total
    assert all(s["total_ms"] > 0 for s in stats.values())
    assert p.ac_plan_read_profile() == []
    p.ac_plan_set_profiling(False)
    with pytest.raises(B.AcError) as ei:
        p.ac_plan_read_profile()
    assert ei.value.status == B.AC_ERR_STATE
    y2 = torch.empty_like(r.dx)
    p.ac_execute(r.dx, y2, ws)
    torch.cuda.synchronize()
    assert torch.equal(y, y2)


def test_two_segments_in_flight_equals_sequential(B):
    """Segments alternate between two streams with separate per-segment workspaces: same bits,
    larger planned (and measured) workspace, nothing outside it touched."""
    import torch
    cfg = I.TransformerConfig("t2s", 37, 3, 1152, 256, 4, 1024, True, "bf16", 0.05)
    r = Runner(B, cfg, bias_std=0.05, ln_jitter=0.1)
    ref = r.oracle()
    for c in ((128, 128, 128), (256, 384, 1152), (200, 136, 72)):
        y1, i1 = r.run(regions(B, *c))
        y2, i2 = r.run(regions(B, *c), flags=B.AC_FLAG_TWO_SEGMENTS_IN_FLIGHT)
        assert torch.equal(y1, y2), c
        assert i2.workspace_bytes >= i1.workspace_bytes
        check(host(y2), ref, "bf16", depth=3)
    # repeated executes of one plan reuse its second stream and events
    p = B.Plan(B.transformer_desc(cfg, flags=B.AC_FLAG_TWO_SEGMENTS_IN_FLIGHT), regions(B, 128, 128, 128))
    p.ac_plan_bind_weights(r.dw)
    ws = B.empty_workspace(p.ac_plan_query().workspace_bytes)
    outs = []
    for _ in range(3):
        y = torch.full_like(r.dx, float("nan"))
        p.ac_execute(r.dx, y, ws)
        outs.append(y)
    torch.cuda.synchronize()
    assert torch.equal(outs[0], outs[1]) and torch.equal(outs[0], outs[2])
    cfg32 = I.TransformerConfig("t2s32", 38, 1, 200, 64, 4, 160, False, "f32", None)
    r32 = Runner(B, cfg32, bias_std=0.2)
    ya, _ = r32.run(regions(B, 33, 77, 50))
    yb, _ = r32.run(regions(B, 33, 77, 50), flags=B.AC_FLAG_TWO_SEGMENTS_IN_FLIGHT)
    assert torch.equal(ya, yb)


@pytest.mark.parametrize("dtype,causal", [("f32", False), ("f32", True), ("bf16", True), ("bf16", False)])
def test_stored_scores_plans_equal_the_oracle(B, dtype, causal):
    """AC_FLAG_MATERIALIZED_SCORES: scores and probabilities are stored tensors of the segment, as
    in an unfused graph.  Same function as the fused kernel: oracle parity for one segment and
    for ragged segments, batch chunks included; close to the fused plan's output; the measured
    peak is the planned one and grows with the segment length as the paper's second activation
    equation says."""
    import torch
    cfg = I.TransformerConfig("tss", 41, 2, 320, 128, 4, 256, causal, dtype, 0.05 if dtype == "bf16" else None, batch=2)
    r = Runner(B, cfg, bias_std=0.1, ln_jitter=0.1)
    ref = r.oracle()
    flag = B.AC_FLAG_MATERIALIZED_SCORES
    y_fused, _ = r.run(regions(B, 320, 320, 320))
    peaks = []
    for c in (320, 128, 72):
        y, info = r.run(regions(B, 320, c, 320, c_out=320), flags=flag)
        check(host(y), ref, dtype, depth=2)
        check(host(y), host(y_fused), dtype, depth=2)
        peaks.append(info.workspace_bytes)
    assert peaks[0] > peaks[1] > peaks[2]
    e = 2 if dtype == "bf16" else 4
    # whole minus 128-row segments: at least the scores + probabilities of (320 - 128) rows
    assert peaks[0] - peaks[1] >= 2 * cfg.heads * (320 - 128) * 320 * e
    # chunked along the batch: one problem per segment
    y, info = r.run(regions(B, 1, 1, 1, dim=B.AC_DIM_BATCH), flags=flag)
    check(host(y), ref, dtype, depth=2)
    y2, _ = r.run(regions(B, 1, 1, 1, dim=B.AC_DIM_BATCH), flags=flag | B.AC_FLAG_TWO_SEGMENTS_IN_FLIGHT)
    assert torch.equal(y, y2)


@pytest.mark.parametrize("dtype,batch", [("f32", 1), ("bf16", 2)])
def test_chunks_planned_on_the_graph_run_in_the_executor(B, dtype, batch):
    """The whole chain: the unfused graph of the stack is chunked to half its estimated peak by
    ac_graph_plan (sections 3.2 to 3.4), the chunks are handed to the executor as region settings,
    and the stored-scores plan they give equals the oracle and really needs less workspace."""
    from paper_2401_10652_amd import graphs as PG
    cfg = I.TransformerConfig("tgp", 43, 2, 384, 128, 4, 256, True, dtype, 0.05 if dtype == "bf16" else None, batch=batch)
    e = 2 if dtype == "bf16" else 4
    spec, names = PG.transformer_stack_graph(cfg.batch, cfg.seq, cfg.d_model, cfg.heads, cfg.d_ffn, cfg.layers)
    nodes = B.graph_nodes(spec)
    _, whole, peak_node = B.ac_graph_estimate(nodes, e)
    assert peak_node == names["scaled"]
    chunks, peak = B.ac_graph_plan(nodes, e, whole // 2, 12, (1.0, 0.0, 0.0, 0.0), beam=2)
    assert chunks and peak <= whole // 2
    settings = PG.executor_regions(chunks, names)
    assert [s[0] for s in settings] == [B.AC_REGION_ATTENTION] and settings[0][2] < cfg.seq
    r = Runner(B, cfg, bias_std=0.1, ln_jitter=0.1)
    flag = B.AC_FLAG_MATERIALIZED_SCORES
    y, info = r.run(settings, flags=flag)
    check(host(y), r.oracle(), dtype, depth=2)
    assert info.regions[B.AC_REGION_ATTENTION].n_segments > 1
    _, info_whole = r.run([], flags=flag)
    assert info.workspace_bytes < info_whole.workspace_bytes
