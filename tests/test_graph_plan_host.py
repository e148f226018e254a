"""Graph memory estimate, selection cost and pass loop of the library (ac_graph_estimate,
ac_graph_chunk_cost, ac_graph_plan; AutoChunk sections 2.1, 2.2, 3.2, 3.4) against the
oracle's, value by value.  Host code only."""
import ctypes as C

import numpy as np
import pytest

from oracle import chunk_search as S
from oracle import graph_memory as GM
from paper_2401_10652_amd import binding as B
from paper_2401_10652_amd import graphs as PG
from paper_2401_10652_amd import inputs as I
from tests import graphs as G
from tests.test_oracle_graph_memory import hoisting_chunks, some_chunks
from tests.test_search_host import library_nodes, oracle_nodes

WEIGHTS = ((1, 0, 0, 0), (0, 0, 0, -1), (1.0, 1e-3, -1e-3, -0.5), (0.3, 2e-7, -1e-7, 0.01))


def test_estimate_equals_the_oracle():
    n_chunked = 0
    for seed in range(60):
        spec = G.random_graph(seed, n_ops=9 + seed % 6)
        on, ln = oracle_nodes(spec), library_nodes(spec)
        rng = np.random.default_rng(seed)
        for chunks in ([], some_chunks(on, rng, 3)):
            for e in (2, 4):
                assert B.ac_graph_estimate(ln, e, chunks) == GM.estimate(on, e, chunks), (seed, chunks)
            n_chunked += len(chunks)
    assert n_chunked > 60


def test_estimate_with_moved_nodes_equals_the_oracle():
    n_moved = 0
    block, nm = S.transformer_block_graph(2, 12, 8, 2, 16)
    kv = tuple(sorted(nm[x + s] for x in "kv" for s in ("_flat", "_split", "_h")))
    cases = [([(nd.op, nd.inputs, nd.shape, nd.attr, None) for nd in block], [(nm["q_flat"], nm["ctx"], 1, 4, kv)])]
    cases += [(G.random_graph(seed, n_ops=12 + seed % 6), None) for seed in range(220)]
    for seed, (spec, chunks) in enumerate(cases):
        on, ln = oracle_nodes(spec), library_nodes(spec)
        if chunks is None:
            chunks = hoisting_chunks(on, np.random.default_rng(seed))
        assert B.ac_graph_estimate(ln, 2, [c[:4] + (1,) for c in chunks]) == GM.estimate(on, 2, chunks), (seed, chunks)
        for c in chunks:
            for w in WEIGHTS:
                assert B.ac_graph_chunk_cost(ln, c[0], c[1], c[2], w, hoist=True) == GM.chunk_cost(on, c[0], c[1], c[2], w, c[4])
        n_moved += sum(len(c[4]) > 0 for c in chunks)
    assert n_moved > 20


def test_cost_equals_the_oracle_bit_for_bit():
    for seed in range(20):
        spec = G.random_graph(seed, n_ops=10)
        on, ln = oracle_nodes(spec), library_nodes(spec)
        first = next(i for i, nd in enumerate(on) if nd.op not in (S.INPUT, S.PARAM))
        for start in range(first, len(on)):
            for end in range(start, min(len(on), start + 4)):
                for d in range(len(on[end].shape)):
                    for w in WEIGHTS:
                        assert B.ac_graph_chunk_cost(ln, start, end, d, w) == GM.chunk_cost(on, start, end, d, w)


def both_plans(on, ln, e, budget, window, w, beam=1, hoist=False):
    try:
        want = GM.plan(on, e, budget, window, w, beam, hoist)
    except ValueError:
        with pytest.raises(B.AcError) as err:
            B.ac_graph_plan(ln, e, budget, window, w, beam, hoist=hoist)
        assert err.value.status == B.AC_ERR_BUDGET_INFEASIBLE
        return None
    got = B.ac_graph_plan(ln, e, budget, window, w, beam, hoist=hoist)
    assert got == ([c[:4] + (1,) for c in want[0]] if hoist else want[0], want[1])
    return want


def test_plan_equals_the_oracle_on_random_graphs():
    planned = failed = rescued = 0
    for seed in range(150):
        spec = G.random_graph(seed, n_ops=10 + seed % 6)
        on, ln = oracle_nodes(spec), library_nodes(spec)
        _, whole, _ = GM.estimate(on, 2)
        for frac in (1.0, 0.95, 0.85, 0.75, 0.6):
            got = both_plans(on, ln, 2, int(whole * frac), 5, WEIGHTS[seed % len(WEIGHTS)])
            planned += bool(got and got[0])
            failed += got is None
            for beam in (2, 5):
                wide = both_plans(on, ln, 2, int(whole * frac), 5, WEIGHTS[seed % len(WEIGHTS)], beam)
                rescued += got is None and wide is not None
            both_plans(on, ln, 2, int(whole * frac), 7, WEIGHTS[seed % len(WEIGHTS)], 2, hoist=True)

    # (a beam of 1 now remembers every extension that fits, so a wider beam rescues it less often than it did)
    assert planned > 40 and failed > 20 and rescued >= 1


def test_plan_equals_the_oracle_on_the_block_graph():
    spec, nm = PG.transformer_stack_graph(2, 32, 8, 2, 64)
    onodes, onm = S.transformer_block_graph(2, 32, 8, 2, 64)
    # the library's builder and the oracle's describe the same graph
    assert nm == onm and spec == [(nd.op, nd.inputs, nd.shape, nd.attr) for nd in onodes]
    ln = B.graph_nodes(spec)
    for budget in (73728, 60000, 40000, 30000, 28672, 28671):
        for w in WEIGHTS:
            both_plans(onodes, ln, 8, budget, 8, w)
    chunks, peak = B.ac_graph_plan(ln, 8, 40000, 8, (1, 0, 0, 0))
    assert len(chunks) == 2 and peak <= 40000


def test_two_layers_take_one_pass_per_peak():
    spec, nm = PG.transformer_stack_graph(1, 64, 16, 2, 32, layers=2)
    ln = B.graph_nodes(spec)
    per_node, whole, peak_node = B.ac_graph_estimate(ln, 2)
    assert peak_node == nm["scaled"] and per_node[nm["l1.scaled"]] == whole
    chunks, peak = B.ac_graph_plan(ln, 2, whole // 2, 8, (1, 0, 0, 0))
    assert len(chunks) == 2 and peak <= whole // 2
    assert nm["scores"] <= chunks[0][0] <= chunks[0][1] <= nm["ctx"]
    assert nm["l1.scores"] <= chunks[1][0] <= chunks[1][1] <= nm["l1.ctx"]


def test_errors():
    spec, nm = PG.transformer_stack_graph(2, 32, 8, 2, 64)
    ln = B.graph_nodes(spec)

    def status(fn):
        with pytest.raises(B.AcError) as err:
            fn()
        return err.value.status

    s, c = nm["scores"], nm["ctx_h"]
    assert status(lambda: B.ac_graph_estimate(ln, 2, [(s, c, 3, 1)])) == B.AC_ERR_ILLEGAL_CHUNK_DIM   # head dim
    assert status(lambda: B.ac_graph_estimate(ln, 2, [(s, c, 2, 0)])) == B.AC_ERR_ARG
    assert status(lambda: B.ac_graph_estimate(ln, 2, [(s, c, 2, 33)])) == B.AC_ERR_ARG
    assert status(lambda: B.ac_graph_estimate(ln, 2, [(s, c, 2, 4), (c, c + 1, 1, 4)])) == B.AC_ERR_ARG   # overlap
    assert status(lambda: B.ac_graph_estimate(ln, 2, [(nm["ctx_h"], nm["ctx"], 2, 3)])) == B.AC_ERR_ARG   # granule 4
    assert status(lambda: B.ac_graph_estimate(ln, 0)) == B.AC_ERR_ARG
    assert status(lambda: B.ac_graph_plan(ln, 8, 40000, 8, (1, 0, 0, 0), max_out=1)) == B.AC_ERR_ARG
    assert status(lambda: B.ac_graph_plan(ln, 8, 40000, 8, (1, 0, 0, 0), beam=0)) == B.AC_ERR_ARG
    assert status(lambda: B.ac_graph_plan(ln, 8, 40000, 0, (1, 0, 0, 0))) == B.AC_ERR_ARG
    assert status(lambda: B.ac_graph_chunk_cost(ln, s, c, 4, (1, 0, 0, 0))) == B.AC_ERR_ARG
    assert status(lambda: B.ac_graph_chunk_cost(ln, s, c, 3, (1, 0, 0, 0), hoist=True)) == B.AC_ERR_ILLEGAL_CHUNK_DIM
    L = B.lib()
    assert L.ac_graph_estimate(ln, len(ln), 2, None, 0, None, None, None) == B.AC_ERR_ARG


def test_pair_block_plan_equals_the_oracle_and_chunks_the_triangle_attention():
    from tests.test_search_host import pair_spec
    spec, nm = pair_spec(n=8, c=4, ch=4, heads=2, dh=2, factor=2)
    on, ln = oracle_nodes(spec), library_nodes(spec)
    assert B.ac_graph_estimate(ln, 2) == GM.estimate(on, 2)
    _, whole, peak_node = GM.estimate(on, 2)
    assert peak_node == nm["tas.biased"]
    for frac in (0.8, 0.6, 0.5):
        for beam in (1, 3):
            both_plans(on, ln, 2, int(whole * frac), 10, (1, 0, 0, 0), beam)
        both_plans(on, ln, 2, int(whole * frac), 12, (-1, 0, 0, 0), 2, hoist=True)
    # at the size of the pair workload: 16.8 GiB unchunked, the scores of both triangle attentions cut along rows
    spec, nm = PG.pair_block_graph(1024, 128, 128, 4, 32, 4)
    big = B.graph_nodes(spec)
    _, whole, peak_node = B.ac_graph_estimate(big, 2)
    # two score-sized tensors, and z, the values, the gate (one pair tensor each) and the bias [H, N, N]
    assert peak_node == nm["tas.biased"] and whole == 2 * (4 * 1024 ** 3) * 2 + (3 * 128 + 4) * 1024 * 1024 * 2
    chunks, peak = B.ac_graph_plan(big, 2, 4 << 30, 16, (1, 0, 0, 0), beam=2)
    assert peak <= 4 << 30 and [(c[0], c[2]) for c in chunks] == [(nm["tas.scores"], 0), (nm["tae.scores"], 0)]


def test_calibration_reads_the_four_terms_of_the_cost():
    from paper_2401_10652_amd import calibrate
    spec, nm = PG.transformer_stack_graph(2, 12, 8, 2, 16)
    ln = B.graph_nodes(spec)
    b, h, sq, dh = 2, 2, 12, 4
    flops = 2 * b * h * sq * sq * dh + b * h * sq * sq + 5 * b * h * sq * sq + 2 * b * h * sq * dh * sq
    assert calibrate.terms(ln, nm["scores"], nm["ctx_h"], 2) == [4.0, float(flops), flops / 4, float(dh)]
    assert list(calibrate.ranks(np.array([0.3, -1.0, 2.0]))) == [1.0, 0.0, 2.0]


def test_chunks_map_to_executor_region_settings():
    """ac_graph_chunks_to_regions: a chunk goes to the region kind that holds its nodes; a kind takes the
    shortest length any layer asks for; the graph side only says which node is what (the tags)."""
    spec, nm = PG.transformer_stack_graph(1, 64, 16, 2, 32, layers=2)
    regs = PG.executor_regions([(nm["scores"], nm["ctx_h"], 2, 24), (nm["l1.scores"], nm["l1.ctx"], 1, 16, 1),
                                (nm["l1.t"], nm["l1.down"], 1, 32)], nm)
    assert regs == [(B.AC_REGION_ATTENTION, B.AC_DIM_SEQ, 16), (B.AC_REGION_FFN, B.AC_DIM_SEQ, 32)]
    assert PG.executor_regions([(nm["u"], nm["qkv"], 0, 1)], nm) == [(B.AC_REGION_QKV, B.AC_DIM_BATCH, 1)]
    # along the heads: a feature chunk of whole heads (head_dim 8 here); along the output columns of the projection
    assert PG.executor_regions([(nm["scores"], nm["ctx_h"], 1, 1)], nm, head_dim=8) == [(B.AC_REGION_ATTENTION, B.AC_DIM_FEATURE, 8)]
    assert PG.executor_regions([(nm["o"], nm["h"], 2, 8)], nm) == [(B.AC_REGION_OUT_PROJ, B.AC_DIM_FEATURE, 8)]
    # ... and the settings are ones the executor takes
    cfg = I.TransformerConfig("tmap", 1, 2, 64, 16, 2, 32, True, "bf16", 0.05)
    info = B.Plan(B.transformer_desc(cfg), PG.executor_regions([(nm["scores"], nm["ctx_h"], 1, 1)], nm, head_dim=8)).ac_plan_query()
    assert info.regions[B.AC_REGION_ATTENTION].n_segments == 2
    for bad, status in (([(nm["scores"], nm["ctx_h"], 3, 4)], B.AC_ERR_UNSUPPORTED),        # along head_dim: no such chunk dim
                        ([(nm["ctx"], nm["h"], 1, 8)], B.AC_ERR_ARG),                       # spans attention and output projection
                        ([(nm["y"], nm["l1.u"], 1, 8)], B.AC_ERR_ARG),                      # spans two layers
                        ([(nm["scores"], nm["ctx_h"], 2, 8), (nm["l1.scores"], nm["l1.ctx_h"], 0, 1)], B.AC_ERR_ARG),   # layers disagree
                        ([(nm["x"], nm["x"], 0, 1)], B.AC_ERR_ARG),                         # no region kind computes an input
                        ([(nm["scores"], len(spec), 2, 8)], B.AC_ERR_ARG)):
        with pytest.raises(B.AcError) as ei:
            PG.executor_regions(bad, nm)
        assert ei.value.status == status


def test_pair_chunks_map_to_executor_region_settings():
    """The plan of the pair block's graph goes to the executor: rows of the starting-node attention, and for
    the ending-node attention (which the graph writes on the transposed pair tensor) columns."""
    n, c, ch, heads, dh = 64, 16, 16, 2, 8
    spec, nm = PG.pair_block_graph(n, c, ch, heads, dh, 4)
    nodes = B.graph_nodes(spec)
    _, whole, peak_node = B.ac_graph_estimate(nodes, 2)
    chunks, peak = B.ac_graph_plan(nodes, 2, whole // 2, 12, (1.0, 0.0, 0.0, 0.0), beam=2)
    assert chunks and peak <= whole // 2
    regs = PG.pair_executor_regions(chunks, nm)
    kinds = {k: (d, l) for k, d, l in regs}
    assert set(kinds) <= {B.AC_REGION_TRIATT_START, B.AC_REGION_TRIATT_END, B.AC_REGION_TRIMUL_OUT, B.AC_REGION_TRIMUL_IN,
                          B.AC_REGION_PAIR_TRANSITION}
    assert kinds[B.AC_REGION_TRIATT_START][0] == B.AC_DIM_ROW and kinds[B.AC_REGION_TRIATT_END][0] == B.AC_DIM_COL
    assert all(1 <= l < n for _, l in kinds.values())
    cfg = I.PairConfig("pmap", 2, n, c, ch, heads, dh, 4, "bf16")
    info = B.Plan(B.pair_desc(cfg), regs).ac_plan_query()
    by_kind = {r.kind: r for r in info.regions[:info.n_regions]}
    assert by_kind[B.AC_REGION_TRIATT_END].chunk_dim == B.AC_DIM_COL
    assert by_kind[B.AC_REGION_TRIATT_START].n_segments > 1
    # by hand: rows of the scores of the starting node; the transposed tensor's rows are z's columns
    assert PG.pair_executor_regions([(nm["tas.scores"], nm["tas.ctx_h"], 0, 5)], nm) == [(B.AC_REGION_TRIATT_START, B.AC_DIM_ROW, 5)]
    assert PG.pair_executor_regions([(nm["tae.scores"], nm["tae.ctx_h"], 0, 5)], nm) == [(B.AC_REGION_TRIATT_END, B.AC_DIM_COL, 5)]
    assert PG.pair_executor_regions([(nm["tae.scores"], nm["tae.ctx_h"], 2, 5)], nm) == [(B.AC_REGION_TRIATT_END, B.AC_DIM_ROW, 5)]
    assert PG.pair_executor_regions([(nm["tmo.o"], nm["tmo.z"], 1, 6)], nm) == [(B.AC_REGION_TRIMUL_OUT, B.AC_DIM_COL, 6)]
    with pytest.raises(B.AcError):      # the b operand is read whole by every segment: it belongs to no chunked part
        PG.pair_executor_regions([(nm["tmo.b"], nm["tmo.z"], 0, 6)], nm)


def test_unet_residual_block_chunks_map_to_the_executor():
    """Chunks of the UNet stage graph: along the batch, those of the residual block and of the spatial transformer
    become the executor's settings; output channels of a convolution and query rows of the scores are legal by the
    rules (section 3.3) but the executor has no such dim there; a chunk across the two blocks belongs to no kind."""
    spec, nm = PG.unet_stage_graph(4, 64, 8, 8, 2, 7, 32, groups=8)
    nodes = B.graph_nodes(spec)
    tags = PG.unet_stage_tags(nm)
    assert B.ac_chunk_trace(nodes, nm["res.n1"], nm["res.y"], 0) is not None
    assert B.ac_graph_chunks_to_regions(tags, [(nm["res.n1"], nm["res.y"], 0, 2)]) == [(B.AC_REGION_RES_BLOCK, B.AC_DIM_BATCH, 2)]
    cfg = I.ResStackConfig("tmapu", 3, 1, 4, 8, 8, 64, 8)
    info = B.Plan(B.res_stack_desc(cfg), B.ac_graph_chunks_to_regions(tags, [(nm["res.n1"], nm["res.y"], 0, 2)])).ac_plan_query()
    assert info.regions[0].n_segments == 2
    for bad, status in (([(nm["res.c2"], nm["res.c2"], 1, 16)], B.AC_ERR_UNSUPPORTED),      # output channels of the convolution
                        ([(nm["tr.sa.scores"], nm["tr.sa.ctx_h"], 2, 16)], B.AC_ERR_UNSUPPORTED),   # query rows of an image
                        ([(nm["tr.ca.scores"], nm["tr.ca.ctx_h"], 3, 4)], B.AC_ERR_UNSUPPORTED),    # context tokens (were it legal)
                        ([(nm["res.n1"], nm["tr.n"], 0, 1)], B.AC_ERR_ARG)):
        with pytest.raises(B.AcError) as ei:
            B.ac_graph_chunks_to_regions(tags, bad)
        assert ei.value.status == status
    # the attention block: batch chunks of the self-attention and of the feed-forward meet in one setting (the shorter)
    assert B.ac_chunk_trace(nodes, nm["tr.sa.u"], nm["tr.sa.h"], 0) is not None
    both = [(nm["tr.sa.u"], nm["tr.ca.h"], 0, 2), (nm["tr.ff.u"], nm["tr.ff.h"], 0, 1), (nm["res.n1"], nm["res.y"], 0, 2)]
    regs = B.ac_graph_chunks_to_regions(tags, both)
    assert regs == [(B.AC_REGION_RES_BLOCK, B.AC_DIM_BATCH, 2), (B.AC_REGION_UNET_ATTN, B.AC_DIM_BATCH, 1)]
    cfga = I.ResStackConfig("tmapa", 3, 1, 4, 8, 8, 64, 8, heads=2, d_ffn=256, context_tokens=7, context_dim=32, gated=True)
    infa = B.Plan(B.res_stack_desc(cfga), regs).ac_plan_query()
    assert [infa.regions[k].n_segments for k in range(2)] == [2, 4]
    # the executor's one legal dim is what the rules say: no other dim of the whole block is legal
    for d in (1, 2, 3):
        assert B.ac_chunk_trace(nodes, nm["res.n1"], nm["res.y"], d) is None
