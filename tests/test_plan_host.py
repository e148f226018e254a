"""Host-side checks that need no GPU: the library loads and exports what the header
declares; plan arithmetic against the paper-style memory model and against the arena
worked out by hand; legality and error codes."""
import dataclasses
import os
import re

import pytest

from oracle import memory_model as M
from paper_2401_10652_amd import binding as B
from paper_2401_10652_amd import inputs as I

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
MIB, GIB = 1 << 20, 1 << 30


def test_library_exports_every_declared_symbol():
    inc = os.path.join(ROOT, "include")
    hdr = "".join(open(os.path.join(inc, f)).read() for f in sorted(os.listdir(inc)) if f.endswith(".h"))
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(ac_[a-z_0-9]+)\s*\(", hdr))
    assert declared == set(B.SIGNATURES), declared ^ set(B.SIGNATURES)
    L = B.lib()
    for name in declared:
        assert getattr(L, name) is not None
    assert L.ac_status_string(0) == b"ok"
    assert L.ac_status_string(B.AC_ERR_ILLEGAL_CHUNK_DIM) == b"illegal chunk dimension"


def regions(c_qkv, c_attn, c_ffn, dim=B.AC_DIM_SEQ, c_out=None):
    """Four regions per layer; the output projection follows the attention's length unless given."""
    return [(B.AC_REGION_QKV, dim, c_qkv), (B.AC_REGION_ATTENTION, dim, c_attn),
            (B.AC_REGION_OUT_PROJ, dim, c_attn if c_out is None else c_out), (B.AC_REGION_FFN, dim, c_ffn)]


def al(v):
    return (v + 255) // 256 * 256


def key_splits_by_hand(sq, sk, heads, batch, dh, dtype):
    """The executor cuts the keys of a launch with fewer than 512 blocks of 128 query rows into
    runs of at least 512 keys, as many as keep the launch within 768 blocks (three per compute
    unit, all resident at once; 512, two per unit, with 128-wide heads), at most 16 (bf16
    matrix-core path)."""
    if dtype != "bf16" or dh not in (32, 64, 128):
        return 1
    blocks = -(-sq // 128) * heads * batch
    if blocks >= 512 or sk < 1024:
        return 1
    return max(1, min((512 if dh > 64 else 768) // blocks, sk // 512, 16))


def arena_by_hand(cfg, c_qkv, c_attn, c_ffn, unfused=False, lanes=1, c_out=None, stored_scores=False):
    """Whole tensors q,k (2Td) + v^T (Td) [bf16] or qkv (3Td) [fp32], context (Td), h (Td),
    inter-layer t (Td if layers > 1), plus the largest per-segment set: nothing for LayerNorm 1 +
    projection (the normalised rows sit in the context buffer, which is idle then) | fp32 split
    partials of the attention (ns c H (d_h + 2) floats) | nothing for the output projection
    (its unfused form holds c d) | the hidden tensor (c F) of the feed-forward (LayerNorm 2 also writes
    into the context buffer; the unfused second projection holds c d more)."""
    c_out = c_attn if c_out is None else c_out
    e = 2 if cfg.dtype == "bf16" else 4
    T, d, F = cfg.seq * cfg.batch, cfg.d_model, cfg.d_ffn
    whole = (al(T * 2 * d * e) + al(T * d * e)) if cfg.dtype == "bf16" else al(T * 3 * d * e)
    if stored_scores and cfg.dtype != "bf16":
        whole += al(T * d * e)             # v transposed, which the bf16 layout has anyway
    whole += 2 * al(T * d * e)
    if cfg.layers > 1:
        whole += al(T * d * e)
    r1 = 0
    groups = attention_groups_by_hand(cfg, c_attn)
    r2 = max(b for _, _, b in groups)
    if stored_scores:                      # scores and probabilities of one segment, every head
        r2 = 2 * al(cfg.heads * c_attn * cfg.seq * e)
        groups = [None] * -(-cfg.seq // c_attn)
    r2b = al(c_out * d * e) if unfused else 0
    r3 = al(c_ffn * F * e) + (al(c_ffn * d * e) if unfused else 0)
    # two segments in flight: a region with more than one segment (launch) holds two per-segment sets
    mult = lambda c: lanes if c < cfg.seq else 1
    return whole + max(r1, r2 * (lanes if len(groups) > 1 else 1), r2b * mult(c_out), r3 * mult(c_ffn))


def attention_launch_bytes_by_hand(cfg, s0, rows):
    """fp32 partial results (unnormalised context, running maximum and sum) of the key splits of one
    attention launch over query rows [s0, s0 + rows) of one sequence; a causal launch splits the keys
    its last row sees."""
    keys = min(cfg.seq, s0 + rows) if cfg.causal else cfg.seq
    ns = key_splits_by_hand(rows, keys, cfg.heads, 1, cfg.head_dim, cfg.dtype)
    return 0 if ns <= 1 else al(ns * rows * cfg.d_model * 4) + al(ns * rows * cfg.heads * 8)


def attention_groups_by_hand(cfg, c_attn):
    """The fused attention keeps nothing of a segment in memory, so the consecutive segments of a
    sequence share one launch, whose key splits are capped so that their partial results stay within
    those of the plan's largest single segment.  Returns (first row, rows, bytes) per launch."""
    segs = [(s, min(c_attn, cfg.seq - s)) for s in range(0, cfg.seq, c_attn)]
    bound = max(attention_launch_bytes_by_hand(cfg, s, r) for s, r in segs)
    rows = cfg.seq
    ns = key_splits_by_hand(rows, cfg.seq, cfg.heads, 1, cfg.head_dim, cfg.dtype)
    size = lambda n: 0 if n <= 1 else al(n * rows * cfg.d_model * 4) + al(n * rows * cfg.heads * 8)
    while ns > 1 and size(ns) > bound:
        ns -= 1
    return [(0, rows, size(ns))]


@pytest.mark.parametrize("cfg,c", [(I.C1, (64, 64, 64)), (I.C3, (512, 512, 512)), (I.C2, (1024, 1024, 1024)),
                                   (I.C5, (8192, 640, 4096)), (I.C2, (8192, 8192, 8192))])
def test_planned_bytes_equal_the_arena_worked_by_hand(cfg, c):
    p = B.Plan(B.transformer_desc(cfg), regions(*c))
    info = p.ac_plan_query()
    e = 2 if cfg.dtype == "bf16" else 4
    assert info.io_bytes == 2 * cfg.seq * cfg.d_model * e
    assert info.workspace_bytes == arena_by_hand(cfg, *c)
    assert info.peak_bytes_planned == info.io_bytes + info.workspace_bytes
    assert info.peak_bytes_unchunked_planned == info.io_bytes + arena_by_hand(cfg, cfg.seq, cfg.seq, cfg.seq)
    assert info.n_weights == 12 * cfg.layers and info.n_regions == 4
    for r, cl in zip(info.regions[:4], (c[0], c[1], c[1], c[2])):
        assert r.chunk_len == cl and r.n_segments == -(-cfg.seq // cl) and r.extent == cfg.seq
    # paper-style region bytes agree with the independent model in oracle/
    a = info.regions[1]
    assert a.model_bytes == M.attention_region(cfg.seq, cfg.d_model, cfg.heads, e, c[1])
    assert a.model_bytes_unchunked == M.attention_region(cfg.seq, cfg.d_model, cfg.heads, e)
    assert info.regions[0].model_bytes == M.qkv_region(cfg.seq, cfg.d_model, e, c[0])
    assert info.regions[3].model_bytes == M.ffn_region(cfg.seq, cfg.d_model, cfg.d_ffn, e, c[2])
    assert info.regions[2].model_bytes == M.out_proj_region(cfg.seq, cfg.d_model, e, c[1])
    assert info.peak_bytes_model == M.transformer_layer_peak(cfg.seq, cfg.d_model, cfg.heads, cfg.d_ffn, e, *c, c_out=c[1])
    assert info.peak_bytes_model_unchunked == M.transformer_layer_peak(cfg.seq, cfg.d_model, cfg.heads, cfg.d_ffn, e)
    p.close()


def test_key_split_rule():
    for sq, sk, h, b, dh, dt in ((1792, 8192, 16, 1, 64, "bf16"), (1024, 8192, 16, 1, 64, "bf16"),
                                 (512, 4096, 12, 1, 64, "bf16"), (640, 65536, 16, 1, 128, "bf16"),
                                 (8192, 8192, 16, 1, 64, "bf16"), (64, 640, 4, 1, 64, "bf16"),
                                 (1024, 1024, 4, 64, 32, "bf16"), (64, 256, 4, 1, 16, "f32")):
        assert B.ac_attention_key_splits(sq, sk, h, b, dh, dt) == key_splits_by_hand(sq, sk, h, b, dh, dt)
    assert B.ac_attention_key_splits(1792, 8192, 16, 1, 64, "bf16") == 3
    assert B.ac_attention_key_splits(512, 4096, 12, 1, 64, "bf16") == 8
    assert B.ac_attention_key_splits(640, 65536, 16, 1, 128, "bf16") == 6
    assert B.ac_attention_split_workspace_bytes(100, 4, 2, 64, 3) == 3 * 2 * 100 * 4 * (64 + 2) * 4
    assert B.ac_attention_split_workspace_bytes(100, 4, 2, 64, 1) == 0


def test_two_segments_in_flight_doubles_the_per_segment_sets():
    for cfg, c in ((I.C3, (512, 512, 512)), (I.C2, (8192, 1792, 8192)), (I.C2, (1024, 1024, 1024))):
        p = B.Plan(B.transformer_desc(cfg, flags=B.AC_FLAG_TWO_SEGMENTS_IN_FLIGHT), regions(*c))
        assert p.ac_plan_query().workspace_bytes == arena_by_hand(cfg, *c, lanes=2)
    # the output projection may be cut differently from the attention core
    p = B.Plan(B.transformer_desc(I.C2), regions(8192, 1792, 8192, c_out=8192))
    info = p.ac_plan_query()
    assert [r.n_segments for r in info.regions[:4]] == [1, 5, 1, 1]
    assert info.workspace_bytes == arena_by_hand(I.C2, 8192, 1792, 8192, c_out=8192)


def test_stored_scores_hold_what_the_paper_counts():
    """With AC_FLAG_MATERIALIZED_SCORES the attention core's share of the workspace is the
    intermediate activation of the paper's equations: scores and probabilities, H c S elements
    each, for the rows of one segment (AutoChunk section 2.1 and 2.2)."""
    for cfg, c in ((I.C1, (256, 64, 256)), (I.C1, (256, 256, 256)), (I.C3, (4096, 512, 4096)), (I.C2, (8192, 1792, 8192))):
        e = 2 if cfg.dtype == "bf16" else 4
        p = B.Plan(B.transformer_desc(cfg, flags=B.AC_FLAG_MATERIALIZED_SCORES), regions(*c, c_out=cfg.seq))
        info = p.ac_plan_query()
        assert info.workspace_bytes == arena_by_hand(cfg, *c, c_out=cfg.seq, stored_scores=True)
        a = M.attention_region(cfg.seq, cfg.d_model, cfg.heads, e, c[1]) - 5 * cfg.seq * cfg.d_model * e
        assert a == 2 * cfg.heads * min(c[1], cfg.seq) * cfg.seq * e
        # the model's peak and the chunk lengths a budget gives do not depend on the flag
        q = B.Plan(B.transformer_desc(cfg), regions(*c, c_out=cfg.seq)).ac_plan_query()
        assert info.peak_bytes_model == q.peak_bytes_model
    expect(B.AC_ERR_UNSUPPORTED, lambda: B.Plan(B.pair_desc(I.C4, flags=B.AC_FLAG_MATERIALIZED_SCORES), []))


def test_unfused_flag_adds_the_temporaries():
    p = B.Plan(B.transformer_desc(I.C3, flags=B.AC_FLAG_UNFUSED_ELEMENTWISE), regions(512, 512, 512))
    assert p.ac_plan_query().workspace_bytes == arena_by_hand(I.C3, 512, 512, 512, unfused=True)


def test_flops_are_the_algorithmic_counts():
    for cfg in (I.C2, I.C3, I.C5):
        S, d, L = cfg.seq, cfg.d_model, cfg.layers
        lin = 24 * S * d * d
        att = 2 * S * (S + 1) * d if cfg.causal else 4 * S * S * d
        ln = 2 * 8 * S * d
        info = B.Plan(B.transformer_desc(cfg), regions(1024, 1024, 1024)).ac_plan_query()
        assert abs(info.flops_per_execute - L * (lin + att + ln)) <= 1e-9 * info.flops_per_execute
        # the count does not depend on the chunk length
        info2 = B.Plan(B.transformer_desc(cfg), regions(S, 640, 128)).ac_plan_query()
        assert abs(info2.flops_per_execute - info.flops_per_execute) <= 1e-9 * info.flops_per_execute


def expect(status, fn):
    with pytest.raises(B.AcError) as ei:
        fn()
    assert ei.value.status == status, str(ei.value)
    assert B.lib().ac_last_error() != b""


def test_budget_bounds_the_executor_bytes():
    """Reading: the budget is the paper's memory_budget (section 3.2) applied to what the executor
    really holds, mem(X) + mem(Y) + the workspace's high-water mark.  The fused attention keeps no
    scores in memory, so C2 at 1 GiB and C5 at 4 GiB run every region as one segment."""
    for cfg, budget in ((I.C2, 1 * GIB), (I.C5, 4 * GIB)):
        info = B.Plan(B.transformer_desc(cfg), regions(0, 0, 0, c_out=0), budget).ac_plan_query()
        assert [r.n_segments for r in info.regions[:4]] == [1, 1, 1, 1]
        assert info.peak_bytes_planned == info.peak_bytes_unchunked_planned <= budget
    # C5, 2.75 GiB: only the feed-forward region (the hidden tensor of a segment on top of the whole
    # tensors) exceeds it; it gets the largest multiple of 128 rows that fits
    e = 2
    S, d, F = I.C5.seq, I.C5.d_model, I.C5.d_ffn
    BUD = 11 * GIB // 4
    whole = 2 * S * d * e + 6 * S * d * e          # x, y; q, k, v, context, h, inter-layer buffer
    info3 = B.Plan(B.transformer_desc(I.C5), regions(0, 0, 0, c_out=0), BUD).ac_plan_query()
    fits = lambda c: whole + c * F * e <= BUD
    assert [r.n_segments for r in info3.regions[:3]] == [1, 1, 1]
    assert info3.regions[3].chunk_len == M.largest_chunk_len(S, 128, fits) == 49152
    assert info3.peak_bytes_planned <= BUD < info3.peak_bytes_unchunked_planned
    assert info3.peak_bytes_planned == arena_by_hand(I.C5, S, S, 49152, c_out=S) + 2 * S * d * e
    # one granule more would not fit
    over = B.Plan(B.transformer_desc(I.C5), regions(S, S, 49152 + 128, c_out=S)).ac_plan_query()
    assert over.peak_bytes_planned > BUD
    # an explicit length that does not fit is an error, as is a budget below the whole tensors
    expect(B.AC_ERR_BUDGET_INFEASIBLE, lambda: B.Plan(B.transformer_desc(I.C5), regions(0, 0, S, c_out=0), BUD))
    expect(B.AC_ERR_BUDGET_INFEASIBLE, lambda: B.Plan(B.transformer_desc(I.C5), regions(0, 0, 0, c_out=0), 2 * GIB))
    # two segments in flight: the budget bounds the doubled per-segment sets too
    info2 = B.Plan(B.transformer_desc(I.C5, flags=B.AC_FLAG_TWO_SEGMENTS_IN_FLIGHT), regions(0, 0, 0, c_out=0),
                   BUD).ac_plan_query()
    assert info2.peak_bytes_planned <= BUD and info2.regions[3].chunk_len <= 49152 // 2 + 128


def test_budget_sizes_batch_chunks():
    """Batch chunks are sized in whole batch elements (granule 1), with and without stored scores."""
    cfg = I.TransformerConfig("b8", 91, 2, 1024, 1024, 16, 4096, True, "bf16", 0.02, batch=8)
    kinds = (B.AC_REGION_QKV, B.AC_REGION_ATTENTION, B.AC_REGION_OUT_PROJ, B.AC_REGION_FFN)
    regs = [(k, B.AC_DIM_BATCH, 0) for k in kinds]
    for flags, budget in ((B.AC_FLAG_MATERIALIZED_SCORES, 400000000), (0, 200000000),
                          (B.AC_FLAG_MATERIALIZED_SCORES | B.AC_FLAG_BUDGET_PAPER_MODEL, 400000000)):
        info = B.Plan(B.transformer_desc(cfg, flags=flags), regs, budget).ac_plan_query()
        assert info.peak_bytes_planned <= budget < info.peak_bytes_unchunked_planned
        assert any(1 <= r.chunk_len < 8 for r in info.regions[:4])
        # the lengths chosen are the largest that fit: one more batch element in the region that
        # holds the peak does not
        worst = max(range(4), key=lambda i: B.Plan(
            B.transformer_desc(cfg, flags=flags & ~B.AC_FLAG_BUDGET_PAPER_MODEL),
            [(k, B.AC_DIM_BATCH, info.regions[j].chunk_len if j == i else 8) for j, k in enumerate(kinds)]
        ).ac_plan_query().peak_bytes_planned)
        r = info.regions[worst]
        if r.chunk_len < 8 and not flags & B.AC_FLAG_BUDGET_PAPER_MODEL:
            more = [(k, B.AC_DIM_BATCH, info.regions[j].chunk_len + (1 if j == worst else 0)) for j, k in enumerate(kinds)]
            assert B.Plan(B.transformer_desc(cfg, flags=flags), more).ac_plan_query().peak_bytes_planned > budget


def test_budget_under_the_paper_model_sizes_the_chunk_lengths():
    """AC_FLAG_BUDGET_PAPER_MODEL: the budget also bounds the bytes the two activation equations give
    for the unfused graph of a region (scores and probabilities stored)."""
    pm = B.AC_FLAG_BUDGET_PAPER_MODEL
    # C2, 1 GiB: only the attention region exceeds it; largest multiple of 128 that fits is 1792
    p = B.Plan(B.transformer_desc(I.C2, flags=pm), regions(0, 0, 0), 1 * GIB)
    info = p.ac_plan_query()
    e = 2
    fits = lambda c: M.attention_region(8192, 1024, 16, e, c) <= GIB
    assert info.regions[1].chunk_len == M.largest_chunk_len(8192, 128, fits) == 1792
    assert info.regions[1].n_segments == 5
    assert info.regions[0].chunk_len == 8192 and info.regions[2].chunk_len == 8192 and info.regions[3].chunk_len == 8192
    assert info.peak_bytes_model <= GIB < info.peak_bytes_model_unchunked
    assert info.peak_bytes_planned <= GIB
    # C5, 4 GiB: attention gets 640 rows, the other regions fit whole (multi-stage: each
    # region is sized on its own until the layer's peak is under the budget)
    info5 = B.Plan(B.transformer_desc(I.C5, flags=pm), regions(0, 0, 0), 4 * GIB).ac_plan_query()
    fits5 = lambda c: M.attention_region(65536, 2048, 16, e, c) <= 4 * GIB
    assert info5.regions[1].chunk_len == M.largest_chunk_len(65536, 128, fits5) == 640
    assert info5.regions[1].n_segments == 103
    assert info5.peak_bytes_model <= 4 * GIB and info5.peak_bytes_planned <= 4 * GIB
    # a tighter budget makes the feed-forward chunk too
    tight = 5 * GIB // 2
    info5b = B.Plan(B.transformer_desc(I.C5, flags=pm), regions(0, 0, 0), tight).ac_plan_query()
    assert info5b.regions[3].chunk_len < 65536 and info5b.regions[1].chunk_len == 256
    for r in info5b.regions[:4]:
        assert r.model_bytes <= tight
    assert info5b.peak_bytes_planned <= tight
    # at 2 GiB the whole tensors of the executor alone (x, y, q, k, v, context, h, t: 8 x 256 MiB) do not fit
    expect(B.AC_ERR_BUDGET_INFEASIBLE, lambda: B.Plan(B.transformer_desc(I.C5, flags=pm), regions(0, 0, 0), 2 * GIB))
    # monotone: more segments never need more bytes
    prev = None
    for c in (8192, 4096, 1024, 256, 64):
        w = B.Plan(B.transformer_desc(I.C2), regions(c, c, c)).ac_plan_query().workspace_bytes
        assert prev is None or w <= prev
        prev = w


def test_legality_and_errors():
    d = B.transformer_desc(I.C3)
    for dim in (B.AC_DIM_FEATURE, B.AC_DIM_HEAD_DIM, B.AC_DIM_KEY):
        for kind in (B.AC_REGION_QKV, B.AC_REGION_ATTENTION, B.AC_REGION_OUT_PROJ, B.AC_REGION_FFN):
            # by the rules the context can be cut in whole heads and the output projection in blocks
            # of columns (tests/test_search_host.py reads both off the graph)
            legal = dim == B.AC_DIM_FEATURE and kind in (B.AC_REGION_ATTENTION, B.AC_REGION_OUT_PROJ)
            if not legal:
                expect(B.AC_ERR_ILLEGAL_CHUNK_DIM, lambda: B.Plan(d, [(kind, dim, 64)]))
                continue
            info = B.Plan(d, [(kind, dim, 128)]).ac_plan_query()
            assert info.regions[kind].n_segments == I.C3.d_model // 128 and info.regions[kind].launches == 1
            # whole heads (64 wide here); blocks of columns that start on 16-byte boundaries
            expect(B.AC_ERR_ARG, lambda: B.Plan(d, [(kind, dim, 96 if kind == B.AC_REGION_ATTENTION else 100)]))
    B.Plan(d, [(B.AC_REGION_ATTENTION, B.AC_DIM_BATCH, 1)]).close()
    expect(B.AC_ERR_ARG, lambda: B.Plan(d, [(B.AC_REGION_ATTENTION, 9, 64)]))
    expect(B.AC_ERR_ARG, lambda: B.Plan(d, [(B.AC_REGION_TRIMUL_OUT, 0, 64)]))
    expect(B.AC_ERR_ARG, lambda: B.Plan(d, [(B.AC_REGION_FFN, 1, 64), (B.AC_REGION_FFN, 1, 32)]))
    expect(B.AC_ERR_ARG, lambda: B.Plan(d, [(B.AC_REGION_FFN, 1, -5)]))
    bad = B.transformer_desc(I.C3)
    bad.heads = 7
    expect(B.AC_ERR_ARG, lambda: B.Plan(bad))
    bad = B.transformer_desc(I.C3)
    bad.activation = B.AC_ACT_SIGMOID
    expect(B.AC_ERR_ARG, lambda: B.Plan(bad))
    bad = B.transformer_desc(I.C3)
    bad.dtype = 5
    expect(B.AC_ERR_ARG, lambda: B.Plan(bad))
    # the floor of the second activation equation: whole tensors alone exceed the budget
    expect(B.AC_ERR_BUDGET_INFEASIBLE, lambda: B.Plan(B.transformer_desc(I.C5), regions(0, 0, 0), 1 * GIB))
    expect(B.AC_ERR_BUDGET_INFEASIBLE, lambda: B.Plan(B.transformer_desc(I.C2, flags=B.AC_FLAG_BUDGET_PAPER_MODEL),
                                                      regions(0, 4096, 0, c_out=0), 1 * GIB))
    # chunk_len larger than the extent means one segment
    info = B.Plan(d, regions(10 ** 9, 10 ** 9, 10 ** 9)).ac_plan_query()
    assert all(r.n_segments == 1 for r in info.regions[:4])
    # query / bind / execute argument checks that need no device
    p = B.Plan(d)
    L = B.lib()
    assert L.ac_plan_query(p._h, None) == B.AC_ERR_ARG
    assert L.ac_plan_query(None, None) == B.AC_ERR_ARG
    assert L.ac_plan_bind_weights(p._h, None, 0) == B.AC_ERR_ARG
    import ctypes as C
    ptrs = (C.c_void_p * 3)(256, 512, 768)
    assert L.ac_plan_bind_weights(p._h, ptrs, 3) == B.AC_ERR_ARG          # wrong count
    n = p.ac_plan_query().n_weights
    ptrs = (C.c_void_p * n)(*[256 * (i + 1) for i in range(n)])
    assert L.ac_execute(p._h, 256, 1 << 30, 256, 1 << 40, None, None) == B.AC_ERR_STATE   # not bound
    ptrs[3] = 257
    assert L.ac_plan_bind_weights(p._h, ptrs, n) == B.AC_ERR_ALIGN
    ptrs[3] = 0
    assert L.ac_plan_bind_weights(p._h, ptrs, n) == B.AC_ERR_ARG
    ptrs[3] = 1024
    assert L.ac_plan_bind_weights(p._h, ptrs, n) == B.AC_OK
    need = p.ac_plan_query().workspace_bytes
    assert L.ac_execute(p._h, 256, 1 << 30, 256, need - 1, None, None) == B.AC_ERR_WORKSPACE
    assert L.ac_execute(p._h, 256, 1 << 30, 257, need, None, None) == B.AC_ERR_ALIGN
    assert L.ac_execute(p._h, 256, 512, 256, need, None, None) == B.AC_ERR_ARG          # x, y overlap
    assert L.ac_execute(p._h, None, 512, 256, need, None, None) == B.AC_ERR_ARG
    wi = p.ac_plan_weight_info(2)
    assert wi.name == b"L0.w_qkv" and (wi.rows, wi.cols) == (3 * 768, 768) and wi.dtype == B.AC_BF16
    assert L.ac_plan_weight_info(p._h, n, C.byref(wi)) == B.AC_ERR_ARG
    assert L.ac_plan_read_profile(p._h, None, 0, None) == B.AC_ERR_ARG
    L.ac_plan_destroy(None)


def test_public_headers_are_plain_c(tmp_path):
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no C compiler")
    inc = os.path.join(ROOT, "include")
    src = tmp_path / "headers.c"
    src.write_text("".join(f'#include "{f}"\n' for f in sorted(os.listdir(inc)) if f.endswith(".h")) + "int main(void) { return 0; }\n")
    r = subprocess.run([gcc, "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-I", inc, "-fsyntax-only", str(src)],
                       capture_output=True, text=True)
    assert r.returncode == 0, r.stderr


def test_unet_residual_stack_plan():
    """The residual stack's arena by hand (inter-block buffers, the bias-plus-embedding table, the GroupNorm
    partial statistics, two tensors of a segment's images), its paper-style bytes (x and y whole, seven
    intermediates of a segment), the one legal chunk dim and what the kernels do not take."""
    cfg = I.ResStackConfig("tu", 9, 3, 6, 16, 16, 128, 32)
    img = 16 * 16 * 128 * 2
    whole = 2 * al(6 * img) + al(6 * 128 * 2) + al(6 * 32 * 64 * 3 * 4)
    for c, lanes in ((6, 1), (2, 1), (4, 1), (1, 2)):
        flags = B.AC_FLAG_TWO_SEGMENTS_IN_FLIGHT if lanes == 2 else 0
        info = B.Plan(B.res_stack_desc(cfg, flags=flags), [(B.AC_REGION_RES_BLOCK, B.AC_DIM_BATCH, c)]).ac_plan_query()
        assert info.io_bytes == 2 * 6 * img and info.n_weights == 27 and info.n_regions == 1
        assert info.workspace_bytes == whole + lanes * 2 * al(c * img)
        assert info.peak_bytes_model == 2 * 6 * img + 7 * c * img and info.peak_bytes_model_unchunked == 9 * 6 * img
        assert info.regions[0].n_segments == -(-6 // c) and info.regions[0].extent == 6
    # the budget sizes the images per segment
    one = B.Plan(B.res_stack_desc(cfg), []).ac_plan_query()
    sized = B.Plan(B.res_stack_desc(cfg), [(B.AC_REGION_RES_BLOCK, B.AC_DIM_BATCH, 0)], one.peak_bytes_planned - 2 * img).ac_plan_query()
    assert sized.regions[0].chunk_len == 5 and sized.peak_bytes_planned <= one.peak_bytes_planned - 2 * img
    expect(B.AC_ERR_BUDGET_INFEASIBLE, lambda: B.Plan(B.res_stack_desc(cfg), [(B.AC_REGION_RES_BLOCK, B.AC_DIM_BATCH, 0)], 2 * 6 * img))
    for dim in (B.AC_DIM_SEQ, B.AC_DIM_FEATURE):
        expect(B.AC_ERR_ILLEGAL_CHUNK_DIM, lambda: B.Plan(B.res_stack_desc(cfg), [(B.AC_REGION_RES_BLOCK, dim, 2)]))
    expect(B.AC_ERR_ARG, lambda: B.Plan(B.res_stack_desc(cfg), [(B.AC_REGION_FFN, B.AC_DIM_BATCH, 2)]))
    expect(B.AC_ERR_UNSUPPORTED, lambda: B.Plan(B.res_stack_desc(I.ResStackConfig("f", 9, 1, 2, 8, 8, 64, 8, dtype="f32")), []))
    expect(B.AC_ERR_UNSUPPORTED, lambda: B.Plan(B.res_stack_desc(I.ResStackConfig("c", 9, 1, 2, 8, 8, 96, 8)), []))
    expect(B.AC_ERR_ARG, lambda: B.Plan(B.res_stack_desc(I.ResStackConfig("g", 9, 1, 2, 8, 8, 64, 7)), []))
    expect(B.AC_ERR_UNSUPPORTED, lambda: B.Plan(B.res_stack_desc(cfg, flags=B.AC_FLAG_UNFUSED_ELEMENTWISE), []))


def test_unet_stage_with_attention_plan():
    """A residual block followed by an attention block per layer: the weight list, the two regions, the attention
    block's arena by hand at 4096 positions (where its attention launch also holds the partial results of its key
    splits), its paper-style bytes, and the shapes the attention kernels do not take."""
    cfg = I.ResStackConfig("tua", 10, 2, 4, 64, 64, 320, 32, heads=5, d_ffn=1280)
    hw, c, f, e = 4096, 320, 1280, 2
    img = hw * c * e
    p = B.Plan(B.res_stack_desc(cfg), [(B.AC_REGION_RES_BLOCK, B.AC_DIM_BATCH, 4), (B.AC_REGION_UNET_ATTN, B.AC_DIM_BATCH, 1)])
    info = p.ac_plan_query()
    names = p.weight_names()
    assert info.n_weights == 2 * 27 and info.n_regions == 2
    assert names[:9] == [f"R0.{n}" for n in I.RES_BLOCK_TENSORS] and names[9:27] == [f"A0.{n}" for n in I.ATTN_BLOCK_TENSORS]
    assert names[27] == "R1.gn1_g" and names[-1] == "A1.b_out"
    shapes = {p.ac_plan_weight_info(i).name.decode(): (p.ac_plan_weight_info(i).rows, p.ac_plan_weight_info(i).cols) for i in range(27)}
    assert shapes["A0.w_qkv"] == (3 * c, c) and shapes["A0.w_1"] == (f, c) and shapes["A0.w_2"] == (c, f) and shapes["A0.b_qkv"] == (1, 3 * c)
    assert [info.regions[k].kind for k in range(2)] == [B.AC_REGION_RES_BLOCK, B.AC_REGION_UNET_ATTN]
    assert [info.regions[k].n_segments for k in range(2)] == [1, 4]
    assert info.regions[1].model_bytes == 2 * 4 * img + 13 * img + 2 * hw * f * e + 2 * 5 * hw * hw * e
    assert info.regions[1].model_bytes_unchunked == 2 * 4 * img + 4 * (13 * img + 2 * hw * f * e + 2 * 5 * hw * hw * e)
    # four modules: two whole buffers between them; one image of the attention block holds u, t, q|k, v^T, the
    # context, the hidden rows (the residual block's segment of four images is smaller: 8 images' worth against 10)
    whole = 2 * al(4 * img) + al(4 * c * e) + al(4 * 32 * 64 * 3 * 4)
    seg = 2 * al(img) + al(2 * img) + 2 * al(img) + al(hw * f * e)
    assert seg + whole <= info.workspace_bytes <= seg + whole + (64 << 20)      # + the key splits' fp32 partials
    # with a context and the gate: seven more tensors per attention block, a first layer twice as wide
    full = dataclasses.replace(cfg, context_tokens=77, context_dim=768, gated=True)
    pf = B.Plan(B.res_stack_desc(full), [(B.AC_REGION_UNET_ATTN, B.AC_DIM_BATCH, 1)])
    inf = pf.ac_plan_query()
    assert inf.n_weights == 2 * (9 + 25) and pf.weight_names()[9:34] == [f"A0.{n}" for n in I.attn_block_tensors(full)]
    sh = {pf.ac_plan_weight_info(i).name.decode(): (pf.ac_plan_weight_info(i).rows, pf.ac_plan_weight_info(i).cols) for i in range(34)}
    assert sh["A0.context"] == (4 * 77, 768) and sh["A0.w_kvc"] == (2 * c, 768) and sh["A0.w_1"] == (2 * f, c) and sh["A0.w_2"] == (c, f)
    assert inf.regions[1].model_bytes == 2 * 4 * img + 13 * img + 4 * hw * f * e + 2 * 5 * hw * hw * e + \
        5 * img + 2 * 77 * c * e + 2 * 5 * hw * 77 * e
    seg_full = seg + al(hw * f * e) + al(hw * f * e) + al(77 * c * e) + al(c * 80 * e)      # 2F-wide first layer, its product, k and v^T
    assert seg_full + whole <= inf.workspace_bytes <= seg_full + whole + (64 << 20)
    expect(B.AC_ERR_ARG, lambda: B.Plan(B.res_stack_desc(dataclasses.replace(cfg, heads=0, d_ffn=0, gated=True)), []))
    expect(B.AC_ERR_ARG, lambda: B.Plan(B.res_stack_desc(dataclasses.replace(cfg, heads=0, d_ffn=0, context_tokens=7, context_dim=64)), []))
    expect(B.AC_ERR_UNSUPPORTED, lambda: B.Plan(B.res_stack_desc(dataclasses.replace(cfg, context_tokens=7, context_dim=12)), []))
    expect(B.AC_ERR_ARG, lambda: B.Plan(B.transformer_desc(I.C1, flags=B.AC_FLAG_GATED_FFN), []))
    expect(B.AC_ERR_UNSUPPORTED, lambda: B.Plan(B.res_stack_desc(dataclasses.replace(cfg, heads=4)), []))       # 80 channels per head
    expect(B.AC_ERR_ARG, lambda: B.Plan(B.res_stack_desc(dataclasses.replace(cfg, heads=7)), []))
    expect(B.AC_ERR_UNSUPPORTED, lambda: B.Plan(B.res_stack_desc(dataclasses.replace(cfg, d_ffn=100)), []))
    expect(B.AC_ERR_UNSUPPORTED, lambda: B.Plan(B.res_stack_desc(dataclasses.replace(cfg, height=5, width=5)), []))
    expect(B.AC_ERR_ILLEGAL_CHUNK_DIM, lambda: B.Plan(B.res_stack_desc(cfg), [(B.AC_REGION_UNET_ATTN, B.AC_DIM_SEQ, 64)]))
    expect(B.AC_ERR_ARG, lambda: B.Plan(B.res_stack_desc(dataclasses.replace(cfg, heads=0, d_ffn=0)),
                                        [(B.AC_REGION_UNET_ATTN, B.AC_DIM_BATCH, 1)]))
