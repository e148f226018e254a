"""Chunk search of the library (ac_chunk_trace, ac_chunk_search; AutoChunk section 3.3) against
the oracle's, candidate by candidate, on the transformer block graph and on seeded random
graphs; plus brute-force pins of the oracle on those random graphs.  Host code only."""
import ctypes as C

import numpy as np
import pytest

from oracle import chunk_search as S
from paper_2401_10652_amd import binding as B
from tests import graphs as G


def oracle_nodes(spec):
    return [S.Node(op, inputs, shape, attr, G.FNS.get(fn)) for op, inputs, shape, attr, fn in spec]


def library_nodes(spec):
    return B.graph_nodes([(op, inputs, shape, attr) for op, inputs, shape, attr, _ in spec])


def block_spec(batch=2, seq=12, d=8, heads=2, f=16):
    nodes, names = S.transformer_block_graph(batch, seq, d, heads, f)
    return [(nd.op, nd.inputs, nd.shape, nd.attr, None) for nd in nodes], names


def oracle_candidates(nodes, peak, window):
    cands, tried, passed = S.search(nodes, peak, window)
    out = []
    for start, end, dim, node_dims, input_dims in cands:
        row = [-1] * len(nodes)
        for i, d in list(node_dims.items()) + list(input_dims.items()):
            row[i] = d
        out.append((start, end, dim, S.chunk_granule(nodes, end, dim, node_dims, input_dims), row))
    return out, tried, passed


def oracle_candidates_hoisting(nodes, peak, window):
    cands, tried, passed = S.search_hoisting(nodes, peak, window)
    out = []
    for start, end, dim, node_dims, input_dims, moved in cands:
        row = [-1] * len(nodes)
        for i, d in list(node_dims.items()) + list(input_dims.items()):
            row[i] = d
        out.append((start, end, dim, S.chunk_granule(nodes, end, dim, node_dims, input_dims), row, sorted(moved)))
    return out, tried, passed


def compare_everywhere(spec, windows, hoist=False):
    on, ln = oracle_nodes(spec), library_nodes(spec)
    total = 0
    for peak in range(len(spec)):
        for w in windows:
            want, tried, passed = (oracle_candidates_hoisting if hoist else oracle_candidates)(on, peak, w)
            got, n_found, n_tried, n_passed = B.ac_chunk_search(ln, peak, w, hoist=hoist)
            assert (n_tried, n_passed, n_found) == (tried, passed, len(want)), (peak, w)
            assert got == want, (peak, w)
            total += sum(bool(c[5]) for c in want) if hoist else len(want)
    return total


def test_search_with_the_graph_optimisation_equals_the_oracle():
    """hoist = 1: candidates, dims and moved nodes, on the block graph, the pair block and random graphs."""
    spec, nm = block_spec()
    assert compare_everywhere(spec, (6, 12, 20), hoist=True) > 50            # counts candidates with moved nodes
    ln = library_nodes(spec)
    dims, moved = B.ac_chunk_trace(ln, nm["q_flat"], nm["ctx"], 1, hoist=True)
    assert moved == sorted(nm[x + s] for x in "kv" for s in ("_flat", "_split", "_h")) and dims[nm["qkv"]] == 1
    assert B.ac_chunk_trace(ln, nm["q_flat"], nm["ctx"], 1) is None          # without it: k and v are read whole
    assert B.ac_chunk_trace(ln, nm["u"], nm["ctx"], 1, hoist=True) is None   # the first node would move
    pair, pnm = pair_spec()
    assert compare_everywhere(pair, (8, 14), hoist=True) > 300
    pl = library_nodes(pair)
    # the triangle update from the a projection on, cut along rows: the b projection moves ahead
    dims, moved = B.ac_chunk_trace(pl, pnm["tmo.a_gate"], pnm["tmo.z"], 0, hoist=True)
    assert moved == sorted(pnm["tmo." + x] for x in ("b_gate", "b_proj", "b"))
    total = 0
    for seed in range(40):
        total += compare_everywhere(G.random_graph(seed, n_ops=13), (5, 10), hoist=True)
    assert total > 100


def test_search_equals_the_oracle_on_the_transformer_block():
    spec, _ = block_spec()
    assert compare_everywhere(spec, (1, 4, 9, len(spec))) > 500


def test_search_equals_the_oracle_on_random_graphs():
    total = 0
    for seed in range(80):
        total += compare_everywhere(G.random_graph(seed, n_ops=8 + seed % 7), (1, 3, 6, 40))
    assert total > 3000


def test_trace_equals_the_oracle_on_every_region_and_dim():
    for seed in (3, 11, 42):
        spec = G.random_graph(seed, n_ops=9)
        on, ln = oracle_nodes(spec), library_nodes(spec)
        first = next(i for i, nd in enumerate(on) if nd.op not in (S.INPUT, S.PARAM))
        n_legal = 0
        for start in range(first, len(on)):
            for end in range(start, len(on)):
                for d in range(len(on[end].shape)):
                    want = S.trace(on, start, end, d)
                    got = B.ac_chunk_trace(ln, start, end, d)
                    if want is None:
                        assert got is None, (seed, start, end, d)
                    else:
                        assert S.some_flow_reaches_an_input(on, start, end, d)   # the first stage loses no chunk
                        row = [-1] * len(on)
                        for i, v in list(want[0].items()) + list(want[1].items()):
                            row[i] = v
                        assert got == row, (seed, start, end, d)
                        n_legal += 1
        assert n_legal > 10


def test_oracle_chunks_of_random_graphs_reproduce_the_unchunked_output():
    """Pins the oracle (flow table of every op kind, granule) by brute force: each chunk it calls
    legal, run segment by segment at its granule, gives segments of exactly that length and the
    unchunked values; a shorter length cuts some tensor inside an element."""
    n_checked, n_coarse, kinds = 0, 0, set()
    for seed in range(60):
        spec = G.random_graph(seed, n_ops=8 + seed % 5)
        nodes = oracle_nodes(spec)
        val = S.run(nodes, S.random_feeds(nodes, seed))
        seen = set()
        for peak in range(len(nodes)):
            if nodes[peak].op in (S.INPUT, S.PARAM):
                continue
            for start, end, dim, node_dims, input_dims in S.search(nodes, peak, 5)[0]:
                if (start, end, dim) in seen:
                    continue
                seen.add((start, end, dim))
                g = S.chunk_granule(nodes, end, dim, node_dims, input_dims)
                extent = nodes[end].shape[dim]
                assert extent % g == 0
                for clen in {g, extent}:
                    got, parts = S.run_chunked(nodes, val, start, end, dim, node_dims, input_dims, clen, parts_too=True)
                    assert all(p.shape[dim] == clen for p in parts), (seed, start, end, dim, clen)
                    assert G.close(got, val[end]), (seed, start, end, dim, clen)
                    n_checked += 1
                if g > 1:
                    n_coarse += 1
                    # at the largest proper divisor of g some cut dim would get a fractional length
                    small = max(k for k in range(1, g) if g % k == 0)
                    exts = [nodes[i].shape[d] for i, d in list(node_dims.items()) + list(input_dims.items())]
                    assert any(small * e % extent for e in exts)
                kinds.update(nodes[i].op for i in range(start, end + 1))
    assert n_checked > 1500 and n_coarse > 20
    assert kinds == set(range(S.LINEAR, S.GROUP_NORM + 1))


def test_granule_of_the_head_merge():
    # context [B, S, H*dh] cut along its features: whole heads only
    spec, nm = block_spec(heads=2, d=8)
    ln = library_nodes(spec)
    got, *_ = B.ac_chunk_search(ln, nm["ctx"], 3)
    by_key = {(s, e, d): g for s, e, d, g, _ in got}
    assert by_key[(nm["ctx_h"], nm["ctx"], 2)] == 4
    assert by_key[(nm["ctx_h"], nm["ctx"], 1)] == 1


def test_region_kinds_of_the_executor_are_chunks_of_the_block_graph():
    """The executor's legality table (batch and sequence legal for every transformer region;
    feature legal for the attention core and the output projection only, where it is not
    implemented; head_dim and key never) read off the graph."""
    spec, nm = block_spec()
    ln = library_nodes(spec)

    def dims(a, b):
        return {d for d in range(len(spec[nm[b]][2])) if B.ac_chunk_trace(ln, nm[a], nm[b], d) is not None}

    assert dims("u", "qkv") == {0, 1}
    assert dims("scores", "ctx") == {0, 1, 2}      # query rows; features in whole heads
    assert dims("scores", "ctx_h") == {0, 1, 2}    # [B, H, S, dh]: not the head dim
    assert dims("scaled", "probs") == {0, 1, 2}    # [B, H, S, S]: not the key dim
    assert dims("o", "h") == {0, 1, 2}
    assert dims("u2", "y") == {0, 1}


def test_count_only_truncation_and_errors():
    spec, nm = block_spec()
    ln = library_nodes(spec)
    full, n_found, _, _ = B.ac_chunk_search(ln, nm["probs"], 6)
    assert n_found == len(full) > 4
    part, n_found2, _, _ = B.ac_chunk_search(ln, nm["probs"], 6, max_out=3)
    assert n_found2 == n_found and part == full[:3]
    L = B.lib()
    found = C.c_int(-1)
    assert L.ac_chunk_search(ln, len(ln), nm["probs"], 6, 0, None, None, None, 2, C.byref(found), None, None) == B.AC_ERR_ARG
    assert L.ac_chunk_search(ln, len(ln), len(ln), 6, 0, None, None, None, 0, C.byref(found), None, None) == B.AC_ERR_ARG
    assert L.ac_chunk_search(ln, len(ln), nm["probs"], 6, 2, None, None, None, 0, C.byref(found), None, None) == B.AC_ERR_ARG
    assert L.ac_chunk_search(ln, len(ln), 0, 0, 0, None, None, None, 0, C.byref(found), None, None) == B.AC_ERR_ARG
    # a peak that is an input: nothing to chunk, no error
    assert L.ac_chunk_search(ln, len(ln), 0, 4, 0, None, None, None, 0, C.byref(found), None, None) == B.AC_OK
    assert found.value == 0
    with pytest.raises(B.AcError):
        B.ac_chunk_trace(ln, nm["x"], nm["u"], 0)       # region holds leaves
    with pytest.raises(B.AcError):
        B.ac_chunk_trace(ln, nm["u"], nm["qkv"], 3)     # no such dim
    # malformed graphs: forward reference, bad permutation, shapes that do not fit the op
    for breaker in ("forward", "perm", "shape", "rank", "huge"):
        bad = library_nodes(spec)
        if breaker == "forward":
            bad[nm["u"]].inputs[0] = nm["y"]
        elif breaker == "perm":
            bad[nm["q_h"]].attr[1] = 0
        elif breaker == "shape":
            bad[nm["scores"]].shape[3] += 1
        elif breaker == "huge":
            bad[nm["x"]].shape[0] = 1 << 41
        else:
            bad[nm["probs"]].rank = 7
        assert L.ac_chunk_search(bad, len(bad), nm["probs"], 6, 0, None, None, None, 0, C.byref(found), None, None) == \
            B.AC_ERR_ARG, breaker


def pair_spec(n=6, c=4, ch=4, heads=2, dh=2, factor=2):
    from paper_2401_10652_amd import graphs as PG
    spec, names = PG.pair_block_graph(n, c, ch, heads, dh, factor)
    # any elementwise function serves the legality checks: pick one by arity
    fn = {1: "tanh", 2: "mul"}
    return [(op, ins, shape, attr, fn[len(ins)] if op == S.ELEMENTWISE else None) for op, ins, shape, attr in spec], names


def test_pair_block_chunks_equal_the_oracle_and_reproduce_the_unchunked_output():
    spec, nm = pair_spec()
    assert compare_everywhere(spec, (1, 5, 12)) > 2000
    nodes = oracle_nodes(spec)
    val = S.run(nodes, S.random_feeds(nodes, 5))
    seen = set()
    for peak in range(len(nodes)):
        if nodes[peak].op in (S.INPUT, S.PARAM):
            continue
        for start, end, dim, node_dims, input_dims in S.search(nodes, peak, 7)[0]:
            if (start, end, dim) in seen:
                continue
            seen.add((start, end, dim))
            g = S.chunk_granule(nodes, end, dim, node_dims, input_dims)
            got = S.run_chunked(nodes, val, start, end, dim, node_dims, input_dims, g)
            assert G.close(got, val[end]), (start, end, dim)
    assert len(seen) > 400


def test_region_kinds_of_the_pair_executor_are_chunks_of_the_pair_graph():
    """Row and column chunks are legal for the chunked part of every pair module, channel chunks
    are not; the projections that every segment reads whole (b of the triangle update; keys,
    values and bias of the triangle attention) cannot be inside the region (rule 4)."""
    spec, nm = pair_spec()
    ln = library_nodes(spec)

    def dims(a, b):
        return {d for d in range(len(spec[nm[b]][2])) if B.ac_chunk_trace(ln, nm[a], nm[b], d) is not None}

    for p in ("tmo.", "tmi."):
        assert dims(p + "o", p + "z") == {0, 1}            # contraction .. residual: rows i, columns j
        assert dims(p + "o", p + "o") == {0, 1, 2}         # the contraction alone: channels too
        assert dims(p + "t", p + "z") == set()             # with the b projection inside: no chunk
    for p in ("tas.", "tae."):
        assert dims(p + "scores", p + "ctx") == {0, 1, 2}  # row, query column, whole heads
        assert dims(p + "scores", p + "probs") == {0, 1, 2}
        assert dims(p + "scores", p + "o") == {0, 1}
        assert dims(p + "t", p + "z") == set()
    assert dims("pt.u", "pt.z") == {0, 1}
    # the ending-node module cut along rows of z: after its two transposes the cut runs along the query column
    row = B.ac_chunk_trace(ln, nm["tae.scores"], nm["tae.z"], 0)
    assert row is not None and row[nm["tae.o"]] == 1 and row[nm["tae.scores"]] == 2


def unet_spec(batch=2, c=4, h=3, w=2, heads=2, t=3, d=5, groups=2):
    from paper_2401_10652_amd import graphs as PG
    spec, names = PG.unet_stage_graph(batch, c, h, w, heads, t, d, groups)
    fn = {1: "tanh", 2: "mul"}
    return [(op, ins, shape, attr, fn[len(ins)] if op == S.ELEMENTWISE else None) for op, ins, shape, attr in spec], names


def test_unet_stage_chunks_equal_the_oracle_and_reproduce_the_unchunked_output():
    spec, nm = unet_spec()
    assert compare_everywhere(spec, (1, 6, 14)) > 2000
    assert compare_everywhere(spec, (10, 16), hoist=True) > 5           # candidates with moved nodes (few here)
    nodes = oracle_nodes(spec)
    val = S.run(nodes, S.random_feeds(nodes, 9))
    seen = set()
    for peak in range(len(nodes)):
        if nodes[peak].op in (S.INPUT, S.PARAM):
            continue
        for start, end, dim, node_dims, input_dims, moved in S.search_hoisting(nodes, peak, 8)[0]:
            if (start, end, dim) in seen:
                continue
            seen.add((start, end, dim))
            g = S.chunk_granule(nodes, end, dim, node_dims, input_dims)
            got = S.run_chunked(nodes, val, start, end, dim, node_dims, input_dims, g, moved=moved)
            assert G.close(got, val[end]), (start, end, dim)
    assert len(seen) > 300
    ln = library_nodes(spec)

    def dims(a, b):
        return {d for d in range(len(spec[nm[b]][2])) if B.ac_chunk_trace(ln, nm[a], nm[b], d) is not None}

    assert dims("res.c1", "res.c1") == {0, 1}          # 3x3 convolution: batch and output channels, not the image dims
    assert dims("tr.in", "tr.in") == {0, 1, 2, 3}      # 1x1 convolution: every pixel on its own
    assert dims("res.n1", "res.c1") == {0}             # behind a group norm: batch only
    assert dims("res.n1", "res.y") == {0}
    assert dims("tr.sa.scores", "tr.sa.ctx") == {0, 1, 2}
    assert dims("tr.ca.scores", "tr.ca.ctx") == {0, 1, 2}
    assert dims("tr.ff.t", "tr.ff.down") == {0, 1}     # the gated feed-forward: rows; its two halves are fixed slices
    # through the 1x1 convolution out and the skip: batch, and rows of the image (whole rows of tokens)
    assert dims("tr.ff.u", "tr.y") == {0, 2}


def test_unet_stage_plan_at_a_latent_diffusion_size():
    from paper_2401_10652_amd import graphs as PG
    spec, nm = PG.unet_stage_graph(2, 320, 64, 64, 8, 77, 768)
    ln = B.graph_nodes(spec)
    per_node, whole, peak_node = B.ac_graph_estimate(ln, 2)
    score = 2 * 8 * 4096 * 4096 * 2
    assert peak_node == nm["tr.sa.scaled"] and whole > 2 * score
    chunks, peak = B.ac_graph_plan(ln, 2, whole // 4, 16, (1, 0, 0, 0), beam=2)
    assert peak <= whole // 4 and len(chunks) == 1
    assert nm["tr.sa.scores"] <= chunks[0][0] <= chunks[0][1] <= nm["tr.sa.ctx"]


def test_corrupted_graphs_are_refused_or_handled_never_trusted():
    """Valid random graphs with a few fields overwritten by arbitrary values: every entry point
    must come back with a status (AC_OK or an error), whatever it is handed."""
    rng = np.random.default_rng(77)
    L = B.lib()
    statuses = set()
    for case in range(1500):
        spec = G.random_graph(case % 40, n_ops=9)
        ln = library_nodes(spec)
        n = len(ln)
        for _ in range(int(rng.integers(1, 4))):
            nd = ln[int(rng.integers(n))]
            field = int(rng.integers(6))
            value = int(rng.choice([-(1 << 31), -7, -1, 0, 1, 2, 5, 6, 7, 100, (1 << 31) - 1]))
            if field == 0:
                nd.op = value
            elif field == 1:
                nd.n_inputs = value
            elif field == 2:
                nd.inputs[int(rng.integers(3))] = value
            elif field == 3:
                nd.rank = value
            elif field == 4:
                nd.shape[int(rng.integers(6))] = int(rng.choice([-(1 << 62), -1, 0, 1, 3, 1 << 20, 1 << 41, (1 << 63) - 1]))
            else:
                nd.attr[int(rng.integers(6))] = int(rng.choice([-(1 << 62), -1, 0, 1, 2, 5, 6, 1 << 40]))
        found, legal, peak_node = C.c_int(0), C.c_int(0), C.c_int(0)
        peak = C.c_uint64(0)
        row = (C.c_int32 * n)()
        moved = (C.c_uint8 * n)()
        out = (B.ac_chunk_candidate * 64)()
        rows = (C.c_int32 * (64 * n))()
        chunks = (B.ac_graph_chunk * 8)()
        w = (C.c_double * 4)(1.0, 1e-9, -1e-9, 0.5)
        cost = C.c_double(0)
        n_out = C.c_int(0)
        hoist = case % 2
        start, end = sorted(int(v) for v in rng.integers(-1, n + 1, size=2))
        statuses.add(L.ac_chunk_search(ln, n, int(rng.integers(-1, n + 1)), int(rng.integers(0, 12)), hoist, out, rows, None,
                                       64, C.byref(found), None, None))
        statuses.add(L.ac_chunk_trace(ln, n, start, end, int(rng.integers(-1, 7)), hoist, row, moved, C.byref(legal)))
        statuses.add(L.ac_graph_estimate(ln, n, 2, None, 0, None, C.byref(peak), C.byref(peak_node)))
        statuses.add(L.ac_graph_chunk_cost(ln, n, start, end, int(rng.integers(-1, 7)), hoist, w, C.byref(cost)))
        statuses.add(L.ac_graph_plan(ln, n, 2, int(rng.integers(0, 4000)), 6, w, 2, hoist, chunks, 8, C.byref(n_out),
                                     C.byref(peak)))
    assert statuses <= {B.AC_OK, B.AC_ERR_ARG, B.AC_ERR_BUDGET_INFEASIBLE, B.AC_ERR_ILLEGAL_CHUNK_DIM}
    assert B.AC_OK in statuses and B.AC_ERR_ARG in statuses
