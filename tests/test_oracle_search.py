"""Pins of the chunk-search oracle (AutoChunk section 3.3): every chunk it calls legal is run
chunked on random data and must reproduce the unchunked output (rules 1 and 2 by brute force),
the dimensions the rules exclude are excluded, and the cases with a textbook answer come out."""
import numpy as np
import pytest

from oracle import chunk_search as S
from tests import graphs as G


def small_block(batch=2, seq=12, d=8, heads=2, f=16):
    nodes, names = S.transformer_block_graph(batch, seq, d, heads, f)
    return nodes, names, S.run(nodes, S.random_feeds(nodes, 3))


def legal_dims(nodes, start, end):
    return {d for d in range(len(nodes[end].shape)) if S.trace(nodes, start, end, d) is not None}


def test_every_legal_chunk_reproduces_the_unchunked_output():
    nodes, names, val = small_block()
    seen = set()
    n_checked = 0
    for peak in range(len(nodes)):
        if nodes[peak].op in (S.INPUT, S.PARAM):
            continue
        cands, tried, passed = S.search(nodes, peak, 9)
        assert 0 < passed <= tried
        for start, end, dim, node_dims, input_dims in cands:
            if (start, end, dim) in seen:
                continue
            seen.add((start, end, dim))
            g = S.granule(nodes[end], dim)
            extent = nodes[end].shape[dim]
            for clen in {g, 2 * g, (extent // g // 2 + 1) * g, extent}:     # incl. a ragged last segment
                got = S.run_chunked(nodes, val, start, end, dim, node_dims, input_dims, clen)
                assert G.close(got, val[end]), (start, end, dim, clen)
                n_checked += 1
    assert n_checked > 200 and len(seen) > 60


def test_region_dims_of_the_block():
    nodes, nm, _ = small_block()
    # layer norm + packed projection -> [B, S, 3d]: batch and sequence; never the feature dim
    assert legal_dims(nodes, nm["u"], nm["qkv"]) == {0, 1}
    # attention core -> [B, H, S, dh]: batch, heads, query; not the head dim (the probabilities
    # would be computed whole in every segment: rule 4)
    assert legal_dims(nodes, nm["scores"], nm["ctx_h"]) == {0, 1, 2}
    # up to the probabilities [B, H, S, S]: the key dim is what the softmax reduces over
    assert legal_dims(nodes, nm["scores"], nm["probs"]) == {0, 1, 2}
    # the scores alone may be cut along the keys too (each key block needs no other)
    assert legal_dims(nodes, nm["scores"], nm["scores"]) == {0, 1, 2, 3}
    # output projection + residual: rows, and also the output features (each block of columns
    # needs its rows of the weight and its columns of the residual, nothing else)
    assert legal_dims(nodes, nm["o"], nm["h"]) == {0, 1, 2}
    # feed-forward: rows only (its layer norm reduces over the features the flow would need)
    assert legal_dims(nodes, nm["u2"], nm["y"]) == {0, 1}
    # the hidden width of the feed-forward cannot be cut: the second GEMM sums over it
    assert legal_dims(nodes, nm["t"], nm["act"]) == {0, 1, 2}          # ...as an output it can
    assert legal_dims(nodes, nm["t"], nm["down"]) == {0, 1}            # ...inside the region not
    # a region that leaks a second value (h feeds both u2 and y) has no chunk form
    assert legal_dims(nodes, nm["o"], nm["u2"]) == set()
    # from the merged context back through the head split: the sequence flows, the heads flow
    # as the outer factor of the merged feature dim (in multiples of dh)
    assert legal_dims(nodes, nm["ctx_h"], nm["ctx"]) == {0, 1, 2}
    assert S.granule(nodes[nm["ctx"]], 2) == nodes[nm["ctx_h"]].shape[3]


def test_interruptions_and_settings():
    N = [S.Node(S.INPUT, shape=(6, 4)), S.Node(S.PARAM, shape=(4,)), S.Node(S.PARAM, shape=(4,)),
         S.Node(S.NORM_LAST, (0, 1, 2), (6, 4)),
         S.Node(S.TRANSPOSE, (3,), (4, 6), (1, 0))]
    assert S.trace(N, 3, 3, 0) is not None and S.trace(N, 3, 3, 1) is None        # reduced dim
    t = S.trace(N, 3, 4, 1)                                                         # rows, seen through the transpose
    assert t is not None and t[0] == {4: 1, 3: 0} and t[1] == {0: 0}
    assert S.trace(N, 3, 4, 0) is None
    # one node reached in two different dims: x * x^T needs two settings for x
    M = [S.Node(S.INPUT, shape=(5, 5)), S.Node(S.ELEMENTWISE, (0,), (5, 5), fn=lambda a: a + 1),
         S.Node(S.TRANSPOSE, (1,), (5, 5), (1, 0)), S.Node(S.ELEMENTWISE, (1, 2), (5, 5), fn=lambda a, b: a * b)]
    assert S.trace(M, 1, 3, 0) is None and S.trace(M, 1, 3, 1) is None
    assert S.trace(M, 2, 3, 0) is None              # nor may an input be cut in two dims at once
    assert S.trace(M, 2, 2, 0) is not None and S.trace(M, 3, 3, 1) is not None


def test_triangle_contraction_dims():
    n, k, c = 5, 7, 3
    N = [S.Node(S.INPUT, shape=(n, k, c)), S.Node(S.INPUT, shape=(n, k, c)),
         S.Node(S.CONTRACT_IKC_JKC, (0, 1), (n, n, c))]
    val = S.run(N, S.random_feeds(N, 5))
    for d in range(3):                         # rows i, columns j and channels are all legal
        t = S.trace(N, 2, 2, d)
        assert t is not None
        got = S.run_chunked(N, val, 2, 2, d, t[0], t[1], 2)
        assert np.allclose(got, val[2], atol=1e-12)
    assert S.trace(N, 2, 2, 0)[1] == {0: 0} and S.trace(N, 2, 2, 1)[1] == {1: 0} and S.trace(N, 2, 2, 2)[1] == {0: 2, 1: 2}


def test_window_bounds_the_regions():
    nodes, nm, _ = small_block()
    peak = nm["probs"]
    for w in (1, 3, 6):
        cands, tried, passed = S.search(nodes, peak, w)
        assert all(e - s < w and s <= peak <= e for s, e, *_ in cands)
    assert len(S.search(nodes, peak, 6)[0]) > len(S.search(nodes, peak, 3)[0]) > len(S.search(nodes, peak, 1)[0]) > 0


def test_graph_optimisation_moves_nodes_off_the_flow_ahead_of_the_region():
    """Section 3.3, graph optimisation.  Every candidate of the search with it, run with the moved
    nodes computed once and whole, reproduces the unchunked output in segments of exactly the
    chunk length; every strict candidate is found unchanged; the cases with a known answer."""
    nodes, nm, val = small_block()
    t = S.trace_hoisting(nodes, nm["q_flat"], nm["ctx"], 1)          # attention cut along the queries
    assert t is not None and t[2] == {nm[x + s] for x in "kv" for s in ("_flat", "_split", "_h")}
    assert t[1] == {nm["qkv"]: 1}
    assert S.trace_hoisting(nodes, nm["u"], nm["ctx"], 1) is None     # the first node would have to move
    assert S.trace_hoisting(nodes, nm["scores"], nm["ctx_h"], 3) is None   # the head dim: probabilities whole -> end's producer moves
    n_checked = n_moved = 0
    graphs = [nodes] + [[S.Node(op, i, sh, at, G.FNS.get(fn)) for op, i, sh, at, fn in G.random_graph(seed, 13)]
                        for seed in range(40)]
    for gi, gr in enumerate(graphs):
        v = val if gi == 0 else S.run(gr, S.random_feeds(gr, gi))
        seen = set()
        for peak in range(len(gr)):
            if gr[peak].op in (S.INPUT, S.PARAM):
                continue
            strict = {(c[0], c[1], c[2]): c for c in S.search(gr, peak, 10)[0]}
            found = S.search_hoisting(gr, peak, 10)[0]
            by_key = {(c[0], c[1], c[2]): c for c in found}
            for key, c in strict.items():
                assert by_key[key][3:] == (c[3], c[4], set())
            for start, end, dim, node_dims, input_dims, moved in found:
                if (start, end, dim) in seen:
                    continue
                seen.add((start, end, dim))
                assert start not in moved and end not in moved and peak not in moved
                g = S.chunk_granule(gr, end, dim, node_dims, input_dims)
                got, parts = S.run_chunked(gr, v, start, end, dim, node_dims, input_dims, g, parts_too=True, moved=moved)
                assert all(p.shape[dim] == g for p in parts)
                assert G.close(got, v[end]), (gi, start, end, dim)
                n_checked += 1
                n_moved += bool(moved)
    assert n_checked > 1500 and n_moved > 60, (n_checked, n_moved)
