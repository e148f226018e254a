"""Chunk search on a small op graph, plain and slow.  Test infrastructure.

AutoChunk, section 3.3.  A chunk region is a run of consecutive nodes of the
(topologically ordered) graph; a candidate chunk is a region plus one dimension
of its output.  Starting from that dimension the chunk flow is traced upwards,
breadth first, through every node of the region: passing a node fixes the
node's chunk dimension and tells, for each of its inputs, which dimension the
flow continues in, that the input lacks the dimension (it is then used whole),
or that the dimension is computed over there (a reduction, a contraction, the
inner factor of a reshape), which interrupts the flow.  The candidate is legal
when (rules 1 to 4 of section 3.3)

  1+2  the region has the chunk form Y^c = F(X^c, X^nc): its only value used
       outside is the last node's, every other node feeds the region only, and
       cutting X^c and concatenating the parts of Y^c reproduces Y (guaranteed
       by the per-op flow rules below; `run_chunked` checks it by brute force);
  3    the flow reaches at least one input of the region without interruption;
  4    every node of the region is passed by the flow, with one setting each
       (a node reached twice must be reached in the same dimension, and a node
       that some consumer inside the region reads whole has no setting at all:
       every segment would have to compute all of it).  An input of the region
       may be read both ways, cut by one operand and whole by another.

Section 3.3 also bounds the work: only regions inside a window of k nodes that
holds the peak node are tried, and a region is searched in full only if a
cheaper first test passes: does any flow lead from the output dimension to an
input of the region at all (followed without the checks of rule 4, and given up
as soon as one input is reached).  A legal chunk always passes it.

This module holds the op table (flow of a dimension through each op kind), the
search, and a numpy executor that runs a region chunked, so that tests can
check every legal candidate against the unchunked result.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field

import numpy as np

# op kinds (shared numbering with the C interface; a format, not arithmetic)
INPUT, PARAM, LINEAR, MATMUL_NT, MATMUL_NN, ELEMENTWISE, NORM_LAST, SOFTMAX_LAST, TRANSPOSE, SPLIT_DIM, MERGE_DIMS, \
    SLICE_LAST, CONTRACT_IKC_JKC, CONV2D, GROUP_NORM = range(15)

FLOW, WHOLE, BROKEN = 0, 1, 2


@dataclass
class Node:
    op: int
    inputs: tuple = ()
    shape: tuple = ()
    attr: tuple = ()        # TRANSPOSE: perm; SPLIT_DIM: (dim, outer); MERGE_DIMS: (dim, inner); SLICE_LAST: (start, stop);
                            # GROUP_NORM: (groups,)
    fn: object = None       # ELEMENTWISE: numpy callable of its inputs (executor only)


def flow_to_input(node: Node, nodes, c: int, which: int):
    """Where the chunk flow that passes `node` in output dim c continues in input `which`:
    (FLOW, dim) | (WHOLE, -1) if the input has no such dimension | (BROKEN, -1)."""
    src = nodes[node.inputs[which]]
    r_out, r_in = len(node.shape), len(src.shape)
    if node.op == ELEMENTWISE:
        d = c - (r_out - r_in)          # trailing dims aligned
        if d < 0 or src.shape[d] == 1 and node.shape[c] != 1:
            return WHOLE, -1
        return FLOW, d
    if node.op in (NORM_LAST, SOFTMAX_LAST):
        if which > 0:                   # gain / shift lie along the normalised dim
            return WHOLE, -1
        return (BROKEN, -1) if c == r_out - 1 else (FLOW, c)
    if node.op == LINEAR:               # x [.., K], w [N, K], bias [N] -> [.., N]
        if c < r_out - 1:
            return (FLOW, c) if which == 0 else (WHOLE, -1)
        return (WHOLE, -1) if which == 0 else (FLOW, 0)
    if node.op in (MATMUL_NT, MATMUL_NN):   # a [.., M, K]; b [.., N, K] (NT) or [.., K, N] (NN) -> [.., M, N]
        if c < r_out - 2:
            return FLOW, c
        if c == r_out - 2:
            return (FLOW, c) if which == 0 else (WHOLE, -1)
        if which == 0:
            return WHOLE, -1
        return FLOW, (r_in - 2 if node.op == MATMUL_NT else r_in - 1)
    if node.op == TRANSPOSE:
        return FLOW, node.attr[c]
    if node.op == SPLIT_DIM:            # [.., A*B, ..] -> [.., A, B, ..] at dim p
        p = node.attr[0]
        if c < p:
            return FLOW, c
        if c == p:
            return FLOW, p              # the outer factor is a slice of the merged dim
        if c == p + 1:
            return BROKEN, -1           # the inner factor is a strided gather, not a slice
        return FLOW, c - 1
    if node.op == MERGE_DIMS:           # [.., A, B, ..] -> [.., A*B, ..] at dim p
        p = node.attr[0]
        if c < p:
            return FLOW, c
        if c == p:
            return FLOW, p              # cut the merged dim in multiples of B: slices of A
        return FLOW, c + 1
    if node.op == SLICE_LAST:           # a fixed range of the last dim: cutting it further is not a plain slice
        return (BROKEN, -1) if c == r_out - 1 else (FLOW, c)
    if node.op == CONTRACT_IKC_JKC:     # a [I, K, C], b [J, K, C] -> [I, J, C]
        if c == 0:
            return (FLOW, 0) if which == 0 else (WHOLE, -1)
        if c == 1:
            return (WHOLE, -1) if which == 0 else (FLOW, 0)
        return FLOW, 2
    if node.op == CONV2D:               # x [B, Ci, H, W], w [Co, Ci, kh, kw], bias [Co] -> [B, Co, H, W], same padding
        w = nodes[node.inputs[1]]
        if c == 0:
            return (FLOW, 0) if which == 0 else (WHOLE, -1)
        if c == 1:
            return (WHOLE, -1) if which == 0 else (FLOW, 0)
        if w.shape[c] != 1:
            return BROKEN, -1           # a window wider than one element reads its neighbours across any cut
        return (FLOW, c) if which == 0 else (WHOLE, -1)
    if node.op == GROUP_NORM:           # x [B, C, H, W] normalised over (C / groups, H, W); gain, shift [C]
        if which > 0:
            return WHOLE, -1
        return (FLOW, 0) if c == 0 else (BROKEN, -1)    # channel chunks in whole groups would be legal: not expressed
    raise ValueError(f"no flow rule for op {node.op}")


def granule(node: Node, c: int) -> int:
    """Chunk lengths along output dim c must be multiples of this (merged dims cut between rows)."""
    if node.op == MERGE_DIMS and c == node.attr[0]:
        return node.attr[1]
    return 1


def chunk_granule(nodes, end: int, out_dim: int, node_dims, input_dims) -> int:
    """Smallest chunk length along out_dim for which every tensor on the flow is cut between
    whole elements: the cut dims all have extents proportional to the output's (a segment of
    len elements of the output is len * ext / ext_out elements of a tensor whose cut dim has
    extent ext), so len must make each of those an integer."""
    ext_out = nodes[end].shape[out_dim]
    g = 1
    for i, d in list(node_dims.items()) + list(input_dims.items()):
        g = math.lcm(g, ext_out // math.gcd(ext_out, nodes[i].shape[d]))
    return g


def trace(nodes, start: int, end: int, out_dim: int):
    """Chunk dims of every node of region [start, end] for a flow that leaves in `out_dim`
    of node `end`, or None when a rule is violated.  Returns (node_dims, input_dims) with
    input_dims = {outside node id: dim} for the chunkable inputs X^c."""
    inside = set(range(start, end + 1))
    # rules 1+2, form: nothing but the last node is visible outside the region
    for i, nd in enumerate(nodes):
        if i in inside:
            continue
        for s in nd.inputs:
            if s in inside and s != end:
                return None
    dims = {end: out_dim}
    xin = {}
    frontier = [end]
    while frontier:
        nxt = []
        for n in frontier:
            nd = nodes[n]
            for which, s in enumerate(nd.inputs):
                kind, d = flow_to_input(nd, nodes, dims[n], which)
                if kind == BROKEN:
                    return None                      # interrupted flow
                if kind == WHOLE:
                    if s in inside:
                        return None                  # rule 4: that node would be needed whole by every segment
                    continue
                if s in inside:
                    if s in dims:
                        if dims[s] != d:
                            return None              # rule 4: two settings for one node
                        continue
                    dims[s] = d
                    nxt.append(s)
                else:
                    if s in xin and xin[s] != d:
                        return None
                    xin[s] = d
        frontier = nxt
    if any(i not in dims for i in inside if nodes[i].op not in (INPUT, PARAM)):
        return None                                  # rule 4: a node no flow passes
    if not xin:
        return None                                  # rule 3: no input reached
    return dims, xin


def trace_hoisting(nodes, start: int, end: int, out_dim: int):
    """Like `trace`, with the graph optimisation of section 3.3 applied: nodes of the region
    that the chunk flow does not pass, or that some node reads whole, are moved ahead of the
    region together with everything inside the region they depend on (they are computed once,
    whole, and not again in every segment), and the rest is traced as a region of its own
    whose inputs include the moved nodes.  Returns (node_dims, input_dims, moved) or None;
    input_dims also names the moved nodes that the rest reads in slices.  A region whose first
    node would be moved is left to the shorter region that starts behind it."""
    inside = set(range(start, end + 1))
    for i, nd in enumerate(nodes):
        if i not in inside:
            for s in nd.inputs:
                if s in inside and s != end:
                    return None
    moved = set()
    while True:
        rest = inside - moved
        dims, xin, whole = {end: out_dim}, {}, set()
        frontier = [end]
        while frontier:
            nxt = []
            for n in frontier:
                nd = nodes[n]
                for which, s in enumerate(nd.inputs):
                    kind, d = flow_to_input(nd, nodes, dims[n], which)
                    if kind == BROKEN:
                        return None
                    if kind == WHOLE:
                        if s in rest:
                            whole.add(s)
                        continue
                    if s in rest:
                        if s in dims:
                            if dims[s] != d:
                                return None
                            continue
                        dims[s] = d
                        nxt.append(s)
                    else:
                        if s in xin and xin[s] != d:
                            return None
                        xin[s] = d
            frontier = nxt
        # move what is read whole or not reached, with its ancestors inside the region
        grow = {i for i in rest if i in whole or i not in dims}
        todo = list(grow)
        while todo:
            for s in nodes[todo.pop()].inputs:
                if s in rest and s not in grow:
                    grow.add(s)
                    todo.append(s)
        if not grow:
            break
        if end in grow or start in grow:
            return None
        moved |= grow
    if start in moved or not xin:
        return None
    return dims, xin, moved


def some_flow_reaches_an_input(nodes, start: int, end: int, out_dim: int) -> bool:
    """First stage of the two-stage search: is there any uninterrupted flow from `out_dim` of
    node `end` to a node outside the region?  No rule is checked on the way."""
    todo, seen = [(end, out_dim)], {(end, out_dim)}
    while todo:
        n, c = todo.pop()
        for which, s in enumerate(nodes[n].inputs):
            kind, d = flow_to_input(nodes[n], nodes, c, which)
            if kind != FLOW:
                continue
            if s < start:
                return True
            if (s, d) not in seen:
                seen.add((s, d))
                todo.append((s, d))
    return False


def region_inputs(nodes, start, end):
    inside = set(range(start, end + 1))
    return sorted({s for i in inside for s in nodes[i].inputs if s not in inside})


def search_hoisting(nodes, peak: int, window: int):
    """`search` with `trace_hoisting`: candidates are (start, end, out_dim, node_dims, input_dims,
    moved); a candidate whose peak node would be moved out of the region is dropped (chunking
    it would not touch the peak)."""
    out, tried, passed = [], 0, 0
    for start in range(max(0, peak - window + 1), peak + 1):
        for end in range(peak, min(len(nodes), start + window)):
            if any(nodes[i].op in (INPUT, PARAM) for i in range(start, end + 1)):
                break
            for d in range(len(nodes[end].shape)):
                tried += 1
                if not some_flow_reaches_an_input(nodes, start, end, d):
                    continue
                passed += 1
                t = trace_hoisting(nodes, start, end, d)
                if t is not None and peak not in t[2]:
                    out.append((start, end, d) + t)
    return out, tried, passed


def search(nodes, peak: int, window: int):
    """All legal chunks whose region lies in a window of `window` nodes and holds `peak`.
    Returns (candidates, tried, passed_first_stage); a candidate is
    (start, end, out_dim, node_dims, input_dims)."""
    out, tried, passed = [], 0, 0
    for start in range(max(0, peak - window + 1), peak + 1):
        if nodes[start].op in (INPUT, PARAM):
            continue
        for end in range(peak, min(len(nodes), start + window)):
            if any(nodes[i].op in (INPUT, PARAM) for i in range(start, end + 1)):
                continue
            for d in range(len(nodes[end].shape)):
                tried += 1
                if not some_flow_reaches_an_input(nodes, start, end, d):
                    continue
                passed += 1
                t = trace(nodes, start, end, d)
                if t is not None:
                    out.append((start, end, d, t[0], t[1]))
    return out, tried, passed


# --------------------------------------------------------------------------------------
# numpy executor: runs the graph, or a region chunked along a traced flow
# --------------------------------------------------------------------------------------

def _apply(nd: Node, args):
    if nd.op == LINEAR:
        y = args[0] @ args[1].T
        return y + args[2] if len(args) > 2 else y
    if nd.op == MATMUL_NT:
        return args[0] @ np.swapaxes(args[1], -1, -2)
    if nd.op == MATMUL_NN:
        return args[0] @ args[1]
    if nd.op == ELEMENTWISE:
        return nd.fn(*args)
    if nd.op == NORM_LAST:
        x = args[0]
        mu = x.mean(-1, keepdims=True)
        y = (x - mu) / np.sqrt(((x - mu) ** 2).mean(-1, keepdims=True) + 1e-5)
        if len(args) > 1:
            y = y * args[1] + args[2]
        return y
    if nd.op == SOFTMAX_LAST:
        e = np.exp(args[0] - args[0].max(-1, keepdims=True))
        return e / e.sum(-1, keepdims=True)
    if nd.op == TRANSPOSE:
        return np.transpose(args[0], nd.attr)
    if nd.op == SPLIT_DIM:
        p, outer = nd.attr
        s = args[0].shape
        return args[0].reshape(s[:p] + (outer, s[p] // outer) + s[p + 1:])
    if nd.op == MERGE_DIMS:
        p = nd.attr[0]
        s = args[0].shape
        return args[0].reshape(s[:p] + (s[p] * s[p + 1],) + s[p + 2:])
    if nd.op == SLICE_LAST:
        return args[0][..., nd.attr[0]:nd.attr[1]]
    if nd.op == CONTRACT_IKC_JKC:
        return np.einsum("ikc,jkc->ijc", args[0], args[1])
    if nd.op == CONV2D:
        x, w = args[0], args[1]
        kh, kw = w.shape[2], w.shape[3]
        xp = np.pad(x, ((0, 0), (0, 0), (kh // 2, kh // 2), (kw // 2, kw // 2)))
        y = np.zeros((x.shape[0], w.shape[0], x.shape[2], x.shape[3]))
        for a in range(kh):
            for b in range(kw):
                y += np.einsum("bchw,oc->bohw", xp[:, :, a:a + x.shape[2], b:b + x.shape[3]], w[:, :, a, b])
        return y + args[2][None, :, None, None] if len(args) > 2 else y
    if nd.op == GROUP_NORM:
        x = args[0]
        b, c, h, w_ = x.shape
        g = x.reshape(b, nd.attr[0], -1)
        mu = g.mean(-1, keepdims=True)
        y = ((g - mu) / np.sqrt(((g - mu) ** 2).mean(-1, keepdims=True) + 1e-5)).reshape(x.shape)
        if len(args) > 1:
            y = y * args[1][None, :, None, None] + args[2][None, :, None, None]
        return y
    raise ValueError(nd.op)


def run(nodes, feeds):
    """Values of every node; feeds = {node id: array} for INPUT and PARAM nodes."""
    val = dict(feeds)
    for i, nd in enumerate(nodes):
        if nd.op in (INPUT, PARAM):
            continue
        val[i] = _apply(nd, [val[s] for s in nd.inputs])
    return val


def run_chunked(nodes, val, start, end, out_dim, node_dims, input_dims, chunk_len, parts_too=False, moved=()):
    """Output of region [start, end] computed segment by segment (section 2.2): the chunkable
    inputs are cut along their traced dims, the others are used whole, the parts of the
    output are concatenated along out_dim.  `val` holds the unchunked values of the inputs."""
    extent = nodes[end].shape[out_dim]
    parts = []
    for a in range(0, extent, chunk_len):
        b = min(extent, a + chunk_len)
        frac0, frac1 = a / extent, b / extent
        local, cut = {}, {}
        for s in region_inputs(nodes, start, end) + sorted(moved):   # moved nodes: computed whole beforehand
            x = val[s]
            if s in input_dims:
                d = input_dims[s]
                lo, hi = round(frac0 * x.shape[d]), round(frac1 * x.shape[d])
                cut[s] = np.take(x, range(lo, hi), axis=d)
        for i in range(start, end + 1):
            if i in moved:
                continue
            nd = nodes[i]
            args = []
            for which, s in enumerate(nd.inputs):
                if s in local:
                    args.append(local[s])
                elif flow_to_input(nd, nodes, node_dims[i], which)[0] == FLOW:
                    args.append(cut[s])         # X^c: this operand takes the segment's part
                else:
                    args.append(val[s])         # X^nc: this operand takes the input whole
            if nd.op == SPLIT_DIM:      # the cut dim's outer factor shrinks with the segment
                p, outer = nd.attr
                inner = nodes[nd.inputs[0]].shape[p] // outer
                s_ = args[0].shape
                local[i] = args[0].reshape(s_[:p] + (s_[p] // inner, inner) + s_[p + 1:])
            else:
                local[i] = _apply(nd, args)
        parts.append(local[end])
    whole = np.concatenate(parts, axis=out_dim)
    return (whole, parts) if parts_too else whole


# --------------------------------------------------------------------------------------
# graphs of the workloads (shapes only matter for the search; the executor needs feeds)
# --------------------------------------------------------------------------------------

def transformer_block_graph(batch, seq, d, heads, f):
    """Pre-LN block on x [B, S, d] as a list of nodes; returns (nodes, names)."""
    dh = d // heads
    N, names = [], {}

    def add(name, op, inputs=(), shape=(), attr=(), fn=None):
        N.append(Node(op, tuple(names[i] for i in inputs), tuple(shape), tuple(attr), fn))
        names[name] = len(N) - 1

    add("x", INPUT, shape=(batch, seq, d))
    for nm, shp in (("g1", (d,)), ("b1", (d,)), ("wqkv", (3 * d, d)), ("bqkv", (3 * d,)), ("wo", (d, d)), ("bo", (d,)),
                    ("g2", (d,)), ("b2", (d,)), ("w1", (f, d)), ("bf1", (f,)), ("w2", (d, f)), ("bf2", (d,))):
        add(nm, PARAM, shape=shp)
    add("u", NORM_LAST, ("x", "g1", "b1"), (batch, seq, d))
    add("qkv", LINEAR, ("u", "wqkv", "bqkv"), (batch, seq, 3 * d))
    for i, nm in enumerate("qkv"):
        add(nm + "_flat", SLICE_LAST, ("qkv",), (batch, seq, d), (i * d, (i + 1) * d))
        add(nm + "_split", SPLIT_DIM, (nm + "_flat",), (batch, seq, heads, dh), (2, heads))
        add(nm + "_h", TRANSPOSE, (nm + "_split",), (batch, heads, seq, dh), (0, 2, 1, 3))
    add("scores", MATMUL_NT, ("q_h", "k_h"), (batch, heads, seq, seq))
    add("scaled", ELEMENTWISE, ("scores",), (batch, heads, seq, seq), fn=lambda s: s / math.sqrt(dh))
    add("probs", SOFTMAX_LAST, ("scaled",), (batch, heads, seq, seq))
    add("ctx_h", MATMUL_NN, ("probs", "v_h"), (batch, heads, seq, dh))
    add("ctx_t", TRANSPOSE, ("ctx_h",), (batch, seq, heads, dh), (0, 2, 1, 3))
    add("ctx", MERGE_DIMS, ("ctx_t",), (batch, seq, d), (2, dh))
    add("o", LINEAR, ("ctx", "wo", "bo"), (batch, seq, d))
    add("h", ELEMENTWISE, ("x", "o"), (batch, seq, d), fn=lambda a, b: a + b)
    add("u2", NORM_LAST, ("h", "g2", "b2"), (batch, seq, d))
    add("t", LINEAR, ("u2", "w1", "bf1"), (batch, seq, f))
    add("act", ELEMENTWISE, ("t",), (batch, seq, f), fn=lambda t: np.maximum(t, 0.0) * 0.5 + np.tanh(t) * 0.5)
    add("down", LINEAR, ("act", "w2", "bf2"), (batch, seq, d))
    add("y", ELEMENTWISE, ("h", "down"), (batch, seq, d), fn=lambda a, b: a + b)
    return N, names


def random_feeds(nodes, seed=0):
    rng = np.random.default_rng(seed)
    return {i: rng.standard_normal(nd.shape) for i, nd in enumerate(nodes) if nd.op in (INPUT, PARAM)}
