"""Activation memory of an op graph with and without chunks, the selection cost, and the
pass loop that chunks a graph until it fits a budget.  Plain and slow.  Test infrastructure.

AutoChunk sections 2.1 and 2.2 (activation of a module: inputs + outputs + intermediates,
the intermediates divided by the number of segments once chunked), section 3.2 (passes of
estimate -> search -> select, repeated until the peak is within the budget) and section 3.4
(memory estimation; L = L_macro + L_micro).

Readings where the paper leaves the matter open:
  * every node's output has storage of its own (a view counts as the contiguous copy it
    becomes); parameters are not activations; a graph input is live from the start to its
    last use, a node's output from the node to its last use, a node nobody reads (a graph
    output) to the end;
  * the activation memory at a node is the sum of the tensors live while it runs (its
    operands and its result together); the peak is the largest of these and the peak node
    the first node that reaches it;
  * inside a chunked region every tensor is the fraction chunk_len / extent of its whole
    size, the region's output is held whole from the region's first node on (segments are
    written into it), and every outside tensor the region reads is held until the region's
    last segment is done;
  * "within the budget" is peak <= budget;
  * one pass: search the window around the peak node, drop candidates that overlap a chunk
    already chosen, give each the longest chunk length (a multiple of its granule, below
    the extent) at which the region fits the budget, drop those with none, take the one
    with the least L (ties: fewer segments, then search order).  The weights of L are the
    caller's: the paper tunes them and prints no values;
  * the search over whole strategies (section 3.4: minimise the sum of L subject to the
    budget, by dynamic programming with a beam) keeps the `beam` cheapest strategies from
    pass to pass; a beam of 1 is the loop above.
"""
from __future__ import annotations

import math

from . import chunk_search as S


def node_bytes(node, elem_bytes):
    return 0 if node.op == S.PARAM else math.prod(node.shape) * elem_bytes


def lifetimes(nodes):
    """(born, dies) per node, in node indices; born = -1 for graph inputs."""
    n = len(nodes)
    last = [-1] * n
    for i, nd in enumerate(nodes):
        for s in nd.inputs:
            last[s] = i
    born = [-1 if nd.op in (S.INPUT, S.PARAM) else i for i, nd in enumerate(nodes)]
    dies = [last[i] if last[i] >= 0 else (-1 if nodes[i].op in (S.INPUT, S.PARAM) else n - 1) for i in range(n)]
    return born, dies


def estimate(nodes, elem_bytes, chunks=()):
    """Activation bytes live at every node (0 for leaves), the peak and the peak node.
    chunks = [(start, end, out_dim, chunk_len)], disjoint legal regions."""
    n = len(nodes)
    born, dies = lifetimes(nodes)
    size = [node_bytes(nd, elem_bytes) for nd in nodes]
    region_of = {}
    for ch in chunks:
        for i in range(ch[0], ch[1] + 1):
            region_of[i] = ch
    mem = [0] * n
    for i, nd in enumerate(nodes):
        if nd.op in (S.INPUT, S.PARAM):
            continue
        if i not in region_of:
            mem[i] = sum(size[j] for j in range(n) if born[j] <= i <= dies[j])
            continue
        start, end, out_dim, clen = region_of[i]
        extent = nodes[end].shape[out_dim]
        held = sum(size[j] for j in range(n) if born[j] < start <= dies[j])   # X, and whatever lives across
        inside = sum(size[j] for j in range(start, i + 1) if j != end and dies[j] >= i)
        assert inside * clen % extent == 0
        mem[i] = held + size[end] + inside * clen // extent                  # X + Y + A / n
    peak = max(mem)
    return mem, peak, mem.index(peak)


def node_flops(node, nodes):
    out = math.prod(node.shape)
    if node.op in (S.LINEAR, S.MATMUL_NT, S.MATMUL_NN):
        return 2 * out * nodes[node.inputs[0]].shape[-1]
    if node.op == S.CONTRACT_IKC_JKC:
        return 2 * out * nodes[node.inputs[0]].shape[1]
    if node.op == S.ELEMENTWISE:
        return out
    if node.op == S.SOFTMAX_LAST:
        return 5 * out      # max, subtract, exponential, sum, divide
    if node.op == S.NORM_LAST:
        return 8 * out      # mean; centre, square, sum; scale by the deviation; gain, shift
    return 0                # views and leaves


def chunk_cost(nodes, start, end, out_dim, weights):
    """L = (alpha N_node + beta N_flop) + (gamma N_density + lambda N_stride), section 3.4."""
    alpha, beta, gamma, lam = weights
    n_node = end - start + 1
    n_flop = float(sum(node_flops(nodes[i], nodes) for i in range(start, end + 1)))
    n_density = n_flop / n_node
    n_stride = float(math.prod(nodes[end].shape[out_dim + 1:]))
    return (alpha * n_node + beta * n_flop) + (gamma * n_density + lam * n_stride)


def longest_fitting_len(nodes, elem_bytes, chunks, cand, granule, budget):
    """Longest chunk length (multiple of granule, below the extent) at which every node of the
    candidate region is within the budget, or 0."""
    start, end, out_dim = cand
    extent = nodes[end].shape[out_dim]
    clen = (extent - 1) // granule * granule
    while clen >= granule:
        mem, _, _ = estimate(nodes, elem_bytes, list(chunks) + [(start, end, out_dim, clen)])
        if max(mem[start:end + 1]) <= budget:
            return clen
        clen -= granule
    return 0


def feasible_candidates(nodes, elem_bytes, budget, window, weights, chunks, peak_node):
    """One pass's choices: (cost, segments, (start, end, out_dim, chunk_len)) in search order."""
    out = []
    for start, end, dim, node_dims, input_dims in S.search(nodes, peak_node, window)[0]:
        if any(start <= c[1] and c[0] <= end for c in chunks):
            continue
        g = S.chunk_granule(nodes, end, dim, node_dims, input_dims)
        clen = longest_fitting_len(nodes, elem_bytes, chunks, (start, end, dim), g, budget)
        if clen == 0:
            continue
        extent = nodes[end].shape[dim]
        out.append((chunk_cost(nodes, start, end, dim, weights), -(-extent // clen), (start, end, dim, clen)))
    return out


def plan(nodes, elem_bytes, budget, window, weights, beam=1):
    """Chunks [(start, end, out_dim, chunk_len)] chosen pass by pass until the peak fits;
    returns (chunks, peak) or raises ValueError when no strategy in the beam gets there.

    The beam holds the `beam` strategies of least summed cost (ties: fewer segments in all,
    then the order they were made in).  Every pass extends each strategy that does not fit yet
    by each candidate around its own peak node; strategies that fit stay as they are.  With
    beam = 1 this is: take the cheapest candidate of every pass."""
    states = [(0.0, 0, [])]                               # (sum of L, segments in all, chunks)
    while True:
        grown, all_fit = [], True
        known = set()
        for total, segments, chunks in states:
            mem, peak, peak_node = estimate(nodes, elem_bytes, chunks)
            if peak <= budget:
                if tuple(sorted(chunks)) not in known:
                    known.add(tuple(sorted(chunks)))
                    grown.append((total, segments, chunks))
                continue
            all_fit = False
            if any(c[0] <= peak_node <= c[1] for c in chunks):
                continue                                  # the peak lies in a region already chunked
            for cost, seg, cand in feasible_candidates(nodes, elem_bytes, budget, window, weights, chunks, peak_node):
                new = chunks + [cand]
                if tuple(sorted(new)) in known:
                    continue                              # the same chunks, chosen in another order
                known.add(tuple(sorted(new)))
                grown.append((total + cost, segments + seg, new))
        if all_fit:
            chunks = states[0][2]
            return chunks, estimate(nodes, elem_bytes, chunks)[1]
        if not grown:
            raise ValueError(f"no chunk strategy brings the peak within {budget}")
        grown.sort(key=lambda st: st[:2])                 # stable: equal keys keep the order of making
        states = grown[:beam]
