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
  * with the graph optimisation of section 3.3 (`hoist`), nodes of a region that are off the
    chunk flow are computed whole and once ahead of the region's segments; N_node and N_flop
    of L then count the nodes that run per segment;
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
    chunks = [(start, end, out_dim, chunk_len[, moved])], disjoint legal regions; `moved` lists
    the nodes of the region that are computed whole, once, ahead of its segments (section 3.3,
    graph optimisation): they run first, in order, and those the segments read stay live to
    the region's end."""
    n = len(nodes)
    born, dies = lifetimes(nodes)
    size = [node_bytes(nd, elem_bytes) for nd in nodes]
    read_at_all = {s for nd in nodes for s in nd.inputs}      # the others are results of the graph: kept to the end
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
        start, end, out_dim, clen = region_of[i][:4]
        moved = set(region_of[i][4]) if len(region_of[i]) > 4 else set()
        rest = [j for j in range(start, end + 1) if j not in moved]
        read_by_rest = {s for j in rest for s in nodes[j].inputs if s in moved}
        extent = nodes[end].shape[out_dim]
        held = sum(size[j] for j in range(n) if born[j] < start <= dies[j])   # X, and whatever lives across
        if i in moved:
            mem[i] = held + sum(size[h] for h in moved if h <= i and (h in read_by_rest or dies[h] >= i))
            continue
        inside = sum(size[j] for j in rest if j <= i and j != end and dies[j] >= i)
        assert inside * clen % extent == 0
        kept = sum(size[h] for h in moved if h in read_by_rest or dies[h] > end or h not in read_at_all)   # still needed
        mem[i] = held + kept + size[end] + inside * clen // extent                 # X + Y + A / n
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
    if node.op in (S.NORM_LAST, S.GROUP_NORM):
        return 8 * out      # mean; centre, square, sum; scale by the deviation; gain, shift
    if node.op == S.CONV2D:
        w = nodes[node.inputs[1]].shape
        return 2 * out * w[1] * w[2] * w[3]
    return 0                # views and leaves


def chunk_cost(nodes, start, end, out_dim, weights, moved=()):
    """L = (alpha N_node + beta N_flop) + (gamma N_density + lambda N_stride), section 3.4,
    over the nodes that run once per segment."""
    alpha, beta, gamma, lam = weights
    rest = [i for i in range(start, end + 1) if i not in moved]
    n_node = len(rest)
    n_flop = float(sum(node_flops(nodes[i], nodes) for i in rest))
    n_density = n_flop / n_node
    n_stride = float(math.prod(nodes[end].shape[out_dim + 1:]))
    return (alpha * n_node + beta * n_flop) + (gamma * n_density + lam * n_stride)


def longest_fitting_len(nodes, elem_bytes, chunks, cand, granule, budget, moved=()):
    """Longest chunk length (multiple of granule, below the extent) at which every node of the
    candidate region is within the budget, or 0."""
    start, end, out_dim = cand
    extent = nodes[end].shape[out_dim]
    clen = (extent - 1) // granule * granule
    while clen >= granule:
        mem, _, _ = estimate(nodes, elem_bytes, list(chunks) + [(start, end, out_dim, clen, tuple(moved))])
        if max(mem[start:end + 1]) <= budget:
            return clen
        clen -= granule
    return 0


def feasible_candidates(nodes, elem_bytes, budget, window, weights, chunks, peak_node, hoist=False):
    """One pass's choices: (cost, segments, (start, end, out_dim, chunk_len[, moved])) in search order."""
    out = []
    found = S.search_hoisting(nodes, peak_node, window)[0] if hoist else \
        [c + (set(),) for c in S.search(nodes, peak_node, window)[0]]
    for start, end, dim, node_dims, input_dims, moved in found:
        if any(start <= c[1] and c[0] <= end for c in chunks):
            continue
        g = S.chunk_granule(nodes, end, dim, node_dims, input_dims)
        clen = longest_fitting_len(nodes, elem_bytes, chunks, (start, end, dim), g, budget, moved)
        if clen == 0:
            continue
        extent = nodes[end].shape[dim]
        chunk = (start, end, dim, clen, tuple(sorted(moved))) if hoist else (start, end, dim, clen)
        out.append((chunk_cost(nodes, start, end, dim, weights, moved), -(-extent // clen), chunk))
    return out


def plan(nodes, elem_bytes, budget, window, weights, beam=1, hoist=False):
    """Chunks [(start, end, out_dim, chunk_len)] chosen pass by pass until the peak fits;
    returns (chunks, peak) or raises ValueError when no strategy the passes build gets there.

    Section 3.4 asks for the strategy of least summed cost among those whose peak is within the
    budget.  Every pass extends each strategy of the beam by each candidate around its own peak
    node.  An extension that fits competes for the answer (least summed cost; ties: fewer segments
    in all, then the order of making) and takes no place in the beam; of those that do not fit
    yet, the `beam` cheapest go on to the next pass.  The search ends when the beam is empty.
    With beam = 1 this is: follow the cheapest candidate that does not fit yet, remembering the
    cheapest that did."""
    _, peak0, _ = estimate(nodes, elem_bytes, [])
    if peak0 <= budget:
        return [], peak0
    best = None                                           # (sum of L, segments in all, chunks, peak)
    states = [(0.0, 0, [])]
    while states:
        grown = []
        known = set()
        for total, segments, chunks in states:
            mem, peak, peak_node = estimate(nodes, elem_bytes, chunks)
            if any(c[0] <= peak_node <= c[1] for c in chunks):
                continue                                  # the peak lies in a region already chunked
            for cost, seg, cand in feasible_candidates(nodes, elem_bytes, budget, window, weights, chunks, peak_node, hoist):
                new = chunks + [cand]
                if tuple(sorted(new)) in known:
                    continue                              # the same chunks, chosen in another order
                known.add(tuple(sorted(new)))
                st = (total + cost, segments + seg, new)
                new_peak = estimate(nodes, elem_bytes, new)[1]
                if new_peak <= budget:
                    if best is None or st[:2] < best[:2]:
                        best = st + (new_peak,)
                else:
                    grown.append(st)
        grown.sort(key=lambda st: st[:2])                 # stable: equal keys keep the order of making
        states = grown[:beam]
    if best is None:
        raise ValueError(f"no chunk strategy brings the peak within {budget}")
    return best[2], best[3]
