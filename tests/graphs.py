"""Seeded random op graphs for the chunk-search tests: plain data, (op, inputs, shape, attr, fn)
tuples with the op numbering of include/autochunk_search.h, leaves first.  No search logic."""
import numpy as np

(INPUT, PARAM, LINEAR, MATMUL_NT, MATMUL_NN, ELEMENTWISE, NORM_LAST, SOFTMAX_LAST, TRANSPOSE, SPLIT_DIM, MERGE_DIMS,
 SLICE_LAST, CONTRACT_IKC_JKC, CONV2D, GROUP_NORM) = range(15)

def close(got, want):
    """Equal up to fp64 rounding of sums taken in another order (values of a random graph can be large)."""
    return np.allclose(got, want, rtol=0, atol=1e-9 * max(1.0, float(np.abs(want).max())))


FNS = {"tanh": np.tanh, "add": lambda a, b: a + b, "mul": lambda a, b: a * b, "add3": lambda a, b, c: a + b * c}


def random_graph(seed, n_ops=10):
    rng = np.random.default_rng(seed)
    sizes = (2, 3, 4, 6)
    nodes = []  # [op, inputs, shape, attr, fn]

    def add(op, inputs=(), shape=(), attr=(), fn=None):
        nodes.append((op, tuple(int(i) for i in inputs), tuple(int(v) for v in shape), tuple(int(v) for v in attr), fn))
        return len(nodes) - 1

    for _ in range(int(rng.integers(1, 3))):
        add(INPUT, shape=rng.choice(sizes, size=int(rng.integers(2, 5))))
    made = 0
    while made < n_ops:
        acts = [i for i, nd in enumerate(nodes) if nd[0] != PARAM]
        # mostly continue from a recent node, so that long runs of dependent nodes appear
        x = acts[-1] if rng.random() < 0.6 else int(rng.choice(acts))
        shp = nodes[x][2]
        r = len(shp)
        op = int(rng.choice([LINEAR, MATMUL_NT, MATMUL_NN, ELEMENTWISE, ELEMENTWISE, NORM_LAST, SOFTMAX_LAST, TRANSPOSE,
                             SPLIT_DIM, MERGE_DIMS, SLICE_LAST, CONTRACT_IKC_JKC, CONV2D, GROUP_NORM]))
        if op == LINEAR:
            n = int(rng.choice(sizes))
            w = add(PARAM, shape=(n, shp[-1]))
            ins = [x, w] + ([add(PARAM, shape=(n,))] if rng.random() < 0.5 else [])
            add(LINEAR, ins, shp[:-1] + (n,))
        elif op in (MATMUL_NT, MATMUL_NN):
            if r < 2:
                continue
            want = shp if op == MATMUL_NT else shp[:-2] + (shp[-1], shp[-2])
            # a partner with the same leading dims and contraction length, else the node itself (transposed)
            partners = [i for i in acts if len(nodes[i][2]) == r and nodes[i][2][:-2] == shp[:-2] and
                        (nodes[i][2][-1] if op == MATMUL_NT else nodes[i][2][-2]) == shp[-1]]
            if partners and rng.random() < 0.7:
                y = int(rng.choice(partners))
            elif op == MATMUL_NT:
                y = x
            else:
                perm = list(range(r - 2)) + [r - 1, r - 2]
                y = add(TRANSPOSE, [x], want, perm)
                made += 1
            n = nodes[y][2][-2] if op == MATMUL_NT else nodes[y][2][-1]
            add(op, [x, y], shp[:-1] + (n,))
        elif op == ELEMENTWISE:
            kind = rng.random()
            same = [i for i in acts if nodes[i][2] == shp and i != x]
            if kind < 0.3:
                add(ELEMENTWISE, [x], shp, fn="tanh")
            elif kind < 0.6 and same:
                add(ELEMENTWISE, [x, int(rng.choice(same))], shp, fn=str(rng.choice(["add", "mul"])))
            elif kind < 0.8:
                # a broadcast operand: trailing dims of x, some of them of size 1
                k = int(rng.integers(1, r + 1))
                bshape = tuple(1 if rng.random() < 0.4 else v for v in shp[r - k:])
                add(ELEMENTWISE, [x, add(PARAM, shape=bshape)], shp, fn="add")
            else:
                add(ELEMENTWISE, [x, x, add(PARAM, shape=shp[-1:])], shp, fn="add3")
        elif op in (NORM_LAST, SOFTMAX_LAST):
            if op == NORM_LAST and rng.random() < 0.5:
                add(op, [x, add(PARAM, shape=shp[-1:]), add(PARAM, shape=shp[-1:])], shp)
            else:
                add(op, [x], shp)
        elif op == TRANSPOSE:
            perm = rng.permutation(r)
            add(TRANSPOSE, [x], [shp[p] for p in perm], perm)
        elif op == SPLIT_DIM:
            cands = [p for p in range(r) if shp[p] in (4, 6)]
            if not cands or r >= 5:
                continue
            p = int(rng.choice(cands))
            outer = 2 if shp[p] == 4 or rng.random() < 0.5 else 3
            add(SPLIT_DIM, [x], shp[:p] + (outer, shp[p] // outer) + shp[p + 1:], (p, outer))
        elif op == MERGE_DIMS:
            if r < 3:
                continue
            p = int(rng.integers(0, r - 1))
            add(MERGE_DIMS, [x], shp[:p] + (shp[p] * shp[p + 1],) + shp[p + 2:], (p, shp[p + 1]))
        elif op == SLICE_LAST:
            if shp[-1] < 2:
                continue
            a = int(rng.integers(0, shp[-1] - 1))
            b = int(rng.integers(a + 1, shp[-1] + 1))
            add(SLICE_LAST, [x], shp[:-1] + (b - a,), (a, b))
        elif op == CONV2D:
            if r != 4:
                continue
            co = int(rng.choice(sizes))
            kh, kw = (int(v) for v in rng.choice([1, 3], size=2))
            ins = [x, add(PARAM, shape=(co, shp[1], kh, kw))] + ([add(PARAM, shape=(co,))] if rng.random() < 0.5 else [])
            add(CONV2D, ins, (shp[0], co) + shp[2:])
        elif op == GROUP_NORM:
            if r != 4:
                continue
            groups = int(rng.choice([g for g in (1, 2, 3) if shp[1] % g == 0]))
            ins = [x] + ([add(PARAM, shape=(shp[1],)), add(PARAM, shape=(shp[1],))] if rng.random() < 0.5 else [])
            add(GROUP_NORM, ins, shp, (groups,))
        elif op == CONTRACT_IKC_JKC:
            if r != 3:
                continue
            partners = [i for i in acts if len(nodes[i][2]) == 3 and nodes[i][2][1:] == shp[1:]]
            y = int(rng.choice(partners))
            add(CONTRACT_IKC_JKC, [x, y], (shp[0], nodes[y][2][0], shp[2]))
        made += 1
    # leaves first, order otherwise kept
    order = [i for i, nd in enumerate(nodes) if nd[0] in (INPUT, PARAM)] + \
            [i for i, nd in enumerate(nodes) if nd[0] not in (INPUT, PARAM)]
    new_id = {old: new for new, old in enumerate(order)}
    return [(nodes[i][0], tuple(new_id[s] for s in nodes[i][1]), nodes[i][2], nodes[i][3], nodes[i][4]) for i in order]
