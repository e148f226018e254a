"""Scalar-loop restatements of the definitions, for tiny shapes only.

These are pins for the fp64 oracle: every sum is an explicit Python loop over
indices, nothing is vectorised, so an index, sign or transposition mistake in the
oracle's array code shows up as a mismatch.
"""
import math


def zeros(*shape):
    if len(shape) == 1:
        return [0.0] * shape[0]
    return [zeros(*shape[1:]) for _ in range(shape[0])]


def ln_row(row, g, b, eps):
    d = len(row)
    mu = sum(row) / d
    var = sum((v - mu) ** 2 for v in row) / d
    return [(row[i] - mu) / math.sqrt(var + eps) * g[i] + b[i] for i in range(d)]


def lin_row(row, w, b=None):
    out = []
    for o in range(len(w)):
        acc = 0.0
        for i in range(len(row)):
            acc += row[i] * w[o][i]
        out.append(acc + (b[o] if b is not None else 0.0))
    return out


def gelu(x):
    return 0.5 * x * (1.0 + math.erf(x / math.sqrt(2.0)))


def sigmoid(x):
    return 1.0 / (1.0 + math.exp(-x))


def softmax(vals):
    m = max(vals)
    e = [math.exp(v - m) if v != -math.inf else 0.0 for v in vals]
    s = sum(e)
    return [v / s for v in e]


def attention(q, k, v, heads, causal, bias=None):
    sq, hd = len(q), len(q[0])
    sk = len(k)
    dh = hd // heads
    out = zeros(sq, hd)
    for h in range(heads):
        for i in range(sq):
            sc = []
            for j in range(sk):
                if causal and j > i:
                    sc.append(-math.inf)
                    continue
                acc = 0.0
                for t in range(dh):
                    acc += q[i][h * dh + t] * k[j][h * dh + t]
                acc /= math.sqrt(dh)
                if bias is not None:
                    acc += bias[h][i][j]
                sc.append(acc)
            p = softmax(sc)
            for t in range(dh):
                acc = 0.0
                for j in range(sk):
                    acc += p[j] * v[j][h * dh + t]
                out[i][h * dh + t] = acc
    return out


def transformer_block(x, w, heads, causal, eps=1e-5):
    s, d = len(x), len(x[0])
    qkv = [lin_row(ln_row(x[i], w["ln1_g"], w["ln1_b"], eps), w["w_qkv"], w["b_qkv"]) for i in range(s)]
    q = [r[:d] for r in qkv]
    k = [r[d:2 * d] for r in qkv]
    v = [r[2 * d:] for r in qkv]
    ctx = attention(q, k, v, heads, causal)
    h = []
    for i in range(s):
        o = lin_row(ctx[i], w["w_o"], w["b_o"])
        h.append([x[i][c] + o[c] for c in range(d)])
    y = []
    for i in range(s):
        u = ln_row(h[i], w["ln2_g"], w["ln2_b"], eps)
        t = [gelu(a) for a in lin_row(u, w["w_1"], w["b_1"])]
        o = lin_row(t, w["w_2"], w["b_2"])
        y.append([h[i][c] + o[c] for c in range(d)])
    return y


def _gated(t, w, p, name):
    val = lin_row(t, w[p + "w_" + name + "p"], w[p + "b_" + name + "p"])
    gate = lin_row(t, w[p + "w_" + name + "g"], w[p + "b_" + name + "g"])
    return [sigmoid(gate[c]) * val[c] for c in range(len(val))]


def tri_mul(z, w, p, outgoing, eps=1e-5):
    n = len(z)
    cz = len(z[0][0])
    t = [[ln_row(z[i][j], w[p + "ln_in_g"], w[p + "ln_in_b"], eps) for j in range(n)] for i in range(n)]
    a = [[_gated(t[i][j], w, p, "a") for j in range(n)] for i in range(n)]
    b = [[_gated(t[i][j], w, p, "b") for j in range(n)] for i in range(n)]
    ch = len(a[0][0])
    out = zeros(n, n, cz)
    for i in range(n):
        for j in range(n):
            o = [0.0] * ch
            for c in range(ch):
                acc = 0.0
                for k in range(n):
                    acc += a[i][k][c] * b[j][k][c] if outgoing else a[k][i][c] * b[k][j][c]
                o[c] = acc
            lo = ln_row(o, w[p + "ln_out_g"], w[p + "ln_out_b"], eps)
            upd = lin_row(lo, w[p + "w_o"], w[p + "b_o"])
            g = lin_row(t[i][j], w[p + "w_g"], w[p + "b_g"])
            for c in range(cz):
                out[i][j][c] = z[i][j][c] + sigmoid(g[c]) * upd[c]
    return out


def tri_att(z, w, p, heads, starting, eps=1e-5):
    n = len(z)
    cz = len(z[0][0])
    t = [[ln_row(z[i][j], w[p + "ln_g"], w[p + "ln_b"], eps) for j in range(n)] for i in range(n)]
    q = [[lin_row(t[i][j], w[p + "w_q"]) for j in range(n)] for i in range(n)]
    k = [[lin_row(t[i][j], w[p + "w_k"]) for j in range(n)] for i in range(n)]
    v = [[lin_row(t[i][j], w[p + "w_v"]) for j in range(n)] for i in range(n)]
    bias = [[lin_row(t[i][j], w[p + "w_bias"]) for j in range(n)] for i in range(n)]
    g = [[lin_row(t[i][j], w[p + "w_g"], w[p + "b_g"]) for j in range(n)] for i in range(n)]
    hd = len(q[0][0])
    dh = hd // heads
    out = zeros(n, n, cz)
    for i in range(n):
        for j in range(n):
            o = [0.0] * hd
            for h in range(heads):
                sc = []
                for kk in range(n):
                    acc = 0.0
                    for d in range(dh):
                        kv = k[i][kk][h * dh + d] if starting else k[kk][j][h * dh + d]
                        acc += q[i][j][h * dh + d] * kv
                    acc /= math.sqrt(dh)
                    acc += bias[j][kk][h] if starting else bias[kk][i][h]
                    sc.append(acc)
                pr = softmax(sc)
                for d in range(dh):
                    acc = 0.0
                    for kk in range(n):
                        vv = v[i][kk][h * dh + d] if starting else v[kk][j][h * dh + d]
                        acc += pr[kk] * vv
                    o[h * dh + d] = sigmoid(g[i][j][h * dh + d]) * acc
            upd = lin_row(o, w[p + "w_o"], w[p + "b_o"])
            for c in range(cz):
                out[i][j][c] = z[i][j][c] + upd[c]
    return out


def pair_transition(z, w, p="pt.", eps=1e-5):
    n = len(z)
    cz = len(z[0][0])
    out = zeros(n, n, cz)
    for i in range(n):
        for j in range(n):
            u = ln_row(z[i][j], w[p + "ln_g"], w[p + "ln_b"], eps)
            t = [max(a, 0.0) for a in lin_row(u, w[p + "w_1"], w[p + "b_1"])]
            o = lin_row(t, w[p + "w_2"], w[p + "b_2"])
            for c in range(cz):
                out[i][j][c] = z[i][j][c] + o[c]
    return out
