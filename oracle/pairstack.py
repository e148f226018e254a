"""fp64 CPU oracle: unchunked AlphaFold-style pair-stack block.  Test infrastructure.

The paper (AutoChunk, section 4) evaluates on AlphaFold without defining its
modules.  The reading bound here follows the mathematical description of the pair
stack in the AlphaFold publication (Jumper et al. 2021, supplementary algorithms
for triangular multiplicative update, triangular self-attention and pair
transition), dropout omitted.  With z [N, N, c_z], "Lin" = matmul + bias, weights
[out, in]:

  TriMulOut   t = LN(z); a = sigmoid(Lin(t)) * Lin(t); b = sigmoid(Lin(t)) * Lin(t)
              g = sigmoid(Lin(t)); o[i,j,:] = sum_k a[i,k,:] * b[j,k,:]
              z <- z + g * Lin(LN(o))
  TriMulIn    same with o[i,j,:] = sum_k a[k,i,:] * b[k,j,:]
  TriAttStart t = LN(z); q,k,v = Lin_nobias(t) as [N,N,H,d_h]; bias = Lin_nobias(t) [N,N,H]
              g = sigmoid(Lin(t))
              alpha[i,j,k,h] = softmax_k(q[i,j,h].k[i,k,h]/sqrt(d_h) + bias[j,k,h])
              o[i,j,h,:] = g[i,j,h,:] * sum_k alpha[i,j,k,h] v[i,k,h,:];  z <- z + Lin(o)
  TriAttEnd   alpha[i,j,k,h] = softmax_k(q[i,j,h].k[k,j,h]/sqrt(d_h) + bias[k,i,h])
              o[i,j,h,:] = g[i,j,h,:] * sum_k alpha[i,j,k,h] v[k,j,h,:];  z <- z + Lin(o)
  Transition  z <- z + Lin(act(Lin(LN(z))))          (hidden width = factor * c_z)
  Block       TriMulOut, TriMulIn, TriAttStart, TriAttEnd, Transition, in this order.

Each function takes ``rows``: the indices i (dim 0 of the output) to evaluate, so
that a few rows of a large problem can be checked; all rows by default.  Nothing
else is blocked or reordered.
"""
from __future__ import annotations

import math

import numpy as np

from .transformer import ACTIVATIONS, layer_norm, linear, softmax_rows


def sigmoid(x):
    return 1.0 / (1.0 + np.exp(-np.asarray(x, np.float64)))


def _rows(rows, n):
    return np.arange(n) if rows is None else np.asarray(rows, np.int64)


def tri_mul(z, w, p, outgoing, eps=1e-5, rows=None):
    """Triangular multiplicative update; returns the new z rows [len(rows), N, c_z]."""
    z = np.asarray(z, np.float64)
    n = z.shape[0]
    rows = _rows(rows, n)
    t = layer_norm(z, w[p + "ln_in_g"], w[p + "ln_in_b"], eps)
    a = sigmoid(linear(t, w[p + "w_ag"], w[p + "b_ag"])) * linear(t, w[p + "w_ap"], w[p + "b_ap"])
    b = sigmoid(linear(t, w[p + "w_bg"], w[p + "b_bg"])) * linear(t, w[p + "w_bp"], w[p + "b_bp"])
    if outgoing:
        # o[i,j,c] = sum_k a[i,k,c] b[j,k,c]: one [rows,N]x[N,N] matmul per channel c
        ac = np.ascontiguousarray(a[rows].transpose(2, 0, 1))          # [c, i, k]
        bc = np.ascontiguousarray(b.transpose(2, 0, 1))                # [c, j, k]
    else:
        # o[i,j,c] = sum_k a[k,i,c] b[k,j,c]
        ac = np.ascontiguousarray(a[:, rows].transpose(2, 1, 0))       # [c, i, k]
        bc = np.ascontiguousarray(b.transpose(2, 1, 0))                # [c, j, k]
    o = np.matmul(ac, bc.transpose(0, 2, 1)).transpose(1, 2, 0)
    g = sigmoid(linear(t[rows], w[p + "w_g"], w[p + "b_g"]))
    upd = g * linear(layer_norm(o, w[p + "ln_out_g"], w[p + "ln_out_b"], eps), w[p + "w_o"], w[p + "b_o"])
    return z[rows] + upd


def tri_att(z, w, p, heads, starting, eps=1e-5, rows=None):
    """Triangular self-attention around the starting / ending node; new z rows."""
    z = np.asarray(z, np.float64)
    n, _, cz = z.shape
    rows = _rows(rows, n)
    t = layer_norm(z, w[p + "ln_g"], w[p + "ln_b"], eps)
    hd = np.asarray(w[p + "w_q"]).shape[0]
    dh = hd // heads
    q = linear(t, w[p + "w_q"]).reshape(n, n, heads, dh)
    k = linear(t, w[p + "w_k"]).reshape(n, n, heads, dh)
    v = linear(t, w[p + "w_v"]).reshape(n, n, heads, dh)
    bias = linear(t, w[p + "w_bias"])                      # [N, N, H]
    g = sigmoid(linear(t, w[p + "w_g"], w[p + "b_g"])).reshape(n, n, heads, dh)
    scale = 1.0 / math.sqrt(dh)
    out = np.empty((len(rows), n, cz), np.float64)
    if not starting:
        # the ending form reads keys and values down column j: hold them as [j, h, k, d]
        kj = np.ascontiguousarray(k.transpose(1, 2, 0, 3))
        vj = np.ascontiguousarray(v.transpose(1, 2, 0, 3))
    for r, i in enumerate(rows):
        o = np.empty((n, heads, dh), np.float64)
        for h in range(heads):
            if starting:
                s = (q[i, :, h, :] @ k[i, :, h, :].T) * scale + bias[:, :, h]      # [j, k]
                o[:, h, :] = softmax_rows(s) @ v[i, :, h, :]
            else:
                # s[j, k] = q[i,j,h] . k[k,j,h] / sqrt(d_h) + bias[k,i,h]
                s = np.matmul(kj[:, h], q[i, :, h, :, None])[:, :, 0] * scale + bias[:, i, h][None, :]
                o[:, h, :] = np.matmul(softmax_rows(s)[:, None, :], vj[:, h])[:, 0, :]
        o = (g[i] * o).reshape(n, hd)
        out[r] = z[i] + linear(o, w[p + "w_o"], w[p + "b_o"])
    return out


def pair_transition(z, w, p="pt.", activation="relu", eps=1e-5, rows=None):
    z = np.asarray(z, np.float64)
    rows = _rows(rows, z.shape[0])
    zr = z[rows]
    u = layer_norm(zr, w[p + "ln_g"], w[p + "ln_b"], eps)
    a = ACTIVATIONS[activation](linear(u, w[p + "w_1"], w[p + "b_1"]))
    return zr + linear(a, w[p + "w_2"], w[p + "b_2"])


PAIR_MODULES = ("tmo", "tmi", "tas", "tae", "pt")


def pair_module(name, z, w, heads, activation="relu", eps=1e-5, rows=None):
    if name == "tmo":
        return tri_mul(z, w, "tmo.", True, eps, rows)
    if name == "tmi":
        return tri_mul(z, w, "tmi.", False, eps, rows)
    if name == "tas":
        return tri_att(z, w, "tas.", heads, True, eps, rows)
    if name == "tae":
        return tri_att(z, w, "tae.", heads, False, eps, rows)
    if name == "pt":
        return pair_transition(z, w, "pt.", activation, eps, rows)
    raise ValueError(name)


def pair_block(z, w, heads, activation="relu", eps=1e-5, modules=PAIR_MODULES):
    z = np.asarray(z, np.float64)
    for name in modules:
        z = pair_module(name, z, w, heads, activation, eps)
    return z


def pair_module_chunked(name, z, w, heads, chunk_len, activation="relu", eps=1e-5):
    """The chunk definition (section 2.2) applied to one pair-stack module.

    Output rows i (dim 0) are split into segments computed one after another; each
    segment sees the whole input z, from which it takes its own slice and the
    non-chunkable operands (section 3.1).
    """
    z = np.asarray(z, np.float64)
    n = z.shape[0]
    out = np.empty_like(z)
    for a in range(0, n, chunk_len):
        b = min(n, a + chunk_len)
        out[a:b] = pair_module(name, z, w, heads, activation, eps, rows=np.arange(a, b))
    return out
