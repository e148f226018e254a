"""fp64 CPU oracle: unchunked pre-LN transformer block and stack.  Test infrastructure.

The paper (AutoChunk, section 2.2 and section 4) names attention and feed-forward
modules of GPT (prefill) and ViT models without defining them; the reading taken
here is the standard pre-LN block:

    u   = LN(x; g1, b1)                      rows over d_model, biased variance
    q,k,v = u Wq^T + bq, u Wk^T + bk, u Wv^T + bv
    s_h[i,j] = q_h[i] . k_h[j] / sqrt(d_h)   all j (non-causal) or j <= i (causal)
    p_h[i,:] = softmax_j s_h[i,:]            masked j excluded from the sum
    ctx[i]   = concat_h sum_j p_h[i,j] v_h[j]
    h   = x + ctx Wo^T + bo
    y   = h + act(LN(h; g2, b2) W1^T + b1) W2^T + b2

Every weight matrix is [out_features, in_features].  All arithmetic is fp64 and
nothing is blocked, fused or reordered, except that attention may be evaluated
one block of query rows at a time (``query_block``) so that the score matrix of
a long sequence need not exist at once; that changes no value of any row.

The ``*_chunked`` functions restate the chunk definition of section 2.2
(split the input along the chunk dimension into segments, apply the module to
each, concatenate) on the CPU; tests use them to show chunked == unchunked for
legal chunk dimensions and a mismatch for illegal ones (section 3.3, rules 1-4).
"""
from __future__ import annotations

import math

import numpy as np
from scipy.special import erf as _erf


def layer_norm(x, gain, shift, eps=1e-5):
    """Rows of x normalised over the last dim with the biased variance."""
    x = np.asarray(x, np.float64)
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    return (x - mu) / np.sqrt(var + eps) * np.asarray(gain, np.float64) + np.asarray(shift, np.float64)


def gelu_erf(x):
    x = np.asarray(x, np.float64)
    return 0.5 * x * (1.0 + _erf(x / math.sqrt(2.0)))


def gelu_tanh(x):
    x = np.asarray(x, np.float64)
    return 0.5 * x * (1.0 + np.tanh(math.sqrt(2.0 / math.pi) * (x + 0.044715 * x ** 3)))


def relu(x):
    return np.maximum(np.asarray(x, np.float64), 0.0)


ACTIVATIONS = {"gelu_erf": gelu_erf, "gelu_tanh": gelu_tanh, "relu": relu}


def linear(x, w, b=None):
    """x [.., in] times w[out, in]^T plus b[out]."""
    y = np.asarray(x, np.float64) @ np.asarray(w, np.float64).T
    if b is not None:
        y = y + np.asarray(b, np.float64)
    return y


def softmax_rows(s):
    """Softmax over the last dim; entries equal to -inf get weight exactly 0."""
    m = s.max(axis=-1, keepdims=True)
    e = np.exp(s - m)
    return e / e.sum(axis=-1, keepdims=True)


def attention(q, k, v, heads, causal, bias=None, query_block=None, q_offset=0):
    """Multi-head scaled dot-product attention for one sequence.

    q [Sq, heads*d_h]; k, v [Sk, heads*d_h]; bias None or [heads, Sq, Sk].
    Query row i stands at absolute position q_offset + i for the causal mask
    (keys j <= q_offset + i are visible).  Returns ctx [Sq, heads*d_h].
    """
    q = np.asarray(q, np.float64)
    k = np.asarray(k, np.float64)
    v = np.asarray(v, np.float64)
    sq, hd = q.shape
    sk = k.shape[0]
    dh = hd // heads
    scale = 1.0 / math.sqrt(dh)
    out = np.empty((sq, hd), np.float64)
    qb = sq if not query_block else int(query_block)
    kpos = np.arange(sk)
    for h in range(heads):
        c = slice(h * dh, (h + 1) * dh)
        for r0 in range(0, sq, qb):
            r1 = min(sq, r0 + qb)
            s = (q[r0:r1, c] @ k[:, c].T) * scale
            if bias is not None:
                s = s + np.asarray(bias[h, r0:r1, :], np.float64)
            if causal:
                qpos = q_offset + np.arange(r0, r1)
                s = np.where(kpos[None, :] <= qpos[:, None], s, -np.inf)
            out[r0:r1, c] = softmax_rows(s) @ v[:, c]
    return out


def attention_region(x, w, heads, causal, eps=1e-5, query_block=None):
    """h = x + attention(LN1(x)) Wo^T + bo for one sequence x [S, d]."""
    d = x.shape[1]
    u = layer_norm(x, w["ln1_g"], w["ln1_b"], eps)
    qkv = linear(u, w["w_qkv"], w["b_qkv"])
    ctx = attention(qkv[:, :d], qkv[:, d:2 * d], qkv[:, 2 * d:], heads, causal,
                    query_block=query_block)
    return np.asarray(x, np.float64) + linear(ctx, w["w_o"], w["b_o"])


def ffn_region(h, w, activation="gelu_erf", eps=1e-5):
    """y = h + act(LN2(h) W1^T + b1) W2^T + b2."""
    u = layer_norm(h, w["ln2_g"], w["ln2_b"], eps)
    a = ACTIVATIONS[activation](linear(u, w["w_1"], w["b_1"]))
    return np.asarray(h, np.float64) + linear(a, w["w_2"], w["b_2"])


def transformer_block(x, w, heads, causal, activation="gelu_erf", eps=1e-5, batch=1,
                      query_block=None):
    """One pre-LN block on x [batch*seq, d]; attention is per batch element."""
    x = np.asarray(x, np.float64)
    t = x.shape[0]
    s = t // batch
    h = np.empty_like(x)
    for b in range(batch):
        r = slice(b * s, (b + 1) * s)
        h[r] = attention_region(x[r], w, heads, causal, eps, query_block)
    return ffn_region(h, w, activation, eps)


def transformer_block_row_blocks(x, w, heads, causal, blocks, activation="gelu_erf", eps=1e-5):
    """Rows [r0, r1) of transformer_block(x), for every (r0, r1) of ``blocks``, one sequence.

    Keys and values come from every row of x (they are what every query sees) and are
    computed once; queries, output projection, residuals and feed-forward are evaluated
    for the requested rows only.  Lets a test check some rows of a sequence too long to
    evaluate whole.  Returns a list of arrays, one per block.
    """
    x = np.asarray(x, np.float64)
    d = x.shape[1]
    u = layer_norm(x, w["ln1_g"], w["ln1_b"], eps)
    wq = np.asarray(w["w_qkv"], np.float64)
    bq = np.asarray(w["b_qkv"], np.float64)
    k = linear(u, wq[d:2 * d], bq[d:2 * d])
    v = linear(u, wq[2 * d:], bq[2 * d:])
    out = []
    for r0, r1 in blocks:
        q = linear(u[r0:r1], wq[:d], bq[:d])
        ctx = attention(q, k, v, heads, causal, q_offset=r0)
        h = x[r0:r1] + linear(ctx, w["w_o"], w["b_o"])
        out.append(ffn_region(h, w, activation, eps))
    return out


def transformer_block_rows(x, w, heads, causal, r0, r1, activation="gelu_erf", eps=1e-5):
    """Rows [r0, r1) of transformer_block(x) for one sequence, without forming the other rows."""
    return transformer_block_row_blocks(x, w, heads, causal, [(r0, r1)], activation, eps)[0]


def transformer_stack(x, layers, heads, causal, activation="gelu_erf", eps=1e-5, batch=1,
                      query_block=None):
    y = np.asarray(x, np.float64)
    for w in layers:
        y = transformer_block(y, w, heads, causal, activation, eps, batch, query_block)
    return y


# --------------------------------------------------------------------------------------
# The chunk definition (section 2.2) restated on the CPU, for the invariance tests.
# --------------------------------------------------------------------------------------

def _segments(n, length):
    return [(a, min(n, a + length)) for a in range(0, n, length)]


def transformer_block_chunked(x, w, heads, causal, chunk_len_qkv, chunk_len_attn, chunk_len_ffn,
                              activation="gelu_erf", eps=1e-5):
    """One block on a single sequence, three regions each chunked along the sequence.

    Region 1 (LN1 + QKV projection) writes whole q, k, v segment by segment; region 2
    (attention on a query segment with whole k, v, then output projection and
    residual) and region 3 (LN2 + feed-forward + residual) write their slice of the
    output.  k and v are the non-chunkable inputs of region 2 (section 3.1).
    """
    x = np.asarray(x, np.float64)
    s, d = x.shape
    qkv = np.empty((s, 3 * d), np.float64)
    for a, b in _segments(s, chunk_len_qkv):
        qkv[a:b] = linear(layer_norm(x[a:b], w["ln1_g"], w["ln1_b"], eps), w["w_qkv"], w["b_qkv"])
    h = np.empty_like(x)
    for a, b in _segments(s, chunk_len_attn):
        ctx = attention(qkv[a:b, :d], qkv[:, d:2 * d], qkv[:, 2 * d:], heads, causal, q_offset=a)
        h[a:b] = x[a:b] + linear(ctx, w["w_o"], w["b_o"])
    y = np.empty_like(x)
    for a, b in _segments(s, chunk_len_ffn):
        y[a:b] = ffn_region(h[a:b], w, activation, eps)
    return y


def attention_chunked_over_keys(q, k, v, heads, chunk_len):
    """ILLEGAL chunk: splitting the key dimension and concatenating nothing sensible.

    Each segment of keys yields a full-size context; the only way to "concatenate"
    such outputs is to pick one per row, here the last segment's.  Used by a test to
    show that chunking a reduced dimension changes the output (rule 2 is violated).
    """
    out = None
    for a, b in _segments(k.shape[0], chunk_len):
        out = attention(q, k[a:b], v[a:b], heads, causal=False)
    return out


def ffn_chunked_over_hidden(h, w, chunk_len, activation="gelu_erf", eps=1e-5):
    """ILLEGAL chunk: splitting the hidden width of the feed-forward.

    Segments of the hidden dim give partial sums of the down projection, which add
    rather than concatenate; concatenation along any output dim cannot rebuild y.
    Returns the per-segment partial outputs so a test can show none equals y.
    """
    u = layer_norm(h, w["ln2_g"], w["ln2_b"], eps)
    f = np.asarray(w["w_1"]).shape[0]
    parts = []
    for a, b in _segments(f, chunk_len):
        act = ACTIVATIONS[activation](linear(u, w["w_1"][a:b], w["b_1"][a:b]))
        parts.append(act @ np.asarray(w["w_2"], np.float64)[:, a:b].T)
    return parts
