"""Activation-memory model of the paper, written out per region.  Test infrastructure.

AutoChunk, section 2.1, first activation equation: a module Y = F(X) holds
M = mem(X) + mem(Y) + mem(A), with A the intermediate activations.  Section 2.2,
second activation equation: split into n segments it holds
M = mem(X) + mem(Y) + mem(A)/n.  Both are plain sums (no liveness analysis), and
weights are not activations (section 1).

The regions are written as an unfused graph would hold them (the paper's baseline
is stock PyTorch, section 4): every op output is its own tensor in the storage
dtype.  With b = bytes per element, c = rows per segment (the largest segment
when the length does not divide), n = ceil(D / c):

  qkv projection   X = x[S,d]               A = u[S,d]                      Y = qkv[S,3d]
  attention core   X = x[S,d] + qkv[S,3d]   A = scores[H,S,S] + probs[H,S,S] Y = ctx[S,d]
  output proj.     X = x[S,d] + ctx[S,d]    A = o[S,d] (before the residual) Y = h[S,d]
  feed-forward     X = h[S,d]               A = u[S,d] + t[S,F] + act[S,F]  Y = y[S,d]
  tri-mul          X = z + a,b[N,N,ch]*2    A = t + g + o[N,N,ch] + LN(o)    Y = z'
  tri-attention    X = z + k,v[N,N,H*dh]*2 + bias[H,N,N]
                   A = t + q + g + scores[N,H,N,N] + o[N,N,H*dh]            Y = z'
  transition       X = z                    A = u + hidden*2                Y = z'

The functions return bytes.  "A/n" is evaluated as A with the chunked extent D
replaced by c, which equals A/n when c divides D.
"""
from __future__ import annotations


def ceil_div(a, b):
    return -(-a // b)


def _rows(seq, chunk_len):
    return seq if not chunk_len or chunk_len >= seq else chunk_len


def qkv_region(seq, d, b, chunk_len=0):
    c = _rows(seq, chunk_len)
    return seq * d * b + 3 * seq * d * b + c * d * b


def attention_region(seq, d, heads, b, chunk_len=0):
    """x + qkv + ctx whole; scores and probabilities for the rows of one segment."""
    c = _rows(seq, chunk_len)
    x = seq * d * b
    qkv = 3 * seq * d * b
    ctx = seq * d * b
    a = 2 * heads * c * seq * b
    return x + qkv + ctx + a


def out_proj_region(seq, d, b, chunk_len=0):
    c = _rows(seq, chunk_len)
    return 3 * seq * d * b + c * d * b


def ffn_region(seq, d, f, b, chunk_len=0):
    c = _rows(seq, chunk_len)
    return 2 * seq * d * b + c * d * b + 2 * c * f * b


def transformer_layer_peak(seq, d, heads, f, b, c_qkv=0, c_attn=0, c_ffn=0, c_out=0):
    """Regions run one after another, so a layer's peak is the largest region sum."""
    return max(qkv_region(seq, d, b, c_qkv),
               attention_region(seq, d, heads, b, c_attn),
               out_proj_region(seq, d, b, c_out),
               ffn_region(seq, d, f, b, c_ffn))


def tri_att_region(n, cz, heads, dh, b, chunk_len=0):
    """z, z', k, v, bias whole; t, q, g, scores, o for the rows of one segment."""
    c = _rows(n, chunk_len)
    hd = heads * dh
    whole = 2 * n * n * cz * b + 2 * n * n * hd * b + heads * n * n * b
    seg = c * n * cz * b + 3 * c * n * hd * b + c * heads * n * n * b
    return whole + seg


def tri_mul_region(n, cz, ch, b, chunk_len=0):
    """z, z', a, b whole (both contraction operands); t, g, o, LN(o) per segment."""
    c = _rows(n, chunk_len)
    whole = 2 * n * n * cz * b + 2 * n * n * ch * b
    seg = 2 * c * n * cz * b + 2 * c * n * ch * b
    return whole + seg


def pair_transition_region(n, cz, factor, b, chunk_len=0):
    c = _rows(n, chunk_len)
    return 2 * n * n * cz * b + c * n * cz * b + 2 * c * n * factor * cz * b


def largest_chunk_len(extent, granule, fits):
    """Largest c that is `extent` itself or a multiple of `granule` below it with
    fits(c) true; 0 if none.  The number of segments is then ceil(extent / c)."""
    if fits(extent):
        return extent
    c = ((extent - 1) // granule) * granule
    while c >= granule:
        if fits(c):
            return c
        c -= granule
    return 0
