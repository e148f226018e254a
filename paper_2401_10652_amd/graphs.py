"""Op graphs of the workloads in the form ac_chunk_search takes: lists of
(op, inputs, shape, attr) tuples, leaves first within each layer's parameters.  Data only."""
from __future__ import annotations

from . import binding as B


class GraphBuilder:
    def __init__(self):
        self.spec = []
        self.names = {}

    def add(self, name, op, inputs=(), shape=(), attr=()):
        self.spec.append((op, tuple(self.names[i] for i in inputs), tuple(shape), tuple(attr)))
        self.names[name] = len(self.spec) - 1
        return name


def transformer_stack_graph(batch, seq, d_model, heads, d_ffn, layers=1):
    """Pre-LN decoder/encoder stack on x [batch, seq, d_model] as the unfused graph of AutoChunk
    section 2.1 (scores, probabilities and head views are nodes of their own).  Returns
    (spec, names); names of layer l carry the prefix "l<l>." except for layer 0."""
    g = GraphBuilder()
    dh = d_model // heads
    g.add("x", B.AC_OP_INPUT, shape=(batch, seq, d_model))
    params = (("g1", (d_model,)), ("b1", (d_model,)), ("wqkv", (3 * d_model, d_model)), ("bqkv", (3 * d_model,)),
              ("wo", (d_model, d_model)), ("bo", (d_model,)), ("g2", (d_model,)), ("b2", (d_model,)),
              ("w1", (d_ffn, d_model)), ("bf1", (d_ffn,)), ("w2", (d_model, d_ffn)), ("bf2", (d_model,)))
    for layer in range(layers):
        for nm, shp in params:
            g.add(f"l{layer}.{nm}" if layer else nm, B.AC_OP_PARAM, shape=shp)
    src = "x"
    for layer in range(layers):
        def n(s, layer=layer):
            return f"l{layer}.{s}" if layer else s
        bsd, bhsd = (batch, seq, d_model), (batch, heads, seq, dh)
        g.add(n("u"), B.AC_OP_NORM_LAST, (src, n("g1"), n("b1")), bsd)
        g.add(n("qkv"), B.AC_OP_LINEAR, (n("u"), n("wqkv"), n("bqkv")), (batch, seq, 3 * d_model))
        for i, t in enumerate("qkv"):
            g.add(n(t + "_flat"), B.AC_OP_SLICE_LAST, (n("qkv"),), bsd, (i * d_model, (i + 1) * d_model))
            g.add(n(t + "_split"), B.AC_OP_SPLIT_DIM, (n(t + "_flat"),), (batch, seq, heads, dh), (2, heads))
            g.add(n(t + "_h"), B.AC_OP_TRANSPOSE, (n(t + "_split"),), bhsd, (0, 2, 1, 3))
        g.add(n("scores"), B.AC_OP_MATMUL_NT, (n("q_h"), n("k_h")), (batch, heads, seq, seq))
        g.add(n("scaled"), B.AC_OP_ELEMENTWISE, (n("scores"),), (batch, heads, seq, seq))
        g.add(n("probs"), B.AC_OP_SOFTMAX_LAST, (n("scaled"),), (batch, heads, seq, seq))
        g.add(n("ctx_h"), B.AC_OP_MATMUL_NN, (n("probs"), n("v_h")), bhsd)
        g.add(n("ctx_t"), B.AC_OP_TRANSPOSE, (n("ctx_h"),), (batch, seq, heads, dh), (0, 2, 1, 3))
        g.add(n("ctx"), B.AC_OP_MERGE_DIMS, (n("ctx_t"),), bsd, (2, dh))
        g.add(n("o"), B.AC_OP_LINEAR, (n("ctx"), n("wo"), n("bo")), bsd)
        g.add(n("h"), B.AC_OP_ELEMENTWISE, (src, n("o")), bsd)
        g.add(n("u2"), B.AC_OP_NORM_LAST, (n("h"), n("g2"), n("b2")), bsd)
        g.add(n("t"), B.AC_OP_LINEAR, (n("u2"), n("w1"), n("bf1")), (batch, seq, d_ffn))
        g.add(n("act"), B.AC_OP_ELEMENTWISE, (n("t"),), (batch, seq, d_ffn))
        g.add(n("down"), B.AC_OP_LINEAR, (n("act"), n("w2"), n("bf2")), bsd)
        src = g.add(n("y"), B.AC_OP_ELEMENTWISE, (n("h"), n("down")), bsd)
    return g.spec, g.names
