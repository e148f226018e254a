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


# What each dimension of a node of transformer_stack_graph is to the executor, by node name:
# (chunk dim, executor units per index).  A head is head_dim features; head_dim and key positions
# are no chunk dims of the executor (section 3.3 excludes them anyway: they are reduced over).
def _transformer_dims(name, head_dim):
    b, s, f, h, no = (B.AC_DIM_BATCH, 1), (B.AC_DIM_SEQ, 1), (B.AC_DIM_FEATURE, 1), (B.AC_DIM_FEATURE, head_dim), (-1, 0)
    if name in ("scores", "scaled", "probs") or name.endswith("_h"):
        return (b, h, s, no)                       # [batch, heads, seq, key | head_dim]
    if name.endswith("_split") or name == "ctx_t":
        return (b, s, h, no)                       # [batch, seq, heads, head_dim]
    return (b, s, f)                               # [batch, seq, feature]


# Node spans of the executor's region kinds within a layer (first node, last node).
_KIND_SPANS = ((B.AC_REGION_QKV, "u", "v_h"), (B.AC_REGION_ATTENTION, "scores", "ctx"),
               (B.AC_REGION_OUT_PROJ, "o", "h"), (B.AC_REGION_FFN, "u2", "y"))


def transformer_stack_tags(names, head_dim):
    """ac_node_tag entries for the nodes of a transformer_stack_graph: which region kind of the executor
    computes a node, in which layer, and what its dims are to the executor.  Data about the graph;
    what is done with it is ac_graph_chunks_to_regions'."""
    tags = [(-1, 0, ())] * len(names)
    for full, idx in names.items():
        prefix, _, last = full.rpartition(".")
        layer = int(prefix[1:]) if prefix else 0
        where = (lambda nm: names.get(f"{prefix}.{nm}" if prefix else nm, -1))
        kind = next((k for k, a, b in _KIND_SPANS if where(a) >= 0 and where(a) <= idx <= where(b)), -1)
        if kind >= 0:
            tags[idx] = (kind, layer, _transformer_dims(last, head_dim))
    return B.node_tags(tags)


def executor_regions(chunks, names, head_dim=1):
    """Region settings for ac_plan_create, [(kind, chunk_dim, chunk_len)], from chunks
    [(start, end, out_dim, chunk_len)] of a transformer_stack_graph (as ac_graph_plan returns
    them).  Raises AcError for a chunk that spans two kinds or layers, that is cut along a dimension
    the executor has no chunk dim for, or when layers disagree on the dimension.  head_dim is needed
    only for chunks along the heads."""
    return B.ac_graph_chunks_to_regions(transformer_stack_tags(names, head_dim), chunks)


# Pair block: the chunked part of each module (what the executor runs per segment; the whole operands of
# a module, a and b, or keys, values and bias, are its non-chunkable inputs and belong to no kind).
_PAIR_PARTS = {
    "tmo": (B.AC_REGION_TRIMUL_OUT, ("gate", "o", "on", "ol", "upd", "z")),
    "tmi": (B.AC_REGION_TRIMUL_IN, ("gate", "o", "on", "ol", "upd", "z")),
    "tas": (B.AC_REGION_TRIATT_START, ("q", "q_split", "q_h", "gate", "scores", "biased", "probs", "ctx_h", "ctx_t", "ctx",
                                        "gated", "o", "z")),
    "tae": (B.AC_REGION_TRIATT_END, ("q", "q_split", "q_h", "gate", "scores", "biased", "probs", "ctx_h", "ctx_t", "ctx",
                                      "gated", "o", "o_t", "z")),
    "pt": (B.AC_REGION_PAIR_TRANSITION, ("u", "t", "act", "down", "z")),
}


def pair_block_tags(names):
    """ac_node_tag entries for a pair_block_graph.  Dim 0 of a module's tensors is the row i of z and the
    dim that holds the other position index its column j - except inside the ending-node attention,
    which the graph writes on the transposed pair tensor: there dim 0 is the column."""
    row, col, no = (B.AC_DIM_ROW, 1), (B.AC_DIM_COL, 1), (-1, 0)
    tags = [(-1, 0, ())] * len(names)
    for full, idx in names.items():
        prefix, _, last = full.rpartition(".")
        if prefix not in _PAIR_PARTS or last not in _PAIR_PARTS[prefix][1]:
            continue
        first, second = (col, row) if prefix == "tae" and last not in ("o_t", "z") else (row, col)
        if last in ("q_h", "scores", "biased", "probs", "ctx_h"):
            dims = (first, no, second, no)            # [i, heads, j, key | head_dim]
        elif last in ("q_split", "ctx_t"):
            dims = (first, second, no, no)            # [i, j, heads, head_dim]
        else:
            dims = (first, second, no)                # [i, j, channels]
        tags[idx] = (_PAIR_PARTS[prefix][0], 0, dims)
    return B.node_tags(tags)


def pair_executor_regions(chunks, names):
    """As executor_regions, for chunks of a pair_block_graph."""
    return B.ac_graph_chunks_to_regions(pair_block_tags(names), chunks)


def unet_stage_tags(names):
    """ac_node_tag entries for a unet_stage_graph.  The executor runs its residual block (nodes "res.*") and its
    spatial transformer ("tr.*": group norm, convolution in, self-attention, cross-attention to the context, gated
    feed-forward, convolution out, skip) as the attention block.  Every tensor of both has the batch as its first
    dim, and the batch is the only dim the executor cuts them along."""
    tags = [(-1, 0, ())] * len(names)
    batch_only = ((B.AC_DIM_BATCH, 1), (-1, 0), (-1, 0), (-1, 0))
    params = {"ln_g", "ln_b", "wq", "wk", "wv", "wo", "bo", "w1", "b1", "w2", "b2", "gn_g", "gn_b", "w_in", "b_in", "w_out", "b_out"}
    for full, idx in names.items():
        prefix, _, last = full.rpartition(".")
        if prefix == "res" and last in ("n1", "a1", "c1", "t", "n2", "a2", "c2", "y"):
            tags[idx] = (B.AC_REGION_RES_BLOCK, 0, batch_only)
        elif full.startswith("tr.") and last not in params:
            tags[idx] = (B.AC_REGION_UNET_ATTN, 0, batch_only)
    return B.node_tags(tags)


def pair_block_graph(n_res, c_z, c_hidden, heads, head_dim, transition_factor):
    """One pair-stack block on z [n_res, n_res, c_z] as an unfused graph: triangle
    multiplicative update (outgoing "tmo", incoming "tmi"), triangle self-attention around the
    starting ("tas") and ending ("tae") node, pair transition ("pt"); node names carry the
    module's prefix.  The ending-node attention is the starting-node one on the transposed
    pair tensor, transposed back.  Returns (spec, names)."""
    g = GraphBuilder()
    n, c, ch, hd = n_res, c_z, c_hidden, heads * head_dim
    nnc = (n, n, c)
    g.add("z", B.AC_OP_INPUT, shape=nnc)

    def param(name, *shape):
        return g.add(name, B.AC_OP_PARAM, shape=shape)

    for p in ("tmo.", "tmi."):
        for nm in ("ln_in_g", "ln_in_b"):
            param(p + nm, c)
        for nm in ("ag", "ap", "bg", "bp"):
            param(p + "w_" + nm, ch, c)
            param(p + "b_" + nm, ch)
        param(p + "w_g", c, c), param(p + "b_g", c)
        param(p + "ln_out_g", ch), param(p + "ln_out_b", ch)
        param(p + "w_o", c, ch), param(p + "b_o", c)
    for p in ("tas.", "tae."):
        param(p + "ln_g", c), param(p + "ln_b", c)
        for nm in ("q", "k", "v"):
            param(p + "w_" + nm, hd, c)
        param(p + "w_bias", heads, c)
        param(p + "w_g", hd, c), param(p + "b_g", hd)
        param(p + "w_o", c, hd), param(p + "b_o", c)
    param("pt.ln_g", c), param("pt.ln_b", c)
    param("pt.w_1", transition_factor * c, c), param("pt.b_1", transition_factor * c)
    param("pt.w_2", c, transition_factor * c), param("pt.b_2", c)

    src = "z"
    for p, outgoing in (("tmo.", True), ("tmi.", False)):
        g.add(p + "t", B.AC_OP_NORM_LAST, (src, p + "ln_in_g", p + "ln_in_b"), nnc)
        for x in "ab":
            g.add(p + x + "_gate", B.AC_OP_LINEAR, (p + "t", p + f"w_{x}g", p + f"b_{x}g"), (n, n, ch))
            g.add(p + x + "_proj", B.AC_OP_LINEAR, (p + "t", p + f"w_{x}p", p + f"b_{x}p"), (n, n, ch))
            g.add(p + x, B.AC_OP_ELEMENTWISE, (p + x + "_gate", p + x + "_proj"), (n, n, ch))
            if not outgoing:     # o[i,j,c] = sum_k a[k,i,c] b[k,j,c]: bring the summed index to the middle
                g.add(p + x + "_t", B.AC_OP_TRANSPOSE, (p + x,), (n, n, ch), (1, 0, 2))
        ops = (p + "a", p + "b") if outgoing else (p + "a_t", p + "b_t")
        g.add(p + "o", B.AC_OP_CONTRACT_IKC_JKC, ops, (n, n, ch))
        g.add(p + "gate", B.AC_OP_LINEAR, (p + "t", p + "w_g", p + "b_g"), nnc)
        g.add(p + "on", B.AC_OP_NORM_LAST, (p + "o", p + "ln_out_g", p + "ln_out_b"), (n, n, ch))
        g.add(p + "ol", B.AC_OP_LINEAR, (p + "on", p + "w_o", p + "b_o"), nnc)
        g.add(p + "upd", B.AC_OP_ELEMENTWISE, (p + "gate", p + "ol"), nnc)
        src = g.add(p + "z", B.AC_OP_ELEMENTWISE, (src, p + "upd"), nnc)
    for p, starting in (("tas.", True), ("tae.", False)):
        zin = src if starting else g.add(p + "zt", B.AC_OP_TRANSPOSE, (src,), nnc, (1, 0, 2))
        g.add(p + "t", B.AC_OP_NORM_LAST, (zin, p + "ln_g", p + "ln_b"), nnc)
        for x in "qkv":
            g.add(p + x, B.AC_OP_LINEAR, (p + "t", p + "w_" + x), (n, n, hd))
            g.add(p + x + "_split", B.AC_OP_SPLIT_DIM, (p + x,), (n, n, heads, head_dim), (2, heads))
            g.add(p + x + "_h", B.AC_OP_TRANSPOSE, (p + x + "_split",), (n, heads, n, head_dim), (0, 2, 1, 3))
        g.add(p + "bias", B.AC_OP_LINEAR, (p + "t", p + "w_bias"), (n, n, heads))
        g.add(p + "bias_t", B.AC_OP_TRANSPOSE, (p + "bias",), (heads, n, n), (2, 0, 1))
        g.add(p + "gate", B.AC_OP_LINEAR, (p + "t", p + "w_g", p + "b_g"), (n, n, hd))
        g.add(p + "scores", B.AC_OP_MATMUL_NT, (p + "q_h", p + "k_h"), (n, heads, n, n))
        g.add(p + "biased", B.AC_OP_ELEMENTWISE, (p + "scores", p + "bias_t"), (n, heads, n, n))
        g.add(p + "probs", B.AC_OP_SOFTMAX_LAST, (p + "biased",), (n, heads, n, n))
        g.add(p + "ctx_h", B.AC_OP_MATMUL_NN, (p + "probs", p + "v_h"), (n, heads, n, head_dim))
        g.add(p + "ctx_t", B.AC_OP_TRANSPOSE, (p + "ctx_h",), (n, n, heads, head_dim), (0, 2, 1, 3))
        g.add(p + "ctx", B.AC_OP_MERGE_DIMS, (p + "ctx_t",), (n, n, hd), (2, head_dim))
        g.add(p + "gated", B.AC_OP_ELEMENTWISE, (p + "gate", p + "ctx"), (n, n, hd))
        g.add(p + "o", B.AC_OP_LINEAR, (p + "gated", p + "w_o", p + "b_o"), nnc)
        upd = p + "o" if starting else g.add(p + "o_t", B.AC_OP_TRANSPOSE, (p + "o",), nnc, (1, 0, 2))
        src = g.add(p + "z", B.AC_OP_ELEMENTWISE, (src, upd), nnc)
    g.add("pt.u", B.AC_OP_NORM_LAST, (src, "pt.ln_g", "pt.ln_b"), nnc)
    g.add("pt.t", B.AC_OP_LINEAR, ("pt.u", "pt.w_1", "pt.b_1"), (n, n, transition_factor * c))
    g.add("pt.act", B.AC_OP_ELEMENTWISE, ("pt.t",), (n, n, transition_factor * c))
    g.add("pt.down", B.AC_OP_LINEAR, ("pt.act", "pt.w_2", "pt.b_2"), nnc)
    g.add("pt.z", B.AC_OP_ELEMENTWISE, (src, "pt.down"), nnc)
    return g.spec, g.names


def unet_stage_graph(batch, channels, height, width, heads, context_tokens, context_dim, groups=32):
    """One stage of a latent-diffusion UNet at a fixed resolution, as an unfused graph: a residual
    block (group norm, SiLU, 3x3 convolution, time embedding added, again, skip) and a spatial
    transformer (group norm, 1x1 convolution in, tokens [B, H*W, C]: self-attention,
    cross-attention to a context [B, T, D], gated feed-forward, each behind a layer norm and
    with a residual; 1x1 convolution out, skip).  Prefixes: "res." and "tr.".  Returns (spec, names)."""
    g = GraphBuilder()
    b, c, hh, ww = batch, channels, height, width
    n, dh = hh * ww, channels // heads
    img, tok = (b, c, hh, ww), (b, n, c)
    g.add("x", B.AC_OP_INPUT, shape=img)
    g.add("temb", B.AC_OP_INPUT, shape=(b, c, 1, 1))
    g.add("context", B.AC_OP_INPUT, shape=(b, context_tokens, context_dim))

    def param(name, *shape):
        return g.add(name, B.AC_OP_PARAM, shape=shape)

    for i in (1, 2):
        param(f"res.gn{i}_g", c), param(f"res.gn{i}_b", c), param(f"res.w{i}", c, c, 3, 3), param(f"res.b{i}", c)
    param("tr.gn_g", c), param("tr.gn_b", c), param("tr.w_in", c, c, 1, 1), param("tr.b_in", c)
    for a, kv_dim in (("sa", c), ("ca", context_dim)):
        param(f"tr.{a}.ln_g", c), param(f"tr.{a}.ln_b", c), param(f"tr.{a}.wq", c, c)
        param(f"tr.{a}.wk", c, kv_dim), param(f"tr.{a}.wv", c, kv_dim), param(f"tr.{a}.wo", c, c), param(f"tr.{a}.bo", c)
    param("tr.ff.ln_g", c), param("tr.ff.ln_b", c), param("tr.ff.w1", 8 * c, c), param("tr.ff.b1", 8 * c)
    param("tr.ff.w2", c, 4 * c), param("tr.ff.b2", c)
    param("tr.w_out", c, c, 1, 1), param("tr.b_out", c)

    # residual block
    g.add("res.n1", B.AC_OP_GROUP_NORM, ("x", "res.gn1_g", "res.gn1_b"), img, (groups,))
    g.add("res.a1", B.AC_OP_ELEMENTWISE, ("res.n1",), img)
    g.add("res.c1", B.AC_OP_CONV2D, ("res.a1", "res.w1", "res.b1"), img)
    g.add("res.t", B.AC_OP_ELEMENTWISE, ("res.c1", "temb"), img)
    g.add("res.n2", B.AC_OP_GROUP_NORM, ("res.t", "res.gn2_g", "res.gn2_b"), img, (groups,))
    g.add("res.a2", B.AC_OP_ELEMENTWISE, ("res.n2",), img)
    g.add("res.c2", B.AC_OP_CONV2D, ("res.a2", "res.w2", "res.b2"), img)
    g.add("res.y", B.AC_OP_ELEMENTWISE, ("x", "res.c2"), img)
    # spatial transformer: image -> tokens
    g.add("tr.n", B.AC_OP_GROUP_NORM, ("res.y", "tr.gn_g", "tr.gn_b"), img, (groups,))
    g.add("tr.in", B.AC_OP_CONV2D, ("tr.n", "tr.w_in", "tr.b_in"), img)
    g.add("tr.flat", B.AC_OP_MERGE_DIMS, ("tr.in",), (b, c, n), (2, ww))
    src = g.add("tr.tok", B.AC_OP_TRANSPOSE, ("tr.flat",), tok, (0, 2, 1))
    for a, kv_src, kv_len in (("sa", None, n), ("ca", "context", context_tokens)):
        p = f"tr.{a}."
        g.add(p + "u", B.AC_OP_NORM_LAST, (src, p + "ln_g", p + "ln_b"), tok)
        kv = kv_src or p + "u"
        for t, inp, w, length in (("q", p + "u", "wq", n), ("k", kv, "wk", kv_len), ("v", kv, "wv", kv_len)):
            g.add(p + t, B.AC_OP_LINEAR, (inp, p + w), (b, length, c))
            g.add(p + t + "_split", B.AC_OP_SPLIT_DIM, (p + t,), (b, length, heads, dh), (2, heads))
            g.add(p + t + "_h", B.AC_OP_TRANSPOSE, (p + t + "_split",), (b, heads, length, dh), (0, 2, 1, 3))
        g.add(p + "scores", B.AC_OP_MATMUL_NT, (p + "q_h", p + "k_h"), (b, heads, n, kv_len))
        g.add(p + "scaled", B.AC_OP_ELEMENTWISE, (p + "scores",), (b, heads, n, kv_len))
        g.add(p + "probs", B.AC_OP_SOFTMAX_LAST, (p + "scaled",), (b, heads, n, kv_len))
        g.add(p + "ctx_h", B.AC_OP_MATMUL_NN, (p + "probs", p + "v_h"), (b, heads, n, dh))
        g.add(p + "ctx_t", B.AC_OP_TRANSPOSE, (p + "ctx_h",), (b, n, heads, dh), (0, 2, 1, 3))
        g.add(p + "ctx", B.AC_OP_MERGE_DIMS, (p + "ctx_t",), tok, (2, dh))
        g.add(p + "o", B.AC_OP_LINEAR, (p + "ctx", p + "wo", p + "bo"), tok)
        src = g.add(p + "h", B.AC_OP_ELEMENTWISE, (src, p + "o"), tok)
    g.add("tr.ff.u", B.AC_OP_NORM_LAST, (src, "tr.ff.ln_g", "tr.ff.ln_b"), tok)
    g.add("tr.ff.t", B.AC_OP_LINEAR, ("tr.ff.u", "tr.ff.w1", "tr.ff.b1"), (b, n, 8 * c))
    g.add("tr.ff.val", B.AC_OP_SLICE_LAST, ("tr.ff.t",), (b, n, 4 * c), (0, 4 * c))
    g.add("tr.ff.gate", B.AC_OP_SLICE_LAST, ("tr.ff.t",), (b, n, 4 * c), (4 * c, 8 * c))
    g.add("tr.ff.act", B.AC_OP_ELEMENTWISE, ("tr.ff.val", "tr.ff.gate"), (b, n, 4 * c))
    g.add("tr.ff.down", B.AC_OP_LINEAR, ("tr.ff.act", "tr.ff.w2", "tr.ff.b2"), tok)
    g.add("tr.ff.h", B.AC_OP_ELEMENTWISE, (src, "tr.ff.down"), tok)
    # tokens -> image
    g.add("tr.back", B.AC_OP_TRANSPOSE, ("tr.ff.h",), (b, c, n), (0, 2, 1))
    g.add("tr.img", B.AC_OP_SPLIT_DIM, ("tr.back",), img, (2, hh))
    g.add("tr.out", B.AC_OP_CONV2D, ("tr.img", "tr.w_out", "tr.b_out"), img)
    g.add("tr.y", B.AC_OP_ELEMENTWISE, ("res.y", "tr.out"), img)
    return g.spec, g.names
