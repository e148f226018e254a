"""ctypes binding of libautochunk_rt.so: argument marshalling only.

Every function here has the name of the C entry point it calls (``ac_*``); tensors are
torch tensors used purely as device buffers (``data_ptr()``), and the stream handed to
the library is torch's current stream.  Nothing is computed in Python, and there is no
fallback: if the shared library has not been built, ``lib()`` raises.
"""
from __future__ import annotations

import ctypes as C
import os

from .build import LIB_PATH

AC_OK = 0
AC_ERR_ARG, AC_ERR_ILLEGAL_CHUNK_DIM, AC_ERR_BUDGET_INFEASIBLE, AC_ERR_WORKSPACE = -1, -2, -3, -4
AC_ERR_ALIGN, AC_ERR_HIP, AC_ERR_STATE, AC_ERR_UNSUPPORTED = -5, -6, -7, -8
AC_TRANSFORMER_STACK, AC_PAIR_STACK, AC_UNET_RES_STACK = 0, 1, 2
AC_F32, AC_BF16 = 0, 1
AC_ACT_NONE, AC_ACT_GELU_ERF, AC_ACT_GELU_TANH, AC_ACT_RELU, AC_ACT_SIGMOID, AC_ACT_SILU = 0, 1, 2, 3, 4, 5
(AC_REGION_QKV, AC_REGION_ATTENTION, AC_REGION_OUT_PROJ, AC_REGION_FFN, AC_REGION_TRIMUL_OUT,
 AC_REGION_TRIMUL_IN, AC_REGION_TRIATT_START, AC_REGION_TRIATT_END, AC_REGION_PAIR_TRANSITION,
 AC_REGION_RES_BLOCK, AC_REGION_UNET_ATTN, AC_REGION_KINDS) = range(12)
AC_DIM_BATCH, AC_DIM_SEQ, AC_DIM_FEATURE, AC_DIM_HEAD_DIM, AC_DIM_KEY = range(5)
AC_DIM_ROW, AC_DIM_COL, AC_DIM_CHANNEL, AC_DIM_CONTRACT = range(4)
AC_FLAG_UNFUSED_ELEMENTWISE = 1
AC_FLAG_LISTED_REGIONS_ONLY = 2
AC_FLAG_TWO_SEGMENTS_IN_FLIGHT = 4
AC_FLAG_MATERIALIZED_SCORES = 8
AC_FLAG_BUDGET_PAPER_MODEL = 16
AC_FLAG_GATED_FFN = 32

ACTIVATIONS = {"none": AC_ACT_NONE, "gelu_erf": AC_ACT_GELU_ERF, "gelu_tanh": AC_ACT_GELU_TANH,
               "relu": AC_ACT_RELU, "sigmoid": AC_ACT_SIGMOID}
DTYPES = {"f32": AC_F32, "bf16": AC_BF16}


class ac_model_desc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in (
        "workload", "dtype", "layers", "batch", "seq", "d_model", "heads", "head_dim", "d_ffn",
        "causal", "activation", "n_res", "c_z", "c_hidden", "tri_heads", "tri_head_dim",
        "transition_factor", "flags")] + [("ln_eps", C.c_float)] + [(n, C.c_int32) for n in (
        "img_h", "img_w", "channels", "groups")]


class ac_region_desc(C.Structure):
    _fields_ = [("kind", C.c_int32), ("chunk_dim", C.c_int32), ("chunk_len", C.c_int64)]


class ac_region_info(C.Structure):
    _fields_ = [("kind", C.c_int32), ("chunk_dim", C.c_int32), ("extent", C.c_int64),
                ("chunk_len", C.c_int64), ("n_segments", C.c_int64), ("launches", C.c_int64),
                ("model_bytes", C.c_uint64),
                ("model_bytes_unchunked", C.c_uint64)]


class ac_plan_info(C.Structure):
    _fields_ = [("workspace_bytes", C.c_uint64), ("io_bytes", C.c_uint64),
                ("peak_bytes_planned", C.c_uint64), ("peak_bytes_unchunked_planned", C.c_uint64),
                ("peak_bytes_model", C.c_uint64), ("peak_bytes_model_unchunked", C.c_uint64),
                ("weight_bytes", C.c_uint64), ("flops_per_execute", C.c_double),
                ("n_weights", C.c_int32), ("n_regions", C.c_int32),
                ("regions", ac_region_info * AC_REGION_KINDS)]


class ac_weight_info(C.Structure):
    _fields_ = [("name", C.c_char * 48), ("rows", C.c_int64), ("cols", C.c_int64),
                ("dtype", C.c_int32), ("index", C.c_int32)]


class ac_proj_part(C.Structure):
    _fields_ = [("w", C.c_void_p), ("bias", C.c_void_p), ("w_gate", C.c_void_p), ("bias_gate", C.c_void_p),
                ("gated", C.c_int32), ("activation", C.c_int32), ("n", C.c_int64),
                ("out", C.c_void_p), ("ldo", C.c_int64), ("o_period", C.c_int64), ("o_s1", C.c_int64),
                ("o_s2", C.c_int64), ("out_t", C.c_void_p), ("t_period", C.c_int64), ("t_s1", C.c_int64),
                ("t_s2", C.c_int64), ("t_s3", C.c_int64)]


class ac_kernel_stat(C.Structure):
    _fields_ = [("name", C.c_char * 32), ("launches", C.c_int64), ("total_ms", C.c_double),
                ("flops", C.c_double), ("bytes", C.c_double)]


AC_GRAPH_MAX_RANK, AC_GRAPH_MAX_INPUTS = 6, 3
(AC_OP_INPUT, AC_OP_PARAM, AC_OP_LINEAR, AC_OP_MATMUL_NT, AC_OP_MATMUL_NN, AC_OP_ELEMENTWISE, AC_OP_NORM_LAST,
 AC_OP_SOFTMAX_LAST, AC_OP_TRANSPOSE, AC_OP_SPLIT_DIM, AC_OP_MERGE_DIMS, AC_OP_SLICE_LAST, AC_OP_CONTRACT_IKC_JKC,
 AC_OP_CONV2D, AC_OP_GROUP_NORM, AC_OP_KINDS) = range(16)


class ac_graph_node(C.Structure):
    _fields_ = [("op", C.c_int32), ("n_inputs", C.c_int32), ("inputs", C.c_int32 * AC_GRAPH_MAX_INPUTS),
                ("rank", C.c_int32), ("shape", C.c_int64 * AC_GRAPH_MAX_RANK), ("attr", C.c_int64 * AC_GRAPH_MAX_RANK)]


class ac_chunk_candidate(C.Structure):
    _fields_ = [("start", C.c_int32), ("end", C.c_int32), ("out_dim", C.c_int32), ("granule", C.c_int32)]


class ac_graph_chunk(C.Structure):
    _fields_ = [("start", C.c_int32), ("end", C.c_int32), ("out_dim", C.c_int32), ("hoist", C.c_int32),
                ("chunk_len", C.c_int64)]


class ac_node_tag(C.Structure):
    _fields_ = [("region_kind", C.c_int32), ("group", C.c_int32), ("dim", C.c_int32 * AC_GRAPH_MAX_RANK),
                ("unit", C.c_int64 * AC_GRAPH_MAX_RANK)]


I64, U64, VP, INT, F32 = C.c_int64, C.c_uint64, C.c_void_p, C.c_int, C.c_float
I32P, INTP, U8P = C.POINTER(C.c_int32), C.POINTER(C.c_int), C.POINTER(C.c_uint8)

# name -> (restype, argtypes): every symbol the headers under include/ declare.
SIGNATURES = {
    "ac_plan_create": (INT, [C.POINTER(ac_model_desc), C.POINTER(ac_region_desc), INT, U64, C.POINTER(VP)]),
    "ac_plan_query": (INT, [VP, C.POINTER(ac_plan_info)]),
    "ac_plan_weight_info": (INT, [VP, INT, C.POINTER(ac_weight_info)]),
    "ac_plan_bind_weights": (INT, [VP, C.POINTER(VP), INT]),
    "ac_execute": (INT, [VP, VP, VP, VP, U64, VP, C.POINTER(U64)]),
    "ac_plan_destroy": (None, [VP]),
    "ac_plan_set_profiling": (INT, [VP, INT]),
    "ac_plan_read_profile": (INT, [VP, C.POINTER(ac_kernel_stat), INT, C.POINTER(INT)]),
    "ac_status_string": (C.c_char_p, [INT]),
    "ac_last_error": (C.c_char_p, []),
    "ac_op_layernorm": (INT, [VP, I64, VP, VP, VP, I64, I64, I64, C.c_float, INT, VP]),
    "ac_op_ln_linear": (INT, [VP, I64, VP, VP, C.c_float, I64, I64, C.POINTER(ac_proj_part), INT, INT, VP]),
    "ac_op_linear": (INT, [VP, I64, VP, I64, VP, VP, I64, VP, I64, VP, I64, VP, I64, I64, I64, I64, I64,
                           I64, I64, I64, INT, INT, VP]),
    "ac_op_attention": (INT, [VP, I64, I64, VP, I64, I64, VP, I64, I64, INT, VP, I64, I64, VP, I64, I64,
                              VP, I64, I64, I64, I64, I64, INT, INT, INT, I64, INT, VP, U64, INT, VP]),
    "ac_op_attention_static_scratch": (INT, [VP, I64, I64, VP, I64, I64, VP, I64, I64, INT, VP, I64, I64, VP, I64, I64,
                                             VP, I64, I64, I64, I64, I64, INT, INT, INT, I64, INT, INT, VP]),
    "ac_static_scratch_bytes": (U64, []),
    "ac_attention_key_splits": (INT, [I64, I64, INT, I64, INT, INT, INT]),
    "ac_attention_split_workspace_bytes": (U64, [I64, INT, I64, INT, INT]),
    "ac_op_bias_act": (INT, [VP, I64, VP, VP, I64, I64, I64, INT, INT, VP]),
    "ac_op_binary": (INT, [VP, I64, VP, I64, VP, I64, I64, I64, INT, INT, VP]),
    "ac_op_softmax_rows": (INT, [VP, I64, VP, I64, I64, I64, F32, INT, I64, I64, INT, VP]),
    "ac_op_transpose": (INT, [VP, I64, VP, I64, I64, I64, INT, VP]),
    "ac_op_triangle_contract": (INT, [VP, I64, I64, VP, I64, I64, VP, I64, I64, I64, I64, I64, INT, INT, VP]),
    "ac_op_transpose_square_inplace": (INT, [VP, I64, I64, I64, I64, INT, VP]),
    "ac_op_layernorm_channel_major": (INT, [VP, I64, VP, VP, VP, I64, I64, I64, C.c_float, INT, VP]),
    "ac_group_norm_workspace_bytes": (U64, [I64, INT]),
    "ac_op_group_norm": (INT, [VP, VP, VP, VP, VP, U64, I64, I64, INT, INT, C.c_float, INT, INT, VP]),
    "ac_op_conv3x3": (INT, [VP, VP, VP, INT, VP, VP, I64, INT, INT, INT, INT, INT, VP]),
    "ac_chunk_trace": (INT, [C.POINTER(ac_graph_node), INT, INT, INT, INT, INT, I32P, U8P, INTP]),
    "ac_chunk_search": (INT, [C.POINTER(ac_graph_node), INT, INT, INT, INT, C.POINTER(ac_chunk_candidate), I32P, U8P,
                              INT, INTP, INTP, INTP]),
    "ac_graph_estimate": (INT, [C.POINTER(ac_graph_node), INT, INT, C.POINTER(ac_graph_chunk), INT, C.POINTER(U64),
                                C.POINTER(U64), INTP]),
    "ac_graph_chunk_cost": (INT, [C.POINTER(ac_graph_node), INT, INT, INT, INT, INT, C.POINTER(C.c_double),
                                  C.POINTER(C.c_double)]),
    "ac_graph_plan": (INT, [C.POINTER(ac_graph_node), INT, INT, U64, INT, C.POINTER(C.c_double), INT, INT,
                            C.POINTER(ac_graph_chunk), INT, INTP, C.POINTER(U64)]),
    "ac_graph_chunks_to_regions": (INT, [C.POINTER(ac_node_tag), INT, C.POINTER(ac_graph_chunk), INT,
                                         C.POINTER(ac_region_desc), INT, INTP]),
}

_lib = None


def lib():
    """The loaded shared library; raises if it has not been built (no fallback)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it first (python -m paper_2401_10652_amd.build)")
        L = C.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(L, name)
            fn.restype = res
            fn.argtypes = args
        _lib = L
    return _lib


class AcError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        msg = lib().ac_last_error().decode()
        super().__init__(f"{where}: {lib().ac_status_string(status).decode()} ({status}): {msg}")


def _check(status, where):
    if status != AC_OK:
        raise AcError(status, where)


def _stream():
    import torch
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t):
    return C.c_void_p(0 if t is None else t.data_ptr())


def _dt(t):
    import torch
    if t.dtype == torch.bfloat16:
        return AC_BF16
    if t.dtype == torch.float32:
        return AC_F32
    raise TypeError(f"unsupported tensor dtype {t.dtype}")


def transformer_desc(cfg, flags=0) -> ac_model_desc:
    m = ac_model_desc()
    m.workload = AC_TRANSFORMER_STACK
    m.dtype = DTYPES[cfg.dtype]
    m.layers, m.batch, m.seq, m.d_model = cfg.layers, cfg.batch, cfg.seq, cfg.d_model
    m.heads, m.head_dim, m.d_ffn = cfg.heads, cfg.head_dim, cfg.d_ffn
    m.causal = int(cfg.causal)
    m.activation = ACTIVATIONS[cfg.activation]
    m.flags = flags
    m.ln_eps = cfg.ln_eps
    return m


def pair_desc(cfg, flags=0) -> ac_model_desc:
    m = ac_model_desc()
    m.workload = AC_PAIR_STACK
    m.dtype = DTYPES[cfg.dtype]
    m.layers = 1
    m.n_res, m.c_z, m.c_hidden = cfg.n_res, cfg.c_z, cfg.c_hidden
    m.tri_heads, m.tri_head_dim, m.transition_factor = cfg.heads, cfg.head_dim, cfg.transition_factor
    m.activation = ACTIVATIONS[cfg.activation]
    m.flags = flags
    m.ln_eps = cfg.ln_eps
    return m


def res_stack_desc(cfg, flags=0) -> ac_model_desc:
    m = ac_model_desc()
    m.workload = AC_UNET_RES_STACK
    m.dtype = DTYPES[cfg.dtype]
    m.layers, m.batch = cfg.layers, cfg.batch
    m.img_h, m.img_w, m.channels, m.groups = cfg.height, cfg.width, cfg.channels, cfg.groups
    m.heads, m.d_ffn = cfg.heads, cfg.d_ffn              # heads > 0: an attention block after every residual block
    m.seq, m.d_model = cfg.context_tokens, cfg.context_dim   # > 0: with a cross-attention to a context per image
    m.activation = ACTIVATIONS[cfg.activation]
    m.flags = flags | (AC_FLAG_GATED_FFN if cfg.gated else 0)
    m.ln_eps = cfg.eps
    return m


class Plan:
    """Owns one ``ac_plan*``; methods carry the names of the entry points they call."""

    def __init__(self, model: ac_model_desc, regions=(), act_budget_bytes=0):
        arr = (ac_region_desc * max(1, len(regions)))()
        for i, (kind, dim, length) in enumerate(regions):
            arr[i].kind, arr[i].chunk_dim, arr[i].chunk_len = kind, dim, length
        self._h = VP()
        self._keep = []
        _check(lib().ac_plan_create(C.byref(model), arr, len(regions), act_budget_bytes, C.byref(self._h)),
               "ac_plan_create")
        self.model = model

    def ac_plan_query(self) -> ac_plan_info:
        info = ac_plan_info()
        _check(lib().ac_plan_query(self._h, C.byref(info)), "ac_plan_query")
        return info

    def ac_plan_weight_info(self, index) -> ac_weight_info:
        wi = ac_weight_info()
        _check(lib().ac_plan_weight_info(self._h, index, C.byref(wi)), "ac_plan_weight_info")
        return wi

    def weight_names(self):
        n = self.ac_plan_query().n_weights
        return [self.ac_plan_weight_info(i).name.decode() for i in range(n)]

    def ac_plan_bind_weights(self, tensors):
        ptrs = (VP * len(tensors))(*[t.data_ptr() for t in tensors])
        _check(lib().ac_plan_bind_weights(self._h, ptrs, len(tensors)), "ac_plan_bind_weights")
        self._keep = list(tensors)

    def ac_execute(self, x, y, workspace) -> int:
        peak = U64(0)
        nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
        _check(lib().ac_execute(self._h, _ptr(x), _ptr(y), _ptr(workspace), nbytes, _stream(), C.byref(peak)),
               "ac_execute")
        return peak.value

    def ac_plan_set_profiling(self, enabled):
        _check(lib().ac_plan_set_profiling(self._h, int(enabled)), "ac_plan_set_profiling")

    def ac_plan_read_profile(self):
        stats = (ac_kernel_stat * 8)()
        n = INT(0)
        _check(lib().ac_plan_read_profile(self._h, stats, 8, C.byref(n)), "ac_plan_read_profile")
        return [dict(name=s.name.decode(), launches=s.launches, total_ms=s.total_ms, flops=s.flops,
                     bytes=s.bytes) for s in stats[:n.value]]

    def close(self):
        if self._h:
            lib().ac_plan_destroy(self._h)
            self._h = VP()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


# ---- single kernels -----------------------------------------------------------------------

def ac_op_layernorm(x, gain, shift, y, eps=1e-5):
    rows, cols = x.shape
    _check(lib().ac_op_layernorm(_ptr(x), x.stride(0), _ptr(gain), _ptr(shift), _ptr(y), y.stride(0),
                                 rows, cols, eps, _dt(x), _stream()), "ac_op_layernorm")


def ac_op_linear(a, w, out, bias=None, mul=None, residual=None, activation=AC_ACT_NONE,
                 out_t=None, n_split=None, t_period=0, t_s1=0, t_s2=1, t_s3=0):
    m, k = a.shape
    n = w.shape[0]
    if n_split is None:
        n_split = n
    _check(lib().ac_op_linear(
        _ptr(a), a.stride(0), _ptr(w), w.stride(0), _ptr(bias),
        _ptr(mul), 0 if mul is None else mul.stride(0),
        _ptr(residual), 0 if residual is None else residual.stride(0),
        _ptr(out), 0 if out is None else out.stride(0),
        _ptr(out_t), n_split, t_period, t_s1, t_s2, t_s3, m, n, k, activation, _dt(a), _stream()),
        "ac_op_linear")


def ac_op_ln_linear(x, gain, shift, parts, eps=1e-5):
    """parts: dicts with w, n (default w.shape[0]) and either out (row-major tensor, optional o_period / o_s1 /
    o_s2) or out_t (+ t_period, t_s1, t_s2, t_s3); optional bias, activation, w_gate, bias_gate."""
    arr = (ac_proj_part * len(parts))()
    for i, d in enumerate(parts):
        a = arr[i]
        addr = lambda t: None if t is None else t.data_ptr()
        a.w, a.bias = addr(d["w"]), addr(d.get("bias"))
        a.w_gate, a.bias_gate = addr(d.get("w_gate")), addr(d.get("bias_gate"))
        a.gated = int(d.get("w_gate") is not None)
        a.activation = d.get("activation", AC_ACT_NONE)
        a.n = d.get("n", d["w"].shape[0])
        out = d.get("out")
        a.out = addr(out)
        a.ldo = 0 if out is None else d.get("ldo", out.stride(0))
        a.o_period, a.o_s1, a.o_s2 = d.get("o_period", 0), d.get("o_s1", 0), d.get("o_s2", 0)
        a.out_t = addr(d.get("out_t"))
        a.t_period, a.t_s1, a.t_s2, a.t_s3 = d.get("t_period", 0), d.get("t_s1", 0), d.get("t_s2", 0), d.get("t_s3", 0)
    _check(lib().ac_op_ln_linear(_ptr(x), x.stride(0), _ptr(gain), _ptr(shift), eps, x.shape[0], x.shape[1],
                                 arr, len(parts), _dt(x), _stream()), "ac_op_ln_linear")


def ac_op_attention(q, k, v, ctx, heads, head_dim, causal=False, q_offset=0, bias=None, gate=None,
                    v_transposed=False, batch=1, strides=None, n_splits=1, split_workspace=None):
    """q [sq, >=heads*head_dim], k [sk, ..], v [sk, ..] or v^T [heads*head_dim, sk]; one problem
    unless ``batch`` and ``strides`` = (q, k, v, gate, ctx batch strides in elements) are given."""
    sq, sk = q.shape[0], k.shape[0]
    sb = strides or (0, 0, 0, 0, 0)
    _check(lib().ac_op_attention(
        _ptr(q), q.stride(0), sb[0], _ptr(k), k.stride(0), sb[1], _ptr(v), v.stride(0), sb[2],
        int(v_transposed),
        _ptr(bias), 0 if bias is None else bias.stride(1), 0 if bias is None else bias.stride(0),
        _ptr(gate), 0 if gate is None else gate.stride(0), sb[3],
        _ptr(ctx), ctx.stride(0), sb[4], batch, sq, sk, heads, head_dim, int(causal), q_offset,
        n_splits, _ptr(split_workspace),
        0 if split_workspace is None else split_workspace.numel() * split_workspace.element_size(),
        _dt(q), _stream()), "ac_op_attention")


def ac_op_attention_static_scratch(q, k, v, ctx, heads, head_dim, causal=False, q_offset=0, bias=None, gate=None,
                                   v_transposed=False, batch=1, strides=None, n_splits=0):
    """ac_op_attention with the key-split partial results in the library's static device array."""
    sq, sk = q.shape[0], k.shape[0]
    sb = strides or (0, 0, 0, 0, 0)
    _check(lib().ac_op_attention_static_scratch(
        _ptr(q), q.stride(0), sb[0], _ptr(k), k.stride(0), sb[1], _ptr(v), v.stride(0), sb[2],
        int(v_transposed),
        _ptr(bias), 0 if bias is None else bias.stride(1), 0 if bias is None else bias.stride(0),
        _ptr(gate), 0 if gate is None else gate.stride(0), sb[3],
        _ptr(ctx), ctx.stride(0), sb[4], batch, sq, sk, heads, head_dim, int(causal), q_offset,
        n_splits, _dt(q), _stream()), "ac_op_attention_static_scratch")


def ac_static_scratch_bytes():
    return lib().ac_static_scratch_bytes()


def ac_attention_key_splits(sq, sk, heads, batch, head_dim, dtype, v_transposed=True):
    return lib().ac_attention_key_splits(sq, sk, heads, batch, head_dim, DTYPES[dtype], int(v_transposed))


def ac_attention_split_workspace_bytes(sq, heads, batch, head_dim, n_splits):
    return lib().ac_attention_split_workspace_bytes(sq, heads, batch, head_dim, n_splits)


def ac_op_bias_act(x, bias, y, activation):
    rows, cols = x.shape
    _check(lib().ac_op_bias_act(_ptr(x), x.stride(0), _ptr(bias), _ptr(y), y.stride(0), rows, cols,
                                activation, _dt(x), _stream()), "ac_op_bias_act")


def ac_op_softmax_rows(s, p, scale, causal=False, q_offset=0, period=None):
    rows, cols = s.shape
    _check(lib().ac_op_softmax_rows(_ptr(s), s.stride(0), _ptr(p), p.stride(0), rows, cols, float(scale),
                                    int(causal), q_offset, rows if period is None else period, _dt(s), _stream()),
           "ac_op_softmax_rows")


def ac_op_binary(a, b, y, op):
    rows, cols = a.shape
    _check(lib().ac_op_binary(_ptr(a), a.stride(0), _ptr(b), b.stride(0), _ptr(y), y.stride(0), rows, cols,
                              op, _dt(a), _stream()), "ac_op_binary")


def ac_op_transpose(src, dst):
    rows, cols = src.shape
    _check(lib().ac_op_transpose(_ptr(src), src.stride(0), _ptr(dst), dst.stride(0), rows, cols, _dt(src),
                                 _stream()), "ac_op_transpose")


def ac_op_triangle_contract(a_t, b_t, out_c):
    """a_t [C, ni, nk], b_t [C, nj, nk] -> out_c [C, ni, nj] (views with strides are fine)."""
    ch, ni, nk = a_t.shape
    nj = b_t.shape[1]
    _check(lib().ac_op_triangle_contract(_ptr(a_t), a_t.stride(1), a_t.stride(0), _ptr(b_t), b_t.stride(1),
                                         b_t.stride(0), _ptr(out_c), out_c.stride(1), out_c.stride(0),
                                         ni, nj, nk, ch, _dt(a_t), _stream()), "ac_op_triangle_contract")


def ac_op_transpose_square_inplace(data):
    """data [batch, n, n], transposed in place per batch entry."""
    batch, n, _ = data.shape
    _check(lib().ac_op_transpose_square_inplace(_ptr(data), data.stride(1), data.stride(0), n, batch, _dt(data),
                                                _stream()), "ac_op_transpose_square_inplace")


def ac_op_layernorm_channel_major(src, gain, shift, dst, eps=1e-5):
    """src [C, P] -> dst [P, C]."""
    ch, pos = src.shape
    _check(lib().ac_op_layernorm_channel_major(_ptr(src), src.stride(0), _ptr(gain), _ptr(shift), _ptr(dst),
                                               dst.stride(0), pos, ch, eps, _dt(src), _stream()),
           "ac_op_layernorm_channel_major")


def ac_group_norm_workspace_bytes(images, groups):
    return int(lib().ac_group_norm_workspace_bytes(images, groups))


def ac_op_group_norm(x, gain, shift, y, workspace, groups, eps=1e-5, activation=AC_ACT_NONE):
    """x, y [images, positions..., channels] channels-last."""
    images, ch = x.shape[0], x.shape[-1]
    positions = x.numel() // (images * ch) if images else 0
    _check(lib().ac_op_group_norm(_ptr(x), _ptr(gain), _ptr(shift), _ptr(y), _ptr(workspace), workspace.numel() * workspace.element_size(),
                                  images, positions, ch, groups, eps, activation, _dt(x), _stream()), "ac_op_group_norm")


def ac_op_conv3x3(x, weight, out, bias=None, bias_per_image=False, residual=None):
    """x [images, H, W, c_in], weight [c_out, 3, 3, c_in] -> out [images, H, W, c_out]."""
    images, h, w, c_in = x.shape
    _check(lib().ac_op_conv3x3(_ptr(x), _ptr(weight), _ptr(bias), int(bias_per_image), _ptr(residual), _ptr(out), images, h, w,
                               c_in, weight.shape[0], _dt(x), _stream()), "ac_op_conv3x3")


# ---- helpers for callers (buffers only) ------------------------------------------------------

def to_device(arr, dtype: str):
    """Upload a host fp32 array that already holds storage-exact values."""
    import numpy as np
    import torch
    t = torch.from_numpy(np.ascontiguousarray(arr, dtype=np.float32))
    return t.to(device="cuda", dtype=torch.bfloat16 if dtype == "bf16" else torch.float32).contiguous()


def empty_workspace(nbytes: int):
    import torch
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device="cuda")


# ------------------------------------------------------------------------------------------
# chunk search (host only)
# ------------------------------------------------------------------------------------------

def graph_nodes(spec):
    """ac_graph_node array from a list of (op, inputs, shape, attr) tuples."""
    arr = (ac_graph_node * len(spec))()
    for nd, (op, inputs, shape, attr) in zip(arr, spec):
        if len(inputs) > AC_GRAPH_MAX_INPUTS or len(shape) > AC_GRAPH_MAX_RANK or len(attr) > AC_GRAPH_MAX_RANK:
            raise ValueError("node exceeds AC_GRAPH_MAX_INPUTS / AC_GRAPH_MAX_RANK")
        nd.op, nd.n_inputs, nd.rank = op, len(inputs), len(shape)
        for i, v in enumerate(inputs):
            nd.inputs[i] = v
        for i, v in enumerate(shape):
            nd.shape[i] = v
        for i, v in enumerate(attr):
            nd.attr[i] = v
    return arr


def ac_chunk_trace(nodes, start, end, out_dim, hoist=False):
    """Chunk dims per node (list, -1 = not cut) of a legal chunk, or None; with hoist, a pair
    (dims, sorted list of the nodes moved ahead of the region)."""
    row = (C.c_int32 * len(nodes))()
    moved = (C.c_uint8 * len(nodes))()
    legal = C.c_int(0)
    _check(lib().ac_chunk_trace(nodes, len(nodes), start, end, out_dim, int(hoist), row, moved, C.byref(legal)),
           "ac_chunk_trace")
    if not legal.value:
        return None
    return (list(row), [i for i, m in enumerate(moved) if m]) if hoist else list(row)


def ac_chunk_search(nodes, peak, window, max_out=None, hoist=False):
    """(candidates, n_found, n_tried, n_passed); a candidate is (start, end, out_dim, granule,
    node_dims), with hoist followed by the sorted list of its moved nodes."""
    n = len(nodes)
    found, tried, passed = C.c_int(0), C.c_int(0), C.c_int(0)
    if max_out is None:
        _check(lib().ac_chunk_search(nodes, n, peak, window, int(hoist), None, None, None, 0, C.byref(found), None, None),
               "ac_chunk_search")
        max_out = found.value
    out = (ac_chunk_candidate * max(max_out, 1))()
    rows = (C.c_int32 * (max(max_out, 1) * n))()
    moved = (C.c_uint8 * (max(max_out, 1) * n))()
    _check(lib().ac_chunk_search(nodes, n, peak, window, int(hoist), out, rows, moved, max_out, C.byref(found),
                                 C.byref(tried), C.byref(passed)), "ac_chunk_search")
    cands = []
    for i, c in enumerate(out[:min(max_out, found.value)]):
        cand = (c.start, c.end, c.out_dim, c.granule, list(rows[i * n:(i + 1) * n]))
        if hoist:
            cand += ([j for j in range(n) if moved[i * n + j]],)
        cands.append(cand)
    return cands, found.value, tried.value, passed.value


def _chunks(chunks):
    """ac_graph_chunk array from (start, end, out_dim, chunk_len[, hoist]) tuples."""
    arr = (ac_graph_chunk * max(len(chunks), 1))()
    for c, ch in zip(arr, chunks):
        c.start, c.end, c.out_dim, c.chunk_len = ch[:4]
        c.hoist = int(bool(ch[4])) if len(ch) > 4 else 0
    return arr


def ac_graph_estimate(nodes, elem_bytes, chunks=()):
    """(bytes per node, peak bytes, peak node) with chunks = [(start, end, out_dim, chunk_len[, hoist])]."""
    per_node = (C.c_uint64 * len(nodes))()
    peak, peak_node = C.c_uint64(0), C.c_int(0)
    _check(lib().ac_graph_estimate(nodes, len(nodes), elem_bytes, _chunks(chunks), len(chunks), per_node,
                                   C.byref(peak), C.byref(peak_node)), "ac_graph_estimate")
    return list(per_node), peak.value, peak_node.value


def ac_graph_chunk_cost(nodes, start, end, out_dim, weights, hoist=False):
    w = (C.c_double * 4)(*weights)
    cost = C.c_double(0)
    _check(lib().ac_graph_chunk_cost(nodes, len(nodes), start, end, out_dim, int(hoist), w, C.byref(cost)),
           "ac_graph_chunk_cost")
    return cost.value


def node_tags(tags):
    """ctypes array of ac_node_tag from [(region_kind, group, ((dim, unit), ...))], one entry per node."""
    arr = (ac_node_tag * len(tags))()
    for t, (kind, group, dims) in zip(arr, tags):
        t.region_kind, t.group = kind, group
        for i in range(AC_GRAPH_MAX_RANK):
            t.dim[i], t.unit[i] = dims[i] if i < len(dims) else (-1, 0)
    return arr


def ac_graph_chunks_to_regions(tags, chunks):
    """[(kind, chunk_dim, chunk_len)] for ac_plan_create from chunks (start, end, out_dim, chunk_len[, hoist])."""
    arr = (ac_graph_chunk * max(1, len(chunks)))()
    for a, c in zip(arr, chunks):
        a.start, a.end, a.out_dim, a.chunk_len = c[:4]
        a.hoist = c[4] if len(c) > 4 else 0
    out = (ac_region_desc * AC_REGION_KINDS)()
    n_out = C.c_int(0)
    _check(lib().ac_graph_chunks_to_regions(tags, len(tags), arr, len(chunks), out, AC_REGION_KINDS, C.byref(n_out)),
           "ac_graph_chunks_to_regions")
    return [(r.kind, r.chunk_dim, r.chunk_len) for r in out[:n_out.value]]


def ac_graph_plan(nodes, elem_bytes, budget_bytes, window, weights, beam=1, max_out=64, hoist=False):
    """(chunks, peak bytes): chunks (start, end, out_dim, chunk_len), with hoist (.., 1), in the order chosen."""
    w = (C.c_double * 4)(*weights)
    out = (ac_graph_chunk * max_out)()
    n_out, peak = C.c_int(0), C.c_uint64(0)
    _check(lib().ac_graph_plan(nodes, len(nodes), elem_bytes, budget_bytes, window, w, beam, int(hoist), out, max_out,
                               C.byref(n_out), C.byref(peak)), "ac_graph_plan")
    return [(c.start, c.end, c.out_dim, c.chunk_len) + ((1,) if hoist else ()) for c in out[:n_out.value]], peak.value
