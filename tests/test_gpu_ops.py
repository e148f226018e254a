"""GPU parity of the single kernels against the fp64 oracle, through the C-ABI."""
import math

import numpy as np
import pytest

from oracle import transformer as O
from util import TOL, check, draw, host, rel_err

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_2401_10652_amd import binding
    binding.lib()
    return binding


def dev(B, arr, dtype):
    return B.to_device(arr, dtype)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("rows,cols", [(5, 64), (300, 128), (257, 768), (130, 1024), (70, 2048), (33, 100), (9, 24),
                                       (70, 320), (33, 640), (21, 1280)])
def test_layernorm(B, dtype, rows, cols):
    import torch
    from paper_2401_10652_amd.inputs import round_to_storage
    x = round_to_storage(draw((rows, cols), 1, "f32", 2.0) + 0.5, dtype)
    g = round_to_storage(draw((cols,), 2, "f32", 0.3) + 1, dtype)
    b = draw((cols,), 3, dtype, 0.3)
    dx, dg, db = dev(B, x, dtype), dev(B, g, dtype), dev(B, b, dtype)
    y = torch.full_like(dx, float("nan"))
    B.ac_op_layernorm(dx, dg, db, y, 1e-5)
    torch.cuda.synchronize()
    ref = O.layer_norm(x, g, b, 1e-5)
    check(host(y), ref, dtype)


@pytest.mark.parametrize("dtype,m,n,k", [
    ("bf16", 300, 200, 192),      # 32x64 tiles, ragged m and n
    ("bf16", 500, 2040, 192),     # 64x64 tiles (256 of them), ragged m and n
    ("bf16", 520, 3000, 128),     # 64x64 tiles in two rounds, ragged m and n
    ("bf16", 2048, 2048, 256),    # 128x128 tiles
    ("bf16", 1100, 3072, 128),    # 128x128 tiles, ragged m
    ("bf16", 77, 37, 100),        # odd shape -> generic kernel
    ("bf16", 64, 4, 128),         # n = 4 (pair-bias projection shape)
    ("f32", 256, 192, 64),
    ("f32", 70, 50, 33),
])
@pytest.mark.parametrize("epi", ["plain", "bias_gelu", "bias_resid", "sigmoid_mul_resid", "tanh", "relu"])
def test_linear(B, dtype, m, n, k, epi):
    import torch
    a = draw((m, k), 10, dtype)
    w = draw((n, k), 11, dtype, 1 / math.sqrt(k))
    bias = draw((n,), 12, dtype, 0.5)
    mul = draw((m, n), 13, dtype)
    res = draw((m, n), 14, dtype)
    da, dw = dev(B, a, dtype), dev(B, w, dtype)
    out = torch.full((m, n), float("nan"), device="cuda", dtype=da.dtype)
    ref = O.linear(a, w)
    kw = {}
    if epi == "bias_gelu":
        kw = dict(bias=dev(B, bias, dtype), activation=B.AC_ACT_GELU_ERF)
        ref = O.gelu_erf(ref + bias)
    elif epi == "bias_resid":
        kw = dict(bias=dev(B, bias, dtype), residual=dev(B, res, dtype))
        ref = ref + bias + res
    elif epi == "sigmoid_mul_resid":
        kw = dict(bias=dev(B, bias, dtype), activation=B.AC_ACT_SIGMOID, mul=dev(B, mul, dtype),
                  residual=dev(B, res, dtype))
        ref = 1 / (1 + np.exp(-(ref + bias))) * mul + res
    elif epi == "tanh":
        kw = dict(activation=B.AC_ACT_GELU_TANH)
        ref = O.gelu_tanh(ref)
    elif epi == "relu":
        kw = dict(activation=B.AC_ACT_RELU)
        ref = O.relu(ref)
    B.ac_op_linear(da, dw, out, **kw)
    torch.cuda.synchronize()
    got = host(out)
    assert np.isfinite(got).all()
    check(got, ref, dtype)


@pytest.mark.parametrize("m,n,k,epi", [(8184, 8168, 2048, "none"), (8184, 8168, 2048, "bias_gelu"),
                                       (8184, 8168, 4096, "bias_resid"), (8192, 8192, 1024, "bias_gelu")])
def test_linear_large_tiles_on_sampled_rows(B, m, n, k, epi):
    """Shapes that take the 256x256 tiles (both kernels: k >= 2048 and below), with ragged last
    tiles in both directions; the oracle computes every column of a sample of rows (the first
    and the last tile's rows among them)."""
    import torch
    a = draw((m, k), 15, "bf16")
    w = draw((n, k), 16, "bf16", 1 / math.sqrt(k))
    bias = draw((n,), 17, "bf16", 0.5)
    res = draw((m, n), 18, "bf16")
    rows = np.unique(np.concatenate([np.arange(40), np.arange(m - 40, m), np.arange(0, m, 97), [255, 256, 4095, 4096]]))
    da, dw = dev(B, a, "bf16"), dev(B, w, "bf16")
    out = torch.full((m, n), float("nan"), device="cuda", dtype=da.dtype)
    ref = O.linear(a[rows], w)
    kw = {}
    if epi == "bias_gelu":
        kw = dict(bias=dev(B, bias, "bf16"), activation=B.AC_ACT_GELU_ERF)
        ref = O.gelu_erf(ref + bias)
    elif epi == "bias_resid":
        kw = dict(bias=dev(B, bias, "bf16"), residual=dev(B, res, "bf16"))
        ref = ref + bias + res[rows]
    B.ac_op_linear(da, dw, out, **kw)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(out.float()).all())
    got = host(out[torch.from_numpy(rows).cuda()])
    check(got, ref, "bf16")


@pytest.mark.parametrize("dtype,m,n,k,split", [("bf16", 384, 256, 128, 128), ("bf16", 200, 96, 64, 0),
                                               ("f32", 100, 48, 32, 16), ("bf16", 50, 30, 20, 10)])
def test_linear_strided_store(B, dtype, m, n, k, split):
    """Columns >= split land transposed, with a period: rows (m / P, m % P) -> [m/P][n][m%P]."""
    import torch
    a = draw((m, k), 20, dtype)
    w = draw((n, k), 21, dtype, 1 / math.sqrt(k))
    bias = draw((n,), 22, dtype, 0.5)
    da, dw, dbias = dev(B, a, dtype), dev(B, w, dtype), dev(B, bias, dtype)
    ref = O.linear(a, w, bias)
    # plain transpose of the tail columns
    out = torch.zeros((m, max(split, 1)), device="cuda", dtype=da.dtype)
    out_t = torch.zeros((n - split, m), device="cuda", dtype=da.dtype)
    B.ac_op_linear(da, dw, out if split else None, bias=dbias, out_t=out_t, n_split=split, t_s2=1, t_s3=m)
    torch.cuda.synchronize()
    if split:
        check(host(out)[:, :split], ref[:, :split], dtype)
    check(host(out_t), ref[:, split:].T, dtype)
    # periodic form: m = p * P + r  ->  out_t[p][n][r]
    if m % 50 == 0:
        P = 50
        out_p = torch.zeros((m // P, n - split, P), device="cuda", dtype=da.dtype)
        B.ac_op_linear(da, dw, out if split else None, bias=dbias, out_t=out_p, n_split=split,
                       t_period=P, t_s1=(n - split) * P, t_s2=1, t_s3=P)
        torch.cuda.synchronize()
        want = ref[:, split:].reshape(m // P, P, n - split).transpose(0, 2, 1)
        check(host(out_p), want, dtype)


def _attn_case(B, dtype, sq, sk, heads, dh, causal, q_offset, use_bias, use_gate, v_t, n_splits=1):
    import torch
    hd = heads * dh
    q = draw((sq, hd), 30, dtype)
    k = draw((sk, hd), 31, dtype)
    v = draw((sk, hd), 32, dtype)
    bias = draw((heads, sq, sk), 33, dtype) if use_bias else None
    gate = draw((sq, hd), 34, dtype) if use_gate else None
    dq, dk, dv = dev(B, q, dtype), dev(B, k, dtype), dev(B, v, dtype)
    if v_t:
        ld = (sk + 7) // 8 * 8
        dvt = torch.zeros((hd, ld), device="cuda", dtype=dq.dtype)
        B.ac_op_transpose(dv, dvt)
        vv = dvt[:, :sk]
    else:
        vv = dv
    ctx = torch.full((sq, hd), float("nan"), device="cuda", dtype=dq.dtype)
    ws = None
    if n_splits > 1:
        need = B.ac_attention_split_workspace_bytes(sq, heads, 1, dh, n_splits)
        ws = torch.full((need,), 0xFF, dtype=torch.uint8, device="cuda")
    B.ac_op_attention(dq, dk, vv, ctx, heads, dh, causal=causal, q_offset=q_offset,
                      bias=None if bias is None else dev(B, bias, dtype),
                      gate=None if gate is None else dev(B, gate, dtype), v_transposed=v_t,
                      n_splits=n_splits, split_workspace=ws)
    torch.cuda.synchronize()
    ref = O.attention(q, k, v, heads, causal, bias=bias, q_offset=q_offset)
    if gate is not None:
        ref = ref * gate
    got = host(ctx)
    assert np.isfinite(got).all()
    return rel_err(got, ref)


@pytest.mark.parametrize("dh", [32, 64, 128])
@pytest.mark.parametrize("sq,sk,causal,q_offset", [
    (300, 520, False, 0),       # ragged query and key tails
    (128, 64, False, 0),
    (200, 456, True, 256),      # a query segment placed at its absolute position
    (333, 336, True, 3),
    (1, 8, True, 7),
])
def test_attention_mfma(B, dh, sq, sk, causal, q_offset):
    assert _attn_case(B, "bf16", sq, sk, 3, dh, causal, q_offset, False, False, True) <= TOL["bf16"]


@pytest.mark.parametrize("dh", [64, 128])
@pytest.mark.parametrize("sq,sk,causal,q_offset", [
    (300, 512, False, 0),       # whole key tiles and no bias: the software-pipelined loop, several tiles
    (384, 640, True, 256),      # diagonal tiles of every wave inside the loop
    (200, 448, True, 248),      # a segment offset that is no multiple of the tile
    (96, 1024, True, 928),      # a short segment at the end of a long sequence
    (64, 128, True, 64),        # two tiles: prologue and last step only
])
def test_attention_whole_key_tiles(B, dh, sq, sk, causal, q_offset):
    assert _attn_case(B, "bf16", sq, sk, 3, dh, causal, q_offset, False, False, True) <= TOL["bf16"]
    assert _attn_case(B, "bf16", sq, sk, 2, dh, causal, q_offset, False, True, True) <= TOL["bf16"]


@pytest.mark.parametrize("dh,causal", [(64, False), (128, True), (128, False)])
def test_attention_256_row_blocks(B, dh, causal):
    """A launch with at least 1024 blocks of 256 query rows runs 8 waves per block."""
    assert _attn_case(B, "bf16", 1024, 1024, 256, dh, causal, 0, False, False, True) <= TOL["bf16"]


@pytest.mark.parametrize("dh", [32, 64, 128])
@pytest.mark.parametrize("n_splits", [2, 3, 7])
def test_attention_key_splits(B, dh, n_splits):
    """Key runs handled by separate blocks and merged: same result to rounding; includes splits
    that are empty for early query blocks (causal) and more splits than key tiles."""
    assert _attn_case(B, "bf16", 300, 1216, 2, dh, True, 916, False, False, True, n_splits) <= TOL["bf16"]
    assert _attn_case(B, "bf16", 200, 200, 2, dh, True, 0, False, False, True, n_splits) <= TOL["bf16"]
    assert _attn_case(B, "bf16", 130, 1000, 3, dh, False, 0, dh != 128, True, True, n_splits) <= TOL["bf16"]


def test_attention_split_workspace_is_checked(B):
    import torch
    q = torch.zeros((64, 64), device="cuda", dtype=torch.bfloat16)
    vt = torch.zeros((64, 64), device="cuda", dtype=torch.bfloat16)
    with pytest.raises(B.AcError) as ei:
        B.ac_op_attention(q, q, vt, q.clone(), 1, 64, v_transposed=True, n_splits=4,
                          split_workspace=torch.zeros(16, dtype=torch.uint8, device="cuda"))
    assert ei.value.status == B.AC_ERR_WORKSPACE


@pytest.mark.parametrize("dh", [32, 64])
def test_attention_mfma_bias_gate(B, dh):
    assert _attn_case(B, "bf16", 260, 392, 4, dh, False, 0, True, True, True) <= TOL["bf16"]
    assert _attn_case(B, "bf16", 100, 128, 2, dh, False, 0, True, False, True) <= TOL["bf16"]


@pytest.mark.parametrize("dtype,dh", [("f32", 16), ("f32", 64), ("bf16", 16), ("bf16", 64)])
@pytest.mark.parametrize("causal", [False, True])
def test_attention_generic(B, dtype, dh, causal):
    off = 40 if causal else 0
    assert _attn_case(B, dtype, 150, 190 + off, 2, dh, causal, off, True, True, False) <= TOL[dtype]
    assert _attn_case(B, dtype, 70, 70, 3, dh, causal, 0, False, False, False) <= TOL[dtype]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("rows,cols", [(100, 256), (37, 51)])
def test_elementwise(B, dtype, rows, cols):
    import torch
    x = draw((rows, cols), 40, dtype, 2.0)
    r = draw((rows, cols), 41, dtype)
    bias = draw((cols,), 42, dtype)
    dx, dr, dbias = dev(B, x, dtype), dev(B, r, dtype), dev(B, bias, dtype)
    y = torch.empty_like(dx)
    for act, fn in ((B.AC_ACT_GELU_ERF, O.gelu_erf), (B.AC_ACT_GELU_TANH, O.gelu_tanh), (B.AC_ACT_RELU, O.relu),
                    (B.AC_ACT_SIGMOID, lambda t: 1 / (1 + np.exp(-t))), (B.AC_ACT_NONE, lambda t: t)):
        B.ac_op_bias_act(dx, dbias, y, act)
        torch.cuda.synchronize()
        check(host(y), fn(x.astype(np.float64) + bias), dtype)
    B.ac_op_bias_act(dx, None, y, B.AC_ACT_GELU_ERF)
    torch.cuda.synchronize()
    check(host(y), O.gelu_erf(x), dtype)
    B.ac_op_binary(dx, dr, y, 0)
    torch.cuda.synchronize()
    check(host(y), x.astype(np.float64) + r, dtype)
    B.ac_op_binary(dx, dr, y, 1)
    torch.cuda.synchronize()
    check(host(y), x.astype(np.float64) * r, dtype)


def test_bf16_store_rounds_to_nearest_even(B):
    """x + 0 through the kernel must equal the host generator's rounding, bit for bit."""
    import torch
    from paper_2401_10652_amd import inputs as I
    v = I.standard_normal(4242, 64 * 256).astype(np.float32).reshape(64, 256)
    want = I.round_to_bf16(v)
    # feed fp32 halves that sum to v exactly is not possible in bf16; instead add two bf16 numbers
    hi = I.round_to_bf16(v)
    lo = I.round_to_bf16(v - hi)
    y = torch.empty((64, 256), device="cuda", dtype=torch.bfloat16)
    B.ac_op_binary(B.to_device(hi, "bf16"), B.to_device(lo, "bf16"), y, 0)
    torch.cuda.synchronize()
    want = I.round_to_bf16(hi.astype(np.float32) + lo.astype(np.float32))
    assert np.array_equal(y.float().cpu().numpy(), want)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("rows,cols,period,q_offset,causal", [
    (12, 100, 4, 0, False), (12, 100, 4, 96, True), (6, 1000, 3, 10, True), (8, 8, 8, 0, True),
    (5, 4097, 5, 4000, True), (3, 1, 3, 0, True),
    (4, 4096, 4, 100, True), (3, 8192, 3, 5000, True), (2, 16384, 2, 0, False), (2, 20000, 2, 12345, True),
])
def test_softmax_rows(B, dtype, rows, cols, period, q_offset, causal):
    """Stored scores -> stored probabilities; row r is query r mod period at position q_offset +
    (r mod period); masked columns get exactly 0.  In place as well."""
    import torch
    s = draw((rows, cols), 70, dtype, 3.0)
    scale = 0.37
    ds = dev(B, s, dtype)
    p = torch.full_like(ds, float("nan"))
    B.ac_op_softmax_rows(ds, p, scale, causal=causal, q_offset=q_offset, period=period)
    torch.cuda.synchronize()
    z = s.astype(np.float64) * scale
    if causal:
        pos = q_offset + np.arange(rows) % period
        z = np.where(np.arange(cols)[None, :] <= pos[:, None], z, -np.inf)
    ref = O.softmax_rows(z)
    got = host(p)
    check(got, ref, dtype)
    assert (got[ref == 0] == 0).all()
    B.ac_op_softmax_rows(ds, ds, scale, causal=causal, q_offset=q_offset, period=period)
    torch.cuda.synchronize()
    assert np.array_equal(host(ds), got)


def test_random_shapes_of_linear_and_attention(B):
    """Seeded random shapes around the tile and split boundaries of both matrix kernels (ragged
    tails in every direction, every epilogue, query segments at random absolute positions),
    each against the oracle."""
    import torch
    rng = np.random.default_rng(2401)
    worst = 0.0
    for case in range(24):
        m = int(rng.choice([1, 31, 64, 65, 127, 128, 129, 255, 257, 300, 513, 700]))
        n = 4 * int(rng.integers(1, 160))
        k = 64 * int(rng.integers(1, 9)) if case % 4 else 8 * int(rng.integers(1, 40))
        epi = ["plain", "bias_gelu", "bias_resid", "relu"][case % 4]
        a, w = draw((m, k), 100 + case, "bf16"), draw((n, k), 200 + case, "bf16", 1 / math.sqrt(k))
        bias, res = draw((n,), 300 + case, "bf16", 0.5), draw((m, n), 400 + case, "bf16")
        out = torch.full((m, n), float("nan"), device="cuda", dtype=torch.bfloat16)
        ref = O.linear(a, w)
        kw = {}
        if epi == "bias_gelu":
            kw, ref = dict(bias=dev(B, bias, "bf16"), activation=B.AC_ACT_GELU_ERF), O.gelu_erf(ref + bias)
        elif epi == "bias_resid":
            kw, ref = dict(bias=dev(B, bias, "bf16"), residual=dev(B, res, "bf16")), ref + bias + res
        elif epi == "relu":
            kw, ref = dict(activation=B.AC_ACT_RELU), O.relu(ref)
        B.ac_op_linear(dev(B, a, "bf16"), dev(B, w, "bf16"), out, **kw)
        torch.cuda.synchronize()
        got = host(out)
        assert np.isfinite(got).all(), (m, n, k, epi)
        err = rel_err(got, ref)
        assert err <= TOL["bf16"], (m, n, k, epi, err)
        worst = max(worst, err)
    for case in range(24):
        dh = int(rng.choice([32, 64, 128]))
        heads = int(rng.integers(1, 5))
        sk = int(rng.integers(1, 1400))
        causal = bool(case % 2)
        sq = int(rng.integers(1, min(sk, 400) + 1)) if causal else int(rng.integers(1, 400))
        q_offset = sk - sq if causal else 0          # the segment's rows end at the last key
        n_splits = int(rng.choice([1, 1, 2, 5])) if sk >= 64 else 1
        err = _attn_case(B, "bf16", sq, sk, heads, dh, causal, q_offset, case % 3 == 0, case % 5 == 0, True, n_splits)
        assert err <= TOL["bf16"], (sq, sk, heads, dh, causal, q_offset, n_splits, err)
        worst = max(worst, err)
    assert worst > 0


@pytest.mark.parametrize("rows,k", [(300, 128), (384, 128), (200, 64), (1, 128)])
def test_ln_linear_parts(B, rows, k):
    """LayerNorm + several projections in one kernel against the oracle's separate steps: a plain part
    with bias and ReLU stored row-major, a gated pair stored channel-major, a 4-column part stored
    strided, a GELU part with its rows regrouped on the way out, a sigmoid part."""
    import torch
    x = draw((rows, k), 400, "bf16")
    g = 1.0 + draw((k,), 401, "bf16", 0.1)
    b = draw((k,), 402, "bf16", 0.1)
    w = {n: draw((c, k), 403 + i, "bf16", k ** -0.5) for i, (n, c) in
         enumerate((("p", 128), ("gw", 64), ("gp", 64), ("s", 4), ("r", 256), ("sg", 72)))}
    bias = {n: draw((w[n].shape[0],), 420 + i, "bf16", 0.2) for i, n in enumerate(w)}
    dev_w = {n: dev(B, v, "bf16") for n, v in w.items()}
    dev_b = {n: dev(B, v, "bf16") for n, v in bias.items()}
    t = O.layer_norm(x, g, b)
    sig = lambda v: 1.0 / (1.0 + np.exp(-v))
    ref_p = O.relu(O.linear(t, w["p"], bias["p"]))
    ref_g = sig(O.linear(t, w["gw"], bias["gw"])) * O.linear(t, w["gp"], bias["gp"])
    ref_s = O.linear(t, w["s"])
    ref_r = O.gelu_erf(O.linear(t, w["r"], bias["r"]))
    ref_sg = sig(O.linear(t, w["sg"], bias["sg"]))
    bf = torch.bfloat16
    out_p = torch.full((rows, 128), float("nan"), dtype=bf, device="cuda")
    out_g = torch.full((64, rows), float("nan"), dtype=bf, device="cuda")        # channel-major
    out_s = torch.full((4, rows), float("nan"), dtype=bf, device="cuda")
    # rows regrouped: row m = (a, c) with c < period lands at (c, a); pad the row count to the period
    period = 8 if rows % 8 == 0 else 1
    out_r = torch.full((rows, 256), float("nan"), dtype=bf, device="cuda")
    out_sg = torch.full((rows, 72), float("nan"), dtype=bf, device="cuda")
    parts = [
        dict(w=dev_w["p"], bias=dev_b["p"], activation=B.AC_ACT_RELU, out=out_p),
        dict(w=dev_w["gp"], bias=dev_b["gp"], w_gate=dev_w["gw"], bias_gate=dev_b["gw"], out_t=out_g, t_s2=1, t_s3=rows),
        dict(w=dev_w["s"], out_t=out_s, t_s2=1, t_s3=rows),
        dict(w=dev_w["r"], bias=dev_b["r"], activation=B.AC_ACT_GELU_ERF, out=out_r, o_period=period,
             o_s1=256, o_s2=(rows // period) * 256),
        dict(w=dev_w["sg"], bias=dev_b["sg"], activation=B.AC_ACT_SIGMOID, out=out_sg),
    ]
    B.ac_op_ln_linear(dev(B, x, "bf16"), dev(B, g, "bf16"), dev(B, b, "bf16"), parts)
    torch.cuda.synchronize()
    check(host(out_p), ref_p, "bf16", what="plain")
    check(host(out_g).T, ref_g, "bf16", what="gated")
    check(host(out_s).T, ref_s, "bf16", what="narrow")
    # row m of the result sits at (m % period) * (rows / period) + m / period
    m = np.arange(rows)
    check(host(out_r)[(m % period) * (rows // period) + m // period], ref_r, "bf16", what="regrouped")
    check(host(out_sg), ref_sg, "bf16", what="sigmoid")
    # shapes the kernel does not cover are refused
    with pytest.raises(B.AcError) as ei:
        B.ac_op_ln_linear(dev(B, draw((8, 96), 1, "bf16"), "bf16"), dev(B, g[:96], "bf16"), dev(B, b[:96], "bf16"),
                          [dict(w=dev(B, draw((8, 96), 2, "bf16"), "bf16"), out=out_p)])
    assert ei.value.status == B.AC_ERR_UNSUPPORTED
