"""Pins of the fp64 pair-stack oracle (no GPU)."""
import numpy as np
import pytest

import brute
from oracle import pairstack as P
from oracle import transformer as O
from paper_2401_10652_amd import inputs as I


def tiny(n=5, cz=6, ch=4, heads=2, dh=3, idx=21):
    cfg = I.PairConfig("tinyp", idx, n, cz, ch, heads, dh, 4, "f32")
    z, w = I.pair_inputs(cfg, bias_std=0.3, ln_jitter=0.2)
    return cfg, z.astype(np.float64), {k: v.astype(np.float64) for k, v in w.items()}


def tolist(w):
    return {k: v.tolist() for k, v in w.items()}


@pytest.mark.parametrize("outgoing", [True, False])
def test_tri_mul_matches_scalar_loops(outgoing):
    cfg, z, w = tiny()
    p = "tmo." if outgoing else "tmi."
    ref = np.array(brute.tri_mul(z.tolist(), tolist(w), p, outgoing))
    assert np.abs(P.tri_mul(z, w, p, outgoing) - ref).max() < 1e-12


@pytest.mark.parametrize("starting", [True, False])
def test_tri_att_matches_scalar_loops(starting):
    cfg, z, w = tiny()
    p = "tas." if starting else "tae."
    ref = np.array(brute.tri_att(z.tolist(), tolist(w), p, cfg.heads, starting))
    assert np.abs(P.tri_att(z, w, p, cfg.heads, starting) - ref).max() < 1e-12


def test_transition_matches_scalar_loops_and_ffn():
    cfg, z, w = tiny()
    ref = np.array(brute.pair_transition(z.tolist(), tolist(w)))
    got = P.pair_transition(z, w)
    assert np.abs(got - ref).max() < 1e-12
    # the transition is the transformer feed-forward applied to the N*N rows
    wf = {"ln2_g": w["pt.ln_g"], "ln2_b": w["pt.ln_b"], "w_1": w["pt.w_1"], "b_1": w["pt.b_1"],
          "w_2": w["pt.w_2"], "b_2": w["pt.b_2"]}
    n, _, cz = z.shape
    assert np.abs(O.ffn_region(z.reshape(n * n, cz), wf, "relu").reshape(n, n, cz) - got).max() < 1e-13


def test_tri_mul_symmetries_and_einsum():
    cfg, z, w = tiny()
    zt = z.transpose(1, 0, 2)
    # o_in(z)[i,j] = sum_k a[k,i] b[k,j] = o_out(z^T)[i,j], while gate and residual read
    # position [i,j] of their own input: the two forms agree on a symmetric input only.
    w2 = {k.replace("tmo.", "tmi."): v for k, v in w.items() if k.startswith("tmo.")}
    out_t = P.tri_mul(zt, w, "tmo.", True) - zt            # g[j,i]*Lin(LN(o^T[j,i]))
    inc = P.tri_mul(z, w2, "tmi.", False) - z
    zs = z + zt
    a = P.tri_mul(zs, w, "tmo.", True)
    b = P.tri_mul(zs, w2, "tmi.", False)
    assert np.abs(a - b).max() < 1e-12
    assert np.abs(out_t - inc).max() > 1e-6       # and they differ in general
    # a == b (same weights for both operands) makes the outgoing contraction symmetric in i,j
    ws = dict(w)
    for s in ("p", "g"):
        ws["tmo.w_b" + s] = w["tmo.w_a" + s]
        ws["tmo.b_b" + s] = w["tmo.b_a" + s]
    ws["tmo.w_g"] = np.zeros_like(w["tmo.w_g"])
    ws["tmo.b_g"] = np.zeros_like(w["tmo.b_g"])        # gate = 1/2 everywhere
    upd = P.tri_mul(z, ws, "tmo.", True) - z
    assert np.abs(upd - upd.transpose(1, 0, 2)).max() < 1e-12
    # einsum witness of the two contractions
    t = O.layer_norm(z, w["tmo.ln_in_g"], w["tmo.ln_in_b"])
    av = P.sigmoid(O.linear(t, w["tmo.w_ag"], w["tmo.b_ag"])) * O.linear(t, w["tmo.w_ap"], w["tmo.b_ap"])
    bv = P.sigmoid(O.linear(t, w["tmo.w_bg"], w["tmo.b_bg"])) * O.linear(t, w["tmo.w_bp"], w["tmo.b_bp"])
    for outgoing, spec in ((True, "ikc,jkc->ijc"), (False, "kic,kjc->ijc")):
        o = np.einsum(spec, av, bv)
        g = P.sigmoid(O.linear(t, w["tmo.w_g"], w["tmo.b_g"]))
        ref = z + g * O.linear(O.layer_norm(o, w["tmo.ln_out_g"], w["tmo.ln_out_b"]), w["tmo.w_o"], w["tmo.b_o"])
        assert np.abs(P.tri_mul(z, w, "tmo.", outgoing) - ref).max() < 1e-12


def test_tri_att_transpose_symmetry_and_reduction_to_plain_attention():
    cfg, z, w = tiny()
    w2 = {k.replace("tas.", "tae."): v for k, v in w.items() if k.startswith("tas.")}
    zt = np.ascontiguousarray(z.transpose(1, 0, 2))
    end = P.tri_att(z, w2, "tae.", cfg.heads, False)
    start_t = P.tri_att(zt, w, "tas.", cfg.heads, True).transpose(1, 0, 2)
    assert np.abs(end - start_t).max() < 1e-12
    # zero bias projection: each row i of the starting form is plain multi-head attention
    w0 = dict(w)
    w0["tas.w_bias"] = np.zeros_like(w["tas.w_bias"])
    got = P.tri_att(z, w0, "tas.", cfg.heads, True)
    t = O.layer_norm(z, w["tas.ln_g"], w["tas.ln_b"])
    for i in range(z.shape[0]):
        q, k, v = (O.linear(t[i], w["tas.w_" + s]) for s in "qkv")
        ctx = O.attention(q, k, v, cfg.heads, False)
        g = P.sigmoid(O.linear(t[i], w["tas.w_g"], w["tas.b_g"]))
        ref = z[i] + O.linear(g * ctx, w["tas.w_o"], w["tas.b_o"])
        assert np.abs(got[i] - ref).max() < 1e-12
    # with the bias: attention() given bias[h, j, k] = (t W_bias^T)[j, k, h]
    bias = O.linear(t, w["tas.w_bias"]).transpose(2, 0, 1)
    i = 2
    q, k, v = (O.linear(t[i], w["tas.w_" + s]) for s in "qkv")
    ctx = O.attention(q, k, v, cfg.heads, False, bias=bias)
    g = P.sigmoid(O.linear(t[i], w["tas.w_g"], w["tas.b_g"]))
    ref = z[i] + O.linear(g * ctx, w["tas.w_o"], w["tas.b_o"])
    assert np.abs(P.tri_att(z, w, "tas.", cfg.heads, True)[i] - ref).max() < 1e-12


def test_rows_subset_and_chunked_equal_unchunked():
    cfg, z, w = tiny(n=6)
    for name in P.PAIR_MODULES:
        full = P.pair_module(name, z, w, cfg.heads)
        sub = P.pair_module(name, z, w, cfg.heads, rows=[4, 1])
        assert np.abs(sub - full[[4, 1]]).max() < 1e-12, name
        for c in (1, 2, 4, 6, 9):
            got = P.pair_module_chunked(name, z, w, cfg.heads, c)
            assert np.abs(got - full).max() < 1e-12, (name, c)


def test_block_is_the_five_modules_in_order():
    cfg, z, w = tiny()
    zz = z
    zz = np.array(brute.tri_mul(zz.tolist(), tolist(w), "tmo.", True))
    zz = np.array(brute.tri_mul(zz.tolist(), tolist(w), "tmi.", False))
    zz = np.array(brute.tri_att(zz.tolist(), tolist(w), "tas.", cfg.heads, True))
    zz = np.array(brute.tri_att(zz.tolist(), tolist(w), "tae.", cfg.heads, False))
    zz = np.array(brute.pair_transition(zz.tolist(), tolist(w)))
    assert np.abs(P.pair_block(z, w, cfg.heads) - zz).max() < 1e-11


def test_chunking_the_contraction_index_is_illegal():
    cfg, z, w = tiny(n=6)
    full = P.tri_mul(z, w, "tmo.", True)
    # a chunk over k hands each segment half of the k range
    t = O.layer_norm(z, w["tmo.ln_in_g"], w["tmo.ln_in_b"])
    a = P.sigmoid(O.linear(t, w["tmo.w_ag"], w["tmo.b_ag"])) * O.linear(t, w["tmo.w_ap"], w["tmo.b_ap"])
    b = P.sigmoid(O.linear(t, w["tmo.w_bg"], w["tmo.b_bg"])) * O.linear(t, w["tmo.w_bp"], w["tmo.b_bp"])
    o_full = np.einsum("ikc,jkc->ijc", a, b)
    o_seg = [np.einsum("ikc,jkc->ijc", a[:, s], b[:, s]) for s in (slice(0, 3), slice(3, 6))]
    ln = lambda o: O.layer_norm(o, w["tmo.ln_out_g"], w["tmo.ln_out_b"])
    assert np.abs(o_seg[0] + o_seg[1] - o_full).max() < 1e-12      # partial sums add ...
    assert all(np.abs(ln(s) - ln(o_full)).max() > 1e-3 for s in o_seg)  # ... they do not concatenate
    assert full.shape == z.shape
