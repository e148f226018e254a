"""Pins of oracle/unet.py against something other than itself: scalar loops, scipy's correlation,
torch's fp64 group_norm / silu / conv2d, closed forms and special cases."""
import numpy as np
import pytest

from oracle import unet as U


def rng(seed):
    return np.random.default_rng(seed)


def conv_loops(x, w, bias):
    b, h, wd, ci = x.shape
    co = w.shape[0]
    out = np.zeros((b, h, wd, co))
    for n in range(b):
        for i in range(h):
            for j in range(wd):
                for o in range(co):
                    acc = bias[o]
                    for kh in range(3):
                        for kw in range(3):
                            ii, jj = i + kh - 1, j + kw - 1
                            if 0 <= ii < h and 0 <= jj < wd:
                                for c in range(ci):
                                    acc += x[n, ii, jj, c] * w[o, kh, kw, c]
                    out[n, i, j, o] = acc
    return out


def test_conv3x3_equals_scalar_loops():
    r = rng(1)
    x, w, b = r.standard_normal((2, 5, 4, 3)), r.standard_normal((4, 3, 3, 3)), r.standard_normal(4)
    np.testing.assert_allclose(U.conv3x3(x, w, b), conv_loops(x, w, b), rtol=0, atol=1e-12)


def test_conv3x3_equals_scipy_correlation():
    from scipy.signal import correlate2d
    r = rng(2)
    x, w = r.standard_normal((1, 9, 7, 3)), r.standard_normal((2, 3, 3, 3))
    want = np.zeros((9, 7, 2))
    for o in range(2):
        for c in range(3):
            want[:, :, o] += correlate2d(x[0, :, :, c], w[o, :, :, c], mode="same", boundary="fill", fillvalue=0.0)
    np.testing.assert_allclose(U.conv3x3(x, w)[0], want, rtol=0, atol=1e-12)


def test_conv3x3_special_kernels():
    r = rng(3)
    x = r.standard_normal((2, 6, 5, 4))
    centre = np.zeros((4, 3, 3, 4))
    centre[np.arange(4), 1, 1, np.arange(4)] = 1.0
    np.testing.assert_array_equal(U.conv3x3(x, centre), x)
    # a tap at (kh, kw) = (0, 2) reads the pixel one row up and one column to the right; zeros outside
    shift = np.zeros((4, 3, 3, 4))
    shift[np.arange(4), 0, 2, np.arange(4)] = 1.0
    want = np.zeros_like(x)
    want[:, 1:, :-1] = x[:, :-1, 1:]
    np.testing.assert_array_equal(U.conv3x3(x, shift), want)
    # not symmetric in the two window indices, nor in the two channel indices
    w = r.standard_normal((4, 3, 3, 4))
    assert np.abs(U.conv3x3(x, w) - U.conv3x3(x, w.transpose(0, 2, 1, 3))).max() > 0.1
    assert np.abs(U.conv3x3(x, w) - U.conv3x3(x, w.transpose(3, 1, 2, 0))).max() > 0.1


def test_group_norm_equals_torch_and_has_unit_moments():
    import torch
    r = rng(4)
    x = r.standard_normal((3, 5, 7, 12)) * 3 + 1
    gain, shift = r.standard_normal(12), r.standard_normal(12)
    want = torch.nn.functional.group_norm(torch.from_numpy(x).permute(0, 3, 1, 2), 4, torch.from_numpy(gain),
                                          torch.from_numpy(shift), 1e-5).permute(0, 2, 3, 1).numpy()
    np.testing.assert_allclose(U.group_norm(x, gain, shift, 4), want, rtol=0, atol=1e-12)
    n = U.group_norm(x, np.ones(12), np.zeros(12), 4, eps=0.0).reshape(3, 35, 4, 3)
    np.testing.assert_allclose(n.mean(axis=(1, 3)), 0, atol=1e-12)
    np.testing.assert_allclose((n ** 2).mean(axis=(1, 3)), 1, atol=1e-12)
    # groups are runs of consecutive channels: another grouping gives another result
    assert np.abs(U.group_norm(x, gain, shift, 4) - U.group_norm(x, gain, shift, 3)).max() > 1e-3


def test_silu_closed_forms():
    v = np.linspace(-6, 6, 49)
    assert U.silu(0.0) == 0.0
    np.testing.assert_allclose(U.silu(v) - U.silu(-v), v, atol=1e-14)          # v s(v) + v s(-v) = v
    np.testing.assert_allclose(U.silu(np.array([1.0])), 1.0 / (1.0 + np.exp(-1.0)), atol=1e-15)
    assert U.silu(np.array([40.0]))[0] == pytest.approx(40.0) and abs(U.silu(np.array([-40.0]))[0]) < 1e-15


def weights(r, c, jitter=0.3):
    return {"gn1_g": 1 + jitter * r.standard_normal(c), "gn1_b": jitter * r.standard_normal(c),
            "w1": r.standard_normal((c, 3, 3, c)) / np.sqrt(9 * c), "b1": jitter * r.standard_normal(c),
            "gn2_g": 1 + jitter * r.standard_normal(c), "gn2_b": jitter * r.standard_normal(c),
            "w2": r.standard_normal((c, 3, 3, c)) / np.sqrt(9 * c), "b2": jitter * r.standard_normal(c)}


def test_res_block_equals_torch_composition_and_special_cases():
    import torch
    import torch.nn.functional as F
    r = rng(5)
    c, groups = 8, 4
    x, temb, w = r.standard_normal((3, 6, 5, c)), r.standard_normal((3, c)), weights(r, c)
    t = lambda a: torch.from_numpy(np.asarray(a, np.float64))
    xt = t(x).permute(0, 3, 1, 2)
    h = F.conv2d(F.silu(F.group_norm(xt, groups, t(w["gn1_g"]), t(w["gn1_b"]), 1e-5)), t(w["w1"]).permute(0, 3, 1, 2),
                 t(w["b1"]), padding=1) + t(temb)[:, :, None, None]
    y = xt + F.conv2d(F.silu(F.group_norm(h, groups, t(w["gn2_g"]), t(w["gn2_b"]), 1e-5)), t(w["w2"]).permute(0, 3, 1, 2),
                      t(w["b2"]), padding=1)
    np.testing.assert_allclose(U.res_block(x, temb, w, groups), y.permute(0, 2, 3, 1).numpy(), rtol=0, atol=1e-12)
    # images are independent: a subset equals those images of the whole (the legal chunk dim)
    np.testing.assert_array_equal(U.res_block(x, temb, w, groups, images=[2, 0]), U.res_block(x, temb, w, groups)[[2, 0]])
    # with the second convolution switched off the block is the identity
    w0 = dict(w, w2=np.zeros_like(w["w2"]), b2=np.zeros(c))
    np.testing.assert_array_equal(U.res_block(x, temb, w0, groups), x)
    # the embedding enters before the second normalisation, which removes a constant per group: the same value
    # added to every channel changes nothing, different values per channel do
    np.testing.assert_allclose(U.res_block(x, temb + 1.0, w, groups), U.res_block(x, temb, w, groups), rtol=0, atol=1e-11)
    assert np.abs(U.res_block(x, temb + np.arange(c), w, groups) - U.res_block(x, temb, w, groups)).max() > 1e-3


# ---- attention block ---------------------------------------------------------------------------

def attn_weights(r, c, f, scale=0.5):
    w = {"gn_g": 1 + 0.1 * r.standard_normal(c), "gn_b": 0.1 * r.standard_normal(c),
         "ln1_g": 1 + 0.1 * r.standard_normal(c), "ln1_b": 0.1 * r.standard_normal(c),
         "ln2_g": 1 + 0.1 * r.standard_normal(c), "ln2_b": 0.1 * r.standard_normal(c)}
    for name, shp in (("w_in", (c, c)), ("w_qkv", (3 * c, c)), ("w_o", (c, c)), ("w_1", (f, c)), ("w_2", (c, f)), ("w_out", (c, c))):
        w[name] = scale * r.standard_normal(shp) / np.sqrt(shp[1])
        w["b_" + name[2:]] = 0.1 * r.standard_normal(shp[0])
    return w


def attn_block_loops(x, w, groups, heads, eps, context=None, gated=False):
    """The block written out scalar by scalar for one image (pure Python, math.erf / math.exp)."""
    import math
    h, wd, c = x.shape
    n, cg, dh = h * wd, c // groups, c // heads
    xs = [[float(x[i // wd, i % wd, ch]) for ch in range(c)] for i in range(n)]

    def lin(rows, wm, bv):
        return [[bv[o] + sum(row[i] * wm[o][i] for i in range(len(row))) for o in range(len(wm))] for row in rows]

    def ln(rows, g, b):
        out = []
        for row in rows:
            mu = sum(row) / len(row)
            var = sum((v - mu) ** 2 for v in row) / len(row)
            out.append([(v - mu) / math.sqrt(var + eps) * g[i] + b[i] for i, v in enumerate(row)])
        return out

    gn = [[0.0] * c for _ in range(n)]
    for g in range(groups):
        vals = [xs[i][ch] for i in range(n) for ch in range(g * cg, (g + 1) * cg)]
        mu = sum(vals) / len(vals)
        var = sum((v - mu) ** 2 for v in vals) / len(vals)
        for i in range(n):
            for ch in range(g * cg, (g + 1) * cg):
                gn[i][ch] = (xs[i][ch] - mu) / math.sqrt(var + eps) * w["gn_g"][ch] + w["gn_b"][ch]
    t = lin(gn, w["w_in"], w["b_in"])
    qkv = lin(ln(t, w["ln1_g"], w["ln1_b"]), w["w_qkv"], w["b_qkv"])
    ctx = [[0.0] * c for _ in range(n)]
    for hd in range(heads):
        for i in range(n):
            sc = [sum(qkv[i][hd * dh + d] * qkv[j][c + hd * dh + d] for d in range(dh)) / math.sqrt(dh) for j in range(n)]
            mx = max(sc)
            ex = [math.exp(v - mx) for v in sc]
            z = sum(ex)
            for d in range(dh):
                ctx[i][hd * dh + d] = sum(ex[j] / z * qkv[j][2 * c + hd * dh + d] for j in range(n))
    o = lin(ctx, w["w_o"], w["b_o"])
    t2 = [[t[i][ch] + o[i][ch] for ch in range(c)] for i in range(n)]
    gelu = lambda v: 0.5 * v * (1.0 + math.erf(v / math.sqrt(2.0)))
    if context is not None:
        tc = len(context)
        q2 = lin(ln(t2, w["lnc_g"], w["lnc_b"]), w["w_qc"], [0.0] * c)
        kv2 = lin([[float(v) for v in row] for row in context], w["w_kvc"], [0.0] * (2 * c))
        ctx2 = [[0.0] * c for _ in range(n)]
        for hd in range(heads):
            for i in range(n):
                sc = [sum(q2[i][hd * dh + d] * kv2[j][hd * dh + d] for d in range(dh)) / math.sqrt(dh) for j in range(tc)]
                mx = max(sc)
                ex = [math.exp(v - mx) for v in sc]
                z = sum(ex)
                for d in range(dh):
                    ctx2[i][hd * dh + d] = sum(ex[j] / z * kv2[j][c + hd * dh + d] for j in range(tc))
        o2 = lin(ctx2, w["w_oc"], w["b_oc"])
        t2 = [[t2[i][ch] + o2[i][ch] for ch in range(c)] for i in range(n)]
    hid = lin(ln(t2, w["ln2_g"], w["ln2_b"]), w["w_1"], w["b_1"])
    if gated:
        f = len(hid[0]) // 2
        act = [[row[j] * gelu(row[f + j]) for j in range(f)] for row in hid]
    else:
        act = [[gelu(v) for v in row] for row in hid]
    dn = lin(act, w["w_2"], w["b_2"])
    t3 = [[t2[i][ch] + dn[i][ch] for ch in range(c)] for i in range(n)]
    out = lin(t3, w["w_out"], w["b_out"])
    return np.array([[xs[i][ch] + out[i][ch] for ch in range(c)] for i in range(n)]).reshape(h, wd, c)


def test_attn_block_equals_scalar_loops():
    r = rng(20)
    x = r.standard_normal((2, 3, 2, 8))
    w = attn_weights(r, 8, 16)
    got = U.attn_block(x, w, groups=2, heads=2, eps=1e-5)
    for b in range(2):
        np.testing.assert_allclose(got[b], attn_block_loops(x[b], w, 2, 2, 1e-5), rtol=0, atol=1e-12)


def test_attn_block_special_cases():
    r = rng(21)
    x = r.standard_normal((3, 4, 4, 8))
    w = attn_weights(r, 8, 32)
    y = U.attn_block(x, w, groups=4, heads=2)
    # images are independent, and `images` picks them
    np.testing.assert_array_equal(U.attn_block(x, w, 4, 2, images=[2, 0]), y[[2, 0]])
    np.testing.assert_allclose(U.attn_block(x[1:2], w, 4, 2)[0], y[1], rtol=0, atol=1e-13)
    # no op of the block knows where a position lies: permuting the positions permutes the result
    perm = r.permutation(16)
    xp = x.reshape(3, 16, 8)[:, perm].reshape(3, 4, 4, 8)
    np.testing.assert_allclose(U.attn_block(xp, w, 4, 2).reshape(3, 16, 8), y.reshape(3, 16, 8)[:, perm], rtol=0, atol=1e-12)
    # a zero output projection leaves the skip alone
    w0 = dict(w, w_out=np.zeros((8, 8)), b_out=np.zeros(8))
    np.testing.assert_array_equal(U.attn_block(x, w0, 4, 2), x)
    # with the attention's and the feed-forward's output projections zero the transformer block is the
    # identity and what is left is two linear maps of the normalised image
    wi = dict(w, w_o=np.zeros((8, 8)), b_o=np.zeros(8), w_2=np.zeros((8, 32)), b_2=np.zeros(8))
    gn = U.group_norm(x, w["gn_g"], w["gn_b"], 4)
    want = x + np.einsum("bhwc,oc->bhwo", np.einsum("bhwc,oc->bhwo", gn, w["w_in"]) + w["b_in"], w["w_out"]) + w["b_out"]
    np.testing.assert_allclose(U.attn_block(x, wi, 4, 2), want, rtol=0, atol=1e-12)
    # one head or four: different results (the head split is really applied)
    assert np.abs(U.attn_block(x, w, 4, 4) - y).max() > 1e-3


def cross_weights(r, c, d, w):
    w = dict(w)
    w["lnc_g"], w["lnc_b"] = 1 + 0.1 * r.standard_normal(c), 0.1 * r.standard_normal(c)
    w["w_qc"] = 0.5 * r.standard_normal((c, c)) / np.sqrt(c)
    w["w_kvc"] = 0.5 * r.standard_normal((2 * c, d)) / np.sqrt(d)
    w["w_oc"], w["b_oc"] = 0.5 * r.standard_normal((c, c)) / np.sqrt(c), 0.1 * r.standard_normal(c)
    return w


def test_attn_block_with_context_and_gate_equals_scalar_loops():
    r = rng(22)
    x = r.standard_normal((2, 2, 3, 8))
    context = r.standard_normal((2, 5, 6))
    w = cross_weights(r, 8, 6, attn_weights(r, 8, 16))
    wg = dict(w, w_1=0.5 * r.standard_normal((32, 8)) / np.sqrt(8), b_1=0.1 * r.standard_normal(32))
    for ww, ctx, gated in ((w, context, False), (wg, None, True), (wg, context, True)):
        got = U.attn_block(x, ww, groups=2, heads=2, context=ctx, gated=gated)
        for b in range(2):
            want = attn_block_loops(x[b], ww, 2, 2, 1e-5, None if ctx is None else ctx[b], gated)
            np.testing.assert_allclose(got[b], want, rtol=0, atol=1e-12)


def test_attn_block_context_special_cases():
    r = rng(23)
    x = r.standard_normal((3, 4, 2, 8))
    context = r.standard_normal((3, 7, 6))
    w = cross_weights(r, 8, 6, attn_weights(r, 8, 16))
    y = U.attn_block(x, w, 4, 2, context=context)
    # the tokens of a context carry no order; every image meets its own context only
    np.testing.assert_allclose(U.attn_block(x, w, 4, 2, context=context[:, r.permutation(7)]), y, rtol=0, atol=1e-12)
    np.testing.assert_array_equal(U.attn_block(x, w, 4, 2, images=[2, 0], context=context), y[[2, 0]])
    other = context.copy(); other[1] = r.standard_normal((7, 6))
    y2 = U.attn_block(x, w, 4, 2, context=other)
    np.testing.assert_array_equal(y2[[0, 2]], y[[0, 2]])
    assert np.abs(y2[1] - y[1]).max() > 1e-3
    # a context of one token: every query attends to it with weight 1, so the cross-attention adds the same row
    # (that token's value, projected) to every position; with a zero output projection it adds nothing
    one = context[:, :1]
    w0 = dict(w, w_oc=np.zeros((8, 8)), b_oc=np.zeros(8))
    np.testing.assert_allclose(U.attn_block(x, w0, 4, 2, context=one), U.attn_block(x, w, 4, 2), rtol=0, atol=1e-12)
    # gate: a value half that is the constant 1 (zero weights, unit bias) leaves gelu(gate half): the plain block
    ones = dict(w, w_1=np.concatenate([np.zeros((16, 8)), w["w_1"]]), b_1=np.concatenate([np.ones(16), w["b_1"]]))
    np.testing.assert_allclose(U.attn_block(x, ones, 4, 2, gated=True), U.attn_block(x, w, 4, 2), rtol=0, atol=1e-12)
    # ... and the two halves are really multiplied: doubling the value half's weights and bias doubles the hidden rows,
    # which is the same as doubling the down projection's weights
    wg = dict(w, w_1=r.standard_normal((32, 8)) / np.sqrt(8), b_1=0.1 * r.standard_normal(32))
    dbl = dict(wg, w_1=np.concatenate([2 * wg["w_1"][:16], wg["w_1"][16:]]), b_1=np.concatenate([2 * wg["b_1"][:16], wg["b_1"][16:]]))
    np.testing.assert_allclose(U.attn_block(x, dbl, 4, 2, gated=True), U.attn_block(x, dict(wg, w_2=2 * wg["w_2"]), 4, 2, gated=True),
                               rtol=0, atol=1e-11)
