"""fp64 CPU oracle: residual block and attention block of a UNet stage.  Test infrastructure.

The paper (AutoChunk, section 4) evaluates a UNet (stable diffusion) without defining its
modules.  The reading bound here is the residual block of the latent-diffusion UNet, written
channels-last, x [B, H, W, C], one time-embedding vector per image already projected to C
channels, temb [B, C]:

  h = conv3x3(SiLU(GroupNorm(x)); w1) + b1 + temb[:, None, None, :]
  y = x + conv3x3(SiLU(GroupNorm(h)); w2) + b2

GroupNorm: the C channels of an image in `groups` runs of C / groups consecutive channels;
mean and biased variance over a run's channels and all H * W positions, then a gain and a
shift per channel.  SiLU(v) = v * sigmoid(v).  conv3x3: stride 1, zero padding 1, weights
[C_out, 3, 3, C_in]: out[b, h, w, o] = sum_{kh, kw, i} in[b, h + kh - 1, w + kw - 1, i] w[o, kh, kw, i].
Dropout omitted; the input and output channel counts are equal (no skip projection).

Images are independent of each other in every op of the block (section 3.3: the batch dim is
the legal chunk dim; GroupNorm reduces over positions and channels, the convolution over its
window and the input channels), so `images` picks the ones to evaluate.  Nothing is blocked
or reordered; the sum over the nine taps is written out, each tap a matrix product.

The attention block that follows a residual block at the attention resolutions of that UNet
(its "spatial transformer") is read here as: the H * W positions of an image are the tokens,

  t = GroupNorm(x) W_in^T + b_in                  (no activation; a 1x1 convolution is a linear map per position)
  t' = T(t)                                       (the pre-LN transformer block of oracle/transformer.py, non-causal:
                                                   self-attention over the positions of one image, then the feed-forward)
  y = x + t' W_out^T + b_out

Two parts of the published block are optional here.  With a context [B, T_c, D] (one sequence per
image, e.g. an encoded prompt) a cross-attention sits between the self-attention and the feed-forward,

  t'' = t' + attention(LN_c(t') W_qc^T,  context W_kc^T,  context W_vc^T) W_oc^T + b_oc

(queries from the image's positions, keys and values from its context; no biases on the three input
projections; w_kvc stacks W_kc over W_vc), and with `gated` the feed-forward's first layer is 2F wide,

  hidden = (u W_1[:F]^T + b_1[:F]) * gelu(u W_1[F:]^T + b_1[F:])

instead of gelu(u W_1^T + b_1).  Images are independent here too; nothing in the block knows a
position's place in the image, so permuting the positions of x permutes y the same way, and
permuting the tokens of a context changes nothing.
"""
from __future__ import annotations

import numpy as np

from oracle import transformer as _T


def silu(v):
    v = np.asarray(v, np.float64)
    return v / (1.0 + np.exp(-v))


def group_norm(x, gain, shift, groups, eps=1e-5):
    """x [B, H, W, C] -> same shape."""
    x = np.asarray(x, np.float64)
    b, h, w, c = x.shape
    assert c % groups == 0
    g = x.reshape(b, h * w, groups, c // groups)
    mean = g.mean(axis=(1, 3), keepdims=True)
    var = ((g - mean) ** 2).mean(axis=(1, 3), keepdims=True)
    n = ((g - mean) / np.sqrt(var + eps)).reshape(b, h, w, c)
    return n * np.asarray(gain, np.float64) + np.asarray(shift, np.float64)


def conv3x3(x, w, bias=None):
    """x [B, H, W, C_in], w [C_out, 3, 3, C_in] -> [B, H, W, C_out]."""
    x = np.asarray(x, np.float64)
    w = np.asarray(w, np.float64)
    b, h, wd, ci = x.shape
    co = w.shape[0]
    assert w.shape == (co, 3, 3, ci)
    xp = np.zeros((b, h + 2, wd + 2, ci))
    xp[:, 1:h + 1, 1:wd + 1] = x
    out = np.zeros((b, h, wd, co))
    for kh in range(3):
        for kw in range(3):
            out += xp[:, kh:kh + h, kw:kw + wd] @ w[:, kh, kw].T
    if bias is not None:
        out += np.asarray(bias, np.float64)
    return out


def res_block(x, temb, w, groups, eps=1e-5, images=None):
    """y [len(images), H, W, C]; w: gn1_g, gn1_b, w1, b1, gn2_g, gn2_b, w2, b2."""
    x = np.asarray(x, np.float64)
    temb = np.asarray(temb, np.float64)
    if images is not None:
        x, temb = x[np.asarray(images)], temb[np.asarray(images)]
    h = conv3x3(silu(group_norm(x, w["gn1_g"], w["gn1_b"], groups, eps)), w["w1"], w["b1"]) + temb[:, None, None, :]
    return x + conv3x3(silu(group_norm(h, w["gn2_g"], w["gn2_b"], groups, eps)), w["w2"], w["b2"])


ATTN_LAYER_TENSORS = ("ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_o", "b_o", "ln2_g", "ln2_b", "w_1", "b_1", "w_2", "b_2")


def attn_block(x, w, groups, heads, eps=1e-5, images=None, context=None, gated=False):
    """y [len(images), H, W, C]; w: gn_g, gn_b, w_in, b_in, the twelve tensors of a transformer block, w_out, b_out,
    and with a context [B, T_c, D] also lnc_g, lnc_b, w_qc [C, C], w_kvc [2C, D], w_oc, b_oc."""
    x = np.asarray(x, np.float64)
    if images is not None:
        x = x[np.asarray(images)]
        context = None if context is None else np.asarray(context, np.float64)[np.asarray(images)]
    b, h, wd, c = x.shape
    n = h * wd
    t = _T.linear(group_norm(x, w["gn_g"], w["gn_b"], groups, eps).reshape(b * n, c), w["w_in"], w["b_in"])
    layer = {k: w[k] for k in ATTN_LAYER_TENSORS}
    out = np.empty_like(t)
    for i in range(b):
        ti = _T.attention_region(t[i * n:(i + 1) * n], layer, heads, False, eps)
        if context is not None:
            u = _T.layer_norm(ti, w["lnc_g"], w["lnc_b"], eps)
            kv = _T.linear(np.asarray(context[i], np.float64), w["w_kvc"])
            ctx = _T.attention(_T.linear(u, w["w_qc"]), kv[:, :c], kv[:, c:], heads, False)
            ti = ti + _T.linear(ctx, w["w_oc"], w["b_oc"])
        u = _T.layer_norm(ti, w["ln2_g"], w["ln2_b"], eps)
        hid = _T.linear(u, w["w_1"], w["b_1"])
        if gated:
            f = hid.shape[1] // 2
            hid = hid[:, :f] * _T.gelu_erf(hid[:, f:])
        else:
            hid = _T.gelu_erf(hid)
        out[i * n:(i + 1) * n] = ti + _T.linear(hid, w["w_2"], w["b_2"])
    return x + _T.linear(out, w["w_out"], w["b_out"]).reshape(b, h, wd, c)
