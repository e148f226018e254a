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
