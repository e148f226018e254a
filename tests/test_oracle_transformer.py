"""Pins of the fp64 transformer oracle (no GPU): brute force, library witnesses,
closed forms, invariants, and chunked == unchunked for every legal chunk."""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import brute
from oracle import transformer as O
from paper_2401_10652_amd import inputs as I


def tiny(seq=7, d=8, heads=2, f=12, causal=False, layers=1, idx=11):
    cfg = I.TransformerConfig("tiny", idx, layers, seq, d, heads, f, causal, "f32", None)
    x, ls = I.transformer_inputs(cfg, bias_std=0.3, ln_jitter=0.2)
    return cfg, x.astype(np.float64), [{k: v.astype(np.float64) for k, v in w.items()} for w in ls]


def tolist(w):
    return {k: v.tolist() for k, v in w.items()}


@pytest.mark.parametrize("causal", [False, True])
def test_block_matches_scalar_loops(causal):
    cfg, x, ls = tiny(causal=causal)
    got = O.transformer_block(x, ls[0], cfg.heads, causal)
    ref = np.array(brute.transformer_block(x.tolist(), tolist(ls[0]), cfg.heads, causal))
    assert np.abs(got - ref).max() < 1e-12


def test_layer_norm_library_and_invariants():
    r = np.random.default_rng(1)
    x = r.standard_normal((5, 16)) * 3 + 1
    g, b = r.standard_normal(16), r.standard_normal(16)
    ref = F.layer_norm(torch.from_numpy(x), (16,), torch.from_numpy(g), torch.from_numpy(b), 1e-5).numpy()
    assert np.abs(O.layer_norm(x, g, b) - ref).max() < 1e-13
    n = O.layer_norm(x, np.ones(16), np.zeros(16), 1e-5)
    var = x.var(axis=1)
    assert np.abs(n.mean(axis=1)).max() < 1e-14
    assert np.abs(n.var(axis=1) - var / (var + 1e-5)).max() < 1e-12


def test_gelu_closed_forms():
    xs = np.linspace(-6, 6, 241)
    assert O.gelu_erf(np.array([0.0]))[0] == 0.0
    assert np.abs(O.gelu_erf(xs) - O.gelu_erf(-xs) - xs).max() < 1e-14
    assert abs(O.gelu_erf(np.array([9.0]))[0] - 9.0) < 1e-15
    ref = np.array([0.5 * v * (1 + math.erf(v / math.sqrt(2))) for v in xs])
    assert np.abs(O.gelu_erf(xs) - ref).max() < 1e-15
    t = F.gelu(torch.from_numpy(xs), approximate="tanh").numpy()
    assert np.abs(O.gelu_tanh(xs) - t).max() < 1e-14
    assert np.abs(O.gelu_tanh(xs) - O.gelu_erf(xs)).max() < 2e-3   # the two variants differ
    assert np.abs(O.gelu_tanh(xs) - O.gelu_erf(xs)).max() > 1e-5


def test_linear_library_witness():
    r = np.random.default_rng(2)
    x, w, b = r.standard_normal((4, 6)), r.standard_normal((5, 6)), r.standard_normal(5)
    ref = F.linear(torch.from_numpy(x), torch.from_numpy(w), torch.from_numpy(b)).numpy()
    assert np.abs(O.linear(x, w, b) - ref).max() < 1e-14
    assert O.linear(x, w).shape == (4, 5)


@pytest.mark.parametrize("causal", [False, True])
def test_attention_library_witness(causal):
    r = np.random.default_rng(3)
    s, h, dh = 9, 3, 4
    q, k, v = (r.standard_normal((s, h * dh)) for _ in range(3))
    tq, tk, tv = (torch.from_numpy(a).reshape(s, h, dh).transpose(0, 1) for a in (q, k, v))
    ref = F.scaled_dot_product_attention(tq, tk, tv, is_causal=causal).transpose(0, 1).reshape(s, h * dh).numpy()
    got = O.attention(q, k, v, h, causal)
    assert np.abs(got - ref).max() < 1e-13
    # evaluating a few query rows at a time changes nothing
    assert np.abs(O.attention(q, k, v, h, causal, query_block=4) - got).max() < 1e-14
    bias = r.standard_normal((h, s, s))
    refb = F.scaled_dot_product_attention(tq, tk, tv, attn_mask=torch.from_numpy(bias)).transpose(0, 1).reshape(s, h * dh).numpy()
    assert np.abs(O.attention(q, k, v, h, False, bias=bias) - refb).max() < 1e-13
    assert np.abs(np.array(brute.attention(q.tolist(), k.tolist(), v.tolist(), h, causal)) - got).max() < 1e-13


def test_softmax_invariants():
    r = np.random.default_rng(4)
    s = r.standard_normal((6, 11)) * 5
    p = O.softmax_rows(s)
    assert np.abs(p.sum(axis=1) - 1).max() < 1e-15
    assert np.abs(O.softmax_rows(s + 123.0) - p).max() < 1e-13
    s[:, 7:] = -np.inf
    p = O.softmax_rows(s)
    assert np.all(p[:, 7:] == 0) and np.abs(p.sum(axis=1) - 1).max() < 1e-15


def test_attention_special_cases():
    cfg, x, ls = tiny(seq=6, causal=True)
    w = dict(ls[0])
    d = cfg.d_model
    r = np.random.default_rng(5)
    q0 = np.zeros((6, d))
    k, v = r.standard_normal((6, d)), r.standard_normal((6, d))
    # zero queries -> uniform weights: mean of v (non-causal) / prefix mean (causal)
    assert np.abs(O.attention(q0, k, v, cfg.heads, False) - v.mean(axis=0)).max() < 1e-14
    pm = np.cumsum(v, axis=0) / np.arange(1, 7)[:, None]
    assert np.abs(O.attention(q0, k, v, cfg.heads, True) - pm).max() < 1e-14
    # causal: row 0 attends to itself only
    q = r.standard_normal((6, d))
    assert np.abs(O.attention(q, k, v, cfg.heads, True)[0] - v[0]).max() < 1e-15
    # causal block: changing a later input row leaves earlier output rows bit-identical
    y = O.transformer_block(x, w, cfg.heads, True)
    x2 = x.copy()
    x2[4] += 1.0
    y2 = O.transformer_block(x2, w, cfg.heads, True)
    assert np.array_equal(y[:4], y2[:4]) and not np.array_equal(y[4:], y2[4:])
    # non-causal block is permutation-equivariant over tokens
    perm = r.permutation(6)
    yn = O.transformer_block(x, w, cfg.heads, False)
    assert np.abs(O.transformer_block(x[perm], w, cfg.heads, False) - yn[perm]).max() < 1e-12
    # q_offset: a query slice placed at its absolute position equals the slice of the whole
    full = O.attention(q, k, v, cfg.heads, True)
    assert np.abs(O.attention(q[2:5], k, v, cfg.heads, True, q_offset=2) - full[2:5]).max() < 1e-14


def test_stack_and_batch():
    cfg, x, ls = tiny(seq=5, layers=3, causal=True)
    y = O.transformer_stack(x, ls, cfg.heads, True)
    z = x
    for w in ls:
        z = np.array(brute.transformer_block(z.tolist(), tolist(w), cfg.heads, True))
    assert np.abs(y - z).max() < 1e-11
    xb = np.concatenate([x, x[::-1]], axis=0)
    yb = O.transformer_stack(xb, ls, cfg.heads, True, batch=2)
    assert np.array_equal(yb[:5], y)
    assert np.abs(yb[5:] - O.transformer_stack(x[::-1], ls, cfg.heads, True)).max() == 0


@pytest.mark.parametrize("causal", [False, True])
def test_chunked_equals_unchunked_every_legal_length(causal):
    cfg, x, ls = tiny(seq=10, causal=causal)
    ref = O.transformer_block(x, ls[0], cfg.heads, causal)
    for c in (1, 2, 3, 4, 7, 10, 13):
        got = O.transformer_block_chunked(x, ls[0], cfg.heads, causal, c, c, c)
        assert np.abs(got - ref).max() < 1e-12, c
    got = O.transformer_block_chunked(x, ls[0], cfg.heads, causal, 3, 10, 4)
    assert np.abs(got - ref).max() < 1e-12


def test_illegal_chunk_dims_change_the_output():
    cfg, x, ls = tiny(seq=8)
    w = ls[0]
    r = np.random.default_rng(6)
    d = cfg.d_model
    q, k, v = (r.standard_normal((8, d)) for _ in range(3))
    ref = O.attention(q, k, v, cfg.heads, False)
    assert np.abs(O.attention_chunked_over_keys(q, k, v, cfg.heads, 4) - ref).max() > 1e-3
    y = O.ffn_region(x, w) - x
    parts = O.ffn_chunked_over_hidden(x, w, 6)
    assert all(np.abs(p - y).max() > 1e-3 for p in parts)
    # layer norm over a split feature dim is not the layer norm of the whole row
    a = O.layer_norm(x, w["ln1_g"], w["ln1_b"])
    b = np.concatenate([O.layer_norm(x[:, :4], w["ln1_g"][:4], w["ln1_b"][:4]),
                        O.layer_norm(x[:, 4:], w["ln1_g"][4:], w["ln1_b"][4:])], axis=1)
    assert np.abs(a - b).max() > 1e-3


@pytest.mark.parametrize("causal", [False, True])
def test_block_rows_equals_rows_of_block(causal):
    cfg, x, ls = tiny(seq=12, causal=causal)
    full = O.transformer_block(x, ls[0], cfg.heads, causal)
    for r0, r1 in ((0, 3), (5, 9), (11, 12), (0, 12)):
        got = O.transformer_block_rows(x, ls[0], cfg.heads, causal, r0, r1)
        assert np.abs(got - full[r0:r1]).max() < 1e-12
    blocks = [(0, 3), (5, 9), (11, 12)]
    for (r0, r1), got in zip(blocks, O.transformer_block_row_blocks(x, ls[0], cfg.heads, causal, blocks)):
        assert got.shape[0] == r1 - r0 and np.abs(got - full[r0:r1]).max() < 1e-12
