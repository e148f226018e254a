"""The seeded generator: published splitmix64 test vector, moments, bf16 rounding."""
import numpy as np

from paper_2401_10652_amd import inputs as I


def test_splitmix64_reference_vector():
    # First outputs of splitmix64 seeded with 0 (state advances by the golden gamma before
    # mixing), as listed with the public-domain reference implementation by S. Vigna.
    gamma = 0x9E3779B97F4A7C15
    ctr = np.array([(i * gamma) & 0xFFFFFFFFFFFFFFFF for i in range(3)], dtype=np.uint64)
    got = [int(v) for v in I.splitmix64(ctr)]
    assert got == [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F]


def test_normal_moments_and_random_access():
    v = I.standard_normal(12345, 400000)
    assert abs(v.mean()) < 0.01 and abs(v.std() - 1.0) < 0.01
    assert abs((v ** 3).mean()) < 0.03 and abs((v ** 4).mean() - 3.0) < 0.1
    w = I.standard_normal(12345, 1000, start=777)
    assert np.array_equal(w, v[777:1777])
    assert not np.array_equal(I.standard_normal(12346, 1000), v[:1000])


def test_bf16_rounding_ties_to_even():
    import torch
    x = np.array([1.0, 1.0 + 2 ** -8, 1.0 + 2 ** -7, 1.0 + 3 * 2 ** -8, -3.14159, 1e-30, 65504.0],
                 np.float32)
    ref = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(I.round_to_bf16(x), ref)
    r = np.random.default_rng(0).standard_normal(100000).astype(np.float32)
    ref = torch.from_numpy(r).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(I.round_to_bf16(r), ref)
    bits = I.bf16_bits(ref)
    back = (bits.astype(np.uint32) << 16).view(np.float32)
    assert np.array_equal(back, ref)


def test_recipes_shapes_and_stats():
    x, layers = I.transformer_inputs(I.C1)
    assert x.shape == (256, 64) and len(layers) == 1
    w = layers[0]
    assert w["w_qkv"].shape == (192, 64) and w["w_1"].shape == (256, 64) and w["w_2"].shape == (64, 256)
    assert abs(w["w_1"].std() - 1 / 8) < 0.01 and abs(w["w_2"].std() - 1 / 16) < 0.005
    assert np.all(w["ln1_g"] == 1) and np.all(w["b_1"] == 0)
    cfg = I.TransformerConfig("t", 7, 2, 16, 32, 2, 64, True, "bf16", 0.02)
    x, layers = I.transformer_inputs(cfg, bias_std=0.02, ln_jitter=0.1)
    assert np.array_equal(I.round_to_bf16(x), x)
    assert abs(layers[1]["w_qkv"].std() - 0.02) < 0.002
    assert layers[0]["b_qkv"].std() > 0 and not np.array_equal(layers[0]["w_o"], layers[1]["w_o"])
    pc = I.PairConfig("p", 8, 6, 8, 8, 2, 4, 4, "bf16")
    z, pw = I.pair_inputs(pc)
    assert z.shape == (6, 6, 8) and pw["tas.w_bias"].shape == (2, 8) and pw["pt.w_1"].shape == (32, 8)
