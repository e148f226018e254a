"""Pins of the paper-style activation-memory model: byte counts worked by hand from the
two activation equations of section 2 for the five workloads."""
from oracle import memory_model as M

KIB, MIB, GIB = 1 << 10, 1 << 20, 1 << 30


def test_attention_region_hand_counts():
    # C1 fp32 S=256 d=64 H=4: x 64 KiB + qkv 192 KiB + ctx 64 KiB + 2 * (4*256*256*4 B = 1 MiB)
    assert M.attention_region(256, 64, 4, 4) == (64 + 192 + 64 + 2048) * KIB
    # four segments of 64 rows: the score part divides by 4
    assert M.attention_region(256, 64, 4, 4, 64) == (64 + 192 + 64 + 512) * KIB
    # C2 bf16 S=8192 d=1024 H=16: 16 + 48 + 16 MiB + 2 * 2 GiB
    assert M.attention_region(8192, 1024, 16, 2) == (16 + 48 + 16 + 4096) * MIB
    assert M.attention_region(8192, 1024, 16, 2, 1024) == (16 + 48 + 16 + 512) * MIB
    # C3 bf16 S=4096 d=768 H=12: 6 + 18 + 6 MiB + 2 * 384 MiB; 512-row segments: 2 * 48 MiB
    assert M.attention_region(4096, 768, 12, 2) == (6 + 18 + 6 + 768) * MIB
    assert M.attention_region(4096, 768, 12, 2, 512) == (6 + 18 + 6 + 96) * MIB
    # C5 bf16 S=65536 d=2048 H=16: 256 + 768 + 256 MiB + 2 * 128 GiB
    assert M.attention_region(65536, 2048, 16, 2) == (256 + 768 + 256) * MIB + 256 * GIB
    assert M.attention_region(65536, 2048, 16, 2, 1024) == (256 + 768 + 256) * MIB + 4 * GIB


def test_intermediate_part_scales_as_one_over_n():
    base = M.attention_region(4096, 768, 12, 2, 4096) - 30 * MIB
    for n in (2, 4, 8, 16):
        part = M.attention_region(4096, 768, 12, 2, 4096 // n) - 30 * MIB
        assert part * n == base
    # n = 1 reproduces the unchunked equation, and the total never grows with n
    assert M.attention_region(4096, 768, 12, 2, 4096) == M.attention_region(4096, 768, 12, 2)
    vals = [M.ffn_region(4096, 768, 3072, 2, c) for c in (4096, 2048, 512, 64, 1)]
    assert vals == sorted(vals, reverse=True)


def test_ffn_and_qkv_hand_counts():
    # C2: h 16 + y 16 + u 16 + two copies of the 64 MiB hidden
    assert M.ffn_region(8192, 1024, 4096, 2) == (16 + 16 + 16 + 128) * MIB
    assert M.ffn_region(8192, 1024, 4096, 2, 1024) == (16 + 16 + 2 + 16) * MIB
    assert M.qkv_region(8192, 1024, 2) == (16 + 48 + 16) * MIB
    # output projection: x, ctx, h whole (16 MiB each) + the projection before the residual
    assert M.out_proj_region(8192, 1024, 2) == (48 + 16) * MIB
    assert M.out_proj_region(8192, 1024, 2, 1024) == (48 + 2) * MIB
    assert M.transformer_layer_peak(8192, 1024, 16, 4096, 2) == (16 + 48 + 16 + 4096) * MIB


def test_pair_stack_hand_counts():
    # C4 bf16 N=1024 cz=128, 4 heads x 32: z, z' 256 MiB each; k, v 256 MiB each; bias 8 MiB;
    # per row: t, q, g, o 256 KiB each; scores 4*1024*1024*2 B = 8 MiB
    whole = (256 * 2 + 256 * 2 + 8) * MIB
    assert M.tri_att_region(1024, 128, 4, 32, 2) == whole + (256 * 4 + 8192) * MIB
    assert M.tri_att_region(1024, 128, 4, 32, 2, 64) == whole + (16 * 4 + 512) * MIB
    assert M.tri_mul_region(1024, 128, 128, 2) == (256 * 4 + 256 * 4) * MIB
    assert M.tri_mul_region(1024, 128, 128, 2, 64) == (256 * 4 + 16 * 4) * MIB
    assert M.pair_transition_region(1024, 128, 4, 2) == (256 * 2 + 256 + 2048) * MIB
    assert M.pair_transition_region(1024, 128, 4, 2, 64) == (256 * 2 + 16 + 128) * MIB


def test_budget_sizing():
    fits = lambda c: M.attention_region(8192, 1024, 16, 2, c) <= 1 * GIB
    # 80 MiB whole + c * 512 KiB <= 1024 MiB  ->  c <= 1888  -> largest multiple of 128 is 1792
    assert M.largest_chunk_len(8192, 128, fits) == 1792
    assert M.largest_chunk_len(8192, 128, lambda c: True) == 8192
    assert M.largest_chunk_len(8192, 128, lambda c: False) == 0
    fits5 = lambda c: M.attention_region(65536, 2048, 16, 2, c) <= 4 * GIB
    # 1280 MiB whole + c * 4 MiB <= 4096 MiB -> c <= 704 -> 640
    assert M.largest_chunk_len(65536, 128, fits5) == 640
    assert M.ffn_region(65536, 2048, 8192, 2) <= 4 * GIB   # the feed-forward fits unchunked
