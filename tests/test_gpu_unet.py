"""GPU parity of the UNet stage: the residual block's two kernels alone, and whole chunk plans of residual blocks
and of residual + attention blocks against the fp64 oracle, through the C-ABI."""
import numpy as np
import pytest

from oracle import unet as U
from paper_2401_10652_amd import inputs as I
from util import check, draw, host

pytestmark = pytest.mark.gpu

CANARY = 0x5A


@pytest.fixture(scope="module")
def B():
    from paper_2401_10652_amd import binding
    binding.lib()
    return binding


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("images,h,w,c,groups,act", [(2, 9, 7, 64, 8, "silu"), (3, 16, 16, 320, 32, "silu"),
                                                     (1, 5, 3, 24, 3, "none"), (2, 1, 1, 16, 2, "none"),
                                                     (1, 6, 5, 2304, 32, "silu")])
def test_group_norm(B, dtype, images, h, w, c, groups, act):
    """Groups of 10 channels straddle the 8-channel vectors; 63 positions do not divide into the 64 shares;
    a single position leaves most shares empty; rows of 2304 channels take the kernel that reads a group's
    channels only."""
    import torch
    x = draw((images, h, w, c), 50, dtype) * 2.0 + 0.5
    x = I.round_to_storage(x, dtype)
    gain, shift = draw((c,), 51, dtype) * 0.3 + 1.0, draw((c,), 52, dtype) * 0.3
    gain, shift = I.round_to_storage(gain, dtype), I.round_to_storage(shift, dtype)
    dx = B.to_device(x, dtype)
    y = torch.full_like(dx, float("nan"))
    need = B.ac_group_norm_workspace_bytes(images, groups)
    ws = torch.full((need + 256,), CANARY, dtype=torch.uint8, device="cuda")
    B.ac_op_group_norm(dx, B.to_device(gain, dtype), B.to_device(shift, dtype), y, ws[:need], groups,
                       activation=B.AC_ACT_SILU if act == "silu" else B.AC_ACT_NONE)
    torch.cuda.synchronize()
    assert bool((ws[need:] == CANARY).all())
    ref = U.group_norm(x, gain, shift, groups)
    check(host(y), U.silu(ref) if act == "silu" else ref, dtype)
    with pytest.raises(B.AcError) as ei:
        B.ac_op_group_norm(dx, B.to_device(gain, dtype), B.to_device(shift, dtype), y, ws[:16], groups)
    assert ei.value.status == B.AC_ERR_WORKSPACE


@pytest.mark.parametrize("images,h,w,ci,co,per_image,resid", [(2, 5, 7, 64, 72, True, False), (1, 16, 16, 128, 320, False, True),
                                                              (3, 8, 8, 64, 64, True, True), (1, 1, 1, 64, 8, False, False),
                                                              (2, 13, 1, 192, 136, True, True)])
def test_conv3x3(B, images, h, w, ci, co, per_image, resid):
    """Borders on every side, one-pixel and one-column images (most window positions outside), output channels that
    end inside a tile, a bias per image, the skip."""
    import torch
    x = draw((images, h, w, ci), 60, "bf16")
    wt = draw((co, 3, 3, ci), 61, "bf16", std=1.0 / np.sqrt(9 * ci))
    bias = draw((images, co) if per_image else (co,), 62, "bf16", std=0.5)
    res = draw((images, h, w, co), 63, "bf16") if resid else None
    out = torch.full((images, h, w, co), float("nan"), dtype=torch.bfloat16, device="cuda")
    B.ac_op_conv3x3(B.to_device(x, "bf16"), B.to_device(wt, "bf16"), out, bias=B.to_device(bias, "bf16"),
                    bias_per_image=per_image, residual=None if res is None else B.to_device(res, "bf16"))
    torch.cuda.synchronize()
    ref = U.conv3x3(x, wt) + (bias[:, None, None, :] if per_image else bias)
    if resid:
        ref = ref + res
    check(host(out), ref, "bf16")


def test_conv3x3_refuses_what_it_cannot_do(B):
    import torch
    x = torch.zeros((1, 4, 4, 32), dtype=torch.bfloat16, device="cuda")
    wt = torch.zeros((8, 3, 3, 32), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(B.AcError) as ei:
        B.ac_op_conv3x3(x, wt, torch.zeros((1, 4, 4, 8), dtype=torch.bfloat16, device="cuda"))
    assert ei.value.status == B.AC_ERR_UNSUPPORTED


def run_stack(B, cfg, chunk, flags=0, budget=0, bias_std=0.2, gn_jitter=0.2):
    import torch
    x, layers = I.res_stack_inputs(cfg, bias_std=bias_std, gn_jitter=gn_jitter)
    dx = B.to_device(x, cfg.dtype)
    dw = [B.to_device(w[n].reshape(w[n].shape[0], -1) if w[n].ndim == 4 else w[n], cfg.dtype) for w in layers for n in I.RES_BLOCK_TENSORS]
    regs = [] if chunk is None else [(B.AC_REGION_RES_BLOCK, B.AC_DIM_BATCH, chunk)]
    p = B.Plan(B.res_stack_desc(cfg, flags=flags), regs, budget)
    info = p.ac_plan_query()
    assert p.weight_names() == [f"R{l}.{n}" for l in range(cfg.layers) for n in I.RES_BLOCK_TENSORS]
    p.ac_plan_bind_weights(dw)
    need = int(info.workspace_bytes)
    ws = torch.full((need + 4096,), CANARY, dtype=torch.uint8, device="cuda")
    y = torch.full_like(dx, float("nan"))
    peak = p.ac_execute(dx, y, ws[:need])
    torch.cuda.synchronize()
    assert bool((ws[need:] == CANARY).all())
    assert torch.equal(dx, B.to_device(x, cfg.dtype))
    assert peak == info.peak_bytes_planned
    p.close()
    return x, layers, y, info


def oracle_stack(cfg, x, layers):
    y = x
    for w in layers:
        y = U.res_block(y, w["temb"], w, cfg.groups, cfg.eps)
    return y


@pytest.mark.parametrize("layers,batch,h,w,c,groups", [(1, 5, 12, 10, 64, 8), (2, 4, 16, 16, 128, 32), (3, 3, 8, 8, 320, 32)])
def test_res_stack_chunked_equals_oracle(B, layers, batch, h, w, c, groups):
    import torch
    cfg = I.ResStackConfig("tu", 46, layers, batch, h, w, c, groups)
    outs = []
    ref = None
    for chunk in (batch, 1, 2, 3):
        x, lw, y, info = run_stack(B, cfg, chunk)
        if ref is None:
            ref = oracle_stack(cfg, x, lw)
        assert info.regions[0].n_segments == -(-batch // min(chunk, batch))
        check(host(y), ref, "bf16", what=f"{chunk} images per segment", depth=layers)
        outs.append((y, info))
    for y, _ in outs[1:]:
        assert torch.equal(y, outs[0][0])          # images never meet: every chunk length gives the same bits
    # a segment holds two tensors of its images: by hand
    al = lambda n: (n + 255) // 256 * 256
    img = h * w * c * 2
    whole = (al(batch * img) if layers > 1 else 0) + (al(batch * img) if layers > 2 else 0) + al(batch * c * 2) + \
        al(batch * groups * 64 * 3 * 4)
    for chunk, (_, info) in zip((batch, 1, 2, 3), outs):
        assert info.workspace_bytes == whole + 2 * al(min(chunk, batch) * img)
        assert info.peak_bytes_model == 2 * batch * img + 7 * min(chunk, batch) * img
    _, _, y2, info2 = run_stack(B, cfg, 1, flags=B.AC_FLAG_TWO_SEGMENTS_IN_FLIGHT)
    assert torch.equal(y2, outs[0][0]) and info2.workspace_bytes == whole + 4 * al(img)


def test_res_stack_budget_and_legality(B):
    cfg = I.ResStackConfig("tub", 47, 2, 6, 8, 8, 64, 8)
    img = 8 * 8 * 64 * 2
    x, lw, y1, i1 = run_stack(B, cfg, None)
    assert i1.regions[0].n_segments == 1
    budget = i1.peak_bytes_planned - 6 * img        # room for two tensors of 3 images instead of 6
    _, _, yb, ib = run_stack(B, cfg, 0, budget=budget)
    assert ib.regions[0].chunk_len == 3 and ib.peak_bytes_planned <= budget
    import torch
    assert torch.equal(yb, y1)
    check(host(yb), oracle_stack(cfg, x, lw), "bf16", depth=2)
    for dim in (B.AC_DIM_SEQ, B.AC_DIM_FEATURE):
        with pytest.raises(B.AcError) as ei:
            B.Plan(B.res_stack_desc(cfg), [(B.AC_REGION_RES_BLOCK, dim, 4)])
        assert ei.value.status == B.AC_ERR_ILLEGAL_CHUNK_DIM
    with pytest.raises(B.AcError) as ei:
        B.Plan(B.res_stack_desc(I.ResStackConfig("bad", 48, 1, 2, 8, 8, 48, 8)), [])
    assert ei.value.status == B.AC_ERR_UNSUPPORTED


# ---- residual block + attention block ------------------------------------------------------------

def stage_tensors(cfg):
    return list(I.RES_BLOCK_TENSORS) + list(I.attn_block_tensors(cfg))


def run_stage(B, cfg, chunk_res, chunk_attn, flags=0, budget=0, inputs=None):
    """A plan of the stage (each layer: residual block, then attention block) with its two regions' chunk lengths."""
    import torch
    x, layers = inputs if inputs is not None else I.res_stack_inputs(cfg, bias_std=0.2, gn_jitter=0.2)
    dx = B.to_device(x, cfg.dtype)
    flat = lambda t: t.reshape(t.shape[0], -1) if t.ndim == 4 else t.reshape(-1, t.shape[-1]) if t.ndim == 3 else t
    dw = [B.to_device(flat(w[n]), cfg.dtype) for w in layers for n in stage_tensors(cfg)]
    regs = []
    if chunk_res is not None:
        regs.append((B.AC_REGION_RES_BLOCK, B.AC_DIM_BATCH, chunk_res))
    if chunk_attn is not None:
        regs.append((B.AC_REGION_UNET_ATTN, B.AC_DIM_BATCH, chunk_attn))
    p = B.Plan(B.res_stack_desc(cfg, flags=flags), regs, budget)
    info = p.ac_plan_query()
    assert p.weight_names() == [f"{'R' if n in I.RES_BLOCK_TENSORS else 'A'}{l}.{n}" for l in range(cfg.layers) for n in stage_tensors(cfg)]
    p.ac_plan_bind_weights(dw)
    need = int(info.workspace_bytes)
    ws = torch.full((need + 4096,), CANARY, dtype=torch.uint8, device="cuda")
    y = torch.full_like(dx, float("nan"))
    peak = p.ac_execute(dx, y, ws[:need])
    torch.cuda.synchronize()
    assert bool((ws[need:] == CANARY).all())
    assert peak == info.peak_bytes_planned
    p.close()
    return x, layers, y, info


def oracle_stage(cfg, x, layers):
    y = x
    for w in layers:
        y = U.res_block(y, w["temb"], w, cfg.groups, cfg.eps)
        y = U.attn_block(y, w, cfg.groups, cfg.heads, cfg.eps, context=w.get("context"), gated=cfg.gated)
    return y


@pytest.mark.parametrize("layers,batch,h,w,c,groups,heads,f", [(1, 3, 8, 8, 64, 8, 2, 128), (2, 4, 16, 8, 128, 32, 2, 256),
                                                              (1, 2, 16, 16, 320, 32, 5, 640), (1, 2, 8, 8, 128, 16, 1, 64)])
def test_stage_with_attention_chunked_equals_oracle(B, layers, batch, h, w, c, groups, heads, f):
    """Heads of 32, 64 and 128 channels; every chunk length of the two regions gives the same bits, because images
    never meet (the attention of an image sees its own positions only)."""
    import torch
    cfg = I.ResStackConfig("tua", 49, layers, batch, h, w, c, groups, heads=heads, d_ffn=f)
    x, lw, y1, i1 = run_stage(B, cfg, None, None)
    assert [i1.regions[k].n_segments for k in range(2)] == [1, 1]
    ref = oracle_stage(cfg, x, lw)
    check(host(y1), ref, "bf16", what="one segment per region", depth=2 * layers)
    for cr, ca in ((1, 1), (2, 1), (batch, 2), (3, batch)):
        _, _, y, info = run_stage(B, cfg, cr, ca, inputs=(x, lw))
        assert info.regions[1].n_segments == -(-batch // min(ca, batch)) and info.regions[1].kind == B.AC_REGION_UNET_ATTN
        assert torch.equal(y, y1), (cr, ca)
        if ca < batch:      # the attention block's segment is the larger of the two
            assert info.peak_bytes_planned < i1.peak_bytes_planned
    _, _, y2, _ = run_stage(B, cfg, 1, 1, flags=B.AC_FLAG_TWO_SEGMENTS_IN_FLIGHT, inputs=(x, lw))
    assert torch.equal(y2, y1)


def test_stage_with_attention_bytes_and_legality(B):
    cfg = I.ResStackConfig("tub2", 50, 1, 4, 8, 8, 64, 8, heads=2, d_ffn=128)
    al = lambda n: (n + 255) // 256 * 256
    hw, c, f, e = 64, 64, 128, 2
    img = hw * c * e
    _, _, _, info = run_stage(B, cfg, 4, 1)
    # whole: one buffer between the two blocks, the bias + embedding table, the GroupNorm statistics; the attention
    # block's segment of one image holds u, t, q|k (two), v^T, the context and the hidden rows; the residual block's
    # segment of four images two tensors
    whole = al(4 * img) + al(4 * c * e) + al(4 * 8 * 64 * 3 * 4)
    attn_seg = 2 * al(img) + al(2 * img) + 2 * al(img) + al(hw * f * e)
    res_seg = 2 * al(4 * img)
    assert info.workspace_bytes == whole + max(attn_seg, res_seg)
    assert info.regions[1].model_bytes == 2 * 4 * img + 13 * img + 2 * hw * f * e + 2 * 2 * hw * hw * e
    for dim in (B.AC_DIM_SEQ, B.AC_DIM_FEATURE):
        with pytest.raises(B.AcError) as ei:
            B.Plan(B.res_stack_desc(cfg), [(B.AC_REGION_UNET_ATTN, dim, 1)])
        assert ei.value.status == B.AC_ERR_ILLEGAL_CHUNK_DIM
    # heads of 48 channels have no attention kernel here; without heads the region kind does not exist
    with pytest.raises(B.AcError) as ei:
        B.Plan(B.res_stack_desc(I.ResStackConfig("bad", 51, 1, 2, 8, 8, 192, 8, heads=4, d_ffn=128)), [])
    assert ei.value.status == B.AC_ERR_UNSUPPORTED
    with pytest.raises(B.AcError) as ei:
        B.Plan(B.res_stack_desc(I.ResStackConfig("bad", 52, 1, 2, 8, 8, 64, 8)), [(B.AC_REGION_UNET_ATTN, B.AC_DIM_BATCH, 1)])
    assert ei.value.status == B.AC_ERR_ARG
    # a budget sizes the attention block's segments
    _, _, y1, i1 = run_stage(B, cfg, None, None)
    budget = i1.peak_bytes_planned - 2 * attn_seg
    _, _, yb, ib = run_stage(B, cfg, 4, 0, budget=budget)
    import torch
    assert ib.regions[1].chunk_len < 4 and ib.peak_bytes_planned <= budget and torch.equal(yb, y1)


@pytest.mark.parametrize("tc,d,gated", [(77, 768, True), (5, 48, False), (64, 128, True), (1, 8, False), (130, 64, False)])
def test_stage_with_cross_attention_and_gate_equals_oracle(B, tc, d, gated):
    """The attention block with a context per image (77 tokens of width 768 as in the published model; fewer tokens
    than one key tile, exactly one tile, a single token, more than two tiles) and with the gated feed-forward."""
    import torch
    cfg = I.ResStackConfig("tuc", 53, 1, 3, 8, 8, 128, 16, heads=2, d_ffn=256, context_tokens=tc, context_dim=d, gated=gated)
    x, lw, y1, i1 = run_stage(B, cfg, None, None)
    names = [f"A0.{n}" for n in I.attn_block_tensors(cfg)]
    assert "A0.context" in names and names.index("A0.lnc_g") == 10
    check(host(y1), oracle_stage(cfg, x, lw), "bf16", what="one segment per region", depth=2)
    for ca in (1, 2):
        _, _, y, info = run_stage(B, cfg, 3, ca, inputs=(x, lw))
        assert torch.equal(y, y1) and info.peak_bytes_planned < i1.peak_bytes_planned
    _, _, y2, _ = run_stage(B, cfg, 1, 1, flags=B.AC_FLAG_TWO_SEGMENTS_IN_FLIGHT, inputs=(x, lw))
    assert torch.equal(y2, y1)
    # the contexts are whole inputs: another image's context changes that image only
    lw2 = [dict(lw[0])]
    ctx = lw2[0]["context"].copy()
    ctx[1] = I.round_to_storage(draw(ctx[1].shape, 70, "bf16"), "bf16")
    lw2[0]["context"] = ctx
    _, _, y3, _ = run_stage(B, cfg, 3, 1, inputs=(x, lw2))
    assert torch.equal(y3[0], y1[0]) and torch.equal(y3[2], y1[2]) and not torch.equal(y3[1], y1[1])
