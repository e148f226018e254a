"""GPU parity of the UNet residual block: its two kernels alone and whole chunk plans against the fp64 oracle,
through the C-ABI."""
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
                                                     (1, 5, 3, 24, 3, "none"), (2, 1, 1, 16, 2, "none")])
def test_group_norm(B, dtype, images, h, w, c, groups, act):
    """Groups of 10 channels straddle the 8-channel vectors; 63 positions do not divide into the 16 shares;
    a single position leaves most shares empty."""
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
        al(batch * groups * 16 * 3 * 4)
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
