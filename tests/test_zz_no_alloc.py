"""The attention entry point that allocates nothing (its key-split partial results live in a
static device array of the library) against the entry point that takes a workspace: same
kernels and the same split count, so the same bits; and both within the parity bar of the fp64
oracle.  Two calls in a row on one stream, the second with a smaller input, so that what the
first call left in the array would show if the second depended on it."""
import numpy as np
import pytest

from oracle import transformer as O
from util import check, draw, host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_2401_10652_amd import binding
    binding.lib()
    return binding


def one_call(B, seed, sq, sk, heads, dh, causal, n_splits):
    import torch
    hd = heads * dh
    q = draw((sq, hd), seed, "bf16")
    k = draw((sk, hd), seed + 1, "bf16")
    v = draw((sk, hd), seed + 2, "bf16")
    dq, dk = B.to_device(q, "bf16"), B.to_device(k, "bf16")
    dvt = B.to_device(np.ascontiguousarray(v.T), "bf16")
    q_offset = sk - sq if causal else 0
    ns = n_splits or B.ac_attention_key_splits(sq, sk, heads, 1, dh, "bf16")
    assert ns > 1, "the case must use the scratch array"
    need = B.ac_attention_split_workspace_bytes(sq, heads, 1, dh, ns)
    assert need <= B.ac_static_scratch_bytes()
    ctx_a = torch.full((sq, hd), float("nan"), dtype=torch.bfloat16, device="cuda")
    ctx_b = torch.full_like(ctx_a, float("nan"))
    B.ac_op_attention_static_scratch(dq, dk, dvt, ctx_a, heads, dh, causal=causal, q_offset=q_offset,
                                     v_transposed=True, n_splits=n_splits)
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    B.ac_op_attention(dq, dk, dvt, ctx_b, heads, dh, causal=causal, q_offset=q_offset, v_transposed=True,
                      n_splits=ns, split_workspace=ws)
    torch.cuda.synchronize()
    assert torch.equal(ctx_a, ctx_b)
    ref = O.attention(q, k, v, heads, causal, q_offset=q_offset)
    check(host(ctx_a), ref, "bf16", what=f"static scratch sq={sq} sk={sk}")


def test_static_scratch_attention_two_calls_in_a_row(B):
    import torch
    before = torch.cuda.memory_allocated()
    one_call(B, 700, 640, 4096, 8, 64, True, 0)       # the executor's own split count
    one_call(B, 710, 200, 1536, 4, 128, False, 3)     # smaller, other head size, explicit count
    one_call(B, 720, 72, 1100, 2, 32, True, 2)        # smaller again, ragged key count
    assert torch.cuda.memory_allocated() >= before     # (torch's own tensors of the test only)
    # too large for the array: refused, nothing launched
    with pytest.raises(B.AcError) as ei:
        big = torch.empty((8, 128), dtype=torch.bfloat16, device="cuda")
        L = B.lib()
        st = L.ac_op_attention_static_scratch(big.data_ptr(), 128, 0, big.data_ptr(), 128, 0, big.data_ptr(), 8, 0, 1,
                                              None, 0, 0, None, 0, 0, big.data_ptr(), 128, 0, 1, 1 << 20, 4096, 16, 128,
                                              0, 0, 16, B.AC_BF16, None)
        B._check(st, "ac_op_attention_static_scratch")
    assert ei.value.status == B.AC_ERR_WORKSPACE
