"""The allocation-free attention backward (bf_op_attention_bwd_static: the delta scratch in an array built into
the library) against bf_op_attention_bwd with a caller's buffer: same kernels, so the results must be bit-identical.
Two calls in a row, the second on a smaller input (the array keeps the first call's contents), then the size limit."""
import pytest
import torch

import paper_2211_05953_amd as bf

pytestmark = pytest.mark.gpu


def _case(seed, S_mb, S_seq, N_heads, S_head, causal):
    h = N_heads * S_head
    g = torch.Generator(device="cuda").manual_seed(seed)
    qkv = torch.randn((S_mb, S_seq, 3 * h), generator=g, device="cuda").bfloat16()
    dctx = torch.randn((S_mb, S_seq, h), generator=g, device="cuda").bfloat16()
    ctx = torch.empty((S_mb, S_seq, h), dtype=torch.bfloat16, device="cuda")
    lse = torch.empty((S_mb, N_heads, S_seq), dtype=torch.float32, device="cuda")
    bf.bf_op_attention_fwd(bf.BF_BF16, 0, S_mb, S_seq, N_heads, S_head, causal, qkv, ctx, lse)
    ref = torch.full_like(qkv, float("nan"))
    delta = torch.empty(S_mb * N_heads * S_seq, dtype=torch.float32, device="cuda")
    bf.bf_op_attention_bwd(bf.BF_BF16, 0, S_mb, S_seq, N_heads, S_head, causal, qkv, ctx, lse, dctx, ref, delta)
    got = torch.full_like(qkv, float("nan"))
    bf.bf_op_attention_bwd_static(bf.BF_BF16, 0, S_mb, S_seq, N_heads, S_head, causal, qkv, ctx, lse, dctx, got)
    torch.cuda.synchronize()
    assert torch.isfinite(ref.float()).all()
    assert torch.equal(got, ref), (S_mb, S_seq, N_heads, S_head, causal)


def test_static_scratch_attention_backward_matches_the_buffer_form_on_two_calls_in_a_row():
    _case(1, 2, 512, 8, 128, 1)      # MFMA kernels, 8192 scratch elements
    _case(2, 1, 256, 4, 64, 1)       # smaller input right after: 1024 elements, the rest of the array is stale
    _case(3, 2, 50, 3, 24, 0)        # plain kernels, ragged sizes, bidirectional
    _case(4, 4, 2048, 64, 128, 1)    # 524288 elements, half the array


def test_static_scratch_rejects_what_does_not_fit():
    t = torch.zeros(8, dtype=torch.bfloat16, device="cuda")
    f = torch.zeros(8, dtype=torch.float32, device="cuda")
    with pytest.raises(bf.BfError) as e:
        bf.bf_op_attention_bwd_static(bf.BF_BF16, 0, 8, 4096, 64, 128, 1, t, t, f, t, t)    # 2 Mi elements > 1 Mi
    assert e.value.status == bf.BF_EINVAL and "exceeds" in str(e.value)
