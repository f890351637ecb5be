"""The entry point that allocates nothing (dllm_op_linear_qkv_rope_static) against the entry point it
is a variant of (dllm_op_linear_qkv_rope): same kernels, so the outputs must be bit-identical.  Two
calls in a row, the second with a smaller input, share the one built-in scratch table."""
import pytest
import torch

from paper_2506_10848_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda"


def binding():
    from paper_2506_10848_amd import binding as b
    b.lib()
    b.reload_env()
    return b


def test_static_scratch_variant_matches_the_workspace_variant_twice_in_a_row():
    b = binding()
    # the first use of the built-in table makes the HIP runtime load the library's code object, which is
    # when the device memory of the table itself is reserved: done once here, outside the measured calls
    warm = torch.zeros((64, 3 * 64), dtype=torch.bfloat16, device=DEV)
    b.op_linear_qkv_rope_static(torch.zeros((64, 64), dtype=torch.bfloat16, device=DEV),
                                torch.zeros((192, 64), dtype=torch.bfloat16, device=DEV), warm, 1, 64, 1, 64, 1e4)
    torch.cuda.synchronize()
    for B, L, H, dh, theta in [(2, 300, 5, 128, 5e5), (1, 96, 4, 64, 1e4), (1, 8192, 1, 128, 5e5), (3, 70, 3, 128, 5e5)]:
        d = H * dh
        A = synth.normal_bf16((B * L, d), 1.0, 52, f"A{d}{L}", DEV)
        W = synth.normal_bf16((3 * d, d), 0.05, 53, f"Wqkv{d}", DEV)
        want = b.op_linear_qkv_rope(A, W, B, L, H, dh, theta)
        got = torch.full((B * L, 3 * d), 7.0, dtype=torch.bfloat16, device=DEV)      # allocated before the call
        free_before = torch.cuda.mem_get_info()[0]
        b.op_linear_qkv_rope_static(A, W, got, B, L, H, dh, theta)
        torch.cuda.synchronize()
        assert torch.cuda.mem_get_info()[0] == free_before                            # the call took no device memory
        assert torch.equal(got.view(torch.int16), want.view(torch.int16)), (B, L, H, dh)
    # beyond the built-in table: refused, nothing enqueued
    A = torch.zeros((8200, 128), dtype=torch.bfloat16, device=DEV)
    W = torch.zeros((384, 128), dtype=torch.bfloat16, device=DEV)
    out = torch.zeros((8200, 384), dtype=torch.bfloat16, device=DEV)
    with pytest.raises(b.DllmError) as e:
        b.op_linear_qkv_rope_static(A, W, out, 1, 8200, 1, 128, 1e4)
    assert e.value.code == b.EINVAL and "scratch" in str(e.value)
