"""GPU test of the allocation-free update entry point: agzo_update_noalloc must give what agzo_update gives,
bit for bit (same kernels, scratch in the library's static device array), on calls in a row of different sizes."""
import numpy as np
import pytest
import torch

from paper_2601_17261_amd import binding

pytestmark = pytest.mark.gpu


def _case(ctx_a, ctx_b, d_out, d_in, r, seed, dtype):
    gen = torch.Generator(device="cuda").manual_seed(seed)
    W = (0.02 * torch.randn(d_out, d_in, device="cuda", generator=gen)).to(dtype)
    B = torch.linalg.qr(torch.randn(d_in, r, device="cuda", generator=gen))[0].contiguous()
    g = torch.tensor([0.37], dtype=torch.float64, device="cuda")
    X = torch.empty(r, d_in, device="cuda", dtype=dtype)      # only its shape and dtype enter the descriptor
    W_ref, W_new = W.clone(), W.clone()
    L = binding.make_layer(W_ref, X, r)
    ctx_a.update(L, W_ref, B, seed, 1e-2, g)
    ctx_a.check()
    ctx_b.update_noalloc(L, W_new, B, seed, 1e-2, g)
    ctx_b.check()
    assert not torch.equal(W_ref, W), "the update must change W"
    assert torch.equal(W_ref.view(torch.int16 if dtype == torch.bfloat16 else torch.int32),
                       W_new.view(torch.int16 if dtype == torch.bfloat16 else torch.int32))


def test_update_noalloc_matches_update_on_successive_calls():
    ctx_a, ctx_b = binding.Context(), binding.Context()
    # a large matrix first, then smaller ones: the scratch keeps the first call's fragments behind the second's
    _case(ctx_a, ctx_b, 1536, 1280, 16, 11, torch.bfloat16)
    _case(ctx_a, ctx_b, 200, 264, 5, 12, torch.bfloat16)
    _case(ctx_a, ctx_b, 96, 520, 40, 13, torch.bfloat16)
    _case(ctx_a, ctx_b, 130, 77, 3, 14, torch.float32)
    ctx_a.close()
    ctx_b.close()


def test_update_noalloc_rejects_sizes_beyond_the_static_scratch():
    ctx = binding.Context()
    d_out, d_in, r = 300000, 64, 64         # 4 * 64 * (300000 + 256) bytes of fragments: far above 8 MiB
    W = torch.zeros(d_out, d_in, device="cuda", dtype=torch.bfloat16)
    B = torch.zeros(d_in, r, device="cuda")
    X = torch.empty(r, d_in, device="cuda", dtype=torch.bfloat16)
    L = binding.make_layer(W, X, r)
    with pytest.raises(binding.AgzoError) as ei:
        ctx.update_noalloc(L, W, B, 1, 1e-2, None)
    assert ei.value.code == binding.EINVAL and "static scratch" in str(ei.value)
    assert torch.count_nonzero(W).item() == 0
    ctx.close()
