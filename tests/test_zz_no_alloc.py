"""The entry point that allocates nothing (npd_kd_loss_fwd_bwd_noalloc: scratch in a fixed device array of the
library) against npd_kd_loss_fwd_bwd with a caller workspace, through the C ABI: same kernels, so every output must be
bit-identical -- on two calls in a row, the second smaller (the array keeps the first call's contents)."""
import numpy as np
import pytest
import torch

from paper_2605_05940_amd import binding, synth

pytestmark = pytest.mark.gpu


def _run(T, V, seed, noalloc, tau=1.0, inplace=False):
    dev = torch.device("cuda:0")
    g = torch.Generator(device=dev).manual_seed(seed)
    s = (3.0 * torch.randn((T, V), device=dev, generator=g)).to(torch.bfloat16)
    t = (0.8 * s.float() + 1.5 * torch.randn((T, V), device=dev, generator=g)).to(torch.bfloat16)
    labels = torch.randint(0, V, (T,), device=dev, generator=g, dtype=torch.int32)
    mask = (torch.rand(T, device=dev, generator=g) > 0.25).to(torch.uint8)
    grad = s if inplace else torch.full_like(s, float("nan"))
    kd, nll, tnll, lse = (torch.full((T,), float("nan"), device=dev) for _ in range(4))
    status = torch.zeros(1, dtype=torch.int32, device=dev)
    binding.npd_kd_loss_fwd_bwd(s, mask, teacher_dense=t, labels=labels, tau=tau, grad_out=grad, kd_tok=kd, nll_tok=nll,
                                teacher_nll_tok=tnll, lse_tok=lse, dev_status=status, noalloc=noalloc)
    torch.cuda.synchronize()
    assert status.item() == 0
    return [synth.bf16_bits(grad)] + [x.cpu().numpy().view(np.uint32) for x in (kd, nll, tnll, lse)]


def test_noalloc_entry_point_matches_the_workspace_entry_point_bitwise():
    # (T, V, tau, in place): 8 slices per row; then a smaller call with 3 slices per row and the wider record of tau != 1
    for i, (T, V, tau, inplace) in enumerate([(384, 151936, 1.0, False), (160, 50264, 2.0, True)]):
        assert binding.npd_workspace_bytes(T, V, tau=tau) > 0        # the row-gang kernels, which use the scratch
        got = _run(T, V, 1234 + i, noalloc=True, tau=tau, inplace=inplace)
        want = _run(T, V, 1234 + i, noalloc=False, tau=tau, inplace=inplace)
        for a, b in zip(got, want):
            np.testing.assert_array_equal(a, b)
        assert np.isfinite(got[1].view(np.float32)).all()
