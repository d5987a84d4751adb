"""The allocation-free permutation entry point (dwdp_permute_static: scratch in a static device
array, no context) against dwdp_permute, bit for bit, on two calls in a row, the second smaller."""
import numpy as np
import pytest
import torch

from oracle import moe_oracle as mo
from paper_2604_01621_amd import inputs

pytestmark = pytest.mark.gpu


def _ids(T, E, K, seed):
    g = torch.Generator().manual_seed(seed)
    # K distinct experts per token, as routing produces them
    return torch.stack([torch.randperm(E, generator=g)[:K] for _ in range(T)]).to(torch.int32)


def _both(binding, ctx, cfg, ids):
    T, K, E = ids.shape[0], cfg.K, cfg.E
    n_off = E + 1 + cfg.has_shared
    d = ids.cuda()
    out = []
    for static in (False, True):
        off = torch.full((n_off,), -7, dtype=torch.int32, device="cuda")
        perm = torch.full((max(T * K, 1),), -7, dtype=torch.int32, device="cuda")
        inv = torch.full((max(T * K, 1),), -7, dtype=torch.int32, device="cuda")
        if static:
            binding.dwdp_permute_static(d, E, K, cfg.has_shared, off, perm, inv)
        else:
            ctx.dwdp_permute(d, off, perm, inv)
        torch.cuda.synchronize()
        out.append((off.cpu().numpy(), perm.cpu().numpy()[:T * K], inv.cpu().numpy()[:T * K]))
    return out


def test_permute_static_matches_permute_twice_second_smaller(gpu_device):
    from paper_2604_01621_amd import binding
    cfg = inputs.r1_layer(8192)
    ctx = binding.Context(cfg)
    try:
        # both sizes take the multi-workgroup path, the one that uses the scratch array; the second
        # call is smaller, so stale histogram entries of the first lie behind the part it rewrites
        for T, seed in ((5000, 1), (2100, 2), (64, 3), (0, 4)):
            print("permute_static T", T, flush=True)
            ids = _ids(T, cfg.E, cfg.K, seed) if T else torch.zeros(0, cfg.K, dtype=torch.int32)
            (o0, p0, i0), (o1, p1, i1) = _both(binding, ctx, cfg, ids)
            np.testing.assert_array_equal(o1, o0)
            np.testing.assert_array_equal(p1, p0)
            np.testing.assert_array_equal(i1, i0)
            if T:   # and both equal the oracle's stable counting sort
                ro, rp, ri = mo.permute(ids.numpy(), mo.spec_from(cfg))
                np.testing.assert_array_equal(o1, ro)
                np.testing.assert_array_equal(p1, rp)
                np.testing.assert_array_equal(i1, ri)
    finally:
        ctx.close()


def test_permute_static_scratch_limit_is_an_error(gpu_device):
    from paper_2604_01621_amd import binding
    ids = torch.zeros(8, 2, dtype=torch.int32, device="cuda")
    off = torch.zeros(1026, dtype=torch.int32, device="cuda")
    with pytest.raises(binding.DwdpError) as ei:
        big = torch.zeros(40000, 2, dtype=torch.int32, device="cuda")      # 313 chunks x 1024 experts x 4 B > 1 MiB
        binding.dwdp_permute_static(big, 1024, 2, 0, off, big.view(-1), big.view(-1).clone())
    assert ei.value.status == binding.ESHAPE
    torch.cuda.synchronize()
