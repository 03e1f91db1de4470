"""GPU test of the allocation-free per-head MSE entry point (sta_head_mse_static): through the C ABI, against
sta_head_mse on the same tensors (same kernels and summation order, so the bits must agree) and against the
oracle, on two calls in a row, the second with a smaller input."""
import numpy as np
import pytest
import torch

import paper_2502_04507_amd as sta
from oracle import sta_oracle as orc

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _pair(B, H, N, D, seed):
    g = torch.Generator().manual_seed(seed)
    a = torch.randn((B, H, N, D), generator=g).to(torch.bfloat16)
    b = (a.float() + 0.05 * torch.randn((B, H, N, D), generator=g)).to(torch.bfloat16)
    return a, b


def test_static_scratch_entry_point_matches_workspace_entry_point_twice():
    # first a larger problem, then a smaller one: the second call finds the first call's partial sums in the array
    for B, H, grid, D, seed in ((2, 5, (3, 8, 8), 128, 77), (1, 3, (1, 4, 8), 64, 78)):
        N = grid[0] * grid[1] * grid[2]
        a, b = _pair(B, H, N, D, seed)
        ad, bd = a.to(DEV), b.to(DEV)
        ws = torch.empty(sta.sta_head_mse_workspace_bytes(B, H), dtype=torch.uint8, device=DEV)
        want = torch.full((H,), float("nan"), dtype=torch.float32, device=DEV)
        got = torch.full((H,), float("nan"), dtype=torch.float32, device=DEV)
        sta.sta_head_mse(ad, bd, grid, ws, want)
        sta.sta_head_mse_static(ad, bd, grid, got)
        torch.cuda.synchronize()
        assert np.array_equal(got.cpu().numpy().view(np.uint32), want.cpu().numpy().view(np.uint32)), (B, H, grid)
        ref = orc.head_mse(a.float().numpy(), b.float().numpy())
        assert np.allclose(got.cpu().numpy(), ref, rtol=1e-5, atol=0.0), (got.cpu().numpy(), ref)


def test_static_scratch_entry_point_rejects_more_slabs_than_the_array_holds():
    a = torch.zeros((1025, 1, 8, 8), dtype=torch.bfloat16, device=DEV)
    mse = torch.zeros((1,), dtype=torch.float32, device=DEV)
    with pytest.raises(sta.StaError) as e:
        sta.sta_head_mse_static(a, a.clone(), (1, 1, 8), mse)
    assert e.value.status == 6
