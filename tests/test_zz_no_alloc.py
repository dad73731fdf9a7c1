"""The allocation-free calibrate entry point against heatkv_calibrate, through the C ABI.

Collected last on purpose (file name): it exercises the library's static device workspace, which every call on
the GPU shares and which keeps the previous call's contents."""
import numpy as np
import pytest
import torch

import heatkv_inputs as hi
import paper_2605_14877_amd as hk
from paper_2605_14877_amd import binding

pytestmark = pytest.mark.gpu


def _case(sides, H, batch, dtype, d, seed):
    t0 = hi.tokens_per_scale(sides)
    c = hi.cumulative_tokens(t0)
    g = torch.Generator().manual_seed(seed)
    td = hi.torch_dtype(dtype)
    q = torch.randn(batch, H, c[-1], d, generator=g).to(td).cuda()
    k = torch.randn(batch, H, c[-1], d, generator=g).to(td).cuda()
    return t0, c, q, k, hk.Shape(1, H, d, t0, batch, dtype)


def _both(t0, c, q, k, shape, k1, sm):
    qs = q[:, :, c[k1] - t0[k1]:c[k1]].contiguous()
    ks = k[:, :, :c[k1]].contiguous()
    want = torch.full((shape.batch, shape.H, shape.K), -1.0, device="cuda")
    got = torch.full_like(want, -2.0)
    ws = torch.empty(max(binding.calibrate_workspace_bytes(shape, k1), 4), dtype=torch.uint8, device="cuda")
    hk.heatkv_calibrate(shape, 0, k1, qs, ks, sm, want, ws)
    hk.heatkv_calibrate_static(shape, 0, k1, qs, ks, sm, got)
    torch.cuda.synchronize()
    return want, got


@pytest.mark.parametrize("dtype,d", [("bf16", 128), ("f32", 64)])
def test_calibrate_static_matches_calibrate_on_two_calls_in_a_row(dtype, d):
    # first a larger problem, then a smaller one over the same static workspace (which still holds the first
    # call's partial sums): both must give the bits of heatkv_calibrate, whose masses the parity tests pin to
    # the oracle at 1e-4
    sm = 1.0 / np.sqrt(d)
    big = _case((1, 2, 5, 9, 14, 23) if dtype == "bf16" else (1, 2, 5, 9, 12), 5, 3, dtype, d, seed=3)
    small = _case((1, 3, 6, 11) if dtype == "bf16" else (1, 3, 5), 2, 1, dtype, d, seed=4)
    for case in (big, small):
        t0, c, q, k, shape = case
        for k1 in (len(t0) - 1, 1):
            want, got = _both(t0, c, q, k, shape, k1, sm)
            assert torch.equal(want, got), (dtype, len(t0), k1)
            rows = got[:, :, :k1 + 1].sum(-1).cpu().numpy()
            assert np.abs(rows - 1.0).max() <= 1e-4 and not got[:, :, k1 + 1:].any()
