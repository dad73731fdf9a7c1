"""Runs the library's generation-order pass on the GPU and the oracle's on the CPU for one layer."""
from __future__ import annotations

import numpy as np
import torch

import heatkv_inputs as hi
import paper_2605_14877_amd as hk
from oracle import heatkv_oracle as orc


def device_generation(plan, layer, q, k, v, t0, sm_scale, append_first=False, arenas=None, fused=False):
    """attend+append for scales 0..K-1 of one layer.  q,k,v: device [batch,H,c_K,d].  Returns list of outputs."""
    c = hi.cumulative_tokens(t0)
    dev = q.device
    if arenas is None:
        nbytes = max(plan.arena_bytes, 16)
        arenas = (torch.zeros(nbytes, dtype=torch.uint8, device=dev), torch.zeros(nbytes, dtype=torch.uint8, device=dev))
    ka, va = arenas
    outs = []
    for kk in range(len(t0)):
        sl = slice(c[kk] - t0[kk], c[kk])
        qk, kc, vc = (x[:, :, sl].contiguous() for x in (q, k, v))
        out = torch.empty_like(qk)
        wsb = plan.attend_workspace_bytes(layer, kk)
        ws = torch.empty(max(wsb, 1), dtype=torch.uint8, device=dev)
        if fused:
            hk.heatkv_attend_append_scale(plan, layer, kk, qk, kc, vc, ka, va, sm_scale, out, ws)
        elif append_first:
            # the arena region of scale kk must stay intact: appending first is only legal because
            # append writes the scale-(kk+1) region into free space
            hk.heatkv_append_scale(plan, layer, kk, kc, vc, ka, va)
            hk.heatkv_attend_scale(plan, layer, kk, qk, kc, vc, ka, va, sm_scale, out, ws)
        else:
            hk.heatkv_attend_scale(plan, layer, kk, qk, kc, vc, ka, va, sm_scale, out, ws)
            hk.heatkv_append_scale(plan, layer, kk, kc, vc, ka, va)
        outs.append(out)
    torch.cuda.synchronize()
    return outs


def oracle_rows(q, k, v, t0, kk, b, h, kept_scales0, sm_scale, rows=None):
    """Oracle attention for head (b,h) at 0-based scale kk; `rows` selects query rows (None = all)."""
    t = orc.one_based(t0)
    c = hi.cumulative_tokens(t0)
    qs = q[b, h].double().numpy()
    ks = k[b, h].double().numpy()
    vs = v[b, h].double().numpy()
    if rows is None:
        return orc.attend_scale(qs, ks, vs, t, kk + 1, [i + 1 for i in kept_scales0], sm_scale)
    cur = np.arange(c[kk] - t0[kk], c[kk])
    idx = np.concatenate([orc.retained_token_indices(t, kk + 1, [i + 1 for i in kept_scales0]), cur])
    return orc.attend(qs[cur[rows]], ks[idx], vs[idx], sm_scale)
