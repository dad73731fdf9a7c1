"""Seeded synthetic inputs for the HeatKV hot path.

This module only manufactures data: scale lists, random Q/K/V activations with a
planted per-head preference for prior scales, random head weights and a seeded
explicit retention pattern.  It holds none of the method's arithmetic (no
softmax, no attention mass, no ranking, no budget rule) so that both the CPU
oracle's tests and the GPU path's tests can draw identical bytes from it
without sharing any code of the method itself.

The real workloads of the paper are activations of a pretrained next-scale
image model on text prompts (Sec. 4, "Base Models"); neither the weights nor the
prompts are available here, so these tensors stand in for them.  Shapes follow
the 13-scale 1024x1024 token-map pyramid of an Infinity-like model.
"""
from __future__ import annotations

import numpy as np
import torch

# Side lengths h_k = w_k of the token maps for a 1024x1024 image (13 scales).
SIDES_1024 = (1, 2, 4, 6, 8, 12, 16, 20, 24, 32, 40, 48, 64)
SIDES_TINY = (1, 2, 4, 8)


def tokens_per_scale(sides):
    """t_k = h_k * w_k (Sec. 3.1 notation); an entry is a side s (square map, s * s tokens) or a pair (h, w)."""
    return [int(s[0]) * int(s[1]) if isinstance(s, (tuple, list)) else int(s) * int(s) for s in sides]


def cumulative_tokens(t):
    """c_k = sum_{tau<=k} t_tau, returned 0-based: c[k] includes scale k."""
    out, acc = [], 0
    for x in t:
        acc += int(x)
        out.append(acc)
    return out


# name -> (L, H, d, dtype, batch, sides, sinks, compression factor)
CONFIGS = {
    "tiny": dict(L=1, H=4, d=64, dtype="f32", batch=1, sides=SIDES_TINY, sinks=1, factor=2),
    "layer2b": dict(L=1, H=16, d=128, dtype="bf16", batch=2, sides=SIDES_1024, sinks=3, factor=4),
    "stack2b": dict(L=32, H=16, d=128, dtype="bf16", batch=2, sides=SIDES_1024, sinks=3, factor=10),
    "stack8b": dict(L=40, H=32, d=128, dtype="bf16", batch=2, sides=SIDES_1024, sinks=3, factor=20),
    "serving": dict(L=32, H=16, d=128, dtype="bf16", batch=32, sides=SIDES_1024, sinks=3, factor=20),
}


def budget_tokens(cfg):
    """Token budget per sequence: T * c_{K-1} / factor (integer for every named config)."""
    t = tokens_per_scale(cfg["sides"])
    c = cumulative_tokens(t)
    total = cfg["L"] * cfg["H"] * c[-2]
    assert total % cfg["factor"] == 0
    return total // cfg["factor"]


def elem_bytes(dtype):
    return {"f32": 4, "bf16": 2}[dtype]


def torch_dtype(dtype):
    return {"f32": torch.float32, "bf16": torch.bfloat16}[dtype]


def head_weights(seed, L, H, K, per_scale_jitter=True):
    """Planted logit multipliers w[l,h,i] > 0 for keys of prior scale i.

    w = g * u with g log-uniform on [0.1, 10] per head and u log-uniform on
    [0.5, 2] per (head, source scale); u == 1 when per_scale_jitter is False.
    """
    rng = np.random.default_rng([int(seed), 0x5EED])
    g = np.exp(rng.uniform(np.log(0.1), np.log(10.0), size=(L, H, 1)))
    if per_scale_jitter:
        u = np.exp(rng.uniform(np.log(0.5), np.log(2.0), size=(L, H, K)))
    else:
        u = np.ones((L, H, K))
    return g * u


def make_qkv(seed, layer, cfg, w=None, sm_scale=None, batch=None):
    """Full-sequence Q, K, V for one layer: torch CPU tensors [batch, H, c_K, d].

    Entries are N(0,1) rounded to the config dtype.  When `w` ([L,H,K]) is
    given the last K channels are reserved to plant a logit offset: a key of
    scale i is one-hot at reserved channel i, and a query of scale k carries
    ln(w[l,h,i]) / sm_scale at reserved channel i for every i < k (0 for
    i >= k).  The dot product then adds ln w[l,h,i] to the logits of scale-k
    queries on scale-i keys, prior scales only.
    """
    H, d = cfg["H"], cfg["d"]
    t = tokens_per_scale(cfg["sides"])
    c = cumulative_tokens(t)
    K = len(t)
    nb = cfg["batch"] if batch is None else batch
    if sm_scale is None:
        sm_scale = 1.0 / np.sqrt(d)
    rng = np.random.default_rng([int(seed), int(layer), 0xA77])
    shape = (nb, H, c[-1], d)
    q = rng.standard_normal(shape, dtype=np.float32)
    k = rng.standard_normal(shape, dtype=np.float32)
    v = rng.standard_normal(shape, dtype=np.float32)
    if w is not None:
        assert d > K
        r0 = d - K
        q[..., r0:] = 0.0
        k[..., r0:] = 0.0
        for i in range(K):
            lo, hi = c[i] - t[i], c[i]
            k[:, :, lo:hi, r0 + i] = 1.0
            for kk in range(i + 1, K):
                qlo, qhi = c[kk] - t[kk], c[kk]
                q[:, :, qlo:qhi, r0 + i] = (np.log(w[layer, :, i]) / sm_scale)[None, :, None]
    td = torch_dtype(cfg["dtype"])
    return tuple(torch.from_numpy(x).to(td) for x in (q, k, v))


def scale_slice(c, t, k):
    """Python slice of the tokens of 0-based scale k in a full sequence."""
    return slice(c[k] - t[k], c[k])


def expected_beta_from_weights(w, t):
    """Mass a planted-weight head is expected to put on each prior scale.

    beta[l,h,k,i] ~= w_i t_i / (t_k + sum_{j<k} w_j t_j) for i < k and
    t_k / (...) for i == k: what uniform-in-expectation logits plus the
    planted offsets give.  Used to fabricate a plausible beta table for the
    large configs without running calibration, and as a statistical
    sanity reference; it is a property of this generator, not of the method.
    """
    L, H, K = w.shape
    beta = np.zeros((L, H, K, K))
    tt = np.asarray(t, dtype=np.float64)
    for k in range(K):
        den = tt[k] + (w[:, :, :k] * tt[:k]).sum(-1)
        beta[:, :, k, :k] = w[:, :, :k] * tt[:k] / den[..., None]
        beta[:, :, k, k] = tt[k] / den
    return beta


def explicit_keep_pattern(seed, L, H, t, budget):
    """Seeded explicit retention pattern for configs too small for the paper's rule.

    Visits the L*H*(K-1) head-scales (l, h, i), i < K-1, in a seeded random
    order and keeps each one whose t_i still fits in the running total
    `budget`.  Returns present[k][l][h][i] (uint8): prior scale i is part of
    head (l,h)'s cache when scale k is generated.
    """
    K = len(t)
    rng = np.random.default_rng([int(seed), 0xCAFE])
    items = [(l, h, i) for l in range(L) for h in range(H) for i in range(K - 1)]
    order = rng.permutation(len(items))
    keep = np.zeros((L, H, K), dtype=bool)
    total = 0
    for j in order:
        l, h, i = items[j]
        if total + t[i] <= budget:
            keep[l, h, i] = True
            total += t[i]
    present = np.zeros((K, L, H, K), dtype=np.uint8)
    for k in range(K):
        present[k, :, :, :k] = keep[:, :, :k]
    return present


def make_qkv_device(seed, layer, cfg, w, device, sm_scale=None, batch=None):
    """Same recipe as make_qkv, drawn with torch's generator on `device` (for the full-size configs).

    Returns Q, K, V as device tensors [batch, H, c_K, d] in the config dtype.  The values differ from
    make_qkv's for the same seed (another generator); callers copy what they need back to the host.
    """
    H, d = cfg["H"], cfg["d"]
    t = tokens_per_scale(cfg["sides"])
    c = cumulative_tokens(t)
    K = len(t)
    nb = cfg["batch"] if batch is None else batch
    if sm_scale is None:
        sm_scale = 1.0 / np.sqrt(d)
    g = torch.Generator(device=device)
    g.manual_seed(int(seed) * 1000003 + int(layer) * 7919 + 17)
    td = torch_dtype(cfg["dtype"])
    out = []
    for _ in range(3):
        out.append(torch.randn((nb, H, c[-1], d), generator=g, device=device, dtype=torch.float32))
    q, k, v = out
    if w is not None:
        r0 = d - K
        q[..., r0:] = 0.0
        k[..., r0:] = 0.0
        lw = torch.from_numpy(np.log(w[layer]) / sm_scale).to(device=device, dtype=torch.float32)  # [H, K]
        for i in range(K):
            k[:, :, c[i] - t[i]:c[i], r0 + i] = 1.0
            if i + 1 < K:
                q[:, :, c[i]:, r0 + i] = lw[None, :, i, None]
    return tuple(x.to(td) for x in (q, k, v))
