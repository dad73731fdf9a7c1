"""Shared helpers for the tests: building the oracle's schedule and the library's plan side by side."""
from __future__ import annotations

import numpy as np

import heatkv_inputs as hi
from oracle import heatkv_oracle as orc


def oracle_schedule(beta0, L, H, t0, s, B, variant=0):
    """Runs the oracle's ranking + Eq. 5 + Alg. 1 on a 0-based fp32 beta table."""
    K = len(t0)
    t = orc.one_based(t0)
    beta1 = orc.beta_one_based(np.asarray(beta0, dtype=np.float32))
    N = orc.heads_to_prune(L * H, t, s, B)
    binary, naive = bool(variant & 1), bool(variant & 2)
    if binary:
        order = orc.cas_order(beta1, L, H, K, s)
        sch = orc.binary_heatkv_schedule(order, N, t, s, L, H, B, naive=naive)
        orders = {i: order for i in range(s + 1, K)}
    else:
        orders = orc.head_orders(beta1, L, H, K, s)
        sch = orc.heatkv_schedule(orders, N, t, s, L, H, B, naive=naive)
    present = orc.to_zero_based_present(sch["A"], K, L, H, s, binary=binary)
    return dict(N=N, orders=orders, sch=sch, present=present, t=t, binary=binary)


def bitmap(S, K, L, H, s, binary):
    """Oracle set -> the library's [K][T] bitmap convention."""
    if not binary:
        return orc.to_zero_based_bitmap(S, K, L, H)
    out = np.zeros((K, L * H), dtype=np.uint8)
    heads = S.m[0, 1:, 1:].reshape(L * H)
    out[s:K - 1, :] = heads[None, :]
    return out


def random_beta(seed, L, H, K):
    rng = np.random.default_rng(seed)
    b = np.tril(rng.random((L, H, K, K))).astype(np.float32)
    b /= b.sum(-1, keepdims=True)
    return b.astype(np.float32)


def config_beta(name, seed=0):
    cfg = hi.CONFIGS[name]
    t0 = hi.tokens_per_scale(cfg["sides"])
    w = hi.head_weights(seed, cfg["L"], cfg["H"], len(t0))
    return hi.expected_beta_from_weights(w, t0).astype(np.float32), w
