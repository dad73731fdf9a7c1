"""Pins for the oracle's attention and scale-mass functions (CPU only).

Each check ties the oracle to something other than itself: a brute-force
masked attention over the whole sequence, torch's own fp64 attention routine,
closed forms that hold when Q = 0, and invariances of softmax attention.
"""
import numpy as np
import torch

import heatkv_inputs as hi
from oracle import heatkv_oracle as orc


def _tiny(seed=1, d=8, sides=(1, 2, 3, 2)):
    t0 = hi.tokens_per_scale(sides)
    t = orc.one_based(t0)
    c = orc.cumulative(t)
    rng = np.random.default_rng(seed)
    q, k, v = (rng.standard_normal((c[-1], d)) for _ in range(3))
    return t, c, q, k, v


def _scale_of_token(t):
    c = orc.cumulative(t)
    out = np.zeros(c[-1], dtype=np.int64)
    for k in range(1, len(t)):
        out[c[k - 1]:c[k]] = k
    return out


def test_keep_everything_equals_bruteforce_block_causal_attention():
    # One masked attention over the whole sequence (mask: scale(key) <= scale(query)),
    # written with explicit loops, must equal the scale-by-scale oracle with all priors kept.
    t, c, q, k, v = _tiny()
    K = len(t) - 1
    sm = 0.37
    sc = _scale_of_token(t)
    n = c[-1]
    ref = np.zeros_like(q)
    for a in range(n):
        logits = [sm * float(np.dot(q[a], k[b])) if sc[b] <= sc[a] else -np.inf for b in range(n)]
        mx = max(logits)
        w = [np.exp(x - mx) for x in logits]
        z = sum(w)
        for b in range(n):
            ref[a] += (w[b] / z) * v[b]
    got = np.concatenate([orc.attend_scale(q, k, v, t, kk, list(range(1, kk)), sm) for kk in range(1, K + 1)])
    np.testing.assert_allclose(got, ref, rtol=0, atol=1e-12)


def test_matches_torch_sdpa_fp64_on_retained_subset():
    t, c, q, k, v = _tiny(seed=3, d=16, sides=(1, 2, 4, 3, 5))
    sm = 1.0 / np.sqrt(16)
    kk, kept = 5, [1, 3]
    idx = np.concatenate([orc.retained_token_indices(t, kk, kept), np.arange(c[kk - 1], c[kk])])
    tq = torch.from_numpy(q[c[kk - 1]:c[kk]])[None, None]
    tk = torch.from_numpy(k[idx])[None, None]
    tv = torch.from_numpy(v[idx])[None, None]
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, scale=sm)[0, 0].numpy()
    got = orc.attend_scale(q, k, v, t, kk, kept, sm)
    np.testing.assert_allclose(got, ref, rtol=0, atol=1e-12)


def test_retained_indices_are_scale_ranges_in_order():
    t = orc.one_based([1, 4, 16, 64])
    idx = orc.retained_token_indices(t, 4, [3, 1])
    assert idx.tolist() == [0] + list(range(5, 21))


def test_zero_queries_give_mean_of_gathered_values_and_proportional_masses():
    t, c, q, k, v = _tiny(seed=5)
    K = len(t) - 1
    q0 = np.zeros_like(q)
    kk, kept = 4, [2]
    idx = np.concatenate([orc.retained_token_indices(t, kk, kept), np.arange(c[kk - 1], c[kk])])
    got = orc.attend_scale(q0, k, v, t, kk, kept, 0.5)
    np.testing.assert_allclose(got, np.tile(v[idx].mean(0), (t[kk], 1)), atol=1e-13)
    for k1 in range(1, K + 1):
        b = orc.beta_row(q0, k, t, k1, 0.5)
        want = [0.0] + [t[k2] / c[k1] if k2 <= k1 else 0.0 for k2 in range(1, K + 1)]
        np.testing.assert_allclose(b, want, atol=1e-14)


def test_key_permutation_and_logit_shift_invariance():
    t, c, q, k, v = _tiny(seed=7)
    sm = 0.3
    qs = q[c[2]:c[3]]
    base = orc.attend(qs, k[:c[3]], v[:c[3]], sm)
    perm = np.random.default_rng(0).permutation(c[3])
    np.testing.assert_allclose(orc.attend(qs, k[:c[3]][perm], v[:c[3]][perm], sm), base, atol=1e-13)
    # adding the same vector u to every key shifts each row's logits by a constant
    u = np.random.default_rng(1).standard_normal(k.shape[1])
    np.testing.assert_allclose(orc.attend(qs, k[:c[3]] + u, v[:c[3]], sm), base, atol=1e-12)


def test_row_masses_sum_to_one_and_match_full_alpha_matrix():
    t, c, q, k, v = _tiny(seed=11, d=8, sides=(1, 2, 4, 3))
    K = len(t) - 1
    sm = 0.41
    for k1 in range(1, K + 1):
        m = orc.row_masses(q, k, t, k1, sm)
        np.testing.assert_allclose(m.sum(1), 1.0, atol=1e-14)
        assert np.all(m[:, k1 + 1:] == 0) and np.all(m[:, 0] == 0)
        # brute force from explicit per-element probabilities
        for n in range(t[k1]):
            qa = q[c[k1 - 1] + n]
            e = np.array([np.exp(sm * np.dot(qa, k[j])) for j in range(c[k1])])
            p = e / e.sum()
            for k2 in range(1, k1 + 1):
                assert abs(p[c[k2 - 1]:c[k2]].sum() - m[n, k2]) < 1e-13
    beta = orc.beta_matrix(q, k, t, sm)
    np.testing.assert_allclose(beta[1:].sum(1), 1.0, atol=1e-14)
    assert np.all(np.triu(beta[1:, 1:], 1) == 0)
    assert beta[1, 1] == 1.0


def test_planted_weights_show_up_in_masses():
    # Statistical pin of the generator + mass function together: the planted logit
    # offsets ln w move mass toward prior scales roughly as w_i t_i / (t_k + sum w_j t_j).
    cfg = dict(hi.CONFIGS["tiny"], H=2)
    t0 = hi.tokens_per_scale(cfg["sides"])
    K = len(t0)
    w = np.ones((1, 2, K))
    w[0, 0, :] = 8.0
    w[0, 1, :] = 0.125
    q, k, v = hi.make_qkv(2, 0, cfg, w=w)
    t = orc.one_based(t0)
    sm = 1.0 / np.sqrt(cfg["d"])
    exp = hi.expected_beta_from_weights(w, t0)
    for h in range(2):
        b = orc.beta_row(q[0, h].double().numpy(), k[0, h].double().numpy(), t, K, sm)
        prior = b[1:K].sum()
        want = exp[0, h, K - 1, :K - 1].sum()
        assert abs(prior - want) < 0.15, (prior, want)
    b_hi = orc.beta_row(q[0, 0].double().numpy(), k[0, 0].double().numpy(), t, K, sm)[1:K].sum()
    b_lo = orc.beta_row(q[0, 1].double().numpy(), k[0, 1].double().numpy(), t, K, sm)[1:K].sum()
    assert b_hi > 0.5 > b_lo
