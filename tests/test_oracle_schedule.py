"""Pins for the oracle's ranking, budget rule and removal-order algorithm (CPU only)."""
import itertools
import os
from fractions import Fraction
from math import ceil

import numpy as np
import pytest

import heatkv_inputs as hi
from oracle import heatkv_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "alg1_hand_example.txt")


def _parse_items(tokens):
    return sorted(tuple(int(x) for x in tok.split(",")) for tok in tokens)


def _load_golden():
    rec = dict(G={}, E={}, A={}, R={}, N=None)
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        p = line.split()
        if p[0] == "N":
            rec["N"] = [int(x) for x in p[1:]]
        elif p[0] in "GEA":
            rec[p[0]][int(p[1])] = _parse_items(p[2:])
        elif p[0] == "R":
            k, l, h = int(p[1]), int(p[2]), int(p[3])
            rec["R"][(k, l, h)] = [int(x) for x in p[5:]]
    return rec


def test_hand_worked_example_of_algorithm_1():
    g = _load_golden()
    L, H, K, s, B = 2, 2, 5, 1, 20
    t = orc.one_based([1, 2, 3, 4, 5])
    a, b, c_, d = (1, 1), (1, 2), (2, 1), (2, 2)
    orders = {2: [c_, a, d, b], 3: [a, c_, b, d], 4: [d, b, a, c_]}
    N = orc.heads_to_prune(L * H, t, s, B)
    assert N[1:] == g["N"]
    sch = orc.heatkv_schedule(orders, N, t, s, L, H, B)
    for name in "GEA":
        for k, want in g[name].items():
            assert sorted(sch[name][k].items()) == want, (name, k)
    for (k, l, h), want in g["R"].items():
        assert orc.retained_scales(sch["A"][k], k, l, h, s) == want


# Eq. 5 evaluated with exact rationals, b as a fraction, exactly as printed.
@pytest.mark.parametrize("name", ["layer2b", "stack2b", "stack8b", "serving"])
def test_eq5_against_rational_arithmetic_and_total_cache_identity(name):
    cfg = hi.CONFIGS[name]
    t = orc.one_based(hi.tokens_per_scale(cfg["sides"]))
    c = orc.cumulative(t)
    K, s, T = len(t) - 1, cfg["sinks"], cfg["L"] * cfg["H"]
    b = Fraction(1, cfg["factor"])
    B = hi.budget_tokens(cfg)
    assert B == b * T * c[K - 1]
    N = orc.heads_to_prune(T, t, s, B)
    for k in range(1, K):
        if k <= s:
            assert N[k] == 0
            continue
        want = max(0, ceil(T * (c[k] - b * c[K - 1]) / Fraction(c[k] - c[s])))
        assert N[k] == want
        # N_k is the minimal count with N c_s + (T-N) c_k <= B (Sec. 3.2)
        assert N[k] * c[s] + (T - N[k]) * c[k] <= B
        if N[k] > 0:
            assert (N[k] - 1) * c[s] + (T - N[k] + 1) * c[k] > B
    assert all(N[k] <= N[k + 1] for k in range(1, K - 1))


def test_eq5_values_for_the_named_configs():
    # Values worked from Eq. 5 by hand arithmetic for k = 10..12 of the 16-head, 4x case:
    # (16*2521-25700)/2500 = 5.85 -> 6, (16*4121-25700)/4100 = 9.81 -> 10, (16*6425-25700)/6404 = 12.04 -> 13
    cfg = hi.CONFIGS["layer2b"]
    t = orc.one_based(hi.tokens_per_scale(cfg["sides"]))
    assert orc.heads_to_prune(16, t, 3, 25700)[1:] == [0] * 9 + [6, 10, 13]
    tt = orc.one_based(hi.tokens_per_scale(hi.SIDES_TINY))
    # Tiny: T=4, s=1, B=42: k=3: ceil((4*21-42)/(21-1)) = ceil(2.1) = 3
    assert orc.heads_to_prune(4, tt, 1, 42)[1:] == [0, 0, 3]


def test_budget_below_sinks_is_rejected():
    t = orc.one_based([1, 4, 16, 64])
    with pytest.raises(ValueError):
        orc.heads_to_prune(4, t, 2, 4 * 5 - 1)


def test_scas_and_cas_against_direct_slices_and_order_direction():
    rng = np.random.default_rng(0)
    L, H, K, s = 2, 3, 6, 2
    beta = np.zeros((L + 1, H + 1, K + 1, K + 1))
    beta[1:, 1:, 1:, 1:] = np.tril(rng.random((L, H, K, K)))
    for l in range(1, L + 1):
        for h in range(1, H + 1):
            for k in range(s + 1, K):
                assert abs(orc.s_cas(beta[l, h], K, k) - beta[l, h, k + 1:, k].mean()) < 1e-15
            assert abs(orc.cas(beta[l, h], K, s) - beta[l, h, K, s + 1:K].sum() / (K - s)) < 1e-15
    orders = orc.head_orders(beta, L, H, K, s)
    assert sorted(orders) == list(range(s + 1, K))
    for i, O in orders.items():
        assert sorted(O) == [(l, h) for l in range(1, L + 1) for h in range(1, H + 1)]
        sc = [orc.s_cas(beta[l, h], K, i) for (l, h) in O]
        assert sc == sorted(sc)  # least dependent first


def test_equal_scores_keep_head_id_order():
    L, H, K, s = 2, 2, 4, 1
    beta = np.zeros((L + 1, H + 1, K + 1, K + 1))
    orders = orc.head_orders(beta, L, H, K, s)
    for O in orders.values():
        assert O == [(1, 1), (1, 2), (2, 1), (2, 2)]


def _random_case(seed, L, H, sides, s, factor_num, factor_den):
    rng = np.random.default_rng(seed)
    t0 = hi.tokens_per_scale(sides)
    t = orc.one_based(t0)
    c = orc.cumulative(t)
    K = len(t0)
    beta0 = np.tril(rng.random((L, H, K, K))).astype(np.float32)
    beta0 /= beta0.sum(-1, keepdims=True)
    T = L * H
    B = (T * c[K - 1] * factor_num) // factor_den
    return t, c, K, T, B, orc.beta_one_based(beta0)


@pytest.mark.parametrize("seed,L,H,sides,s,num,den", [
    (0, 3, 4, (1, 2, 3, 4, 5, 6), 2, 1, 2),
    (1, 4, 2, (1, 2, 4, 6, 8, 12, 16), 3, 1, 4),
    (2, 2, 8, hi.SIDES_1024, 3, 1, 10),
    (3, 5, 3, (1, 2, 4, 6, 8, 12), 1, 1, 3),
])
def test_schedule_invariants(seed, L, H, sides, s, num, den):
    t, c, K, T, B, beta = _random_case(seed, L, H, sides, s, num, den)
    N = orc.heads_to_prune(T, t, s, B)
    orders = orc.head_orders(beta, L, H, K, s)
    sch = orc.heatkv_schedule(orders, N, t, s, L, H, B)
    G, E, A = sch["G"], sch["E"], sch["A"]
    empty = orc._Sets(K, L, H)
    for k in range(1, K):
        Gk, Gp = G[k], (G[k - 1] if k > 1 else empty)
        # each prunable source scale i <= k is removed in exactly N_k heads (Sec. 3.2)
        for i in range(1, K + 1):
            want = N[k] if s < i <= k else 0
            assert int(Gk.m[i].sum()) == want
        assert not np.any(Gp.m & ~Gk.m)                      # G_{k-1} subset of G_k
        assert not np.any(E[k].m & ~(Gk.m & ~Gp.m))          # E_k subset of G_k \ G_{k-1}
        assert np.array_equal(A[k].m, Gp.m | E[k].m)         # A_k = G_{k-1} u E_k
        assert not np.any(A[k].m & ~A[k + 1].m)              # absent sets only grow
        # budget after every layer, by the accounting of Alg. 2, and the end-of-scale closed form
        for layer in range(1, L + 1):
            assert orc.cache_size_after_layer(k, layer, Gk, Gp, E[k], t, c, s, L, H) <= B
        # end of scale: every prunable source scale i <= k is missing from exactly N_k heads
        # (for k <= s the printed CachedTokens is the constant c_s)
        total = orc.cache_size_after_layer(k, L, Gk, Gp, E[k], t, c, s, L, H)
        kept = T * c[max(k, s)] - sum(t[i] * N[k] for i in range(s + 1, k + 1))
        assert total == kept
    assert np.array_equal(A[K].m, G[K - 1].m)


def test_greedy_is_minimal_along_its_own_order():
    # Dropping the last popped element must break feasibility at some layer.
    t, c, K, T, B, beta = _random_case(5, 4, 4, (1, 2, 4, 6, 8, 12, 16), 2, 1, 3)
    L, H, s = 4, 4, 2
    N = orc.heads_to_prune(T, t, s, B)
    orders = orc.head_orders(beta, L, H, K, s)
    rank = {(i, l, h): r for i, O in orders.items() for r, (l, h) in enumerate(O)}
    sch = orc.heatkv_schedule(orders, N, t, s, L, H, B)
    seen = 0
    empty = orc._Sets(K, L, H)
    for k in range(1, K):
        Gp = sch["G"][k - 1] if k > 1 else empty
        E, popped = orc.greedy_early_pruning(k, Gp, sch["G"][k], B, rank, t, c, s, L, H)
        assert sorted(E.items()) == sorted(sch["E"][k].items())
        keys = [(-it[1], -it[0], rank[it]) for it in popped]
        assert keys == sorted(keys)
        if popped:
            seen += 1
            smaller = orc._Sets(K, L, H, popped[:-1])
            sizes = [orc.cache_size_after_layer(k, l, sch["G"][k], Gp, smaller, t, c, s, L, H) for l in range(1, L + 1)]
            assert max(sizes) > B
    assert seen > 0


def test_full_budget_prunes_nothing_and_naive_policy_is_feasible():
    t, c, K, T, B, beta = _random_case(7, 2, 3, (1, 2, 4, 6, 8), 1, 1, 1)
    L, H, s = 2, 3, 1
    N = orc.heads_to_prune(T, t, s, B)
    assert all(n == 0 for n in N)
    orders = orc.head_orders(beta, L, H, K, s)
    sch = orc.heatkv_schedule(orders, N, t, s, L, H, B)
    assert all(len(sch[n][k]) == 0 for n in "GE" for k in range(1, K))
    t, c, K, T, B, beta = _random_case(8, 3, 3, (1, 2, 4, 6, 8, 12), 1, 1, 3)
    L, H, s = 3, 3, 1
    N = orc.heads_to_prune(T, t, s, B)
    orders = orc.head_orders(beta, L, H, K, s)
    nv = orc.heatkv_schedule(orders, N, t, s, L, H, B, naive=True)
    gr = orc.heatkv_schedule(orders, N, t, s, L, H, B)
    empty = orc._Sets(K, L, H)
    for k in range(1, K):
        Gp = nv["G"][k - 1] if k > 1 else empty
        assert np.array_equal(nv["E"][k].m, nv["G"][k].m & ~Gp.m)
        assert len(gr["E"][k]) <= len(nv["E"][k])
        for layer in range(1, L + 1):
            assert orc.cache_size_after_layer(k, layer, nv["G"][k], Gp, nv["E"][k], t, c, s, L, H) <= B


@pytest.mark.parametrize("seed", [0, 1, 2, 3])
def test_binary_greedy_has_minimum_cardinality_by_brute_force(seed):
    # Prop. 1: among all feasible subsets of G_k \ G_{k-1}, the greedy one is smallest.
    rng = np.random.default_rng(seed)
    L, H, s = 3, 2, 1
    t = orc.one_based([1, 2, 4, 6, 9])
    c = orc.cumulative(t)
    K, T = 5, L * H
    B = int(T * c[K - 1] * 0.45)
    N = orc.heads_to_prune(T, t, s, B)
    heads = [(l, h) for l in range(1, L + 1) for h in range(1, H + 1)]
    order = [heads[j] for j in rng.permutation(T)]
    sch = orc.binary_heatkv_schedule(order, N, t, s, L, H, B)
    empty = orc._Sets(K, L, H)
    checked = 0
    for k in range(1, K):
        Gp = sch["G"][k - 1] if k > 1 else empty
        cand = [it for it in sch["G"][k].items() if it not in Gp]
        best = None
        for r in range(len(cand) + 1):
            for sub in itertools.combinations(cand, r):
                Es = orc._Sets(K, L, H, sub)
                if all(orc.cache_size_after_layer(k, l, sch["G"][k], Gp, Es, t, c, s, L, H, binary=True) <= B
                       for l in range(1, L + 1)):
                    best = r
                    break
            if best is not None:
                break
        assert best is not None and len(sch["E"][k]) == best
        checked += len(cand) > 0
    assert checked > 0


def test_zero_based_present_view_matches_retained_scales():
    t, c, K, T, B, beta = _random_case(9, 2, 2, (1, 2, 4, 6, 8), 1, 1, 2)
    L, H, s = 2, 2, 1
    N = orc.heads_to_prune(T, t, s, B)
    sch = orc.heatkv_schedule(orc.head_orders(beta, L, H, K, s), N, t, s, L, H, B)
    pres = orc.to_zero_based_present(sch["A"], K, L, H, s)
    assert pres.shape == (K, L, H, K)
    for k in range(K):
        assert not pres[k, :, :, k:].any()
        assert pres[k, :, :, :min(s, k)].all()
    # once dropped a prior scale never returns
    for k in range(1, K - 1):
        assert np.all(pres[k + 1, :, :, :k] <= pres[k, :, :, :k])


def _beta_with_scores(L, H, K, i_scores):
    """A 1-based beta table whose S-CAS sum for source scale i of flat head j is i_scores[i][j]
    (all of it placed in row tau = i + 1)."""
    beta = np.zeros((L + 1, H + 1, K + 1, K + 1))
    for i, sc in i_scores.items():
        for j, v in enumerate(sc):
            beta[j // H + 1, j % H + 1, i + 1, i] = v
    return beta


def test_rank_dispersion_closed_forms():
    # App. C: identical runs give zero; two runs with exactly reversed orders put head at ranks r and T-1-r,
    # so its deviation is |r - (T-1)/2| and the mean over heads is T/4 for even T.
    L, H, K, s = 2, 3, 5, 1
    T = L * H
    up = {i: [float(j) for j in range(T)] for i in range(s + 1, K)}
    down = {i: [float(T - j) for j in range(T)] for i in range(s + 1, K)}
    a, b = _beta_with_scores(L, H, K, up), _beta_with_scores(L, H, K, down)
    same = orc.rank_dispersion([a, a, a], L, H, K, s)
    assert all(v == 0.0 for v in same.values()) and sorted(same) == list(range(s + 1, K))
    rev = orc.rank_dispersion([a, b], L, H, K, s)
    for i in range(s + 1, K):
        assert abs(rev[i] - T / 4) < 1e-12
    # one head swaps places with its neighbour in one of three runs: two heads have ranks (r, r, r+1) and
    # (r+1, r+1, r): population std sqrt(2)/3 each, all others 0
    sw = {i: list(up[i]) for i in up}
    sw[2][0], sw[2][1] = up[2][1], up[2][0]
    c = _beta_with_scores(L, H, K, sw)
    one = orc.rank_dispersion([a, a, c], L, H, K, s)
    assert abs(one[2] - 2 * (np.sqrt(2) / 3) / T) < 1e-12 and one[3] == 0.0


@pytest.mark.parametrize("seed", [0, 1])
def test_rank_dispersion_against_numpy_argsort_and_std(seed):
    # independent route: numpy's stable argsort of the S-CAS sums, rank = inverse permutation, numpy's std
    from tests import harness
    L, H, K, s, R = 3, 4, 6, 2, 5
    T = L * H
    betas0 = [harness.random_beta(seed * 10 + r, L, H, K) for r in range(R)]
    got = orc.rank_dispersion([orc.beta_one_based(b) for b in betas0], L, H, K, s)
    for i in range(s + 1, K):  # 1-based source scale
        ranks = np.empty((R, T))
        for r, b in enumerate(betas0):
            score = b.reshape(T, K, K).astype(np.float64)[:, i:, i - 1].sum(axis=1)  # rows tau = i+1..K (0-based i..K-1)
            order = np.argsort(score, kind="stable")
            ranks[r, order] = np.arange(T)
        want = np.std(ranks, axis=0).mean()
        assert abs(got[i] - want) < 1e-9
    # binary variant: one CAS order for every source scale
    gb = orc.rank_dispersion([orc.beta_one_based(b) for b in betas0], L, H, K, s, binary=True)
    ranks = np.empty((R, T))
    for r, b in enumerate(betas0):
        score = b.reshape(T, K, K).astype(np.float64)[:, K - 1, s:K - 1].sum(axis=1)
        ranks[r, np.argsort(score, kind="stable")] = np.arange(T)
    want = np.std(ranks, axis=0).mean()
    assert all(abs(v - want) < 1e-9 for v in gb.values())


def test_scale_dependent_greedy_is_not_minimum_cardinality():
    # The paper proves minimum cardinality of E_k for the binary variant only.  This hand-worked instance
    # (tests/golden/alg1_scale_dependent_not_minimal.txt) shows that the scale-dependent variant, followed as
    # printed, can pop more elements than necessary; the oracle must reproduce the printed order, not repair it.
    path = os.path.join(os.path.dirname(__file__), "golden", "alg1_scale_dependent_not_minimal.txt")
    rec = {}
    for line in open(path):
        if line.startswith("#") or not line.strip():
            continue
        key, *rest = line.split()
        rec[key] = rest
    items = lambda toks: [tuple(int(x) for x in tok.split(",")) for tok in toks]
    L, H, s, B = 3, 1, 1, 15
    t = orc.one_based([1, 4, 9, 16])
    c = orc.cumulative(t)
    K, T = 4, L * H
    N = orc.heads_to_prune(T, t, s, B)
    assert N[1:] == [int(x) for x in rec["N"]]
    order = [(1, 1), (2, 1), (3, 1)]
    sch = orc.heatkv_schedule({2: order, 3: order}, N, t, s, L, H, B)
    k = int(rec["GREEDY_E"][0])
    assert sorted(sch["E"][k].items()) == sorted(items(rec["GREEDY_E"][1:]))
    Gp = sch["G"][k - 1]
    sizes = lambda E: [orc.cache_size_after_layer(k, l, sch["G"][k], Gp, orc._Sets(K, L, H, E), t, c, s, L, H)
                       for l in range(1, L + 1)]
    assert sizes(items(rec["GREEDY_E"][1:])) == [int(x) for x in rec["SIZES_GREEDY"]]
    smaller = items(rec["SMALLER_FEASIBLE_E"][1:])
    assert sizes(smaller) == [int(x) for x in rec["SIZES_SMALLER"]] and max(sizes(smaller)) <= B
    assert len(smaller) < len(sch["E"][k])
    # brute force agrees that 2 is the minimum
    cand = [it for it in sch["G"][k].items() if it not in Gp]
    best = min(r for r in range(len(cand) + 1) for sub in itertools.combinations(cand, r) if max(sizes(sub)) <= B)
    assert best == len(smaller)


# --------------------------------------------------------------------------
# Binary-HeatKV (Alg. 1, binary form; App. A binary CachedTokens) and the Naive policy (Sec. 4.2)
# --------------------------------------------------------------------------

BINARY_GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "alg1_binary_hand_example.txt")


def _load_binary_golden():
    rec = dict(G={}, E={}, A={}, M={}, NAIVE_E={}, NAIVE_A={}, R={}, N=None)
    for line in open(BINARY_GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        p = line.split()
        if p[0] == "N":
            rec["N"] = [int(x) for x in p[1:]]
        elif p[0] == "M":
            rec["M"][int(p[1])] = [int(x) for x in p[2:]]
        elif p[0] == "R":
            rec["R"][(int(p[1]), int(p[2]), int(p[3]))] = [int(x) for x in p[5:]]
        else:
            rec[p[0]][int(p[1])] = _parse_items(p[2:])
    return rec


def _heads_of(S):
    """Heads (l, h) of a binary set (the oracle keeps them in slot i = 0)."""
    return sorted((l, h) for (i, l, h) in S.items() if i == 0)


def _pin_binary_hand_example():
    g = _load_binary_golden()
    L, H, s, B = 3, 2, 1, 39
    t = orc.one_based([1, 2, 4, 6, 9])
    c = orc.cumulative(t)
    K = 5
    a, b, c_, d, e, f = (1, 1), (1, 2), (2, 1), (2, 2), (3, 1), (3, 2)
    order = [d, a, f, c_, b, e]
    N = orc.heads_to_prune(L * H, t, s, B)
    assert N[1:] == g["N"]
    sch = orc.binary_heatkv_schedule(order, N, t, s, L, H, B)
    for name in "GEA":
        for k, want in g[name].items():
            assert _heads_of(sch[name][k]) == want, (name, k)
    empty = orc._Sets(K, L, H)
    for k, want in g["M"].items():
        Gp = sch["G"][k - 1] if k > 1 else empty
        got = [orc.cache_size_after_layer(k, l, sch["G"][k], Gp, sch["E"][k], t, c, s, L, H, binary=True)
               for l in range(1, L + 1)]
        assert got == want, (k, got)
    for (k, l, h), want in g["R"].items():
        assert orc.retained_scales(sch["A"][k], k, l, h, s, binary=True) == want
    nv = orc.binary_heatkv_schedule(order, N, t, s, L, H, B, naive=True)
    for k, want in g["NAIVE_E"].items():
        assert _heads_of(nv["E"][k]) == want
    for k, want in g["NAIVE_A"].items():
        assert _heads_of(nv["A"][k]) == want


def test_hand_worked_example_of_binary_algorithm_1_and_naive_policy():
    _pin_binary_hand_example()


def _binary_random_case(seed, L, H, sides, s, num, den):
    rng = np.random.default_rng(seed)
    t = orc.one_based(hi.tokens_per_scale(sides))
    c = orc.cumulative(t)
    K, T = len(t) - 1, L * H
    B = (T * c[K - 1] * num) // den
    heads = [(l, h) for l in range(1, L + 1) for h in range(1, H + 1)]
    order = [heads[j] for j in rng.permutation(T)]
    return t, c, K, T, B, order, orc.heads_to_prune(T, t, s, B)


BINARY_CASES = [
    (0, 3, 4, (1, 2, 3, 4, 5, 6), 2, 1, 2),
    (1, 4, 2, (1, 2, 4, 6, 8, 12, 16), 3, 1, 4),
    (2, 2, 8, hi.SIDES_1024, 3, 1, 10),
    (3, 5, 3, (1, 2, 4, 6, 8, 12), 1, 1, 3),
    (4, 6, 2, (1, 2, 4, 6, 8, 12, 16, 20), 3, 3, 20),
]


def _pin_binary_totals_and_early_set(seed, L, H, sides, s, num, den, naive):
    """Sec. 3.2 fixes the cache total at the end of scale k: N_k c_s + (T - N_k) c_k <= B.  Eq. 5 makes N_k
    minimal, so one head more at c_k instead of c_s would exceed B: a newly pruned head of any layer but the
    first that were left in the cache would push the total after layer 1 over the budget, and a newly pruned
    head of layer 1 is already gone in that total.  Hence, for Binary-HeatKV, E_k is exactly the newly pruned
    heads outside layer 1, and the Alg. 2 total equals the Sec. 3.2 figure after every layer; for the Naive
    policy E_k is all newly pruned heads and the same total holds."""
    t, c, K, T, B, order, N = _binary_random_case(seed, L, H, sides, s, num, den)
    sch = orc.binary_heatkv_schedule(order, N, t, s, L, H, B, naive=naive)
    empty = orc._Sets(K, L, H)
    pruned_something = False
    for k in range(1, K):
        Gk, Gp = sch["G"][k], (sch["G"][k - 1] if k > 1 else empty)
        assert _heads_of(Gk) == sorted(order[:N[k]])                      # prefix of the one order
        fresh = [lh for lh in _heads_of(Gk) if (0,) + lh not in Gp]
        want_E = fresh if naive else [lh for lh in fresh if lh[0] >= 2]
        assert _heads_of(sch["E"][k]) == want_E, (k, naive)
        assert _heads_of(sch["A"][k]) == sorted(set(_heads_of(Gp)) | set(want_E))
        if k > s:
            total = N[k] * c[s] + (T - N[k]) * c[k]
            assert total <= B
            for layer in range(1, L + 1):
                got = orc.cache_size_after_layer(k, layer, Gk, Gp, sch["E"][k], t, c, s, L, H, binary=True)
                assert got == total, (k, layer, got, total)
        pruned_something |= bool(want_E)
    assert _heads_of(sch["A"][K]) == _heads_of(sch["G"][K - 1])
    assert pruned_something


@pytest.mark.parametrize("naive", [False, True])
@pytest.mark.parametrize("seed,L,H,sides,s,num,den", BINARY_CASES)
def test_binary_cache_total_is_the_sec32_figure_after_every_layer(seed, L, H, sides, s, num, den, naive):
    _pin_binary_totals_and_early_set(seed, L, H, sides, s, num, den, naive)


def _replay_cache(sch, t, s, L, H, B, N, c, binary, check_end_total=True):
    """Plays a schedule on explicit per-head cache contents (sets of scale indices), independent of the
    oracle's accounting functions: before scale k the heads (head-scales) of A_k are dropped, after each layer
    the layer's heads gain scale k unless G_k says otherwise and lose what G_k names.  What a head holds when a
    scale starts must be what retained_scales reports; the token count never exceeds B (the accounting of
    Alg. 2 counts layers that have not run as if they already held scale k, so the true count is below it)."""
    K, T = len(t) - 1, L * H
    held = {(l, h): set() for l in range(1, L + 1) for h in range(1, H + 1)}
    gone = (lambda S, i, lh: (0,) + lh in S) if binary else (lambda S, i, lh: (i,) + lh in S)
    for k in range(1, K + 1):
        for lh in held:
            held[lh] = {i for i in held[lh] if i <= s or not gone(sch["A"][k], i, lh)}
            assert sorted(held[lh]) == orc.retained_scales(sch["A"][k], k, lh[0], lh[1], s, binary=binary)
        if k == K:
            break
        for layer in range(1, L + 1):
            for h in range(1, H + 1):
                lh = (layer, h)
                held[lh].add(k)
                held[lh] = {i for i in held[lh] if i <= s or not gone(sch["G"][k], i, lh)}
            assert sum(t[i] for v in held.values() for i in v) <= B
        if check_end_total and k > s:
            kept = T * c[k] - sum(t[i] * N[k] for i in range(s + 1, k + 1))
            assert sum(t[i] for v in held.values() for i in v) == kept


@pytest.mark.parametrize("naive", [False, True])
@pytest.mark.parametrize("seed,L,H,sides,s,num,den", BINARY_CASES)
def test_binary_schedule_replayed_on_explicit_cache_contents(seed, L, H, sides, s, num, den, naive):
    t, c, K, T, B, order, N = _binary_random_case(seed, L, H, sides, s, num, den)
    sch = orc.binary_heatkv_schedule(order, N, t, s, L, H, B, naive=naive)
    _replay_cache(sch, t, s, L, H, B, N, c, binary=True)


@pytest.mark.parametrize("naive", [False, True])
@pytest.mark.parametrize("seed,L,H,sides,s,num,den", BINARY_CASES[:4])
def test_scale_dependent_schedule_replayed_on_explicit_cache_contents(seed, L, H, sides, s, num, den, naive):
    t, c, K, T, B, beta = _random_case(seed, L, H, sides, s, num, den)
    N = orc.heads_to_prune(T, t, s, B)
    sch = orc.heatkv_schedule(orc.head_orders(beta, L, H, K, s), N, t, s, L, H, B, naive=naive)
    _replay_cache(sch, t, s, L, H, B, N, c, binary=False)


def test_binary_pins_catch_a_wrong_cached_tokens(monkeypatch):
    # The pins above are only worth something if a plausible slip in the binary accounting fails them: count
    # a kept head with c_{k-1} instead of c_k (scale k's own tokens forgotten) and run them again.
    def forgot_current_scale(k, t, c, s, P):
        return np.where(P.m[0], c[s], c[k - 1]).astype(np.int64)

    monkeypatch.setattr(orc, "cached_tokens_binary", forgot_current_scale)
    with pytest.raises(AssertionError):
        _pin_binary_hand_example()
    for naive in (False, True):
        with pytest.raises(AssertionError):
            _pin_binary_totals_and_early_set(*BINARY_CASES[0], naive)
