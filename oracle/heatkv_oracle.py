"""CPU oracle for the HeatKV hot path (NumPy, fp64).  TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may use
this file.  It shares no code with the HIP library and imports nothing from
it; it is deliberately plain and slow so that it can be checked against the
paper by eye.

Indices in this file are the paper's: scales k, i in 1..K, layers l in 1..L,
heads h in 1..H (Sec. 3.1).  Arrays indexed by scale therefore carry an unused
slot 0.  `to_zero_based_*` helpers at the bottom convert results to the
0-based form that the C ABI of the library uses.

Pins (tests/test_oracle_*.py): attention against brute-force masked attention
of the whole sequence, against torch's scaled_dot_product_attention in fp64,
Q = 0 closed forms, permutation and shift invariance; masses against row sums
and the Q = 0 closed form; Eq. 5 against exact rational arithmetic and the
total-cache identity; Alg. 1, scale-dependent form, against a hand-worked
example (tests/golden/alg1_hand_example.txt) and the budget/containment
invariants; Alg. 1, binary form, against a second hand-worked example
(tests/golden/alg1_binary_hand_example.txt, which also carries the Naive
policy on the same instance), against the total of Sec. 3.2,
N_k c_s + (T - N_k) c_k, after every layer, against the closed form of E_k
that Eq. 5 and that total imply (every newly pruned head outside the first
layer is pruned early, none of the first layer is), against a replay of the
cache contents head by head, and brute-force minimum cardinality (Prop. 1);
the rank dispersion of App. C against closed forms (identical runs, reversed
orders) and against numpy's argsort/std on random tables; the 8-bit cache
format against the values the OCP FP8 specification fixes (smallest subnormal,
smallest normal, one, 448, NaN), the round trip of all 256 codes, hand-worked
ties, saturation, and torch's float8_e4m3fn cast on random values inside the
finite range.
Minimum cardinality of E_k is not a property of the scale-dependent variant
(the paper proves it for the binary case only): a hand-worked instance,
tests/golden/alg1_scale_dependent_not_minimal.txt, has the greedy order of
Alg. 1 pop three head-scales where two suffice.  There the algorithm's steps
are followed in the paper's order and pinned by the hand-worked examples and
the invariants.
"""
from __future__ import annotations

import math

import numpy as np

# --------------------------------------------------------------------------
# Sec. 3.1 notation
# --------------------------------------------------------------------------


def cumulative(t):
    """c[k] = sum_{tau=1..k} t[tau]; t and c are 1-based (slot 0 = 0)."""
    c = [0] * len(t)
    for k in range(1, len(t)):
        c[k] = c[k - 1] + int(t[k])
    return c


def one_based(t0):
    """[t_1..t_K] given 0-based -> 1-based list with a leading 0."""
    return [0] + [int(x) for x in t0]


# --------------------------------------------------------------------------
# Attention (Sec. 3.1: alpha_{l,h,k} in R^{t_k x c_k}, rows softmax-normalised)
# --------------------------------------------------------------------------


def softmax_rows(s):
    """Row softmax of a 2-D fp64 array (textbook definition, max-shifted)."""
    s = np.asarray(s, dtype=np.float64)
    e = np.exp(s - s.max(axis=1, keepdims=True))
    return e / e.sum(axis=1, keepdims=True)


def attention_probabilities(q, keys, sm_scale):
    """alpha = softmax(q keys^T * sm_scale): [t_k, n] for q [t_k, d], keys [n, d]."""
    q = np.asarray(q, dtype=np.float64)
    keys = np.asarray(keys, dtype=np.float64)
    return softmax_rows((q @ keys.T) * float(sm_scale))


def attend(q, keys, values, sm_scale):
    """softmax(q keys^T * sm_scale) values, everything in fp64."""
    return attention_probabilities(q, keys, sm_scale) @ np.asarray(values, dtype=np.float64)


def retained_token_indices(t, k, retained_scales):
    """0-based token positions, in the full sequence, of the prior scales kept.

    `retained_scales` holds 1-based scale indices i < k; their token ranges
    (c_{i-1}, c_i] are concatenated in ascending scale order.
    """
    c = cumulative(t)
    idx = []
    for i in sorted(retained_scales):
        assert 1 <= i < k
        idx.extend(range(c[i - 1], c[i]))
    return np.asarray(idx, dtype=np.int64)


def attend_scale(q_seq, k_seq, v_seq, t, k, retained_scales, sm_scale):
    """Next-scale attention of one head over its compressed cache.

    q_seq, k_seq, v_seq: [c_K, d] for one (batch row, layer, head).  The t_k
    queries of scale k attend over the tokens of the retained prior scales
    followed by all tokens of scale k itself (block-causal by scale: the
    current scale is always visible, Sec. 3.1).  Returns [t_k, d] fp64.
    """
    c = cumulative(t)
    cur = np.arange(c[k - 1], c[k])
    keys_idx = np.concatenate([retained_token_indices(t, k, retained_scales), cur])
    return attend(q_seq[cur], k_seq[keys_idx], v_seq[keys_idx], sm_scale)


# --------------------------------------------------------------------------
# 8-bit storage of the retained K/V (an extension: the paper leaves quantisation of the cache to future work,
# Sec. 5, and fixes no format; the format taken here is the one described below)
#
# Stored rows are OCP FP8 E4M3 codes: 1 sign bit, 4 exponent bits (bias 7), 3 mantissa bits; exponent field 0
# holds subnormals m * 2^-9; exponent 15 with mantissa 7 is NaN; there are no infinities; the largest finite
# magnitude is 448.  A value is stored as the nearest representable one, ties to the code with an even mantissa,
# magnitudes above 448 as 448 (saturating), NaN as NaN.  No scale factors.  Only what the cache holds is
# rounded: the current scale's K/V are attended as the caller passes them.
# --------------------------------------------------------------------------


def fp8_e4m3_decode(codes):
    """Values of E4M3 codes (uint8 array) as fp64, straight from the bit fields."""
    codes = np.asarray(codes, dtype=np.uint8)
    sign = np.where(codes & 0x80, -1.0, 1.0)
    e = ((codes >> 3) & 0xF).astype(np.int64)
    m = (codes & 0x7).astype(np.float64)
    normal = (1.0 + m / 8.0) * np.exp2((e - 7).astype(np.float64))
    subnormal = (m / 8.0) * 2.0 ** -6
    out = sign * np.where(e == 0, subnormal, normal)
    return np.where((e == 15) & ((codes & 0x7) == 7), np.nan, out)


def fp8_e4m3_encode(x):
    """Nearest E4M3 code of every value of x (any shape): the definition written out as a search over the 127
    non-negative finite values, ties to the even code, saturating at 448; the sign is carried over."""
    x = np.asarray(x, dtype=np.float64)
    grid = fp8_e4m3_decode(np.arange(127, dtype=np.uint8))  # codes 0x00..0x7E, ascending
    mag = np.minimum(np.abs(x), 448.0)
    hi = np.clip(np.searchsorted(grid, mag, side="left"), 1, 126)  # grid[hi-1] <= mag <= grid[hi]
    lo = hi - 1
    d_lo, d_hi = mag - grid[lo], grid[hi] - mag
    take_hi = (d_hi < d_lo) | ((d_hi == d_lo) & (hi % 2 == 0))  # a code is even iff its mantissa's last bit is 0
    code = np.where(take_hi, hi, lo).astype(np.uint8)
    code = np.where(np.signbit(x), code | 0x80, code).astype(np.uint8)
    return np.where(np.isnan(x), np.uint8(0x7F), code).astype(np.uint8)


def fp8_e4m3_round(x):
    """What a value reads back as after being stored in the 8-bit cache."""
    return fp8_e4m3_decode(fp8_e4m3_encode(x))


def attend_scale_fp8_cache(q_seq, k_seq, v_seq, t, k, retained_scales, sm_scale):
    """attend_scale with the retained prior-scale rows of K and V read back from 8-bit storage; the rows of the
    current scale keep their full precision."""
    c = cumulative(t)
    cur = np.arange(c[k - 1], c[k])
    prior = retained_token_indices(t, k, retained_scales)
    k_seq = np.asarray(k_seq, dtype=np.float64)
    v_seq = np.asarray(v_seq, dtype=np.float64)
    keys = np.concatenate([fp8_e4m3_round(k_seq[prior]), k_seq[cur]])
    values = np.concatenate([fp8_e4m3_round(v_seq[prior]), v_seq[cur]])
    return attend(np.asarray(q_seq, dtype=np.float64)[cur], keys, values, sm_scale)


# --------------------------------------------------------------------------
# Scale attention mass (Eq. 2)
# --------------------------------------------------------------------------


def row_masses(q_seq, k_seq, t, k1, sm_scale):
    """m[n, k2] = sum of alpha_{k1}[n, m] over the tokens m of scale k2.

    Uses the uncompressed keys of scales 1..k1.  Returns [t_{k1}, K+1]
    (column 0 unused, columns k2 > k1 zero).
    """
    c = cumulative(t)
    K = len(t) - 1
    cur = np.arange(c[k1 - 1], c[k1])
    alpha = attention_probabilities(q_seq[cur], k_seq[: c[k1]], sm_scale)
    m = np.zeros((t[k1], K + 1))
    for k2 in range(1, k1 + 1):
        m[:, k2] = alpha[:, c[k2 - 1]: c[k2]].sum(axis=1)
    return m


def beta_row(q_seq, k_seq, t, k1, sm_scale):
    """beta^d[k1, :] of Eq. 2: mean over the t_{k1} query rows of row_masses."""
    return row_masses(q_seq, k_seq, t, k1, sm_scale).mean(axis=0)


def beta_matrix(q_seq, k_seq, t, sm_scale):
    """beta^d in R^{(K+1)x(K+1)} (row/column 0 unused) for one head, one data point."""
    K = len(t) - 1
    beta = np.zeros((K + 1, K + 1))
    for k1 in range(1, K + 1):
        beta[k1] = beta_row(q_seq, k_seq, t, k1, sm_scale)
    return beta


# --------------------------------------------------------------------------
# Head-scale importance (Eq. 3, Eq. 4) and the orders O_i
# --------------------------------------------------------------------------


def s_cas(beta_lh, K, k):
    """Eq. 4 for one head: 1/(K-k) * sum_{tau=k+1..K} beta[tau, k], summed in fp64, tau ascending."""
    acc = 0.0
    for tau in range(k + 1, K + 1):
        acc += float(beta_lh[tau, k])
    return acc / (K - k)


def cas(beta_lh, K, s):
    """Eq. 3 for one head: 1/(K-s) * sum_{tau=s+1..K-1} beta[K, tau]."""
    acc = 0.0
    for tau in range(s + 1, K):
        acc += float(beta_lh[K, tau])
    return acc / (K - s)


def scas_sum(beta_lh, K, k):
    """The un-normalised sum of Eq. 4 (the 1/(K-k) factor does not change an order)."""
    acc = 0.0
    for tau in range(k + 1, K + 1):
        acc += float(beta_lh[tau, k])
    return acc


def head_orders(beta, L, H, K, s):
    """Orders {O_i : s < i < K}: heads sorted from least to most dependent on source scale i.

    beta: [L+1, H+1, K+1, K+1] (1-based, fp32 or fp64 values; sums are taken
    in fp64).  Returns dict i -> list of (l, h).  Equal scores keep ascending
    (l, h) order (the paper does not say; a stable sort on the flat head id).
    """
    orders = {}
    for i in range(s + 1, K):
        scored = []
        for l in range(1, L + 1):
            for h in range(1, H + 1):
                scored.append((scas_sum(beta[l, h], K, i), l, h))
        scored.sort(key=lambda x: x[0])  # Python's sort is stable; input is in (l,h) order
        orders[i] = [(l, h) for _, l, h in scored]
    return orders


def cas_sum(beta_lh, K, s):
    """The un-normalised sum of Eq. 3 (the 1/(K-s) factor does not change the order)."""
    acc = 0.0
    for tau in range(s + 1, K):
        acc += float(beta_lh[K, tau])
    return acc


def cas_order(beta, L, H, K, s):
    """Single order O of the binary variant, ascending CAS (Eq. 3); ties keep (l,h) order."""
    scored = []
    for l in range(1, L + 1):
        for h in range(1, H + 1):
            scored.append((cas_sum(beta[l, h], K, s), l, h))
    scored.sort(key=lambda x: x[0])
    return [(l, h) for _, l, h in scored]


def rank_dispersion(betas, L, H, K, s, binary=False):
    """Stability of the head rankings over calibration runs (App. C, S-CAS stability).

    betas: list of R tables, each [L+1, H+1, K+1, K+1] (1-based), one per calibration run.  For every source
    scale i (s < i < K) each run's order O_i gives every head a rank position (0 = pruned first).  Per head:
    the standard deviation of its R positions around the head's own mean position (population form, divide
    by R: the appendix does not say which); the result for scale i is the mean of these over all heads.
    Returns dict i -> float.  With `binary` the single CAS order is used for every i.
    """
    R = len(betas)
    T = L * H
    out = {}
    per_run_binary = [cas_order(b, L, H, K, s) for b in betas] if binary else None
    per_run = None if binary else [head_orders(b, L, H, K, s) for b in betas]
    for i in range(s + 1, K):
        pos = {}
        for r in range(R):
            order = per_run_binary[r] if binary else per_run[r][i]
            for rank, lh in enumerate(order):
                pos.setdefault(lh, []).append(rank)
        total = 0.0
        for l in range(1, L + 1):
            for h in range(1, H + 1):
                ranks = pos[(l, h)]
                mean = sum(ranks) / R
                var = 0.0
                for x in ranks:
                    var += (x - mean) * (x - mean)
                total += math.sqrt(var / R)
        out[i] = total / T
    return out


# --------------------------------------------------------------------------
# Budget allocation (Eq. 5)
# --------------------------------------------------------------------------


def heads_to_prune(T, t, s, B):
    """N_k of Eq. 5 for k = 1..K-1 with B = b*T*c_{K-1} integer tokens.

    N_k = ceil(T (c_k - b c_{K-1}) / (c_k - c_s)) = ceil((T c_k - B)/(c_k - c_s))
    for k > s, clamped below at 0; 0 for k <= s.  Raises if N_k > T (the
    sinks alone exceed the budget, no feasible answer).  Returns a 1-based
    list of length K (slot 0 unused).
    """
    c = cumulative(t)
    K = len(t) - 1
    N = [0] * K
    for k in range(s + 1, K):
        num = T * c[k] - B
        den = c[k] - c[s]
        n = -((-num) // den)  # integer ceiling
        n = max(n, 0)
        if n > T:
            raise ValueError("budget below the sink scales: N_k > T")
        N[k] = n
    return N


# --------------------------------------------------------------------------
# Removal order optimisation (Alg. 1, Alg. 2 and CachedTokens of App. A)
# --------------------------------------------------------------------------


class _Sets:
    """A set of head-scales (i, l, h) as a boolean array member[i, l, h] (1-based)."""

    def __init__(self, K, L, H, items=()):
        self.m = np.zeros((K + 1, L + 1, H + 1), dtype=bool)
        for (i, l, h) in items:
            self.m[i, l, h] = True

    def copy(self):
        o = _Sets.__new__(_Sets)
        o.m = self.m.copy()
        return o

    def add(self, item):
        self.m[item] = True

    def union(self, other):
        o = self.copy()
        o.m |= other.m
        return o

    def items(self):
        return [tuple(int(x) for x in r) for r in np.argwhere(self.m)]

    def __contains__(self, item):
        return bool(self.m[item])

    def __len__(self):
        return int(self.m.sum())


def cached_tokens_scale_dependent(k, t, c, s, P):
    """Tokens each head holds once scale k is in, scale-dependent form (App. A), all heads at once.

    The sinks (c_s tokens) plus t_i for every source scale s < i <= k whose head-scale (i,l,h) is not in
    the pruned set P  ->  array [L+1, H+1].
    """
    out = np.full(P.m.shape[1:], c[s], dtype=np.int64)
    for i in range(s + 1, k + 1):
        out += t[i] * (~P.m[i]).astype(np.int64)
    return out


def cached_tokens_binary(k, t, c, s, P):
    """Tokens each head holds once scale k is in, binary form (App. A): a head of the pruned set P holds
    the sinks only (c_s), any other head everything up to scale k (c_k).  P.m[0] carries the head set."""
    return np.where(P.m[0], c[s], c[k]).astype(np.int64)


def cache_size_after_layer(k, layer, G_k, G_km1, E_k, t, c, s, L, H, binary=False):
    """Alg. 2 (App. A): the cache total the budget is checked against after `layer` of scale k has run.

    A layer that has run holds what it will hold at the end of the scale (everything in G_k is gone from
    it); a layer that has not run yet is only missing what was taken out before the scale started,
    G_{k-1} and the early-pruned set E_k.  Both per-head tables count scale k itself as cached.
    """
    gone_before_scale = G_km1.union(E_k)
    count = cached_tokens_binary if binary else cached_tokens_scale_dependent
    per_head_run = count(k, t, c, s, G_k)                  # [L+1, H+1]
    per_head_pending = count(k, t, c, s, gone_before_scale)
    return int(per_head_run[1:layer + 1, 1:H + 1].sum() + per_head_pending[layer + 1:L + 1, 1:H + 1].sum())


def greedy_early_pruning(k, G_km1, G_k, B, rank, t, c, s, L, H, binary=False, naive=False):
    """The early-pruning step of Alg. 1 (Sec. 3.3).  Returns (E_k as _Sets, the items in the order taken).

    The head(-scale)s that scale k newly marks for removal, G_k minus G_{k-1}, are queued deepest layer
    first, then latest source scale first, then lowest rank in their order first.  Walking the layers in
    execution order, the queue's front is moved into E_k for as long as the total of Alg. 2 after that layer
    is above the budget B.  `naive` is the boundary policy of Sec. 4.2 ("Pruning Algorithm"): the whole
    queue is pruned early, E_k = G_k minus G_{k-1}.
    """
    K = len(t) - 1
    fresh = [it for it in G_k.items() if it not in G_km1]
    queue = sorted(fresh, key=lambda it: (-it[1], -it[0], rank[it]))
    E = _Sets(K, L, H)
    taken = []
    if naive:
        for it in queue:
            E.add(it)
            taken.append(it)
        return E, taken
    for layer in range(1, L + 1):
        while cache_size_after_layer(k, layer, G_k, G_km1, E, t, c, s, L, H, binary) > B:
            if not queue:
                raise ValueError("early pruning cannot reach the budget")
            it = queue.pop(0)
            E.add(it)
            taken.append(it)
    return E, taken


def heatkv_schedule(orders, N, t, s, L, H, B, naive=False):
    """Alg. 1, scale-dependent (green) variant.

    orders: dict i -> list of (l, h) for s < i < K.  N: 1-based list from
    heads_to_prune.  Returns dict with G, E, A: dict k -> _Sets for k = 1..K
    (A[K] := G[K-1]: nothing is cached at the last scale so no early pruning
    applies; G[K], E[K] are not defined and are left out).
    """
    K = len(t) - 1
    c = cumulative(t)
    rank = {}
    for i, O in orders.items():
        for r, (l, h) in enumerate(O):
            rank[(i, l, h)] = r
    G, E, A = {0: _Sets(K, L, H)}, {}, {}
    for k in range(1, K):
        Gk = _Sets(K, L, H)
        for i in range(s + 1, k + 1):
            for (l, h) in orders[i][: N[k]]:
                Gk.add((i, l, h))
        Ek, _ = greedy_early_pruning(k, G[k - 1], Gk, B, rank, t, c, s, L, H, naive=naive)
        G[k], E[k] = Gk, Ek
        A[k] = G[k - 1].union(Ek)
    A[K] = G[K - 1].copy()
    del G[0]
    return dict(G=G, E=E, A=A)


def binary_heatkv_schedule(order, N, t, s, L, H, B, naive=False):
    """Alg. 1, binary (blue) variant: the prunable unit is a head; sets use slot i = 0."""
    K = len(t) - 1
    c = cumulative(t)
    rank = {(0, l, h): r for r, (l, h) in enumerate(order)}
    G, E, A = {0: _Sets(K, L, H)}, {}, {}
    for k in range(1, K):
        Gk = _Sets(K, L, H)
        for (l, h) in order[: N[k]]:
            Gk.add((0, l, h))
        Ek, _ = greedy_early_pruning(k, G[k - 1], Gk, B, rank, t, c, s, L, H, binary=True, naive=naive)
        G[k], E[k] = Gk, Ek
        A[k] = G[k - 1].union(Ek)
    A[K] = G[K - 1].copy()
    del G[0]
    return dict(G=G, E=E, A=A)


def retained_scales(A_k, k, l, h, s, binary=False):
    """Prior scales i < k whose tokens head (l,h) still holds when scale k is generated.

    Sink scales i <= s always; a later scale i iff (i,l,h) is not in A_k
    (binary: iff the head is not in A_k).
    """
    out = []
    for i in range(1, k):
        if i <= s:
            out.append(i)
        elif binary:
            if (0, l, h) not in A_k:
                out.append(i)
        elif (i, l, h) not in A_k:
            out.append(i)
    return out


# --------------------------------------------------------------------------
# 0-based views for comparison with the C ABI
# --------------------------------------------------------------------------


def to_zero_based_present(A, K, L, H, s, binary=False):
    """present[k0][l0][h0][i0] = 1 iff prior scale i0 is attended at scale k0 by head (l0,h0)."""
    present = np.zeros((K, L, H, K), dtype=np.uint8)
    for k in range(1, K + 1):
        for l in range(1, L + 1):
            for h in range(1, H + 1):
                for i in retained_scales(A[k], k, l, h, s, binary):
                    present[k - 1, l - 1, h - 1, i - 1] = 1
    return present


def to_zero_based_bitmap(S, K, L, H):
    """_Sets -> uint8 [K][L*H] with [i0][l0*H+h0] = 1 iff (i0+1, l0+1, h0+1) in S."""
    return S.m[1:, 1:, 1:].reshape(K, L * H).astype(np.uint8)


def beta_one_based(beta0):
    """[L,H,K,K] 0-based -> [L+1,H+1,K+1,K+1] 1-based (same dtype)."""
    L, H, K, _ = beta0.shape
    out = np.zeros((L + 1, H + 1, K + 1, K + 1), dtype=beta0.dtype)
    out[1:, 1:, 1:, 1:] = beta0
    return out


def orders_zero_based(orders, H):
    """dict i -> [(l,h)]  ->  dict i0 -> list of flat head ids l0*H + h0."""
    return {i - 1: [(l - 1) * H + (h - 1) for (l, h) in O] for i, O in orders.items()}
