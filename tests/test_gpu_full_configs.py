"""GPU parity at the full sizes of the stack configs (2B-like stack with calibration, 8B-like stack, serving).

Every layer of a stack runs in generation order over one shared pair of arenas.  The planner's sets are compared
in full and bit-exactly with the oracle's on the same fp32 beta bytes.  Attention is compared (max-abs 2e-2, the
bf16 bar) on
  * a seeded sample of query rows for EVERY (layer, head, scale): one batch row per head (rotating over the
    heads), four rows per scale, the first or the last row of the scale always among them (the last row sits in
    the ragged tail of the last query tile);
  * all query rows of a seeded subset of head-scales, among them the heads with the longest and the shortest
    retained run of every layer at the last scale.
Rows are independent, so a sampled row is checked exactly as in the small tests.  Calibration masses: 1e-4.
The coverage is printed.
"""
import sys
import time

import numpy as np
import pytest
import torch

import heatkv_inputs as hi
import paper_2605_14877_amd as hk
from paper_2605_14877_amd import binding
from oracle import heatkv_oracle as orc
from tests import harness

pytestmark = pytest.mark.gpu
DEV = "cuda"
ROWS_PER_HEAD_SCALE = 4


def _calibrate_stack(cfg, shape, w, t0, c, sm, n_sets, seed, rng, n_mass_samples):
    """Runs heatkv_calibrate over n_sets activation sets and all layers; returns beta (host) and mass checks."""
    L, H, K, nb = cfg["L"], cfg["H"], len(t0), cfg["batch"]
    beta = torch.zeros(L, H, K, K, device=DEV)
    beta_sets = torch.zeros(n_sets, L, H, K, K, device=DEV)  # one table per activation set (App. C runs)
    mass = torch.empty(nb, H, K, device=DEV)
    ws = [torch.empty(max(binding.calibrate_workspace_bytes(shape, k1), 4), dtype=torch.uint8, device=DEV)
          for k1 in range(K)]
    mass_all = [torch.empty(nb, H, K, device=DEV) for _ in range(K)]
    ws_all = torch.empty(binding.calibrate_scales_workspace_bytes(shape, list(range(K))), dtype=torch.uint8, device=DEV)
    picks = {(int(rng.integers(n_sets)), int(rng.integers(L)), int(rng.integers(K))) for _ in range(n_mass_samples)}
    picks.add((1 % n_sets, L - 1, K - 1))
    picks.add((0, 0, K - 1))
    checks = []
    for st in range(n_sets):
        for l in range(L):
            q, k, _ = hi.make_qkv_device(seed + st, l, cfg, w, DEV)
            qs = [q[:, :, c[k1] - t0[k1]:c[k1]].contiguous() for k1 in range(K)]
            kas = [k[:, :, :c[k1]].contiguous() for k1 in range(K)]
            if st % 2:  # odd sets: all scales of the layer in one launch, masses kept per scale
                hk.heatkv_calibrate_scales_accumulate(shape, l, list(range(K)), qs, kas, sm, 1.0 / (n_sets * nb),
                                                      beta, mass_all, ws_all)
            for k1 in range(K):
                if st % 2:
                    m = mass_all[k1]
                else:
                    m = mass
                    hk.heatkv_calibrate(shape, l, k1, qs[k1], kas[k1], sm, mass, ws[k1])
                    hk.heatkv_accumulate_beta(shape, l, k1, mass, 1.0 / (n_sets * nb), beta)
                hk.heatkv_accumulate_beta(shape, l, k1, m, 1.0 / nb, beta_sets[st])
                if (st, l, k1) in picks:
                    b, h = int(rng.integers(nb)), int(rng.integers(H))
                    checks.append((k1, m[b, h].cpu().double().numpy(), q[b, h].cpu(), k[b, h].cpu()))
    torch.cuda.synchronize()
    return beta.cpu().numpy(), checks, beta_sets.cpu().numpy()


def _sample_rows(rng, t_k, l, h, kk):
    """Four query rows of a scale (all of them when it has fewer); row 0 or the last row is always one of them."""
    n = min(ROWS_PER_HEAD_SCALE, t_k)
    rows = rng.choice(t_k, size=n, replace=False)
    rows[0] = 0 if (l + h + kk) % 2 else t_k - 1
    return np.unique(rows)


def _run_stack(name, n_calib_sets, seed, capsys, n_full_extra=12):
    def say(msg):  # progress lines reach the terminal even under pytest's capture
        with capsys.disabled():
            print(f"[{name}] {msg}", flush=True)

    t_begin = time.time()
    cfg = hi.CONFIGS[name]
    L, H, d, s, nb = cfg["L"], cfg["H"], cfg["d"], cfg["sinks"], cfg["batch"]
    t0 = hi.tokens_per_scale(cfg["sides"])
    c = hi.cumulative_tokens(t0)
    K = len(t0)
    sm = 1.0 / np.sqrt(d)
    B = hi.budget_tokens(cfg)
    rng = np.random.default_rng(seed)
    w = hi.head_weights(seed, L, H, K)
    shape = hk.Shape(L, H, d, t0, nb, "bf16")
    t1 = orc.one_based(t0)

    if n_calib_sets:
        beta_h, checks, beta_sets = _calibrate_stack(cfg, shape, w, t0, c, sm, n_calib_sets, seed, rng, 10)
        for k1, got, q_bh, k_bh in checks:
            want = orc.beta_row(q_bh.double().numpy(), k_bh.double().numpy(), t1, k1 + 1, sm)[1:]
            assert np.abs(got - want).max() <= 1e-4, (name, k1)
        assert np.abs(beta_h.sum(-1) - 1.0).max() <= 1e-4
        # Stability of the head orders over the activation sets (App. C): library against oracle on the same
        # per-set beta bytes; the figure itself is reported as a fraction of the ordering range T.
        disp = hk.heatkv_rank_dispersion(shape, beta_sets, s)
        want = orc.rank_dispersion([orc.beta_one_based(b) for b in beta_sets], L, H, K, s)
        for i in range(s, K - 1):
            assert abs(disp[i] - want[i + 1]) <= 1e-9 * max(1.0, want[i + 1])
        say(f"calibrated {n_calib_sets} sets; rank dispersion, % of T={L * H} per source scale: "
            f"{np.round(100.0 * disp[s:K - 1] / (L * H), 3).tolist()}")
    else:
        beta_h = hi.expected_beta_from_weights(w, t0).astype(np.float32)

    plan = hk.heatkv_build_schedule(shape, beta_h, B * 2 * d * 2, s)
    ref = harness.oracle_schedule(beta_h, L, H, t0, s, B)
    assert plan.N().tolist() == ref["N"][1:]
    for k in range(K):
        assert np.array_equal(plan.sets(k, binding.SET_A), harness.bitmap(ref["sch"]["A"][k + 1], K, L, H, s, False))
    present = ref["present"]

    # what will be compared, fixed before anything runs
    b_of = np.array([[(l * H + h + seed) % nb for h in range(H)] for l in range(L)])
    rows_of = {(l, h, kk): _sample_rows(rng, t0[kk], l, h, kk) for l in range(L) for h in range(H) for kk in range(K)}
    full = set()
    for l in range(L):
        ln = plan.runs(K - 1, l)[1]
        full.add((l, int(np.argmax(ln)), K - 1))
        full.add((l, int(np.argmin(ln)), K - 1))
    while len(full) < 2 * L + n_full_extra:
        full.add((int(rng.integers(L)), int(rng.integers(H)), int(rng.integers(K - 1))))

    data = [hi.make_qkv_device(seed, l, cfg, w, DEV) for l in range(L)]
    torch.cuda.synchronize()
    say(f"inputs resident ({sum(x.numel() * 2 for x in data[0]) * L / 1e9:.1f} GB), {time.time() - t_begin:.0f} s")
    ka = torch.zeros(max(plan.arena_bytes, 16), dtype=torch.uint8, device=DEV)
    va = torch.zeros_like(ka)
    hsel = torch.arange(H, device=DEV)
    got_rows, got_full = {}, {}
    for kk in range(K):
        sl = slice(c[kk] - t0[kk], c[kk])
        n_r = max(len(rows_of[(0, h, kk)]) for h in range(H))
        for l in range(L):
            q, k, v = data[l]
            qk, kc, vc = q[:, :, sl].contiguous(), k[:, :, sl].contiguous(), v[:, :, sl].contiguous()
            out = torch.empty_like(qk)
            if l % 2:  # alternate the fused launch and the two separate launches
                hk.heatkv_attend_append_scale(plan, l, kk, qk, kc, vc, ka, va, sm, out)
            else:
                hk.heatkv_attend_scale(plan, l, kk, qk, kc, vc, ka, va, sm, out)
                hk.heatkv_append_scale(plan, l, kk, kc, vc, ka, va)
            # keep only what will be compared: the sampled rows of every head, whole heads of the `full` set
            rsel = np.zeros((H, n_r), dtype=np.int64)
            for h in range(H):
                r = rows_of[(l, h, kk)]
                rsel[h, :len(r)] = r
            bsel = torch.from_numpy(b_of[l]).to(DEV)
            got_rows[(l, kk)] = out[bsel[:, None], hsel[:, None], torch.from_numpy(rsel).to(DEV)].float().cpu()
            for h in range(H):
                if (l, h, kk) in full:
                    got_full[(l, h, kk)] = out[b_of[l, h], h].float().cpu()
    torch.cuda.synchronize()
    say(f"generation order done: {L} layers x {K} scales, {time.time() - t_begin:.0f} s")

    worst, checked_rows, checked_hs = 0.0, 0, 0
    for l in range(L):
        for h in range(H):
            b = int(b_of[l, h])
            q, k, v = (x[b, h].cpu().double().numpy() for x in data[l])
            for kk in range(K):
                kept = [i + 1 for i in range(kk) if present[kk, l, h, i]]
                idx_prior = orc.retained_token_indices(t1, kk + 1, kept)
                assert np.array_equal(plan.retained(kk, l, h), idx_prior)
                cur = np.arange(c[kk] - t0[kk], c[kk])
                idx = np.concatenate([idx_prior, cur])
                rows = rows_of[(l, h, kk)]
                if (l, h, kk) in full:
                    want = orc.attend(q[cur], k[idx], v[idx], sm)
                    err = float(np.abs(got_full[(l, h, kk)].double().numpy() - want).max())
                    assert err <= 2e-2, (name, "all rows", l, h, b, kk, err)
                    worst = max(worst, err)
                    checked_rows += t0[kk]
                want = orc.attend(q[cur[rows]], k[idx], v[idx], sm)
                got = got_rows[(l, kk)][h, :len(rows)].double().numpy()
                err = float(np.abs(got - want).max())
                assert err <= 2e-2, (name, l, h, b, kk, rows.tolist(), err)
                worst = max(worst, err)
                checked_rows += len(rows)
                checked_hs += 1
        if l % 8 == 7 or l == L - 1:
            say(f"oracle compared through layer {l}, worst |err| so far {worst:.4f}, {time.time() - t_begin:.0f} s")
    total_rows = L * H * nb * c[-1]
    assert checked_hs == L * H * K
    say(f"layers run {L}/{L}; every (layer, head, scale) sampled: {checked_hs} head-scales; all rows of "
        f"{len(full)} head-scales; rows compared {checked_rows} of {total_rows} "
        f"({100.0 * checked_rows / total_rows:.3f} %); worst |err| {worst:.4f}; "
        f"arena/budget {plan.arena_tokens / B:.3f}; {time.time() - t_begin:.0f} s")


def test_stack2b_calibrate_schedule_generate(capsys):
    # 32 layers x 16 heads, batch 2, 10x budget: 8 calibration sets -> beta -> schedule -> generation order.
    _run_stack("stack2b", n_calib_sets=8, seed=31, capsys=capsys)


def test_stack8b_skewed_retention(capsys):
    # 40 layers x 32 heads, 20x budget; schedule from the planted weights' closed-form beta; all 40 layers.
    _run_stack("stack8b", n_calib_sets=0, seed=41, capsys=capsys)


def test_serving_batch32(capsys):
    # 32 layers x 16 heads, batch 32, 20x budget; all 32 layers, 132 GB of activations resident.
    _run_stack("serving", n_calib_sets=0, seed=51, capsys=capsys)
