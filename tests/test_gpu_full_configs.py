"""GPU parity at the full sizes of the stack configs (2B-like stack with calibration, 8B-like stack, serving).

The planner's sets are compared in full and bit-exactly with the oracle's on the same fp32 beta bytes.
Attention and calibration outputs are compared on a seeded sample of (layer, head, batch row, scale, query
rows): rows are independent, so a sampled row is checked exactly as in the small tests (max-abs 2e-2 for
bf16 attention, 1e-4 for masses).  The coverage fraction is printed.
"""
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


def _run_stack(name, layers, n_calib_sets, seed, n_samples, rows_per_sample=24):
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
        print(f"{name}: rank dispersion over {n_calib_sets} sets, % of T={L * H} per source scale:",
              np.round(100.0 * disp[s:K - 1] / (L * H), 3).tolist())
    else:
        beta_h = hi.expected_beta_from_weights(w, t0).astype(np.float32)

    plan = hk.heatkv_build_schedule(shape, beta_h, B * 2 * d * 2, s)
    ref = harness.oracle_schedule(beta_h, L, H, t0, s, B)
    assert plan.N().tolist() == ref["N"][1:]
    for k in range(K):
        assert np.array_equal(plan.sets(k, binding.SET_A), harness.bitmap(ref["sch"]["A"][k + 1], K, L, H, s, False))
    present = ref["present"]

    data = {l: hi.make_qkv_device(seed, l, cfg, w, DEV) for l in layers}
    ka = torch.zeros(max(plan.arena_bytes, 16), dtype=torch.uint8, device=DEV)
    va = torch.zeros_like(ka)
    outs = {}
    for kk in range(K):
        sl = slice(c[kk] - t0[kk], c[kk])
        for l in layers:
            q, k, v = data[l]
            qk, kc, vc = q[:, :, sl].contiguous(), k[:, :, sl].contiguous(), v[:, :, sl].contiguous()
            out = torch.empty_like(qk)
            if l % 2:  # alternate the fused launch and the two separate launches
                hk.heatkv_attend_append_scale(plan, l, kk, qk, kc, vc, ka, va, sm, out)
            else:
                hk.heatkv_attend_scale(plan, l, kk, qk, kc, vc, ka, va, sm, out)
                hk.heatkv_append_scale(plan, l, kk, kc, vc, ka, va)
            outs[(l, kk)] = out
    torch.cuda.synchronize()

    worst, checked_rows = 0.0, 0
    samples = [(layers[int(rng.integers(len(layers)))], int(rng.integers(H)), int(rng.integers(nb)),
                int(rng.integers(K))) for _ in range(n_samples)]
    samples += [(layers[-1], h, 0, K - 1) for h in range(0, H, max(H // 4, 1))]  # the largest scale, several heads
    for (l, h, b, kk) in samples:
        q, k, v = (x[b, h].cpu().double().numpy() for x in data[l])
        kept = [i + 1 for i in range(kk) if present[kk, l, h, i]]
        assert np.array_equal(plan.retained(kk, l, h), orc.retained_token_indices(t1, kk + 1, kept))
        rows = np.sort(rng.choice(t0[kk], size=min(rows_per_sample, t0[kk]), replace=False))
        cur = np.arange(c[kk] - t0[kk], c[kk])
        idx = np.concatenate([orc.retained_token_indices(t1, kk + 1, kept), cur])
        want = orc.attend(q[cur[rows]], k[idx], v[idx], sm)
        got = outs[(l, kk)][b, h].float().cpu().double().numpy()[rows]
        err = float(np.abs(got - want).max())
        worst = max(worst, err)
        assert err <= 2e-2, (name, l, h, b, kk, err)
        checked_rows += len(rows)
    total_rows = len(layers) * H * nb * c[-1]
    print(f"{name}: layers run {len(layers)}/{L}, sampled rows {checked_rows} of {total_rows} "
          f"({100.0 * checked_rows / total_rows:.4f} %), worst |err| {worst:.4f}, "
          f"arena/budget {plan.arena_tokens / B:.3f}")


def test_stack2b_calibrate_schedule_generate():
    # 32 layers x 16 heads, batch 2, 10x budget: 8 calibration sets -> beta -> schedule -> generation order.
    _run_stack("stack2b", layers=list(range(32)), n_calib_sets=8, seed=31, n_samples=60)


def test_stack8b_skewed_retention():
    # 40 layers x 32 heads, 20x budget; schedule from the planted weights' closed-form beta; a subset of layers.
    _run_stack("stack8b", layers=[0, 7, 19, 20, 38, 39], n_calib_sets=0, seed=41, n_samples=60)


def test_serving_batch32():
    # 32 layers x 16 heads, batch 32, 20x budget; three layers run through all scales.
    _run_stack("serving", layers=[0, 15, 31], n_calib_sets=0, seed=51, n_samples=50)
