"""CPU-side checks of the C ABI: exported symbols, host planner bit-exact against the oracle,
error paths and the static memory layout.  No GPU needed."""
import ctypes
import os
import re

import numpy as np
import pytest

import heatkv_inputs as hi
import paper_2605_14877_amd as hk
from paper_2605_14877_amd import probe as hp
from paper_2605_14877_amd import binding
from oracle import heatkv_oracle as orc
from tests import harness

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_libraries_export_every_declared_symbol():
    # every header under include/ belongs to one shared library, which must export each function it declares
    from paper_2605_14877_amd import probe
    libs = {"heatkv.h": hk.library_path(), "heatkv_probe.h": probe.library_path()}
    inc = os.path.join(ROOT, "include")
    assert sorted(os.listdir(inc)) == sorted(libs)
    for header, path in libs.items():
        text = open(os.path.join(inc, header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names = set(re.findall(r"\b(heatkv_[a-z_A-Z0-9]+)\s*\(", text))
        if header == "heatkv.h":
            assert {"heatkv_calibrate", "heatkv_build_schedule", "heatkv_append_scale", "heatkv_attend_scale"} <= names
            assert not any(n.startswith("heatkv_probe") for n in names)  # measurement aids stay out of the product ABI
        lib = ctypes.CDLL(path)
        for n in sorted(names):
            assert hasattr(lib, n), (header, n)


def _compare(plan, ref, K, L, H, s):
    binary = ref["binary"]
    assert plan.N().tolist() == ref["N"][1:]
    oz = orc.orders_zero_based(ref["orders"], H)
    for i in range(s, K - 1):
        assert plan.order(i).tolist() == oz[i]
    for k in range(K - 1):
        assert np.array_equal(plan.sets(k, binding.SET_G), harness.bitmap(ref["sch"]["G"][k + 1], K, L, H, s, binary)), k
        assert np.array_equal(plan.sets(k, binding.SET_E), harness.bitmap(ref["sch"]["E"][k + 1], K, L, H, s, binary)), k
    for k in range(K):
        assert np.array_equal(plan.sets(k, binding.SET_A), harness.bitmap(ref["sch"]["A"][k + 1], K, L, H, s, binary)), k
    t = ref["t"]
    for k in range(K):
        for l in range(L):
            for h in range(H):
                kept = [i + 1 for i in range(k) if ref["present"][k, l, h, i]]
                want = orc.retained_token_indices(t, k + 1, kept)
                assert np.array_equal(plan.retained(k, l, h), want)


@pytest.mark.parametrize("name", ["layer2b", "stack2b", "stack8b", "serving"])
def test_planner_bit_exact_on_named_configs(name):
    cfg = hi.CONFIGS[name]
    L, H, s = cfg["L"], cfg["H"], cfg["sinks"]
    t0 = hi.tokens_per_scale(cfg["sides"])
    K = len(t0)
    beta0, _ = harness.config_beta(name)
    B = hi.budget_tokens(cfg)
    shape = hk.Shape(L, H, cfg["d"], t0, cfg["batch"], cfg["dtype"])
    plan = hk.heatkv_build_schedule(shape, beta0, B * 2 * cfg["d"] * hi.elem_bytes(cfg["dtype"]), s)
    assert plan.budget_tokens == B
    ref = harness.oracle_schedule(beta0, L, H, t0, s, B)
    if name in ("stack8b", "serving", "stack2b"):
        # full set comparison; retained lists only on a sample of heads to keep the run short
        assert plan.N().tolist() == ref["N"][1:]
        for k in range(K):
            assert np.array_equal(plan.sets(k, binding.SET_A), harness.bitmap(ref["sch"]["A"][k + 1], K, L, H, s, False))
        for k in range(K - 1):
            assert np.array_equal(plan.sets(k, binding.SET_E), harness.bitmap(ref["sch"]["E"][k + 1], K, L, H, s, False))
            assert np.array_equal(plan.sets(k, binding.SET_G), harness.bitmap(ref["sch"]["G"][k + 1], K, L, H, s, False))
        rng = np.random.default_rng(0)
        for _ in range(40):
            k, l, h = int(rng.integers(K)), int(rng.integers(L)), int(rng.integers(H))
            kept = [i + 1 for i in range(k) if ref["present"][k, l, h, i]]
            assert np.array_equal(plan.retained(k, l, h), orc.retained_token_indices(ref["t"], k + 1, kept))
    else:
        _compare(plan, ref, K, L, H, s)


@pytest.mark.parametrize("variant", [0, 1, 2, 3])
@pytest.mark.parametrize("seed,L,H,sides,s,num,den", [
    (0, 3, 4, (1, 2, 3, 4, 5, 6), 2, 1, 2),
    (1, 4, 2, (1, 2, 4, 6, 8, 12, 16), 3, 1, 4),
    (2, 2, 8, hi.SIDES_1024, 3, 1, 10),
    (3, 5, 3, (1, 2, 4, 6, 8, 12), 1, 1, 3),
    (4, 1, 4, hi.SIDES_TINY, 1, 1, 2),
    (5, 6, 1, (1, 2, 4, 6, 8), 0, 2, 5),
    (6, 2, 3, tuple(range(1, 32)), 3, 1, 5),   # 31 scales: the largest K the ABI takes
])
def test_planner_bit_exact_on_random_beta_all_variants(variant, seed, L, H, sides, s, num, den):
    t0 = hi.tokens_per_scale(sides)
    K = len(t0)
    c = hi.cumulative_tokens(t0)
    B = L * H * c[K - 2] * num // den
    beta0 = harness.random_beta(seed, L, H, K)
    # plant exact ties to exercise the tie-break
    beta0[:, 0] = beta0[:, -1]
    shape = hk.Shape(L, H, 64, t0, 1, "f32")
    plan = hk.heatkv_build_schedule(shape, beta0, B * 2 * 64 * 4, s, variant)
    ref = harness.oracle_schedule(beta0, L, H, t0, s, B, variant)
    _compare(plan, ref, K, L, H, s)


def test_more_scales_than_the_abi_takes_are_rejected():
    t0 = hi.tokens_per_scale(tuple(range(1, 33)))  # 32 scales
    assert len(t0) == 32
    with pytest.raises(hk.HeatKVError) as e:
        hk.heatkv_build_schedule(hk.Shape(1, 2, 64, t0, 1, "f32"), harness.random_beta(0, 1, 2, 32), 1 << 30, 2)
    assert e.value.code == -1


def test_layout_is_a_valid_fifo_and_respects_the_budget_accounting():
    for name in ["layer2b", "stack2b", "stack8b", "serving"]:
        cfg = hi.CONFIGS[name]
        L, H, s = cfg["L"], cfg["H"], cfg["sinks"]
        t0 = hi.tokens_per_scale(cfg["sides"])
        K = len(t0)
        beta0, _ = harness.config_beta(name)
        B = hi.budget_tokens(cfg)
        shape = hk.Shape(L, H, cfg["d"], t0, cfg["batch"], cfg["dtype"])
        plan = hk.heatkv_build_schedule(shape, beta0, B * 512, s)
        cap = plan.arena_tokens
        ref = harness.oracle_schedule(beta0, L, H, t0, s, B)
        t, c1 = ref["t"], orc.cumulative(ref["t"])
        runs = {(k, l): plan.runs(k, l) for k in range(K) for l in range(L)}
        # run lengths = retained tokens; runs of a layer are packed back to back
        for (k, l), (row, ln) in runs.items():
            want = [sum(t0[i] for i in range(k) if ref["present"][k, l, h, i]) for h in range(H)]
            assert ln.tolist() == want
            assert np.all(row + ln <= cap)
            assert np.all(row[1:] == row[:-1] + ln[:-1])
        # generation-order replay: the region written by append(l,k) never overlaps a live region
        live = {l: (0, 0) for l in range(L)}
        peak = 0
        for k in range(K - 1):
            for l in range(L):
                row, ln = runs[(k + 1, l)]
                new = (int(row[0]), int(ln.sum()))
                for l2, (b0, sz) in live.items():
                    if sz and new[1]:
                        assert new[0] + new[1] <= b0 or b0 + sz <= new[0], (k, l, l2)
                live[l] = new
                tot = sum(sz for _, sz in live.values())
                peak = max(peak, tot)
                assert tot == plan.live_tokens(k, l)
                # physical rows never exceed what Alg. 2 accounts for at the same checkpoint
                empty = orc._Sets(K, L, H)
                if k >= s and k + 1 <= K - 1 and name == "layer2b":
                    Gp = ref["sch"]["G"][k] if k >= 1 else empty
                    acc = orc.cache_size_after_layer(k + 1, l + 1, ref["sch"]["G"][k + 1], Gp, ref["sch"]["E"][k + 1],
                                                     t, c1, s, L, H)
                    assert tot <= acc <= B
        assert peak <= B
        biggest = max(int(runs[(k, l)][1].sum()) for k in range(K) for l in range(L))
        assert cap <= B + 2 * biggest


def test_load_schedule_accepts_seeded_pattern_and_rejects_bad_ones():
    cfg = hi.CONFIGS["tiny"]
    t0 = hi.tokens_per_scale(cfg["sides"])
    K, L, H = len(t0), cfg["L"], cfg["H"]
    present = hi.explicit_keep_pattern(7, L, H, t0, 42)
    kept_tokens = sum(t0[i] for l in range(L) for h in range(H) for i in range(K - 1) if present[K - 1, l, h, i])
    assert 0 < kept_tokens <= 42
    shape = hk.Shape(L, H, cfg["d"], t0, 1, "f32")
    plan = hk.heatkv_load_schedule(shape, present)
    for k in range(K):
        for h in range(H):
            want = orc.retained_token_indices(orc.one_based(t0), k + 1, [i + 1 for i in range(k) if present[k, 0, h, i]])
            assert np.array_equal(plan.retained(k, 0, h), want)
    with pytest.raises(hk.HeatKVError) as e:
        plan.N()
    assert e.value.code == -1
    bad = present.copy()
    bad[1, 0, 0, 2] = 1  # a future scale
    with pytest.raises(hk.HeatKVError):
        hk.heatkv_load_schedule(shape, bad)
    bad = np.zeros_like(present)
    bad[3, 0, 0, 0] = 1  # scale 0 absent at k=1,2 and back at k=3
    with pytest.raises(hk.HeatKVError):
        hk.heatkv_load_schedule(shape, bad)


def test_error_codes():
    t0 = hi.tokens_per_scale(hi.SIDES_TINY)
    shape = hk.Shape(1, 4, 64, t0, 1, "f32")
    beta = harness.random_beta(0, 1, 4, 4)
    with pytest.raises(hk.HeatKVError) as e:
        hk.heatkv_build_schedule(shape, beta, (4 * 5 - 1) * 512, 2)  # below the sinks (c_s = 5 per head)
    assert e.value.code == -2
    with pytest.raises(hk.HeatKVError) as e:
        hk.heatkv_build_schedule(shape, beta, 42 * 512, 3)  # sinks > K-2
    assert e.value.code == -1
    with pytest.raises(hk.HeatKVError) as e:
        hk.heatkv_build_schedule(hk.Shape(1, 4, 48, t0, 1, "f32"), beta, 42 * 512, 1)
    assert e.value.code == -1
    plan = hk.heatkv_build_schedule(shape, beta, 42 * 512, 1)
    assert plan.N().tolist() == [0, 0, 3]
    with pytest.raises(hk.HeatKVError):
        plan.order(0)
    with pytest.raises(hk.HeatKVError):
        plan.retained(4, 0, 0)
    # null tensor pointers are rejected before any GPU call
    with pytest.raises(hk.HeatKVError) as e:
        hk.heatkv_attend_scale(plan, 0, 1, None, None, None, None, None, 0.125, None, stream=0)
    assert e.value.code == -1
    with pytest.raises(hk.HeatKVError) as e:
        hk.heatkv_append_scale(plan, 0, 1, None, None, None, None, stream=0)
    assert e.value.code == -1
    with pytest.raises(hk.HeatKVError) as e:
        hp.heatkv_probe_mfma(None, None, 1, 1, stream=0)
    assert e.value.code == -1
    assert hp.heatkv_probe_mfma_operand_bytes() == 65536


def test_calibrate_scales_argument_checks():
    # everything that can be wrong with the scale list is rejected before any GPU call
    import ctypes as C
    from paper_2605_14877_amd import binding
    L = binding.lib()
    t0 = hi.tokens_per_scale(hi.SIDES_TINY)
    shape = hk.Shape(1, 4, 64, t0, 1, "f32")
    K = len(t0)
    fake = (C.c_void_p * K)(*[0x1000] * K)  # never dereferenced by the calls below

    def call(k1_list, ws_bytes, beta=0x1000, q=fake, k_all=fake):
        k1 = (C.c_int32 * max(len(k1_list), 1))(*k1_list)
        return L.heatkv_calibrate_scales_accumulate(shape.ref, 0, len(k1_list), k1, q, k_all, 0.125, 1.0, beta, None,
                                                    0x1000, ws_bytes, None)

    assert call([], 1 << 20) == -1                      # no scale
    assert call([0, 1, 2, 3, 0], 1 << 20) == -1         # more scales than the shape has
    assert call([0, 4], 1 << 20) == -1                  # index out of range
    assert call([2, 1, 2], 1 << 20) == -1               # listed twice
    assert b"twice" in L.heatkv_last_error()
    assert call([1, 2], 1 << 20, beta=None) == -1       # no beta
    assert call([1, 2], 1 << 20, q=None) == -1          # no pointer array
    need = binding.calibrate_scales_workspace_bytes(shape, [3, 1, 2])
    # per scale: batch*H * ceil(t/16) query tiles * K floats, rounded up to 256 bytes
    want = sum((1 * 4 * -(-int(t0[k]) // 16) * K * 4 + 255) // 256 * 256 for k in (3, 1, 2))
    assert need == want
    assert call([3, 1, 2], need - 1) == -1              # workspace too small
    assert b"workspace" in L.heatkv_last_error()
    assert binding.calibrate_scales_workspace_bytes(shape, [0, 7]) == 0
    with pytest.raises(ValueError, match="same length"):
        hk.heatkv_calibrate_scales_accumulate(shape, 0, [1, 2], [None], [None, None], 0.125, 1.0, None, None, None)


def test_bench_refuses_more_than_one_gpu_before_touching_any():
    # one GPU only: the benchmark says so and exits instead of starting ranks
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "one GPU" in (r.stdout + r.stderr)


def test_full_budget_plan_keeps_everything():
    t0 = hi.tokens_per_scale(hi.SIDES_TINY)
    c = hi.cumulative_tokens(t0)
    shape = hk.Shape(2, 2, 64, t0, 1, "f32")
    plan = hk.heatkv_build_schedule(shape, harness.random_beta(1, 2, 2, 4), 4 * c[-2] * 512, 1)
    for k in range(4):
        for l in range(2):
            for h in range(2):
                assert plan.retained(k, l, h).tolist() == list(range(c[k] - t0[k]))


@pytest.mark.parametrize("variant", [binding.VARIANT_HEATKV, binding.VARIANT_BINARY])
def test_head_scores_and_rank_dispersion_match_oracle(variant):
    # App. C diagnostic and the Eq. 3 / Eq. 4 sums behind the orders, on the same fp32 beta bytes
    L, H, sides, s, R = 3, 4, (1, 2, 3, 4, 6, 8), 2, 5
    t0 = hi.tokens_per_scale(sides)
    K, T = len(t0), L * H
    shape = hk.Shape(L, H, 64, t0, 1, "f32")
    betas0 = np.stack([harness.random_beta(40 + r, L, H, K) for r in range(R)])
    binary = variant == binding.VARIANT_BINARY
    # scores: sorting them (stable) reproduces the plan's orders, and they equal the oracle's sums bit for bit
    sc = hk.heatkv_head_scores(shape, betas0[0], s, variant)
    b1 = orc.beta_one_based(betas0[0])
    c = hi.cumulative_tokens(t0)
    plan = hk.heatkv_build_schedule(shape, betas0[0], T * c[-2] * 512 // 2, s, variant)
    for i in range(s, K - 1):
        for head in range(T):
            l, h = head // H + 1, head % H + 1
            want = orc.cas_sum(b1[l, h], K, s) if binary else orc.scas_sum(b1[l, h], K, i + 1)
            assert sc[i, head] == want
        assert np.argsort(sc[i], kind="stable").tolist() == plan.order(i).tolist()
    assert not sc[:s].any() and not sc[K - 1:].any()
    got = hk.heatkv_rank_dispersion(shape, betas0, s, variant)
    want = orc.rank_dispersion([orc.beta_one_based(b) for b in betas0], L, H, K, s, binary=binary)
    for i in range(K):
        if s <= i < K - 1:
            assert abs(got[i] - want[i + 1]) <= 1e-12 * max(1.0, want[i + 1])
        else:
            assert got[i] == 0.0
    # one run: no dispersion; bad arguments are rejected
    assert not hk.heatkv_rank_dispersion(shape, betas0[:1], s, variant).any()
    with pytest.raises(hk.HeatKVError):
        hk.heatkv_rank_dispersion(shape, betas0, K - 1, variant)
    with pytest.raises(hk.HeatKVError):
        hk.heatkv_head_scores(shape, betas0[0], s, 7)


def test_sink_count_sweep_matches_oracle():
    # Table 3b varies the number of sink scales s = 1..6 at a fixed budget: planner against oracle for each
    cfg = hi.CONFIGS["layer2b"]
    t0 = hi.tokens_per_scale(cfg["sides"])
    K, L, H = len(t0), cfg["L"], cfg["H"]
    beta0, _ = harness.config_beta("layer2b")
    B = hi.budget_tokens(cfg)
    shape = hk.Shape(L, H, cfg["d"], t0, cfg["batch"], cfg["dtype"])
    for s in range(1, 7):
        plan = hk.heatkv_build_schedule(shape, beta0, B * 2 * cfg["d"] * hi.elem_bytes(cfg["dtype"]), s)
        ref = harness.oracle_schedule(beta0, L, H, t0, s, B)
        _compare(plan, ref, K, L, H, s)


def test_library_follows_printed_greedy_order_where_it_is_not_minimal():
    # the instance of tests/golden/alg1_scale_dependent_not_minimal.txt: the planner pops three head-scales
    # exactly as the printed sort dictates, although two would do
    L, H, s, B = 3, 1, 1, 15
    t0 = [1, 4, 9, 16]
    K = len(t0)
    beta0 = np.zeros((L, H, K, K), dtype=np.float32)
    for l in range(L):
        beta0[l, 0, 3, 1] = beta0[l, 0, 3, 2] = beta0[l, 0, 2, 1] = 0.1 * (l + 1)  # heads ranked (1,1) < (2,1) < (3,1)
    shape = hk.Shape(L, H, 64, t0, 1, "f32")
    plan = hk.heatkv_build_schedule(shape, beta0, B * 2 * 64 * 4, s)
    ref = harness.oracle_schedule(beta0, L, H, t0, s, B)
    _compare(plan, ref, K, L, H, s)
    E = plan.sets(2, binding.SET_E)  # 0-based scale 2 = paper scale 3; bitmap [source scale][head]
    got = sorted((i + 1, head // H + 1, head % H + 1) for i in range(K) for head in range(L * H) if E[i, head])
    assert got == [(2, 3, 1), (3, 2, 1), (3, 3, 1)]


def test_binding_rejects_wrong_operands_before_any_gpu_call():
    # the kernels trust the plan's sizes; the binding checks tensors on the host (device, shape, dtype, size)
    import torch
    t0 = hi.tokens_per_scale(hi.SIDES_TINY)
    shape = hk.Shape(1, 4, 64, t0, 1, "f32")
    plan = hk.heatkv_build_schedule(shape, harness.random_beta(1, 1, 4, 4), 42 * 512, 1)
    good = torch.zeros(1, 4, t0[1], 64)  # right shape and dtype, but host memory
    with pytest.raises(ValueError, match="device tensor"):
        hk.heatkv_attend_scale(plan, 0, 1, good, good, good, good, good, 0.125, good, stream=0)
    with pytest.raises(ValueError, match="device tensor"):
        hk.heatkv_append_scale(plan, 0, 1, good, good, good, good, stream=0)
    with pytest.raises(TypeError):
        hk.heatkv_attend_scale(plan, 0, 1, np.zeros(4), None, None, None, None, 0.125, None, stream=0)
    with pytest.raises(ValueError, match="device tensor"):
        hk.heatkv_calibrate(shape, 0, 1, good, good, 0.125, good, None, stream=0)


@pytest.mark.parametrize("variant", [binding.VARIANT_BINARY, binding.VARIANT_BINARY_NAIVE])
def test_library_binary_variants_on_the_hand_worked_instance(variant):
    # the instance of tests/golden/alg1_binary_hand_example.txt, checked against the pencil-worked sets directly
    L, H, s, B = 3, 2, 1, 39
    t0 = [1, 2, 4, 6, 9]
    K, T = len(t0), L * H
    order = [(2, 2), (1, 1), (3, 2), (2, 1), (1, 2), (3, 1)]  # O = [d, a, f, c, b, e], 1-based (layer, head)
    beta0 = np.zeros((L, H, K, K), dtype=np.float32)
    for r, (l, h) in enumerate(order):  # CAS = sum over tau in (s, K) of beta[K][tau]: rising along the order
        beta0[l - 1, h - 1, K - 1, s:K - 1] = 0.01 * (r + 1)
    shape = hk.Shape(L, H, 64, t0, 1, "f32")
    plan = hk.heatkv_build_schedule(shape, beta0, B * 2 * 64 * 4, s, variant)
    assert plan.N().tolist() == [0, 0, 1, 4]
    assert plan.order(s).tolist() == [(l - 1) * H + (h - 1) for (l, h) in order]

    def heads(k0, which):  # 1-based (layer, head) of the heads the set names at 0-based scale k0
        bm = plan.sets(k0, which)
        assert all(np.array_equal(bm[s], bm[i]) for i in range(s, K - 1)) and not bm[:s].any() and not bm[K - 1].any()
        return sorted((head // H + 1, head % H + 1) for head in range(T) if bm[s, head])

    assert heads(2, binding.SET_G) == [(2, 2)]
    assert heads(3, binding.SET_G) == [(1, 1), (2, 1), (2, 2), (3, 2)]
    assert heads(2, binding.SET_E) == [(2, 2)]
    if variant == binding.VARIANT_BINARY:
        assert heads(3, binding.SET_E) == [(2, 1), (3, 2)]
        assert heads(3, binding.SET_A) == [(2, 1), (2, 2), (3, 2)]
    else:
        assert heads(3, binding.SET_E) == [(1, 1), (2, 1), (3, 2)]
        assert heads(3, binding.SET_A) == [(1, 1), (2, 1), (2, 2), (3, 2)]
    assert heads(4, binding.SET_A) == [(1, 1), (2, 1), (2, 2), (3, 2)]
    # head (1,1) at paper scale 4 keeps scales 1-3 under Binary-HeatKV (evicted after its layer), sinks only if naive
    want = list(range(0, 7)) if variant == binding.VARIANT_BINARY else [0]
    assert plan.retained(3, 0, 0).tolist() == want


def test_calibrate_static_rejects_what_does_not_fit_before_any_gpu_call():
    # 16 x 64 heads x ceil(4096/128) tiles x 13 scales x 4 bytes = 1.7 MB of partial sums: over the 1 MiB of the
    # library's static workspace.  The size is checked before any HIP call or pointer use, so dummy addresses do.
    t0 = hi.tokens_per_scale(hi.SIDES_1024)
    shape = hk.Shape(1, 64, 128, t0, 16, "bf16")
    assert binding.calibrate_workspace_bytes(shape, 12) > (1 << 20)
    rc = binding.lib().heatkv_calibrate_static(shape.ref, 0, 12, 256, 256, 0.1, 256, None)
    assert rc == -1 and b"exceed the static workspace" in binding.lib().heatkv_last_error()
    fits = hk.Shape(1, 16, 128, t0, 32, "bf16")
    assert binding.calibrate_workspace_bytes(fits, 12) <= (1 << 20)


def test_8_bit_cache_format_doubles_the_tokens_a_byte_budget_holds():
    cfg = hi.CONFIGS["layer2b"]
    t0 = hi.tokens_per_scale(cfg["sides"])
    beta0, _ = harness.config_beta("layer2b")
    shape = hk.Shape(1, cfg["H"], 128, t0, 2, "bf16")
    B = hi.budget_tokens(cfg)
    native = hk.heatkv_build_schedule(shape, beta0, B * 512, 3)
    same_tokens = hk.heatkv_build_schedule(shape, beta0, B * 256, 3, kv_format=hk.KV_FP8_E4M3)
    same_bytes = hk.heatkv_build_schedule(shape, beta0, B * 512, 3, kv_format=hk.KV_FP8_E4M3)
    assert native.kv_format == hk.KV_NATIVE and same_tokens.kv_format == hk.KV_FP8_E4M3
    assert native.budget_tokens == same_tokens.budget_tokens == B and same_bytes.budget_tokens == 2 * B
    # the schedule is a function of the token budget alone: same sets, same rows, half the bytes
    assert native.N().tolist() == same_tokens.N().tolist() and native.arena_tokens == same_tokens.arena_tokens
    assert same_tokens.arena_bytes * 2 == native.arena_bytes
    for k in range(len(t0)):
        assert np.array_equal(native.sets(k, binding.SET_A), same_tokens.sets(k, binding.SET_A))
    assert sum(same_bytes.N().tolist()) < sum(native.N().tolist())  # twice the tokens: fewer heads pruned
    for bad in (dict(shape=hk.Shape(1, 4, 64, t0[:4], 1, "f32"), fmt=hk.KV_FP8_E4M3), dict(shape=shape, fmt=5)):
        with pytest.raises(hk.HeatKVError) as e:
            hk.heatkv_build_schedule(bad["shape"], harness.random_beta(0, bad["shape"].L, bad["shape"].H, bad["shape"].K),
                                     1 << 20, 1, kv_format=bad["fmt"])
        assert e.value.code == -1
