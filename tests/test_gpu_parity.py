"""GPU parity: the HIP path behind the C ABI against the fp64 oracle on the same seeded bytes.

Tolerances (max-abs): attention 1e-5 for fp32 inputs, 2e-2 for bf16 inputs; calibration masses 1e-4.
Rankings, schedules and retained-index lists are compared bit-exactly in test_abi_cpu.py.
"""
import numpy as np
import pytest
import torch

import heatkv_inputs as hi
import paper_2605_14877_amd as hk
from paper_2605_14877_amd import probe as hp
from oracle import heatkv_oracle as orc
from tests import harness
from tests.gpu_driver import device_generation, oracle_rows

pytestmark = pytest.mark.gpu
TOL = {"f32": 1e-5, "bf16": 2e-2}


def _dev(*xs):
    return tuple(x.cuda() for x in xs)


def _check_all(outs, q, k, v, t0, present, layer, sm, tol, sample_from=None, sample_rows=192, seed=0):
    """Compares every (b,h,k); from scale `sample_from` on only a seeded sample of query rows."""
    rng = np.random.default_rng(seed)
    worst = 0.0
    nb, H = q.shape[0], q.shape[1]
    for kk in range(len(t0)):
        got = outs[kk].float().cpu().double().numpy()
        for b in range(nb):
            for h in range(H):
                kept = [i for i in range(kk) if present[kk, layer, h, i]]
                rows = None
                if sample_from is not None and kk >= sample_from and t0[kk] > sample_rows:
                    rows = np.sort(rng.choice(t0[kk], size=sample_rows, replace=False))
                    rows[-1] = t0[kk] - 1
                want = oracle_rows(q, k, v, t0, kk, b, h, kept, sm, rows)
                g = got[b, h] if rows is None else got[b, h][rows]
                err = np.abs(g - want).max()
                worst = max(worst, err)
                assert err <= tol, (kk, b, h, err)
    return worst


def test_tiny_fp32_explicit_half_budget_schedule():
    cfg = hi.CONFIGS["tiny"]
    t0 = hi.tokens_per_scale(cfg["sides"])
    K, L, H = len(t0), cfg["L"], cfg["H"]
    sm = 1.0 / np.sqrt(cfg["d"])
    w = hi.head_weights(3, L, H, K)
    q, k, v = hi.make_qkv(11, 0, cfg, w=w)
    present = hi.explicit_keep_pattern(7, L, H, t0, hi.budget_tokens(cfg))
    shape = hk.Shape(L, H, cfg["d"], t0, cfg["batch"], "f32")
    plan = hk.heatkv_load_schedule(shape, present)
    outs = device_generation(plan, 0, *_dev(q, k, v), t0, sm)
    _check_all(outs, q, k, v, t0, present, 0, sm, TOL["f32"])
    # the order of append and attend within a scale does not change the result
    outs2 = device_generation(plan, 0, *_dev(q, k, v), t0, sm, append_first=True)
    for a, b in zip(outs, outs2):
        assert torch.equal(a, b)
    # neither does running both in one launch
    outs3 = device_generation(plan, 0, *_dev(q, k, v), t0, sm, fused=True)
    for a, b in zip(outs, outs3):
        assert torch.equal(a, b)


def test_tiny_fp32_full_budget_equals_uncompressed_attention():
    cfg = hi.CONFIGS["tiny"]
    t0 = hi.tokens_per_scale(cfg["sides"])
    c = hi.cumulative_tokens(t0)
    K, H = len(t0), cfg["H"]
    sm = 1.0 / np.sqrt(cfg["d"])
    q, k, v = hi.make_qkv(5, 0, cfg)
    shape = hk.Shape(1, H, cfg["d"], t0, 1, "f32")
    plan = hk.heatkv_build_schedule(shape, harness.random_beta(0, 1, H, K), H * c[-2] * 512, 1)
    outs = device_generation(plan, 0, *_dev(q, k, v), t0, sm)
    got = torch.cat(outs, dim=2).cpu().double().numpy()
    # brute force: one block-causal attention over the whole sequence in fp64
    sc = np.concatenate([np.full(t0[i], i) for i in range(K)])
    mask = sc[None, :] <= sc[:, None]
    for h in range(H):
        s = (q[0, h].double().numpy() @ k[0, h].double().numpy().T) * sm
        s[~mask] = -np.inf
        p = np.exp(s - s.max(1, keepdims=True))
        want = (p / p.sum(1, keepdims=True)) @ v[0, h].double().numpy()
        assert np.abs(got[0, h] - want).max() <= TOL["f32"]


@pytest.mark.parametrize("d,L,H,sides,s,den,batch", [
    (64, 2, 3, (1, 2, 4, 8, 5), 1, 2, 2),
    (128, 1, 2, (1, 3, 4, 6, 9), 2, 3, 1),
])
def test_fp32_schedule_from_alg1_multi_layer(d, L, H, sides, s, den, batch):
    t0 = hi.tokens_per_scale(sides)
    c = hi.cumulative_tokens(t0)
    K = len(t0)
    sm = 1.0 / np.sqrt(d)
    cfg = dict(L=L, H=H, d=d, dtype="f32", batch=batch, sides=sides)
    B = L * H * c[-2] // den
    beta0 = harness.random_beta(4, L, H, K)
    shape = hk.Shape(L, H, d, t0, batch, "f32")
    plan = hk.heatkv_build_schedule(shape, beta0, B * 2 * d * 4, s)
    ref = harness.oracle_schedule(beta0, L, H, t0, s, B)
    nbytes = max(plan.arena_bytes, 16)
    arenas = (torch.zeros(nbytes, dtype=torch.uint8, device="cuda"), torch.zeros(nbytes, dtype=torch.uint8, device="cuda"))
    qkv = [hi.make_qkv(21, l, cfg) for l in range(L)]
    dq = [_dev(*x) for x in qkv]
    # generation order: scale outer, layer inner, one shared arena
    cN = hi.cumulative_tokens(t0)
    outs = [[None] * K for _ in range(L)]
    for kk in range(K):
        sl = slice(cN[kk] - t0[kk], cN[kk])
        for l in range(L):
            qk, kc, vc = (x[:, :, sl].contiguous() for x in dq[l])
            out = torch.empty_like(qk)
            hk.heatkv_attend_scale(plan, l, kk, qk, kc, vc, arenas[0], arenas[1], sm, out)
            hk.heatkv_append_scale(plan, l, kk, kc, vc, arenas[0], arenas[1])
            outs[l][kk] = out
    torch.cuda.synchronize()
    for l in range(L):
        _check_all(outs[l], *qkv[l], t0, ref["present"], l, sm, TOL["f32"])


def _bf16_case(L, H, sides, s, den, batch, seed, sample_from=None, fused=False, d=128):
    t0 = hi.tokens_per_scale(sides)
    c = hi.cumulative_tokens(t0)
    K = len(t0)
    sm = 1.0 / np.sqrt(d)
    cfg = dict(L=L, H=H, d=d, dtype="bf16", batch=batch, sides=sides)
    B = L * H * c[-2] // den
    w = hi.head_weights(seed, L, H, K)
    beta0 = hi.expected_beta_from_weights(w, t0).astype(np.float32)
    shape = hk.Shape(L, H, d, t0, batch, "bf16")
    plan = hk.heatkv_build_schedule(shape, beta0, B * 2 * d * 2, s)
    ref = harness.oracle_schedule(beta0, L, H, t0, s, B)
    q, k, v = hi.make_qkv(seed, 0, cfg, w=w)
    outs = device_generation(plan, 0, *_dev(q, k, v), t0, sm, fused=fused)
    if fused:  # the fused launch must reproduce the two separate launches bit for bit
        outs_sep = device_generation(plan, 0, *_dev(q, k, v), t0, sm)
        for a, b in zip(outs, outs_sep):
            assert torch.equal(a, b)
    return _check_all(outs, q, k, v, t0, ref["present"], 0, sm, TOL["bf16"], sample_from=sample_from)


def _generation_all_layers(plan, dq, t0, sm, fused_layers=()):
    """Generation order over a whole stack: scale outer, layer inner, one shared pair of arenas.
    dq[l] = (q, k, v) device tensors of layer l.  Returns outs[l][k]."""
    c = hi.cumulative_tokens(t0)
    K, L = len(t0), len(dq)
    nbytes = max(plan.arena_bytes, 16)
    ka = torch.zeros(nbytes, dtype=torch.uint8, device="cuda")
    va = torch.zeros(nbytes, dtype=torch.uint8, device="cuda")
    outs = [[None] * K for _ in range(L)]
    for kk in range(K):
        sl = slice(c[kk] - t0[kk], c[kk])
        for l in range(L):
            qk, kc, vc = (x[:, :, sl].contiguous() for x in dq[l])
            out = torch.empty_like(qk)
            if l in fused_layers:
                hk.heatkv_attend_append_scale(plan, l, kk, qk, kc, vc, ka, va, sm, out)
            else:
                hk.heatkv_attend_scale(plan, l, kk, qk, kc, vc, ka, va, sm, out)
                hk.heatkv_append_scale(plan, l, kk, kc, vc, ka, va)
            outs[l][kk] = out
    torch.cuda.synchronize()
    return outs


@pytest.mark.parametrize("variant", [hk.VARIANT_BINARY, hk.VARIANT_NAIVE, hk.VARIANT_BINARY_NAIVE])
@pytest.mark.parametrize("dtype,d", [("bf16", 128), ("f32", 64)])
def test_generation_under_binary_and_naive_plans(variant, dtype, d):
    # Alg. 1's binary path (one CAS order, a head keeps all or only the sinks), the Naive policy of Sec. 4.2
    # (E_k = G_k minus G_{k-1}) and both together: three layers in generation order over one arena, every
    # (layer, batch row, head, scale, query row) against the oracle's attention over the oracle's retained
    # scales for that variant.  The budget is tight enough that every variant prunes early somewhere.
    L, H, s, batch = 3, 4, 2, 2
    sides = (1, 2, 4, 6, 9, 12, 17) if dtype == "bf16" else (1, 2, 4, 6, 9, 11)
    t0 = hi.tokens_per_scale(sides)
    c = hi.cumulative_tokens(t0)
    K = len(t0)
    sm = 1.0 / np.sqrt(d)
    esz = hi.elem_bytes(dtype)
    cfg = dict(L=L, H=H, d=d, dtype=dtype, batch=batch, sides=sides)
    B = (L * H * c[-2] * 2) // 5
    w = hi.head_weights(40 + variant, L, H, K)
    beta0 = hi.expected_beta_from_weights(w, t0).astype(np.float32)
    shape = hk.Shape(L, H, d, t0, batch, dtype)
    plan = hk.heatkv_build_schedule(shape, beta0, B * 2 * d * esz, s, variant)
    ref = harness.oracle_schedule(beta0, L, H, t0, s, B, variant=variant)
    binary = bool(variant & 1)
    assert any(len(ref["sch"]["E"][k]) > 0 for k in range(1, K))
    for k in range(K):
        assert np.array_equal(plan.sets(k, hk.binding.SET_A), harness.bitmap(ref["sch"]["A"][k + 1], K, L, H, s, binary))
    if binary:  # every head holds either everything or the sinks only
        for k in range(K):
            for l in range(L):
                assert set(plan.runs(k, l)[1].tolist()) <= {c[k - 1] if k else 0, c[min(s, k) - 1] if min(s, k) else 0}
    qkv = [hi.make_qkv(50 + variant, l, cfg, w=w) for l in range(L)]
    outs = _generation_all_layers(plan, [_dev(*x) for x in qkv], t0, sm, fused_layers=(1,))
    worst = 0.0
    for l in range(L):
        for kk in range(K):
            for h in range(H):
                kept = [i + 1 for i in range(kk) if ref["present"][kk, l, h, i]]
                assert kept == orc.retained_scales(ref["sch"]["A"][kk + 1], kk + 1, l + 1, h + 1, s, binary=binary)
                assert np.array_equal(plan.retained(kk, l, h), orc.retained_token_indices(ref["t"], kk + 1, kept))
        worst = max(worst, _check_all(outs[l], *qkv[l], t0, ref["present"], l, sm, TOL[dtype]))
    print(f"variant {variant} {dtype}: worst |err| {worst:.2e}")


def test_bf16_small_ragged_scales():
    # several key tiles, ragged tails in both the query and the key direction
    _bf16_case(1, 4, (1, 2, 4, 6, 8, 11, 13), 3, 3, 2, seed=2)


def test_bf16_non_square_token_maps():
    # a 2:1 pyramid (h x 2h token maps), token counts that are no squares and no multiples of the tile sizes
    sides = ((1, 2), (2, 3), (3, 6), (5, 10), (7, 13), (9, 19), (12, 23))
    _bf16_case(2, 3, sides, 2, 3, 2, seed=8, fused=True)


def test_bf16_fused_attend_append_medium():
    # attend + append in one launch, scales up to 32x32 tokens, several key tiles per head
    _bf16_case(1, 6, (1, 2, 4, 6, 8, 12, 16, 20, 24, 32), 3, 4, 2, seed=5, fused=True)


def test_bf16_two_key_streams_per_workgroup():
    # Launches that give every compute unit at most one workgroup use the instance with two key streams per
    # workgroup (scales of 384 tokens and more).  Token counts 400, 441 and 529 with ragged query and key tiles:
    # heads whose walk has an odd number of tiles leave the second stream idle in the last step, the last query
    # tile has idle wavefronts, and the two streams merge partial sums taken against different references.
    _bf16_case(1, 5, (1, 2, 4, 20, 21, 23), 2, 3, 2, seed=21, fused=True)
    _bf16_case(2, 3, (1, 3, 20, 22), 1, 2, 1, seed=22)


def test_bf16_two_query_sets_per_workgroup():
    # Scales of 1024 tokens and more whose launch gives every compute unit at least two rounds of them use the
    # instance whose workgroups take 256 queries (eight wavefronts sharing every K/V tile), unless the last such
    # tile would be mostly empty.
    # 1225 tokens on 104 (batch row, head) pairs: the last query tile holds 201 rows (second set: two full
    # wavefronts, one with 9 rows, one idle); ragged key tiles; fused = separate bit for bit.
    _bf16_case(1, 13, (1, 2, 4, 8, 35), 2, 3, 8, seed=91, sample_from=4, fused=True)
    # 4150 tokens (a 50 x 83 map) on 32 pairs, every prior scale retained: 17 query tiles, the last with 54 rows
    # (first set: one full wavefront and one with 22 rows; the second set idle but still copying its share).
    _bf16_case(1, 4, ((1, 1), (2, 2), (4, 4), (35, 35), (50, 83)), 1, 1, 8, seed=92, sample_from=3)


def test_bf16_head_dimension_64():
    # rows of 128 bytes: 8 KB tiles, four MFMA steps per score block, two accumulator blocks, its own swizzles.
    # Ragged tails in both directions, several tiles per head, fused = separate, and 1024-token scales.
    _bf16_case(1, 4, (1, 2, 4, 6, 8, 11, 13), 3, 3, 2, seed=81, d=64)
    _bf16_case(2, 3, ((1, 2), (2, 3), (3, 6), (5, 10), (7, 13), (9, 19), (12, 23)), 2, 3, 2, seed=82, fused=True, d=64)
    _bf16_case(1, 6, (1, 2, 4, 6, 8, 12, 16, 20, 24, 32), 3, 4, 2, seed=83, fused=True, d=64)
    _bf16_case(1, 2, (1, 2, 4, 9, 20, 22), 2, 1, 1, seed=84, d=64)  # full budget: the longest runs


def test_bf16_budget_extremes():
    # Full budget: nothing is pruned, every head walks all prior scales (the longest runs the layout can hold).
    # Smallest legal budget (the sink scales only): every head keeps just the sinks.  Both at sizes that use the
    # two-stream instance (400 and 484 tokens) and the plain one.
    sides = (1, 2, 4, 9, 20, 22)
    t0 = hi.tokens_per_scale(sides)
    c = hi.cumulative_tokens(t0)
    _bf16_case(1, 2, sides, 2, 1, 1, seed=25)                     # den = 1: B = all prior tokens
    L, H, s = 1, 3, 2
    K = len(t0)
    w = hi.head_weights(26, L, H, K)
    beta0 = hi.expected_beta_from_weights(w, t0).astype(np.float32)
    shape = hk.Shape(L, H, 128, t0, 2, "bf16")
    plan = hk.heatkv_build_schedule(shape, beta0, L * H * c[s - 1] * 2 * 128 * 2, s)
    assert plan.N().tolist()[s:K - 1] == [L * H] * (K - 1 - s)
    ref = harness.oracle_schedule(beta0, L, H, t0, s, L * H * c[s - 1])
    cfg = dict(L=L, H=H, d=128, dtype="bf16", batch=2, sides=sides)
    q, k, v = hi.make_qkv(26, 0, cfg, w=w)
    outs = device_generation(plan, 0, *_dev(q, k, v), t0, 1.0 / np.sqrt(128), fused=True)
    _check_all(outs, q, k, v, t0, ref["present"], 0, 1.0 / np.sqrt(128), TOL["bf16"])


def test_bf16_thirty_one_scales():
    # The largest scale count the ABI takes (the kernel parameter tables are sized for it): schedule, attention
    # against the oracle, and all 31 scales calibrated in one launch against the per-scale calls.
    sides = tuple(range(1, 32))
    _bf16_case(1, 2, sides, 3, 3, 1, seed=27, sample_from=12)
    t0 = hi.tokens_per_scale(sides)
    c = hi.cumulative_tokens(t0)
    K, H, d, batch = len(t0), 2, 128, 1
    sm = 1.0 / np.sqrt(d)
    g = torch.Generator().manual_seed(28)
    q = torch.randn(batch, H, c[-1], d, generator=g).to(torch.bfloat16)
    k = torch.randn(batch, H, c[-1], d, generator=g).to(torch.bfloat16)
    dq, dk = _dev(q, k)
    shape = hk.Shape(1, H, d, t0, batch, "bf16")
    qs = [dq[:, :, c[i] - t0[i]:c[i]].contiguous() for i in range(K)]
    ks = [dk[:, :, :c[i]].contiguous() for i in range(K)]
    beta_a = torch.zeros(1, H, K, K, device="cuda")
    beta_b = torch.zeros(1, H, K, K, device="cuda")
    for k1 in range(K):
        ws = torch.empty(max(hk.binding.calibrate_workspace_bytes(shape, k1), 4), dtype=torch.uint8, device="cuda")
        hk.heatkv_calibrate_accumulate(shape, 0, k1, qs[k1], ks[k1], sm, 1.0, beta_a, None, ws)
    ws = torch.empty(hk.binding.calibrate_scales_workspace_bytes(shape, list(range(K))), dtype=torch.uint8, device="cuda")
    hk.heatkv_calibrate_scales_accumulate(shape, 0, list(range(K)), qs, ks, sm, 1.0, beta_b, None, ws)
    torch.cuda.synchronize()
    assert torch.equal(beta_a, beta_b)
    rows = beta_b[0].sum(-1).cpu().numpy()
    assert np.abs(rows - 1.0).max() <= 1e-4  # every query scale's masses sum to one


def test_bf16_layer2b_full_size():
    # One Infinity-2B-like layer at its real shape (16 heads, 13 scales, batch 2, 4x budget).
    cfg = hi.CONFIGS["layer2b"]
    worst = _bf16_case(1, cfg["H"], cfg["sides"], cfg["sinks"], cfg["factor"], cfg["batch"], seed=9, sample_from=8)
    print("layer2b worst abs err", worst)


def test_calibrate_tiny_fp32_and_bf16_small():
    for dtype, d, sides, batch, H in (("f32", 64, hi.SIDES_TINY, 1, 4), ("bf16", 128, (1, 2, 4, 6, 8, 12, 16), 2, 3),
                                      ("bf16", 64, (1, 2, 4, 6, 8, 12, 17), 2, 3)):
        t0 = hi.tokens_per_scale(sides)
        c = hi.cumulative_tokens(t0)
        K = len(t0)
        sm = 1.0 / np.sqrt(d)
        cfg = dict(L=1, H=H, d=d, dtype=dtype, batch=batch, sides=sides)
        w = hi.head_weights(1, 1, H, K)
        q, k, v = hi.make_qkv(13, 0, cfg, w=w)
        dq, dk = _dev(q, k)
        shape = hk.Shape(1, H, d, t0, batch, dtype)
        t1 = orc.one_based(t0)
        for k1 in range(K):
            qk = dq[:, :, c[k1] - t0[k1]:c[k1]].contiguous()
            ka = dk[:, :, :c[k1]].contiguous()
            mass = torch.full((batch, H, K), -1.0, device="cuda")
            ws = torch.empty(max(hk.binding.calibrate_workspace_bytes(shape, k1), 4), dtype=torch.uint8, device="cuda")
            hk.heatkv_calibrate(shape, 0, k1, qk, ka, sm, mass, ws)
            got = mass.cpu().double().numpy()
            # deterministic: a second run gives the same bits
            mass2 = torch.empty_like(mass)
            hk.heatkv_calibrate(shape, 0, k1, qk, ka, sm, mass2, ws)
            assert torch.equal(mass, mass2)
            for b in range(batch):
                for h in range(H):
                    want = orc.beta_row(q[b, h].double().numpy(), k[b, h].double().numpy(), t1, k1 + 1, sm)[1:]
                    assert np.abs(got[b, h] - want).max() <= 1e-4, (dtype, k1, b, h)
            assert np.abs(got.sum(-1) - 1.0).max() <= 1e-4
            # the accumulating variant gives the bits of calibrate followed by accumulate_beta
            beta_a = torch.zeros(1, H, K, K, device="cuda")
            beta_b = torch.zeros(1, H, K, K, device="cuda")
            hk.heatkv_accumulate_beta(shape, 0, k1, mass, 0.5, beta_a)
            mass3 = torch.empty_like(mass)
            hk.heatkv_calibrate_accumulate(shape, 0, k1, qk, ka, sm, 0.5, beta_b, mass3, ws)
            assert torch.equal(beta_a, beta_b) and torch.equal(mass, mass3)
            beta_c = torch.zeros(1, H, K, K, device="cuda")
            hk.heatkv_calibrate_accumulate(shape, 0, k1, qk, ka, sm, 0.5, beta_c, None, ws)
            assert torch.equal(beta_a, beta_c)


def test_bf16_rising_logits_exercise_lazy_rescale():
    # Keys are laid out so that, in the order the kernel walks them (current scale first, then the retained
    # run), the row maxima keep rising: slowly inside a scale (many tiles below the rescaling threshold, a few
    # crossings) and by a large jump at the change of segment.  Head 1 sees the mirror image (falling logits).
    sides = (1, 2, 4, 8, 16, 24)
    t0 = hi.tokens_per_scale(sides)
    c = hi.cumulative_tokens(t0)
    K, H, d, batch = len(t0), 2, 128, 1
    sm = 1.0 / np.sqrt(d)
    g = torch.Generator().manual_seed(17)
    q = (0.1 * torch.randn(batch, H, c[-1], d, generator=g))
    k = (0.1 * torch.randn(batch, H, c[-1], d, generator=g))
    v = torch.randn(batch, H, c[-1], d, generator=g)
    for i in range(K):
        lo = c[i] - t0[i]
        ramp = torch.linspace(0.0, 21.0, t0[i]) + 30.0 * (K - 1 - i)   # earlier scales sit higher
        k[:, :, lo:c[i], 0] = ramp
    q[:, 0, :, 0] = 16.0
    q[:, 1, :, 0] = -16.0
    q, k, v = (x.to(torch.bfloat16) for x in (q, k, v))
    present = np.zeros((K, 1, H, K), dtype=np.uint8)
    for kk in range(K):
        present[kk, 0, :, :kk] = 1
    shape = hk.Shape(1, H, d, t0, batch, "bf16")
    plan = hk.heatkv_load_schedule(shape, present)
    outs = device_generation(plan, 0, *_dev(q, k, v), t0, sm)
    worst = _check_all(outs, q, k, v, t0, present, 0, sm, TOL["bf16"])
    for o in outs:
        assert torch.isfinite(o.float()).all()
    print("rising logits worst abs err", worst)


def test_mfma_probe_runs_and_is_deterministic():
    # measurement aid: same operands, same sums; zero operands give zeros
    n = hp.heatkv_probe_mfma_operand_bytes() // 2
    g = torch.Generator(device="cuda").manual_seed(3)
    ops = torch.randn(n, device="cuda", generator=g).to(torch.bfloat16)
    out1 = torch.empty(4 * 256, device="cuda")
    out2 = torch.empty(4 * 256, device="cuda")
    hp.heatkv_probe_mfma(ops, out1, 4, 3)
    hp.heatkv_probe_mfma(ops, out2, 4, 3)
    torch.cuda.synchronize()
    assert torch.equal(out1, out2) and torch.isfinite(out1).all() and out1.abs().max() > 0
    hp.heatkv_probe_mfma(torch.zeros_like(ops), out1, 4, 3)
    torch.cuda.synchronize()
    assert (out1 == 0).all()
    with pytest.raises(hk.HeatKVError):
        hp.heatkv_probe_mfma(ops, out1, 0, 3)


def test_rank_dispersion_over_gpu_calibration_runs():
    # App. C on synthetic data: three seeded activation sets of one small stack, beta of each from the GPU
    # calibration pass, head-rank dispersion from the library against the oracle on the same beta bytes.
    sides, L, H, d, batch, s = (1, 2, 4, 6, 8, 12), 2, 3, 128, 2, 2
    t0 = hi.tokens_per_scale(sides)
    c = hi.cumulative_tokens(t0)
    K = len(t0)
    sm = 1.0 / np.sqrt(d)
    cfg = dict(L=L, H=H, d=d, dtype="bf16", batch=batch, sides=sides)
    w = hi.head_weights(6, L, H, K)
    shape = hk.Shape(L, H, d, t0, batch, "bf16")
    betas = []
    for run in range(3):
        beta = torch.zeros(L, H, K, K, device="cuda")
        for l in range(L):
            q, k, _ = hi.make_qkv(100 + run, l, cfg, w=w)
            dq, dk = _dev(q, k)
            for k1 in range(K):
                qk = dq[:, :, c[k1] - t0[k1]:c[k1]].contiguous()
                ka = dk[:, :, :c[k1]].contiguous()
                ws = torch.empty(max(hk.binding.calibrate_workspace_bytes(shape, k1), 4), dtype=torch.uint8, device="cuda")
                hk.heatkv_calibrate_accumulate(shape, l, k1, qk, ka, sm, 1.0 / batch, beta, None, ws)
        betas.append(beta.cpu().numpy())
    betas = np.stack(betas)
    got = hk.heatkv_rank_dispersion(shape, betas, s)
    want = orc.rank_dispersion([orc.beta_one_based(b) for b in betas], L, H, K, s)
    for i in range(s, K - 1):
        assert abs(got[i] - want[i + 1]) <= 1e-12 * max(1.0, want[i + 1])
    # the planted per-head preferences dominate the sampling noise: heads keep their places
    print("rank dispersion per source scale (heads:", L * H, "):", got[s:K - 1])
    assert got.max() <= 0.25 * L * H


def test_rank_positions_from_gpu_beta_against_oracle_beta_are_reported(capsys):
    # Rankings are compared bit-exactly on identical beta bytes elsewhere.  Here the two betas differ: the GPU's
    # (bf16 products, fp32 sums) and the oracle's (fp64), both for one 2B-like layer at full size (16 heads, 13
    # scales, both batch rows as data points).  Masses must agree to 1e-4; how many rank positions of the orders
    # O_i and of the CAS order then differ is printed, not gated: near-ties may flip.
    cfg = hi.CONFIGS["layer2b"]
    t0 = hi.tokens_per_scale(cfg["sides"])
    c = hi.cumulative_tokens(t0)
    K, L, H, d, s, nb = len(t0), 1, cfg["H"], cfg["d"], cfg["sinks"], cfg["batch"]
    sm = 1.0 / np.sqrt(d)
    w = hi.head_weights(61, L, H, K)
    q, k, _ = hi.make_qkv(61, 0, cfg, w=w)
    dq, dk = _dev(q, k)
    shape = hk.Shape(L, H, d, t0, nb, "bf16")
    beta = torch.zeros(L, H, K, K, device="cuda")
    qs = [dq[:, :, c[i] - t0[i]:c[i]].contiguous() for i in range(K)]
    ks = [dk[:, :, :c[i]].contiguous() for i in range(K)]
    ws = torch.empty(hk.binding.calibrate_scales_workspace_bytes(shape, list(range(K))), dtype=torch.uint8, device="cuda")
    hk.heatkv_calibrate_scales_accumulate(shape, 0, list(range(K)), qs, ks, sm, 1.0 / nb, beta, None, ws)
    torch.cuda.synchronize()
    beta_gpu = beta.cpu().numpy()
    t1 = orc.one_based(t0)
    beta_orc = np.zeros((L, H, K, K))
    for h in range(H):
        for b in range(nb):
            beta_orc[0, h] += orc.beta_matrix(q[b, h].double().numpy(), k[b, h].double().numpy(), t1, sm)[1:, 1:] / nb
    assert np.abs(beta_gpu - beta_orc).max() <= 1e-4
    og = orc.head_orders(orc.beta_one_based(beta_gpu), L, H, K, s)
    oo = orc.head_orders(orc.beta_one_based(beta_orc.astype(np.float32)), L, H, K, s)
    differ = {i: sum(a != b for a, b in zip(og[i], oo[i])) for i in og}
    cg = orc.cas_order(orc.beta_one_based(beta_gpu), L, H, K, s)
    co = orc.cas_order(orc.beta_one_based(beta_orc.astype(np.float32)), L, H, K, s)
    with capsys.disabled():
        print(f"\n[rank positions] GPU beta vs oracle beta, one 2B-like layer (T = {L * H}): max |beta diff| "
              f"{np.abs(beta_gpu - beta_orc).max():.2e}; positions that differ per source scale "
              f"{differ} (of {L * H} each), CAS order {sum(a != b for a, b in zip(cg, co))}", flush=True)


def test_binding_rejects_wrong_shapes_and_dtypes_on_device():
    t0 = hi.tokens_per_scale(hi.SIDES_TINY)
    shape = hk.Shape(1, 4, 64, t0, 1, "f32")
    plan = hk.heatkv_build_schedule(shape, harness.random_beta(1, 1, 4, 4), 42 * 512, 1)
    ok = torch.zeros(1, 4, t0[2], 64, device="cuda")
    arena = torch.zeros(max(plan.arena_bytes, 16), dtype=torch.uint8, device="cuda")
    with pytest.raises(ValueError, match="shape"):
        hk.heatkv_attend_scale(plan, 0, 2, ok[:, :, :3].contiguous(), ok, ok, arena, arena, 0.125, ok)
    with pytest.raises(ValueError, match="dtype"):
        hk.heatkv_attend_scale(plan, 0, 2, ok.to(torch.bfloat16), ok, ok, arena, arena, 0.125, ok)
    with pytest.raises(ValueError, match="bytes"):
        hk.heatkv_attend_scale(plan, 0, 2, ok, ok, ok, arena[:8], arena, 0.125, ok)
    with pytest.raises(ValueError, match="contiguous"):
        hk.heatkv_attend_scale(plan, 0, 2, ok.transpose(1, 2).contiguous().transpose(1, 2), ok, ok, arena, arena, 0.125, ok)
    hk.heatkv_attend_scale(plan, 0, 2, ok, ok, ok, arena, arena, 0.125, ok)  # the well-formed call goes through
    torch.cuda.synchronize()


def test_generation_pass_replays_from_a_hip_graph():
    # Once the plan is uploaded the entry points only enqueue kernels on the caller's stream, so a whole
    # generation pass can be captured and replayed; every replay must reproduce the eager results bit for bit,
    # also with other work and synchronisations between the replays.
    # (the last two scales, 400 and 484 tokens, use the kernel instance with two key streams per workgroup)
    sides, L, H, d, batch, s = (1, 2, 4, 6, 8, 12, 16, 20, 22), 1, 4, 128, 2, 2
    t0 = hi.tokens_per_scale(sides)
    c = hi.cumulative_tokens(t0)
    K = len(t0)
    sm = 1.0 / np.sqrt(d)
    cfg = dict(L=L, H=H, d=d, dtype="bf16", batch=batch, sides=sides)
    w = hi.head_weights(12, L, H, K)
    beta0 = hi.expected_beta_from_weights(w, t0).astype(np.float32)
    shape = hk.Shape(L, H, d, t0, batch, "bf16")
    plan = hk.heatkv_build_schedule(shape, beta0, (L * H * c[-2] // 3) * 2 * d * 2, s)
    plan.upload()
    q, k, v = _dev(*hi.make_qkv(12, 0, cfg, w=w))
    sl = [slice(c[i] - t0[i], c[i]) for i in range(K)]
    q_s = [q[:, :, x].contiguous() for x in sl]
    k_s = [k[:, :, x].contiguous() for x in sl]
    v_s = [v[:, :, x].contiguous() for x in sl]
    ka = torch.zeros(max(plan.arena_bytes, 16), dtype=torch.uint8, device="cuda")
    va = torch.zeros_like(ka)
    outs = [torch.empty_like(x) for x in q_s]

    def one_pass():
        for kk in range(K):
            hk.heatkv_attend_append_scale(plan, 0, kk, q_s[kk], k_s[kk], v_s[kk], ka, va, sm, outs[kk])

    one_pass()
    torch.cuda.synchronize()
    eager = [o.clone() for o in outs]
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            one_pass()
    torch.cuda.synchronize()
    for rep in range(3):
        for o in outs:
            o.fill_(float("nan"))
        ka.random_(0, 255)  # stale arena contents must not matter: every region is rewritten before it is read
        va.random_(0, 255)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for a, b in zip(outs, eager):
            assert torch.equal(a, b), rep


def test_bf16_calibrate_rising_and_falling_logits():
    # The calibration kernel keeps a lazy softmax reference; logits that climb steadily along the key blocks
    # (head 0) force the exact path again and again in the middle of a walk, head 1 sees them falling.
    sides = (1, 2, 4, 8, 16, 24)
    t0 = hi.tokens_per_scale(sides)
    c = hi.cumulative_tokens(t0)
    K, H, d, batch = len(t0), 2, 128, 1
    sm = 1.0 / np.sqrt(d)
    g = torch.Generator().manual_seed(23)
    q = 0.1 * torch.randn(batch, H, c[-1], d, generator=g)
    k = 0.1 * torch.randn(batch, H, c[-1], d, generator=g)
    k[:, :, :, 0] = torch.linspace(-20.0, 20.0, c[-1])  # keys are walked in sequence order here
    q[:, 0, :, 0] = 16.0
    q[:, 1, :, 0] = -16.0
    q, k = q.to(torch.bfloat16), k.to(torch.bfloat16)
    dq, dk = _dev(q, k)
    shape = hk.Shape(1, H, d, t0, batch, "bf16")
    t1 = orc.one_based(t0)
    for k1 in range(K):
        qk = dq[:, :, c[k1] - t0[k1]:c[k1]].contiguous()
        ka = dk[:, :, :c[k1]].contiguous()
        mass = torch.full((batch, H, K), -1.0, device="cuda")
        ws = torch.empty(max(hk.binding.calibrate_workspace_bytes(shape, k1), 4), dtype=torch.uint8, device="cuda")
        hk.heatkv_calibrate(shape, 0, k1, qk, ka, sm, mass, ws)
        got = mass.cpu().double().numpy()
        assert np.isfinite(got).all()
        for h in range(H):
            want = orc.beta_row(q[0, h].double().numpy(), k[0, h].double().numpy(), t1, k1 + 1, sm)[1:]
            assert np.abs(got[0, h] - want).max() <= 1e-4, (k1, h, np.abs(got[0, h] - want).max())


@pytest.mark.parametrize("dtype,d,sides", [("bf16", 128, (1, 2, 4, 8, 13, 20)), ("f32", 64, (1, 2, 4, 7, 9))])
def test_calibrate_all_scales_in_one_launch_has_the_bits_of_the_per_scale_calls(dtype, d, sides):
    # Calibration data of all scales is available at once, so the library can take them in one launch; masses
    # and the accumulated beta must be bit-identical to the per-scale calls, for all scales and for a subset
    # given in arbitrary order.
    t0 = hi.tokens_per_scale(sides)
    c = hi.cumulative_tokens(t0)
    K, H, batch = len(t0), 3, 2
    sm = 1.0 / np.sqrt(d)
    g = torch.Generator().manual_seed(41)
    td = torch.bfloat16 if dtype == "bf16" else torch.float32
    q = torch.randn(batch, H, c[-1], d, generator=g).to(td)
    k = torch.randn(batch, H, c[-1], d, generator=g).to(td)
    dq, dk = _dev(q, k)
    shape = hk.Shape(2, H, d, t0, batch, dtype)
    qs = [dq[:, :, c[i] - t0[i]:c[i]].contiguous() for i in range(K)]
    ks = [dk[:, :, :c[i]].contiguous() for i in range(K)]
    for k1_list in (list(range(K)), [K - 2, 0, K - 1, 2]):
        beta_a = torch.zeros(2, H, K, K, device="cuda")
        mass_a = [torch.full((batch, H, K), -1.0, device="cuda") for _ in k1_list]
        for i, k1 in enumerate(k1_list):
            ws = torch.empty(max(hk.binding.calibrate_workspace_bytes(shape, k1), 4), dtype=torch.uint8, device="cuda")
            hk.heatkv_calibrate_accumulate(shape, 1, k1, qs[k1], ks[k1], sm, 0.25, beta_a, mass_a[i], ws)
        beta_b = torch.zeros(2, H, K, K, device="cuda")
        mass_b = [torch.full((batch, H, K), -2.0, device="cuda") for _ in k1_list]
        mass_b[1] = None  # a scale whose per-row masses are not wanted
        ws = torch.empty(hk.binding.calibrate_scales_workspace_bytes(shape, k1_list), dtype=torch.uint8, device="cuda")
        hk.heatkv_calibrate_scales_accumulate(shape, 1, k1_list, [qs[i] for i in k1_list], [ks[i] for i in k1_list],
                                              sm, 0.25, beta_b, mass_b, ws)
        torch.cuda.synchronize()
        assert torch.equal(beta_a, beta_b)
        assert float(beta_b[0].abs().max()) == 0.0 and float(beta_b[1].abs().max()) > 0.0
        for i in range(len(k1_list)):
            if mass_b[i] is not None:
                assert torch.equal(mass_a[i], mass_b[i]), (k1_list, i)
    # and against the oracle for one head of the largest scale
    t1 = orc.one_based(t0)
    want = orc.beta_row(q[0, 1].double().numpy(), k[0, 1].double().numpy(), t1, K, sm)[1:]
    got = mass_a[2][0, 1].cpu().double().numpy()
    assert np.abs(got - want).max() <= 1e-4


def test_calibrate_instances_write_the_same_bits():
    # The bf16 kernel has an instance with one and one with two query sets per wavefront; the launcher takes the
    # second when its workgroups fill the chip.  Here the one-launch call over all scales gets the second (64
    # pairs, 768 workgroups), every per-scale call the first; masses and beta must still agree bit for bit, and
    # a large single scale (second instance) must agree with the oracle.
    sides = (1, 2, 4, 6, 8, 12, 16, 20, 24)
    t0 = hi.tokens_per_scale(sides)
    c = hi.cumulative_tokens(t0)
    K, H, d, batch = len(t0), 16, 128, 4
    sm = 1.0 / np.sqrt(d)
    g = torch.Generator().manual_seed(43)
    q = torch.randn(batch, H, c[-1], d, generator=g).to(torch.bfloat16)
    k = torch.randn(batch, H, c[-1], d, generator=g).to(torch.bfloat16)
    dq, dk = _dev(q, k)
    shape = hk.Shape(1, H, d, t0, batch, "bf16")
    qs = [dq[:, :, c[i] - t0[i]:c[i]].contiguous() for i in range(K)]
    ks = [dk[:, :, :c[i]].contiguous() for i in range(K)]
    beta_a = torch.zeros(1, H, K, K, device="cuda")
    mass_a = [torch.empty(batch, H, K, device="cuda") for _ in range(K)]
    for k1 in range(K):
        ws = torch.empty(max(hk.binding.calibrate_workspace_bytes(shape, k1), 4), dtype=torch.uint8, device="cuda")
        hk.heatkv_calibrate_accumulate(shape, 0, k1, qs[k1], ks[k1], sm, 0.25, beta_a, mass_a[k1], ws)
    beta_b = torch.zeros(1, H, K, K, device="cuda")
    mass_b = [torch.empty(batch, H, K, device="cuda") for _ in range(K)]
    ws = torch.empty(hk.binding.calibrate_scales_workspace_bytes(shape, list(range(K))), dtype=torch.uint8, device="cuda")
    hk.heatkv_calibrate_scales_accumulate(shape, 0, list(range(K)), qs, ks, sm, 0.25, beta_b, mass_b, ws)
    torch.cuda.synchronize()
    assert torch.equal(beta_a, beta_b)
    for k1 in range(K):
        assert torch.equal(mass_a[k1], mass_b[k1]), k1
    t1 = orc.one_based(t0)
    for b, h in ((0, 0), (3, 15), (2, 7)):
        want = orc.beta_row(q[b, h].double().numpy(), k[b, h].double().numpy(), t1, K, sm)[1:]
        assert np.abs(mass_b[K - 1][b, h].cpu().double().numpy() - want).max() <= 1e-4


def test_tile_step_probe_runs_and_is_deterministic():
    n = hp.heatkv_probe_tile_step_bytes() // 2
    g = torch.Generator(device="cuda").manual_seed(4)
    tiles = torch.randn(n, device="cuda", generator=g).to(torch.bfloat16)
    out1 = torch.empty(6 * 256, device="cuda")
    out2 = torch.empty(6 * 256, device="cuda")
    hp.heatkv_probe_tile_step(tiles, out1, 6, 4)
    hp.heatkv_probe_tile_step(tiles, out2, 6, 4)
    torch.cuda.synchronize()
    assert torch.equal(out1, out2)
    with pytest.raises(hk.HeatKVError):
        hp.heatkv_probe_tile_step(tiles, out1, 6, 3)  # odd step count
    with pytest.raises(ValueError):
        hp.heatkv_probe_tile_step(tiles[:100], out1, 6, 4)


def test_tile_stream_probe_copies_what_it_claims():
    # The read-bandwidth probe is the attention kernel's tile copy without arithmetic; its checksum words prove
    # that every step of every workgroup went through LDS in source order.
    wgs, steps = 6, 5
    nbytes = hp.heatkv_probe_tile_stream_bytes(wgs, steps)
    assert nbytes == wgs * steps * 32768
    g = torch.Generator(device="cuda").manual_seed(7)
    src = torch.randint(-2**31, 2**31 - 1, (wgs, steps, 8192), dtype=torch.int32, device="cuda", generator=g)
    out = torch.zeros(wgs, 256, dtype=torch.int32, device="cuda")
    hp.heatkv_probe_tile_stream(src, out, wgs, steps)
    torch.cuda.synchronize()
    want = src[:, 0, :256].clone()
    for t in range(1, steps):
        want ^= src[:, t, :256]
    assert torch.equal(out, want)
    with pytest.raises(hk.HeatKVError):
        hp.heatkv_probe_tile_stream(src, out, wgs, steps + 1)  # source too small
    with pytest.raises(hk.HeatKVError):
        hp.heatkv_probe_tile_stream(src, out, 0, steps)

