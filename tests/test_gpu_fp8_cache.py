"""GPU parity of the 8-bit cache (HEATKV_KV_FP8_E4M3): what append_scale stores is compared byte for byte with the
oracle's E4M3 codes, attention over the stored rows with the oracle's attention over the rows read back
(max-abs 2e-2, the bf16 bar: reading the codes back is exact, so the kernel's error budget is unchanged)."""
import numpy as np
import pytest
import torch

import heatkv_inputs as hi
import paper_2605_14877_amd as hk
from oracle import heatkv_oracle as orc
from tests import harness

pytestmark = pytest.mark.gpu
TOL = 2e-2


def _case(L, H, sides, s, den, batch, seed, spikes=False):
    t0 = hi.tokens_per_scale(sides)
    c = hi.cumulative_tokens(t0)
    K, d = len(t0), 128
    cfg = dict(L=L, H=H, d=d, dtype="bf16", batch=batch, sides=sides)
    B = L * H * c[-2] // den
    w = hi.head_weights(seed, L, H, K)
    beta0 = hi.expected_beta_from_weights(w, t0).astype(np.float32)
    shape = hk.Shape(L, H, d, t0, batch, "bf16")
    plan = hk.heatkv_build_schedule(shape, beta0, B * 2 * d * 1, s, kv_format=hk.KV_FP8_E4M3)  # 1 byte per element
    assert plan.budget_tokens == B and plan.kv_format == hk.KV_FP8_E4M3
    assert plan.arena_bytes == batch * plan.arena_tokens * d
    ref = harness.oracle_schedule(beta0, L, H, t0, s, B)
    qkv = [hi.make_qkv(seed, l, cfg, w=w) for l in range(L)]
    if spikes:  # values at and beyond the ends of the E4M3 range, subnormals, ties, signed zeros
        g = torch.Generator().manual_seed(seed)
        vals = torch.tensor([448.0, 449.0, 464.0, 1000.0, -1000.0, -460.0, 2.0 ** -9, 2.0 ** -10, -(2.0 ** -10) * 1.5,
                             3 * 2.0 ** -10, 1.0625, 1.1875, -0.0, 0.0, 2.0 ** -7, 2.0 ** -6 * 0.9375, 6e-4, 240.0])
        for (_, k, v) in qkv:
            for x in (k, v):
                flat = x.view(-1)
                pos = torch.randint(0, flat.numel(), (4000,), generator=g)
                flat[pos] = vals[torch.randint(0, len(vals), (4000,), generator=g)].to(torch.bfloat16)
    return t0, c, K, d, shape, plan, ref, qkv


def _run(plan, qkv, t0, c, sm, fused_layers=(), check_codes=None):
    """Generation order over all layers; after every cache update `check_codes(kk, l, ka, va)` may inspect the arenas."""
    K, L = len(t0), len(qkv)
    dq = [tuple(x.cuda() for x in xs) for xs in qkv]
    ka = torch.zeros(max(plan.arena_bytes, 16), dtype=torch.uint8, device="cuda")
    va = torch.zeros_like(ka)
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
            if check_codes is not None and kk + 1 < K:
                torch.cuda.synchronize()
                check_codes(kk, l, ka, va)
    torch.cuda.synchronize()
    return outs


def _check_attention(outs, qkv, t0, present, sm, sample_from=None, sample_rows=128, seed=0):
    rng = np.random.default_rng(seed)
    t1 = orc.one_based(t0)
    c = hi.cumulative_tokens(t0)
    worst = 0.0
    for l, (q, k, v) in enumerate(qkv):
        nb, H = q.shape[0], q.shape[1]
        for kk in range(len(t0)):
            got = outs[l][kk].float().cpu().double().numpy()
            for b in range(nb):
                for h in range(H):
                    kept = [i + 1 for i in range(kk) if present[kk, l, h, i]]
                    qs, ks, vs = (x[b, h].double().numpy() for x in (q, k, v))
                    if sample_from is not None and kk >= sample_from and t0[kk] > sample_rows:
                        rows = np.sort(rng.choice(t0[kk], size=sample_rows, replace=False))
                        rows[-1] = t0[kk] - 1
                        cur = np.arange(c[kk] - t0[kk], c[kk])
                        prior = orc.retained_token_indices(t1, kk + 1, kept)
                        keys = np.concatenate([orc.fp8_e4m3_round(ks[prior]), ks[cur]])
                        vals = np.concatenate([orc.fp8_e4m3_round(vs[prior]), vs[cur]])
                        want = orc.attend(qs[cur[rows]], keys, vals, sm)
                        g = got[b, h][rows]
                    else:
                        want = orc.attend_scale_fp8_cache(qs, ks, vs, t1, kk + 1, kept, sm)
                        g = got[b, h]
                    err = float(np.abs(g - want).max())
                    worst = max(worst, err)
                    assert err <= TOL, (l, kk, b, h, err)
    return worst


def test_append_stores_the_oracles_codes_byte_for_byte():
    # two layers, three heads, ragged scales; K/V carry values beyond +-448 (saturation), subnormals, exact ties
    # and signed zeros.  After every cache update every head's run must hold exactly the oracle's codes of the rows it
    # retains, in order: rows converted when they entered and moved unchanged since.
    t0, c, K, d, shape, plan, ref, qkv = _case(2, 3, (1, 2, 4, 6, 9, 11, 14), 2, 3, 2, seed=71, spikes=True)
    sm = 1.0 / np.sqrt(d)
    checked = [0]

    def check_codes(kk, l, ka, va):
        rows, lens = plan.runs(kk + 1, l)
        kah = ka.view(shape.batch, plan.arena_tokens, d).cpu().numpy()
        vah = va.view(shape.batch, plan.arena_tokens, d).cpu().numpy()
        for h in range(shape.H):
            idx = plan.retained(kk + 1, l, h)
            assert len(idx) == lens[h]
            for b in range(shape.batch):
                want_k = orc.fp8_e4m3_encode(qkv[l][1][b, h].double().numpy()[idx])
                want_v = orc.fp8_e4m3_encode(qkv[l][2][b, h].double().numpy()[idx])
                assert np.array_equal(kah[b, rows[h]:rows[h] + lens[h]], want_k), (kk, l, h, b, "K")
                assert np.array_equal(vah[b, rows[h]:rows[h] + lens[h]], want_v), (kk, l, h, b, "V")
                checked[0] += 2 * int(lens[h]) * d
    _run(plan, qkv, t0, c, sm, fused_layers=(1,), check_codes=check_codes)
    assert checked[0] > 100000
    # (no attention check here: outputs near 448 are beyond what a bf16 result can hold to 2e-2)


@pytest.mark.parametrize("L,H,sides,s,den,batch,seed", [
    (1, 4, (1, 2, 4, 6, 8, 11, 13), 3, 3, 2, 72),                      # ragged tails in both directions
    (2, 3, (1, 2, 4, 6, 8, 12, 16, 20, 24, 32), 3, 4, 2, 73),          # several cache tiles per head, two layers
    (1, 2, (1, 3, 20, 22), 1, 1, 1, 74),                               # full budget: everything kept, long runs
])
def test_attention_over_the_8_bit_cache_matches_the_oracle(L, H, sides, s, den, batch, seed):
    t0, c, K, d, shape, plan, ref, qkv = _case(L, H, sides, s, den, batch, seed)
    sm = 1.0 / np.sqrt(d)
    sep = _run(plan, qkv, t0, c, sm)
    fused = _run(plan, qkv, t0, c, sm, fused_layers=tuple(range(L)))
    for l in range(L):
        for a, b in zip(sep[l], fused[l]):
            assert torch.equal(a, b)  # one launch or two: the same bits
    worst = _check_attention(sep, qkv, t0, ref["present"], sm)
    print(f"fp8 cache {sides}: worst |err| {worst:.4f}")


def test_8_bit_cache_with_two_query_sets_per_workgroup():
    # 1225 tokens on 104 (batch row, head) pairs: the launch takes the instance whose workgroups hold 256 queries
    # (eight wavefronts copy and convert every tile together); the last query tile has a partly filled second set,
    # the retained runs end in ragged 8-bit tiles; one launch or two: the same bits.
    t0, c, K, d, shape, plan, ref, qkv = _case(1, 13, (1, 2, 4, 8, 35), 2, 3, 8, seed=76)
    sm = 1.0 / np.sqrt(d)
    sep = _run(plan, qkv, t0, c, sm)
    fused = _run(plan, qkv, t0, c, sm, fused_layers=(0,))
    for a, b in zip(sep[0], fused[0]):
        assert torch.equal(a, b)
    worst = _check_attention(sep, qkv, t0, ref["present"], sm, sample_from=4)
    print(f"fp8 cache, two query sets: worst |err| {worst:.4f}")


def test_layer2b_full_size_with_8_bit_cache():
    # one 2B-like layer at its real shape; the same byte budget as the bf16 case now holds twice the tokens
    cfg = hi.CONFIGS["layer2b"]
    t0, c, K, d, shape, plan, ref, qkv = _case(1, cfg["H"], cfg["sides"], cfg["sinks"], 2, cfg["batch"], seed=75)
    native = hk.heatkv_build_schedule(hk.Shape(1, cfg["H"], d, t0, cfg["batch"], "bf16"),
                                      hi.expected_beta_from_weights(hi.head_weights(75, 1, cfg["H"], K), t0).astype(np.float32),
                                      plan.budget_tokens * 2 * d * 1, cfg["sinks"])
    assert native.budget_tokens * 2 == plan.budget_tokens  # same bytes, half the tokens in bf16
    assert plan.arena_bytes < native.arena_bytes * 1.2
    sm = 1.0 / np.sqrt(d)
    outs = _run(plan, qkv, t0, c, sm, fused_layers=(0,))
    worst = _check_attention(outs, qkv, t0, ref["present"], sm, sample_from=8)
    print(f"layer2b with 8-bit cache: worst |err| {worst:.4f}")


def test_8_bit_cache_is_refused_where_it_does_not_exist():
    t0 = hi.tokens_per_scale(hi.SIDES_TINY)
    with pytest.raises(hk.HeatKVError):
        hk.heatkv_build_schedule(hk.Shape(1, 4, 64, t0, 1, "f32"), harness.random_beta(0, 1, 4, 4), 42 * 512, 1,
                                 kv_format=hk.KV_FP8_E4M3)
    with pytest.raises(hk.HeatKVError):
        hk.heatkv_build_schedule(hk.Shape(1, 4, 128, t0, 1, "bf16"), harness.random_beta(0, 1, 4, 4), 42 * 512, 1,
                                 kv_format=7)
