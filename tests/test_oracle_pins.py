"""Pins for the CPU oracle: every check here compares it with something other than itself
(hand-derived counts, set enumeration, library routines, closed forms, pure-Python loops)."""
import itertools
import math
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import amskv_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
VAR_T = [s * s for s in (1, 2, 3, 4, 5, 6, 8, 10, 13, 16)]


def _golden_rows(name="kept_tokens.txt"):
    rows = []
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            name, sides, c, w, ka, counts = [x.strip() for x in line.split(";")]
            rows.append((name, [int(x) for x in sides.split(",")], int(c), int(w), bool(int(ka)),
                         [int(x) for x in counts.split(",")]))
    return rows


# ------------------------------------------------------------------ schedule / kept sets
def test_schedule_680_tokens_and_5_condensed():
    # Section 3.2 (sides 1..16, ten scales) and Appendix A (first two scales = 5 tokens)
    t = orc.scale_tokens((1, 2, 3, 4, 5, 6, 8, 10, 13, 16), (1, 2, 3, 4, 5, 6, 8, 10, 13, 16))
    assert sum(t) == 680 and t[0] + t[1] == 5
    assert orc.scale_starts(t) == [0, 1, 5, 14, 30, 55, 91, 155, 255, 424]
    sc = orc.scale_of_token(t)
    assert sc.shape == (680,) and sc[0] == 0 and sc[4] == 1 and sc[5] == 2 and sc[679] == 9 and sc[423] == 8


@pytest.mark.parametrize("row", _golden_rows(), ids=lambda r: r[0])
def test_kept_token_counts_golden(row):
    _, sides, c, w, ka, counts = row
    t = orc.scale_tokens(sides, sides)
    got = [orc.kept_token_count(t, (c, w, ka), s) for s in range(len(t))]
    assert got == counts
    assert orc.cache_capacity(t, (c, w, ka)) == max(counts)


@pytest.mark.parametrize("row", _golden_rows("stored_tokens.txt"), ids=lambda r: r[0])
def test_stored_token_counts_golden(row):
    _, sides, c, w, ka, counts = row
    t = orc.scale_tokens(sides, sides)
    got = [sum(t[k] for k in orc.stored_scales((c, w, ka), s, len(t))) for s in range(len(t))]
    assert got == counts
    assert orc.stored_capacity(t, (c, w, ka)) == max(counts)


def test_stored_scales_by_set_enumeration():
    n = 5
    for c, w in itertools.product(range(4), range(4)):
        for s in range(n):
            kept = {k for k in (set(range(c)) | set(range(s - w, s)) | {s}) if 0 <= k <= s}
            # the current scale is written only if it is condensed or the window reaches it next step
            want = kept - ({s} if (s == n - 1 or not (s < c or w >= 1)) else set())
            assert orc.stored_scales((c, w, False), s, n) == sorted(want)
        for s in range(n):
            assert orc.stored_scales((c, w, True), s, n) == [k for k in range(s + 1) if k < n - 1]


@pytest.mark.parametrize("n_scales", [3, 5])
def test_kept_sets_by_set_enumeration(n_scales):
    # taxonomy of Section 4.1: condensed = first c scales, local = the w scales before the
    # current one, plus the current scale; everything clipped to what exists
    for c, w in itertools.product(range(5), range(5)):
        prev = set()
        for s in range(n_scales):
            condensed = set(range(c))
            local = set(range(s - w, s))
            want = {k for k in (condensed | local | {s}) if 0 <= k <= s}
            got = orc.kept_scales((c, w, False), s)
            assert got == sorted(want)
            assert orc.evicted_scales((c, w, False), s) == sorted((prev | {s}) - want - {s} if s else [])
            prev = want
        for s in range(n_scales):
            assert orc.kept_scales((c, w, True), s) == list(range(s + 1))
            assert orc.evicted_scales((c, w, True), s) == []


def test_evicted_example_last_var_step():
    # {0,1}+w2 at step 9 drops scale 6 (64 tokens) and keeps 0,1,7,8,9
    assert orc.evicted_scales((2, 2, False), 9) == [6]
    assert orc.kept_scales((2, 2, False), 9) == [0, 1, 7, 8, 9]
    assert orc.segment_offsets(VAR_T, (2, 2, False), 9) == [0, 1, 5, 105, 274]


def test_bytes_held_and_eq4():
    B, H, D, e, L = 256, 30, 64, 2, 30
    pol = (2, 2, False)
    held = orc.bytes_held(VAR_T, pol, 9, B, H, D, e)
    assert held == 2 * 2 * 256 * 30 * 64 * 530
    assert orc.bytes_held(VAR_T, pol, 9, B, H, D, e, include_current=False) == 2 * 2 * 256 * 30 * 64 * 274
    vanilla = orc.bytes_held(VAR_T, (0, 0, True), 9, B, H, D, e)
    # Eq. 4 with the constant 2e: saving = vanilla - held, all layers cache-efficient
    sav_mb = orc.kv_mem_saving_eq4(VAR_T, B, H, D, L, [], 0, [0, 1, 7, 8, 9], L, bytes_per_pair=2 * e)
    assert sav_mb * 1024 ** 2 == pytest.approx(L * (vanilla - held), rel=1e-12)
    # mixed: 7 demanding layers keep everything, 23 efficient layers keep {0,1,7,8,9}
    sav2 = orc.kv_mem_saving_eq4(VAR_T, B, H, D, L, list(range(10)), 7, [0, 1, 7, 8, 9], 23, bytes_per_pair=2 * e)
    assert sav2 * 1024 ** 2 == pytest.approx(23 * (vanilla - held), rel=1e-12)
    # the printed constant is 16: Eq. 4 at B=50, nothing kept anywhere, is the vanilla footprint
    full = orc.kv_mem_saving_eq4(VAR_T, 50, 30, 64, 30, [], 0, [], 0)
    assert full == pytest.approx(16 * 50 * 30 * 64 * 680 * 30 / 1024 ** 2)


# ------------------------------------------------------------------ attention
def _rand_scales(sides, B, H, D, seed):
    g = np.random.default_rng(seed)
    mk = lambda: [g.standard_normal((B, H, s * s, D)) for s in sides]
    return mk(), mk(), mk()


def _sdpa64(q, k, v, scale=None):
    tq, tk, tv = (torch.from_numpy(np.ascontiguousarray(x)).double() for x in (q, k, v))
    return F.scaled_dot_product_attention(tq, tk, tv, scale=scale).numpy()


def test_full_window_equals_block_causal_library_attention():
    sides = (1, 2, 3, 4, 5, 6)
    t = [s * s for s in sides]
    q, k, v = _rand_scales(sides, 2, 3, 16, 1)
    sc = orc.scale_of_token(t)
    causal = sc[None, :] <= sc[:, None]
    for pol in [(0, 0, True), (0, len(sides) - 1, False), (2, 9, False), (len(sides), 0, False)]:
        assert np.array_equal(orc.allow_mask(t, pol), causal)
        for s in range(len(sides)):
            want = _sdpa64(q[s], np.concatenate(k[: s + 1], 2), np.concatenate(v[: s + 1], 2))
            got = orc.attend_step(q, k, v, t, pol, s)
            np.testing.assert_allclose(got, want, rtol=0, atol=1e-12)


@pytest.mark.parametrize("pol", [(2, 2, False), (1, 1, False), (0, 0, False), (3, 1, False), (2, 0, False), (0, 3, False)])
def test_policy_attention_equals_library_attention_on_gathered_scales(pol):
    sides = (1, 2, 3, 4, 5, 6, 8)
    t = [s * s for s in sides]
    q, k, v = _rand_scales(sides, 1, 2, 8, 7)
    c, w, _ = pol
    for s in range(len(sides)):
        keep = sorted({x for x in set(range(c)) | set(range(s - w, s + 1)) if 0 <= x <= s})
        want = _sdpa64(q[s], np.concatenate([k[i] for i in keep], 2), np.concatenate([v[i] for i in keep], 2))
        got = orc.attend_step(q, k, v, t, pol, s)
        np.testing.assert_allclose(got, want, rtol=0, atol=1e-12)


def test_all_steps_equals_step_by_step():
    sides = (1, 2, 3, 4, 5)
    t = [s * s for s in sides]
    q, k, v = _rand_scales(sides, 2, 2, 8, 31)
    for pol in [(2, 1, False), (0, 0, True), (1, 0, False)]:
        every = orc.attend_all_steps(q, k, v, t, pol)
        for s in range(len(sides)):
            np.testing.assert_allclose(every[s], orc.attend_step(q, k, v, t, pol, s), rtol=0, atol=1e-13)


def test_softmax_scale_override_and_default():
    sides = (1, 2, 3)
    t = [1, 4, 9]
    q, k, v = _rand_scales(sides, 1, 1, 4, 3)
    want = _sdpa64(q[2], np.concatenate(k, 2), np.concatenate(v, 2), scale=0.37)
    np.testing.assert_allclose(orc.attend_step(q, k, v, t, (0, 0, True), 2, 0.37), want, atol=1e-12)
    want = _sdpa64(q[2], np.concatenate(k, 2), np.concatenate(v, 2), scale=0.5)  # 1/sqrt(4)
    np.testing.assert_allclose(orc.attend_step(q, k, v, t, (0, 0, True), 2), want, atol=1e-12)


def test_rows_of_p_sum_to_one_and_masked_entries_are_zero():
    t = VAR_T[:7]
    q, k, v = _rand_scales((1, 2, 3, 4, 5, 6, 8), 1, 2, 8, 11)
    allow = orc.allow_mask(t, (2, 1, False))
    o, p = orc.masked_attention(np.concatenate(q, 2), np.concatenate(k, 2), np.concatenate(v, 2), allow, return_probs=True)
    np.testing.assert_allclose(p.sum(-1), 1.0, rtol=0, atol=1e-12)
    assert np.all(p[..., ~allow] == 0.0)
    assert np.all(p[..., allow] > 0.0)


def test_scale0_output_is_v_exactly_and_constant_v():
    q, k, v = _rand_scales((1, 2, 3, 4), 2, 2, 8, 5)
    t = [1, 4, 9, 16]
    for pol in [(2, 2, False), (0, 0, False), (0, 0, True)]:
        assert np.array_equal(orc.attend_step(q, k, v, t, pol, 0), v[0])
    vc = [np.full_like(x, 0.75) for x in v]
    for s in range(4):
        np.testing.assert_allclose(orc.attend_step(q, k, vc, t, (1, 1, False), s), 0.75, atol=1e-14)
    # convexity: every output component lies between the min and max of the visible values
    pol = (1, 1, False)
    for s in range(4):
        keep = orc.kept_scales(pol, s)
        vv = np.concatenate([v[i] for i in keep], 2)
        o = orc.attend_step(q, k, v, t, pol, s)
        assert np.all(o <= vv.max(2, keepdims=True) + 1e-12) and np.all(o >= vv.min(2, keepdims=True) - 1e-12)


def test_poisoned_evicted_scales_change_nothing():
    sides = (1, 2, 3, 4, 5, 6)
    t = [s * s for s in sides]
    q, k, v = _rand_scales(sides, 1, 2, 8, 13)
    pol = (1, 1, False)
    s = 5
    base = orc.attend_step(q, k, v, t, pol, s)
    kp = [x.copy() for x in k]
    vp = [x.copy() for x in v]
    for i in range(s + 1):
        if i not in orc.kept_scales(pol, s):
            kp[i][:] = 1e30
            vp[i][:] = -1e30
    assert np.array_equal(orc.attend_step(q, kp, vp, t, pol, s), base)
    # and a visible scale does matter (the mask is not vacuous)
    kp[4][:] += 1.0
    assert not np.allclose(orc.attend_step(q, kp, vp, t, pol, s), base)


def test_token_permutation_inside_a_kept_scale():
    sides = (1, 2, 3, 4)
    t = [1, 4, 9, 16]
    q, k, v = _rand_scales(sides, 1, 1, 8, 17)
    perm = np.random.default_rng(0).permutation(9)
    k2 = list(k)
    v2 = list(v)
    k2[2] = k[2][:, :, perm]
    v2[2] = v[2][:, :, perm]
    np.testing.assert_allclose(orc.attend_step(q, k2, v2, t, (0, 1, False), 3),
                               orc.attend_step(q, k, v, t, (0, 1, False), 3), atol=1e-13)


def test_brute_force_triple_loops_tiny():
    sides = (1, 2, 3)
    t = [1, 4, 9]
    D = 4
    q, k, v = _rand_scales(sides, 1, 1, D, 23)
    Q = np.concatenate(q, 2)[0, 0]
    K = np.concatenate(k, 2)[0, 0]
    V = np.concatenate(v, 2)[0, 0]
    scale_id = [0] + [1] * 4 + [2] * 9
    for c, w in itertools.product(range(3), range(3)):
        for s in range(3):
            got = orc.attend_step(q, k, v, t, (c, w, False), s)[0, 0]
            rows = [g for g in range(14) if scale_id[g] == s]
            for ri, g in enumerate(rows):
                ws, js = [], []
                for j in range(14):
                    sj = scale_id[j]
                    if sj > s:
                        continue
                    if not (sj < c or s - sj <= w):
                        continue
                    dot = 0.0
                    for d in range(D):
                        dot += Q[g][d] * K[j][d]
                    ws.append(math.exp(dot / math.sqrt(D)))
                    js.append(j)
                z = sum(ws)
                for d in range(D):
                    acc = 0.0
                    for wgt, j in zip(ws, js):
                        acc += wgt / z * V[j][d]
                    assert abs(acc - got[ri][d]) < 1e-12


def test_cache_contents_bit_patterns():
    g = np.random.default_rng(3)
    xs = [g.integers(-2 ** 15, 2 ** 15, size=(2, 2, s * s, 4), dtype=np.int16) for s in (1, 2, 3, 4, 5)]
    out = orc.cache_contents(xs, (1, 1, False), 4)
    assert out.dtype == np.int16 and out.shape == (2, 2, 1 + 16 + 25, 4)
    assert np.array_equal(out[:, :, 0:1], xs[0]) and np.array_equal(out[:, :, 1:17], xs[3]) and np.array_equal(out[:, :, 17:], xs[4])


# ------------------------------------------------------------------ bilinear resize / similarity
def test_bilinear_identity_constant_replication():
    g = np.random.default_rng(5)
    x = g.standard_normal((2, 3, 16, 5))
    np.testing.assert_allclose(orc.bilinear_upsample(x, 4, 4, 4, 4), x, atol=1e-15)
    c = np.full((1, 1, 9, 2), 2.5)
    np.testing.assert_allclose(orc.bilinear_upsample(c, 3, 3, 5, 5), 2.5, atol=1e-15)
    one = g.standard_normal((1, 1, 1, 3))
    np.testing.assert_allclose(orc.bilinear_upsample(one, 1, 1, 2, 2), np.repeat(one, 4, axis=2), atol=1e-15)


def test_bilinear_reproduces_affine_ramp_in_the_interior():
    hi, wi, ho, wo = 6, 5, 8, 10
    r, c = np.meshgrid(np.arange(hi), np.arange(wi), indexing="ij")
    ramp = (2.0 * r - 3.0 * c + 1.0).reshape(1, 1, hi * wi, 1)
    out = orc.bilinear_upsample(ramp, hi, wi, ho, wo).reshape(ho, wo)
    for i in range(ho):
        for j in range(wo):
            sr = (i + 0.5) * hi / ho - 0.5
            scn = (j + 0.5) * wi / wo - 0.5
            if 0 <= sr <= hi - 1 and 0 <= scn <= wi - 1:
                assert abs(out[i, j] - (2.0 * sr - 3.0 * scn + 1.0)) < 1e-12


@pytest.mark.parametrize("sides", [(1, 2), (2, 3), (3, 4), (5, 6), (6, 8), (10, 13), (13, 16), (4, 6), (48, 64)])
def test_bilinear_matches_library_resize(sides):
    a, b = sides
    g = np.random.default_rng(a * 100 + b)
    x = g.standard_normal((1, 2, a * a, 3))
    t = torch.from_numpy(x).reshape(2, a, a, 3).permute(0, 3, 1, 2)
    want = F.interpolate(t, size=(b, b), mode="bilinear", align_corners=False).permute(0, 2, 3, 1).reshape(1, 2, b * b, 3).numpy()
    np.testing.assert_allclose(orc.bilinear_upsample(x, a, a, b, b), want, atol=1e-12)


def test_bilinear_non_square():
    g = np.random.default_rng(9)
    x = g.standard_normal((1, 1, 2 * 5, 2))
    t = torch.from_numpy(x).reshape(1, 2, 5, 2).permute(0, 3, 1, 2)
    want = F.interpolate(t, size=(3, 7), mode="bilinear", align_corners=False).permute(0, 2, 3, 1).reshape(1, 1, 21, 2).numpy()
    np.testing.assert_allclose(orc.bilinear_upsample(x, 2, 5, 3, 7), want, atol=1e-12)


def test_similarity_special_cases():
    g = np.random.default_rng(21)
    prev = g.standard_normal((3, 4, 25, 8))
    up = orc.bilinear_upsample(prev, 5, 5, 6, 6)
    cos, sums = orc.interscale_similarity(up, prev, (6, 6), (5, 5))
    np.testing.assert_allclose(cos, 1.0, atol=1e-12)
    np.testing.assert_allclose(orc.neg_l2_from_sums(sums), 0.0, atol=1e-5)
    cos, sums = orc.interscale_similarity(-up, prev, (6, 6), (5, 5))
    np.testing.assert_allclose(cos, -1.0, atol=1e-12)
    np.testing.assert_allclose(orc.neg_l2_from_sums(sums), -2.0 * np.sqrt((up * up).sum(axis=(0, 2, 3))), rtol=1e-12)
    # independent draws: |mean cos| is of order 1/sqrt(B*T*D)
    cur = g.standard_normal((3, 4, 36, 8))
    cos, _ = orc.interscale_similarity(cur, prev, (6, 6), (5, 5))
    assert np.all(np.abs(cos) < 4.0 / math.sqrt(3 * 36))


def test_similarity_matches_library_route():
    g = np.random.default_rng(22)
    B, H, D = 2, 3, 8
    prev = g.standard_normal((B, H, 16, D))
    cur = 0.7 * orc.bilinear_upsample(prev, 4, 4, 5, 5) + 0.5 * g.standard_normal((B, H, 25, D))
    cos, sums = orc.interscale_similarity(cur, prev, (5, 5), (4, 4))
    tp = torch.from_numpy(prev).reshape(B * H, 4, 4, D).permute(0, 3, 1, 2)
    up = F.interpolate(tp, size=(5, 5), mode="bilinear", align_corners=False).permute(0, 2, 3, 1).reshape(B, H, 25, D)
    tc = torch.from_numpy(cur)
    want = F.cosine_similarity(tc, up, dim=-1).mean(dim=(0, 2)).numpy()
    np.testing.assert_allclose(cos, want, atol=1e-12)
    np.testing.assert_allclose(sums[:, 0], (tc * up).sum(dim=(0, 2, 3)).numpy(), rtol=1e-12)
    np.testing.assert_allclose(sums[:, 1], (tc * tc).sum(dim=(0, 2, 3)).numpy(), rtol=1e-12)
    np.testing.assert_allclose(sums[:, 2], (up * up).sum(dim=(0, 2, 3)).numpy(), rtol=1e-12)
    l2 = -torch.linalg.vector_norm((tc - up).permute(1, 0, 2, 3).reshape(H, -1), dim=1).numpy()
    np.testing.assert_allclose(orc.neg_l2_from_sums(sums), l2, rtol=1e-10)


def test_similarity_monotone_in_rho():
    from amskv_inputs import correlated_qkv
    vals = []
    for rho in (0.2, 0.5, 0.8, 0.95):
        _, k, _ = correlated_qkv((4, 5, 6), 4, 2, 16, "f32", 99, rho)
        cos, _ = orc.interscale_similarity(k[2].double().numpy(), k[1].double().numpy(), (6, 6), (5, 5))
        vals.append(cos.mean())
    assert vals == sorted(vals) and vals[0] < 0.4 and vals[-1] > 0.7


# ------------------------------------------------------------------ Algorithms 1 and 2 (literal, token lists)
def test_clru_identity_and_slicing():
    assert orc.clru(list(range(10)), 10, 2) == list(range(10))
    assert orc.clru(list(range(10)), 12, 2) == list(range(10))
    assert orc.clru(list(range(10)), 6, 2) == [0, 1, 6, 7, 8, 9]
    assert orc.clru(list(range(10)), 2, 2) == [0, 1]


def test_alg1_trace_hand_derived():
    # budgets of the experimental set-up read as token counts: condensed = 5 tokens,
    # C_min = 5 + 169, C_max = 5 + 100 + 169; never below theta -> budget stays C_min
    tr = orc.alg1_cache_trace(VAR_T, 174, 274, 5, [False] * 10)
    ids7, b7 = tr[7]
    st = orc.scale_starts(VAR_T)
    # step 7: 5 condensed + last 169 tokens = all of scales 7 (100) and 6 (64) + 5 tokens of scale 5
    assert b7 == 174 and len(ids7) == 174
    assert ids7[:5] == [0, 1, 2, 3, 4]
    assert ids7[5:] == list(range(st[8] - 169, st[8]))
    assert sum(1 for g in ids7 if st[5] <= g < st[6]) == 5
    # step 8 (169 tokens) fits exactly with the condensed tokens; step 9 (256 > C_max) is skipped
    assert tr[8][0] == [0, 1, 2, 3, 4] + list(range(st[8], st[9]))
    assert tr[9] == tr[8]
    # always below theta: the first overflow (step 7, 255 > 174) expands the budget once
    tr = orc.alg1_cache_trace(VAR_T, 174, 274, 5, [True] * 10)
    assert [b for _, b in tr] == [174] * 7 + [274] * 3
    assert tr[7][0] == list(range(0, st[8]))              # 255 tokens fit in 274
    assert tr[8][0] == [0, 1, 2, 3, 4] + list(range(st[9] - 269, st[9]))
    # the last scale (256 <= C_max) is admitted: 5 condensed + last 269 tokens =
    # 13 tokens of scale 8 beside all of scale 9
    last = tr[9][0]
    assert last == [0, 1, 2, 3, 4] + list(range(680 - 269, 680))
    assert sum(1 for g in last if st[8] <= g < st[9]) == 13 and sum(1 for g in last if g >= st[9]) == 256
    tr2 = orc.alg1_cache_trace(VAR_T, 274, 274, 5, [False] * 10)
    assert tr2[8][0] == tr[8][0] and tr2[9][0] == last
    # a scale larger than C_max is skipped outright and leaves the cache untouched
    small = orc.alg1_cache_trace(VAR_T, 174, 255, 5, [True] * 10)
    assert small[9] == small[8]
    big = orc.alg1_cache_trace(VAR_T, 174, 300, 5, [True] * 10)
    last = big[9][0]
    assert len(last) == 300 and sum(1 for g in last if g >= st[9]) == 256 and sum(1 for g in last if st[8] <= g < st[9]) == 39


def test_alg1_mask_closed_forms():
    tokens = [s * s for s in (1, 2, 3, 4, 5, 6)]
    st = orc.scale_starts(tokens)
    n = sum(tokens)
    # a budget that is never reached: every earlier token stays -> the block-causal mask
    tr = orc.alg1_cache_trace(tokens, n, n, 3, [False] * len(tokens))
    assert np.array_equal(orc.alg1_allow_mask(tokens, tr), orc.allow_mask(tokens, (0, 0, True)))
    # no condensed tokens, one budget k >= every scale: a sliding window of the k newest tokens
    for k in (36, 40, 57):
        tr = orc.alg1_cache_trace(tokens, k, k, 0, [False] * len(tokens))
        m = orc.alg1_allow_mask(tokens, tr)
        for i, t in enumerate(tokens):
            want = np.zeros(n, dtype=bool)
            want[max(0, st[i] - k): st[i] + t] = True
            assert np.array_equal(m[st[i]], want) and np.array_equal(m[st[i] + t - 1], want)
    # condensed tokens stay visible to every later scale, own scale always whole
    tr = orc.alg1_cache_trace(tokens, 30, 30, 5, [False] * len(tokens))
    m = orc.alg1_allow_mask(tokens, tr)
    assert m[st[5]:, :5].all() and not m[st[5], 5: st[5] - 25].any() and m[st[5], st[5] - 25:].all()
    # whole-scale budgets reproduce the scale-window policy at the steps where they line up:
    # C = condensed(2 scales) + penultimate scale -> step s sees {0, 1, s-1, s} once s-1 fills the tail exactly
    for s in (4, 5):
        c = 5 + tokens[s - 1]
        tr = orc.alg1_cache_trace(tokens, c, c, 5, [False] * len(tokens))
        assert np.array_equal(orc.alg1_allow_mask(tokens, tr)[st[s]], orc.allow_mask(tokens, (2, 1, False))[st[s]])


def test_alg1_theta_test_is_asked_once_and_only_on_overflow():
    calls = []

    def ask(i, cached):
        calls.append((i, len(cached)))
        return True

    tr = orc.alg1_cache_trace(VAR_T, 174, 274, 5, ask)
    # the first overflow of C_min is at the 100-token scale (155 cached + 100 > 174)
    assert calls == [(7, 155)]
    assert tr == orc.alg1_cache_trace(VAR_T, 174, 274, 5, [True] * 10)
    calls.clear()
    orc.alg1_cache_trace(VAR_T, 174, 274, 5, lambda i, c: calls.append(i) or False)
    # a layer that stays at C_min is asked again at every later overflow (the 256-token scale
    # is within C_max = 274, so it reaches the test too before being skipped for exceeding C_min)
    assert calls == [7, 8, 9]


# ------------------------------------------------------------------ token windows: the SWA / STA kept sets
def test_token_window_hand_trace():
    # 1 + 4 + 9 tokens, budget 6 with one sink token.  After step 0: {0}.  After step 1: five tokens, all fit.
    # After step 2 fourteen tokens were seen: the sink 0 and the five newest, 9..13 -- the 3x3 scale is cut.
    assert orc.token_window_cache([1, 4, 9], 6, 1) == [[0], [0, 1, 2, 3, 4], [0, 9, 10, 11, 12, 13]]
    # no sink: the six newest
    assert orc.token_window_cache([1, 4, 9], 6, 0)[2] == [8, 9, 10, 11, 12, 13]
    m = orc.token_window_allow_mask([1, 4, 9, 4], 6, 1)
    # queries of the 3x3 scale (ids 5..13) see their own scale and the five cached tokens
    assert m[5].tolist() == [True] * 14 + [False] * 4
    # queries of the last scale (ids 14..17) see the sink, ids 9..13 and themselves
    assert np.flatnonzero(m[14]).tolist() == [0, 9, 10, 11, 12, 13, 14, 15, 16, 17]
    assert np.array_equal(m[14], m[17])


def test_token_window_against_a_token_by_token_queue():
    # the same policy simulated one token at a time: a queue that, once full, drops its oldest
    # entry behind the sink for every token that arrives
    rng = np.random.default_rng(11)
    for _ in range(40):
        tokens = [int(x) for x in rng.integers(1, 12, size=int(rng.integers(1, 7)))]
        window = int(rng.integers(1, 30))
        n_sink = int(rng.integers(0, window + 1))
        queue, after = [], []
        g = 0
        for t in tokens:
            for _ in range(t):
                queue.append(g)
                g += 1
                if len(queue) > window:
                    del queue[n_sink]
            after.append(list(queue))
        if n_sink == window:      # nothing but sinks: the queue keeps the first `window` tokens
            after = [list(range(min(window, sum(tokens[: i + 1])))) for i in range(len(tokens))]
        assert orc.token_window_cache(tokens, window, n_sink) == after
        # mask rows: own scale plus the cache of the step before
        m = orc.token_window_allow_mask(tokens, window, n_sink)
        st = orc.scale_starts(tokens)
        for i, t in enumerate(tokens):
            want = np.zeros(sum(tokens), dtype=bool)
            want[st[i]: st[i] + t] = True
            if i:
                want[after[i - 1]] = True
            assert np.array_equal(m[st[i]], want) and np.array_equal(m[st[i] + t - 1], want)


def test_token_window_special_cases():
    tokens = [s * s for s in (1, 2, 3, 4, 5, 6)]
    n = sum(tokens)
    st = orc.scale_starts(tokens)
    # a window that holds everything is the block-causal mask; every row count is T_s + min(seen before, window)
    assert np.array_equal(orc.token_window_allow_mask(tokens, n, 0), orc.allow_mask(tokens, (0, 0, True)))
    assert np.array_equal(orc.token_window_allow_mask(tokens, n, 7), orc.allow_mask(tokens, (0, 0, True)))
    for window, n_sink in ((10, 0), (10, 3), (40, 5), (1, 1), (0, 0)):
        m = orc.token_window_allow_mask(tokens, window, n_sink)
        for i, t in enumerate(tokens):
            assert m[st[i]].sum() == t + min(st[i], window)
    # while no scale exceeds the budget Algorithm 1 never skips, and with C_min = C_max it never tests:
    # its cache is then this window with the condensed tokens as sinks
    for window, n_sink in ((36, 0), (40, 5), (57, 14)):
        tr = orc.alg1_cache_trace(tokens, window, window, n_sink, [False] * len(tokens))
        assert [ids for ids, _ in tr] == orc.token_window_cache(tokens, window, n_sink)
        assert np.array_equal(orc.alg1_allow_mask(tokens, tr), orc.token_window_allow_mask(tokens, window, n_sink))
    # a scale larger than the window: Algorithm 1 skips it, the window keeps its newest tokens
    tr = orc.alg1_cache_trace(tokens, 30, 30, 5, [False] * len(tokens))
    tw = orc.token_window_cache(tokens, 30, 5)
    assert tr[5][0] == tr[4][0] and tw[5] == [0, 1, 2, 3, 4] + list(range(n - 25, n))


# ------------------------------------------------------------------ attention density (Section 4.1)
def test_attention_density_invariants_and_closed_forms():
    rng = np.random.default_rng(5)
    tokens = [1, 4, 9, 16]
    st = orc.scale_starts(tokens)
    B, H, D = 2, 3, 8
    k_all = rng.standard_normal((B, H, sum(tokens), D))
    s = 3
    q = rng.standard_normal((B, H, tokens[s], D))
    pol = (1, 1, False)                       # step 3 sees scales {0, 2, 3}
    rows = orc.allow_mask(tokens, pol)[st[s]: st[s] + tokens[s]]
    pieces = [(st[k], tokens[k]) for k in orc.kept_scales(pol, s)]
    dens, mass = orc.attention_density(q, k_all, rows, pieces)
    # every query spends exactly one unit of attention on what it can see
    assert np.allclose(mass.sum(axis=-1), tokens[s], rtol=0, atol=1e-12)
    assert np.allclose(dens * [n for _, n in pieces], mass)
    # brute force, element by element
    for h in range(H):
        want = np.zeros(len(pieces))
        for b in range(B):
            for qi in range(tokens[s]):
                vis = [j for j in range(sum(tokens)) if rows[qi, j]]
                e = [math.exp(float(q[b, h, qi] @ k_all[b, h, j]) / math.sqrt(D)) for j in vis]
                z = sum(e)
                for pi, (a, n) in enumerate(pieces):
                    want[pi] += sum(x for x, j in zip(e, vis) if a <= j < a + n) / z / B
        assert np.allclose(mass[h], want, rtol=1e-12, atol=1e-12)
    # uniform attention (all-zero queries): every visible token receives T_s / T_kv
    dens0, _ = orc.attention_density(np.zeros_like(q), k_all, rows, pieces)
    assert np.allclose(dens0, tokens[s] / sum(n for _, n in pieces))
    # one key that dominates: its piece takes (almost) all of the mass
    k_big = k_all.copy()
    k_big[..., st[2] + 4, :] = 50.0 * np.sign(q.mean(axis=-2))     # aligned with the mean query of each (b, h)
    q_pos = np.abs(q) * np.sign(q.mean(axis=-2, keepdims=True))
    _, m_big = orc.attention_density(q_pos, k_big, rows, pieces)
    assert (m_big[:, 1] > tokens[s] - 1e-6).all()
    # partial pieces of one scale add up to the scale
    halves = [(st[2], 4), (st[2] + 4, 5)]
    _, m_halves = orc.attention_density(q, k_all, rows, halves)
    assert np.allclose(m_halves.sum(axis=-1), mass[:, 1])
