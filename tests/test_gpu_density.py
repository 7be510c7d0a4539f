"""GPU parity of the attention density (Section 4.1) against the oracle: fp32 arithmetic (on exact bf16
products, or fp32 dot products for fp32 caches) versus fp64, so mass and density agree to rtol 2e-4 / atol 1e-5;
the group list is bit-exact."""
import numpy as np
import pytest
import torch

import amskv_inputs as inp
import paper_2511_16047_amd as amskv
from oracle import amskv_oracle as orc

pytestmark = pytest.mark.gpu

VAR = (1, 2, 3, 4, 5, 6, 8, 10, 13, 16)
BF16 = amskv.AMSKV_DTYPE_BF16


def _f64(t):
    return t.detach().to("cpu", torch.float64).numpy()


def _runs_by_scale(ids, tokens):
    """Token ids -> maximal runs of consecutive ids that stay inside one scale, as (first id, length)."""
    st = orc.scale_starts(tokens)
    scale_of = orc.scale_of_token(tokens)
    out = []
    for g in ids:
        if out and out[-1][0] + out[-1][1] == g and scale_of[g] == scale_of[out[-1][0]]:
            out[-1][1] += 1
        else:
            out.append([g, 1])
    return [(a, n) for a, n in out]


def _check(h, layer, s, tokens, q_dev, k_all, H, pieces, rows, softmax_scale=None):
    """Compare the library's density of step s with the oracle's.  `pieces` (groups of keys) and `rows` (what the
    queries of s may see) come from the oracle's own kept set / token list; the library's group list must be
    the same list."""
    st = orc.scale_starts(tokens)
    segs = amskv.amskv_cache_segments(h, layer)
    assert [(st[sc] + first, ln) for sc, first, _, ln in segs] == list(pieces)
    want_d, want_m = orc.attention_density(_f64(q_dev), k_all, rows, pieces, softmax_scale)
    got_d, got_m = amskv.amskv_attention_density(h, layer, s, q_dev, H)
    got_d, got_m = np.asarray(got_d), np.asarray(got_m)
    assert got_m.shape == want_m.shape
    assert np.allclose(got_m, want_m, rtol=2e-4, atol=1e-5), np.abs(got_m - want_m).max()
    assert np.allclose(got_d, want_d, rtol=2e-4, atol=1e-5)
    assert np.allclose(got_m.sum(axis=-1), tokens[s], rtol=1e-4)
    return got_d


def _window_view(tokens, pol, s):
    st = orc.scale_starts(tokens)
    pieces = [(st[k], tokens[k]) for k in orc.kept_scales(pol, s)]
    rows = orc.allow_mask(tokens, pol)[st[s]: st[s] + tokens[s]]
    return pieces, rows


@pytest.mark.parametrize("flags", [dict(), dict(layout=amskv.AMSKV_LAYOUT_PLANNED, borrow_unretained=True, fuse_append=True)],
                         ids=["compact", "planned_borrow_fuse"])
@pytest.mark.parametrize("D", [64, 128])
def test_density_scale_window(D, flags):
    B, H = 2, 3
    tokens = [x * x for x in VAR]
    pols = [(2, 2, False), (0, 0, True), (1, 0, False)]
    q, k, v = inp.correlated_qkv(VAR, B, H, D, "bf16", inp.layer_seed(8, D), 0.7)
    k_all = np.concatenate([_f64(x) for x in k], axis=-2)
    qd, kd, vd = ([x.cuda() for x in t] for t in (q, k, v))
    kw = dict(flags)
    layout = kw.pop("layout", amskv.AMSKV_LAYOUT_COMPACT)
    need = amskv.amskv_cache_required_bytes(len(pols), H, D, VAR, VAR, B, BF16, pols, 0.0, layout, **kw)
    arena = torch.empty(need, dtype=torch.uint8, device="cuda")
    arena.fill_(0xFF)
    h = amskv.amskv_cache_create(len(pols), H, D, VAR, VAR, B, BF16, pols, 0.0, layout, arena=arena, **kw)
    try:
        for s in range(len(VAR)):
            for l, pol in enumerate(pols):
                amskv.amskv_append_scale(h, l, s, kd[s], vd[s])
                assert [x[0] for x in amskv.amskv_cache_segments(h, l)] == orc.kept_scales(pol, s)
                pieces, rows = _window_view(tokens, pol, s)
                _check(h, l, s, tokens, qd[s], k_all, H, pieces, rows)   # before the attention of the step ...
                o = torch.empty_like(qd[s])
                amskv.amskv_attend(h, l, s, qd[s], o)
                if s in (4, 9):
                    _check(h, l, s, tokens, qd[s], k_all, H, pieces, rows)   # ... and after it (fused append has filled the slot)
    finally:
        amskv.amskv_cache_destroy(h)


def test_density_token_budget_partial_groups():
    sides = (6, 3, 4, 5, 2, 7)
    tokens = [x * x for x in sides]
    B, H, D = 2, 2, 64
    q, k, v = inp.correlated_qkv(sides, B, H, D, "bf16", inp.layer_seed(8, 1), 0.6)
    k_all = np.concatenate([_f64(x) for x in k], axis=-2)
    qd, kd, vd = ([x.cuda() for x in t] for t in (q, k, v))
    budgets = [(40, 40, 10, -2.0), (30, 60, 20, 2.0)]   # the first keeps head and tail of the 6x6 scale apart
    need = amskv.amskv_cache_required_bytes(2, H, D, sides, sides, B, BF16, None, 0.3, budgets=budgets)
    arena = torch.empty(need, dtype=torch.uint8, device="cuda")
    h = amskv.amskv_cache_create(2, H, D, sides, sides, B, BF16, None, 0.3, arena=arena, budgets=budgets)
    # the oracle's own token lists: Algorithm 1 with the outcome of the Eq. 3 test fixed by the thresholds
    # (-2: never below, the budget stays; 2: always below, the budget grows at the first overflow)
    traces = [orc.alg1_cache_trace(tokens, b[0], b[1], b[2], [b[3] > 1.0] * len(sides)) for b in budgets]
    masks = [orc.alg1_allow_mask(tokens, t) for t in traces]
    st = orc.scale_starts(tokens)
    try:
        split = False
        for s in range(len(sides)):
            for l in range(2):
                amskv.amskv_append_scale(h, l, s, kd[s], vd[s])
                segs = amskv.amskv_cache_segments(h, l)
                split |= len({x[0] for x in segs}) < len(segs)     # one scale present as head and tail
                # what step s attends to: the list iteration s-1 left, then its own scale
                ids = (traces[l][s - 1][0] if s else []) + list(range(st[s], st[s] + tokens[s]))
                rows = masks[l][st[s]: st[s] + tokens[s]]
                assert sorted(np.flatnonzero(rows[0]).tolist()) == sorted(ids)
                _check(h, l, s, tokens, qd[s], k_all, H, _runs_by_scale(ids, tokens), rows, 0.3)
                o = torch.empty_like(qd[s])
                amskv.amskv_attend(h, l, s, qd[s], o)
                with pytest.raises(amskv.AmskvError) as e:          # the step's trim has run: no longer the step's view
                    amskv.amskv_attention_density(h, l, s, qd[s], H)
                assert e.value.status == amskv.AMSKV_ERR_ORDER
        assert split
    finally:
        amskv.amskv_cache_destroy(h)


def test_density_uniform_queries_and_errors():
    # all-zero queries attend uniformly: every visible token receives T_s / T_kv, whatever the keys
    B, H, D = 1, 4, 64
    tokens = [x * x for x in VAR]
    q, k, v = inp.iid_qkv(VAR, B, H, D, "bf16", inp.layer_seed(8, 2))
    qd, kd, vd = ([x.cuda() for x in t] for t in (q, k, v))
    pol = (2, 1, False)
    need = amskv.amskv_cache_required_bytes(1, H, D, VAR, VAR, B, BF16, [pol])
    arena = torch.empty(need, dtype=torch.uint8, device="cuda")
    h = amskv.amskv_cache_create(1, H, D, VAR, VAR, B, BF16, [pol], arena=arena)
    try:
        for s in range(len(VAR)):
            amskv.amskv_append_scale(h, 0, s, kd[s], vd[s])
        s = len(VAR) - 1
        dens, mass = amskv.amskv_attention_density(h, 0, s, torch.zeros_like(qd[s]), H)
        t_kv = orc.kept_token_count(tokens, pol, s)
        assert np.allclose(np.asarray(dens), tokens[s] / t_kv, rtol=1e-5)
        with pytest.raises(amskv.AmskvError) as e:
            amskv.amskv_attention_density(h, 0, s - 1, qd[s - 1], H)
        assert e.value.status == amskv.AMSKV_ERR_ORDER
    finally:
        amskv.amskv_cache_destroy(h)
    # an fp32 cache with one cached token: all of the single query's mass lands on it
    need = amskv.amskv_cache_required_bytes(1, H, D, (1, 2), (1, 2), B, amskv.AMSKV_DTYPE_F32, [pol])
    arena = torch.empty(need, dtype=torch.uint8, device="cuda")
    h = amskv.amskv_cache_create(1, H, D, (1, 2), (1, 2), B, amskv.AMSKV_DTYPE_F32, [pol], arena=arena)
    try:
        x = torch.zeros(B, H, 1, D, device="cuda")
        amskv.amskv_append_scale(h, 0, 0, x, x)
        dens, mass = amskv.amskv_attention_density(h, 0, 0, x, H)
        assert np.array_equal(np.asarray(mass), np.ones((H, 1))) and np.array_equal(np.asarray(dens), np.ones((H, 1)))
    finally:
        amskv.amskv_cache_destroy(h)


def test_density_full_batch_launch_configuration():
    """Batch 256 x 30 heads at the last scale of the 256x256 schedule (the launch the benchmark times).  The batch
    repeats two distinct samples, so the batch mean equals the oracle's over those two; the masses of a head
    add up to T_s whatever the size."""
    B, B0, H, D = 256, 2, 30, 64
    tokens = [x * x for x in VAR]
    q0, k0, v0 = inp.correlated_qkv(VAR, B0, H, D, "bf16", inp.layer_seed(8, 3), 0.7)
    rep = lambda t: t.repeat(B // B0, 1, 1, 1).cuda()
    pol = (2, 2, False)
    need = amskv.amskv_cache_required_bytes(1, H, D, VAR, VAR, B, BF16, [pol], 0.0, amskv.AMSKV_LAYOUT_PLANNED, True, True)
    arena = torch.empty(need, dtype=torch.uint8, device="cuda")
    h = amskv.amskv_cache_create(1, H, D, VAR, VAR, B, BF16, [pol], 0.0, amskv.AMSKV_LAYOUT_PLANNED, arena=arena,
                                 borrow_unretained=True, fuse_append=True)
    try:
        keep = []
        for s in range(len(VAR)):
            kd, vd = rep(k0[s]), rep(v0[s])
            keep += [kd, vd]
            amskv.amskv_append_scale(h, 0, s, kd, vd)
            if s < len(VAR) - 1:
                qd = rep(q0[s])
                o = torch.empty_like(qd)
                amskv.amskv_attend(h, 0, s, qd, o)
        s = len(VAR) - 1
        qd = rep(q0[s])
        got_d, got_m = amskv.amskv_attention_density(h, 0, s, qd, H)
        st = orc.scale_starts(tokens)
        kept = orc.kept_scales(pol, s)
        pieces = [(st[k], tokens[k]) for k in kept]
        rows = orc.allow_mask(tokens, pol)[st[s]: st[s] + tokens[s]]
        k_all = np.concatenate([_f64(x) for x in k0], axis=-2)
        want_d, want_m = orc.attention_density(_f64(q0[s]), k_all, rows, pieces)
        assert np.allclose(np.asarray(got_m), want_m, rtol=2e-4, atol=1e-5)
        assert np.allclose(np.asarray(got_d), want_d, rtol=2e-4, atol=1e-5)
        assert np.allclose(np.asarray(got_m).sum(axis=-1), tokens[s], rtol=1e-4)
    finally:
        amskv.amskv_cache_destroy(h)


@pytest.mark.parametrize("D", [64, 128])
def test_density_fp32_cache(D):
    """fp32 caches: dot products on the vector ALUs in fp32 against the oracle's fp64, odd group lengths (a lane
    half that sees no key of a group, a one-token first scale), borrowed final scale, ragged query count."""
    F32 = amskv.AMSKV_DTYPE_F32
    sides = (1, 2, 3, 5, 7)
    tokens = [x * x for x in sides]
    B, H = 2, 2
    pols = [(1, 1, False), (0, 0, True)]
    q, k, v = inp.correlated_qkv(sides, B, H, D, "f32", inp.layer_seed(8, 300 + D), 0.6)
    k_all = np.concatenate([_f64(x) for x in k], axis=-2)
    qd, kd, vd = ([x.cuda() for x in t] for t in (q, k, v))
    need = amskv.amskv_cache_required_bytes(len(pols), H, D, sides, sides, B, F32, pols, 0.0, amskv.AMSKV_LAYOUT_COMPACT, True)
    arena = torch.empty(need, dtype=torch.uint8, device="cuda")
    arena.fill_(0xFF)
    h = amskv.amskv_cache_create(len(pols), H, D, sides, sides, B, F32, pols, 0.0, amskv.AMSKV_LAYOUT_COMPACT, arena=arena,
                                 borrow_unretained=True)
    try:
        for s in range(len(sides)):
            for l, pol in enumerate(pols):
                amskv.amskv_append_scale(h, l, s, kd[s], vd[s])
                pieces, rows = _window_view(tokens, pol, s)
                _check(h, l, s, tokens, qd[s], k_all, H, pieces, rows)
    finally:
        amskv.amskv_cache_destroy(h)


def test_density_enqueue_matches_the_waiting_call():
    """The form without a wait leaves the same bits in the caller's device buffer, layer after layer on one stream."""
    B, H, D = 2, 3, 64
    tokens = [x * x for x in VAR]
    pols = [(2, 2, False), (0, 0, True)]
    q, k, v = inp.correlated_qkv(VAR, B, H, D, "bf16", inp.layer_seed(8, 77), 0.7)
    qd, kd, vd = ([x.cuda() for x in t] for t in (q, k, v))
    need = amskv.amskv_cache_required_bytes(len(pols), H, D, VAR, VAR, B, BF16, pols)
    arena = torch.empty(need, dtype=torch.uint8, device="cuda")
    h = amskv.amskv_cache_create(len(pols), H, D, VAR, VAR, B, BF16, pols, arena=arena)
    try:
        for s in range(len(VAR)):
            for l in range(len(pols)):
                amskv.amskv_append_scale(h, l, s, kd[s], vd[s])
        s = len(VAR) - 1
        outs = [torch.full((H * amskv.AMSKV_MAX_SCALES,), float("nan"), dtype=torch.float32, device="cuda") for _ in pols]
        lens = [amskv.amskv_attention_density_enqueue(h, l, s, qd[s], outs[l]) for l in range(len(pols))]
        torch.cuda.synchronize()
        for l, pol in enumerate(pols):
            assert lens[l] == [tokens[kk] for kk in orc.kept_scales(pol, s)]
            _, want_m = amskv.amskv_attention_density(h, l, s, qd[s], H)
            got = outs[l].cpu().numpy().reshape(H, amskv.AMSKV_MAX_SCALES)[:, : len(lens[l])]
            assert np.array_equal(got, np.asarray(want_m, dtype=np.float32))
        with pytest.raises(amskv.AmskvError):
            amskv.amskv_attention_density_enqueue(h, 0, s, qd[s], None)
    finally:
        amskv.amskv_cache_destroy(h)


def _mass_rows(buf, H, n):
    return buf.cpu().numpy().reshape(H, amskv.AMSKV_MAX_SCALES)[:, :n].astype(np.float64)


def _bits(t):
    it = torch.int16 if t.dtype == torch.bfloat16 else torch.int32
    return t.contiguous().view(it).cpu().numpy()


@pytest.mark.parametrize("flags", [dict(), dict(layout=amskv.AMSKV_LAYOUT_PLANNED, borrow_unretained=True, fuse_append=True)],
                         ids=["compact", "planned_borrow_fuse"])
@pytest.mark.parametrize("D,dtype", [(64, "bf16"), (128, "bf16"), (64, "f32")])
def test_attend_density_in_one_call(D, dtype, flags):
    """amskv_attend_density: O bit-identical to amskv_attend on a twin cache, the masses against the oracle, the
    caches bit-identical afterwards.  The schedule covers the by-product form (more than 32 queries; two workgroups
    per unit from 169 queries on at head dim 64, at 169 and 256 at head dim 128) and the two-call form (coarse
    scales; the whole fp32 case); groups of 1 and 4 keys end inside the first 32-key block."""
    B, H = 2, 3
    DT = amskv.AMSKV_DTYPE_BF16 if dtype == "bf16" else amskv.AMSKV_DTYPE_F32
    tokens = [x * x for x in VAR]
    pols = [(2, 2, False), (0, 0, True), (1, 0, False)]
    q, k, v = inp.correlated_qkv(VAR, B, H, D, dtype, inp.layer_seed(8, 500 + D), 0.7)
    k_all = np.concatenate([_f64(x) for x in k], axis=-2)
    qd, kd, vd = ([x.cuda() for x in t] for t in (q, k, v))
    kw = dict(flags)
    layout = kw.pop("layout", amskv.AMSKV_LAYOUT_COMPACT)
    need = amskv.amskv_cache_required_bytes(len(pols), H, D, VAR, VAR, B, DT, pols, 0.0, layout, **kw)
    arenas = [torch.empty(need, dtype=torch.uint8, device="cuda") for _ in range(2)]
    for a in arenas:
        a.fill_(0xFF)
    one, two = (amskv.amskv_cache_create(len(pols), H, D, VAR, VAR, B, DT, pols, 0.0, layout, arena=a, **kw) for a in arenas)
    st = orc.scale_starts(tokens)
    try:
        for s in range(len(VAR)):
            for l, pol in enumerate(pols):
                for h in (one, two):
                    amskv.amskv_append_scale(h, l, s, kd[s], vd[s])
                o1 = torch.full_like(qd[s], float("nan"))
                o2 = torch.full_like(qd[s], float("nan"))
                mass = torch.full((H * amskv.AMSKV_MAX_SCALES,), float("nan"), dtype=torch.float32, device="cuda")
                lens = amskv.amskv_attend_density(one, l, s, qd[s], o1, mass)
                amskv.amskv_attend(two, l, s, qd[s], o2)
                torch.cuda.synchronize()
                kept = orc.kept_scales(pol, s)
                assert lens == [tokens[j] for j in kept]
                assert np.array_equal(_bits(o1), _bits(o2)), "O differs at step %d layer %d" % (s, l)
                pieces, rows = _window_view(tokens, pol, s)
                _, want_m = orc.attention_density(_f64(qd[s]), k_all, rows, pieces)
                got_m = _mass_rows(mass, H, len(lens))
                assert np.allclose(got_m, want_m, rtol=2e-4, atol=1e-5), (s, l, np.abs(got_m - want_m).max())
                assert np.allclose(got_m.sum(axis=-1), tokens[s], rtol=1e-4)
        for l, pol in enumerate(pols):
            tk = sum(tokens[j] for j in orc.kept_scales(pol, len(VAR) - 1))
            exp = [torch.empty(B, H, tk, D, dtype=kd[0].dtype, device="cuda") for _ in range(4)]
            amskv.amskv_cache_export(one, l, exp[0], exp[1])
            amskv.amskv_cache_export(two, l, exp[2], exp[3])
            torch.cuda.synchronize()
            assert torch.equal(exp[0], exp[2]) and torch.equal(exp[1], exp[3])
    finally:
        amskv.amskv_cache_destroy(one)
        amskv.amskv_cache_destroy(two)


def test_attend_density_token_budget_and_token_major():
    """The by-product form over partial groups (head and tail of one scale cached apart, a current scale read in
    place from token-major tensors), against the oracle's own token lists; then the step's iteration runs as after
    amskv_attend (the next append sees the trimmed list)."""
    sides = (6, 3, 4, 5, 2, 7)
    tokens = [x * x for x in sides]
    B, H, D = 2, 2, 64
    q, k, v = inp.correlated_qkv(sides, B, H, D, "bf16", inp.layer_seed(8, 601), 0.6)
    k_all = np.concatenate([_f64(x) for x in k], axis=-2)
    budgets = [(40, 40, 10, -2.0), (30, 60, 20, 2.0)]
    need = amskv.amskv_cache_required_bytes(2, H, D, sides, sides, B, BF16, None, 0.3, budgets=budgets)
    arena = torch.empty(need, dtype=torch.uint8, device="cuda")
    h = amskv.amskv_cache_create(2, H, D, sides, sides, B, BF16, None, 0.3, arena=arena, budgets=budgets)
    stride = 3 * H * D
    amskv.amskv_cache_set_io_layout(h, amskv.AMSKV_IO_TOKEN_MAJOR, stride, stride, H * D)
    traces = [orc.alg1_cache_trace(tokens, b[0], b[1], b[2], [b[3] > 1.0] * len(sides)) for b in budgets]
    masks = [orc.alg1_allow_mask(tokens, t) for t in traces]
    st = orc.scale_starts(tokens)
    cat = lambda xs: np.concatenate([_f64(x) for x in xs], axis=-2)
    want_o = [orc.masked_attention(cat(q), cat(k), cat(v), m, 0.3) for m in masks]
    keep = []   # K/V of a scale stay the caller's until the step's iteration has run
    try:
        for s in range(len(sides)):
            # fused projection output [B][T][3][H][D]
            packed = torch.stack([x.permute(0, 2, 1, 3) for x in (q[s], k[s], v[s])], dim=2).contiguous().cuda()
            keep.append(packed)
            flat = packed.view(-1)
            qp, kp, vp = flat, flat[H * D:], flat[2 * H * D:]
            for l in range(2):
                amskv.amskv_append_scale(h, l, s, kp, vp)
                ids = (traces[l][s - 1][0] if s else []) + list(range(st[s], st[s] + tokens[s]))
                pieces = _runs_by_scale(ids, tokens)
                rows = masks[l][st[s]: st[s] + tokens[s]]
                o = torch.full((B, tokens[s], H * D), float("nan"), dtype=torch.bfloat16, device="cuda")
                mass = torch.full((H * amskv.AMSKV_MAX_SCALES,), float("nan"), dtype=torch.float32, device="cuda")
                lens = amskv.amskv_attend_density(h, l, s, qp, o, mass)
                torch.cuda.synchronize()
                assert lens == [n for _, n in pieces]
                _, want_m = orc.attention_density(_f64(q[s]), k_all, rows, pieces, 0.3)
                got_m = _mass_rows(mass, H, len(lens))
                assert np.allclose(got_m, want_m, rtol=2e-4, atol=1e-5), (s, l, np.abs(got_m - want_m).max())
                got_o = _f64(o.view(B, tokens[s], H, D).permute(0, 2, 1, 3))
                assert np.abs(got_o - want_o[l][..., st[s]: st[s] + tokens[s], :]).max() <= 2e-2
                # the iteration of the step has run or will run with the next call: the list is the oracle's
                segs = amskv.amskv_cache_segments(h, l)
                got_ids = [st[sc] + first + i for sc, first, _, ln in segs for i in range(ln)]
                assert got_ids == traces[l][s][0]
    finally:
        amskv.amskv_cache_destroy(h)


def test_attend_density_argument_checks():
    B, H, D = 1, 2, 64
    sides = (1, 2, 7)
    q, k, v = inp.iid_qkv(sides, B, H, D, "bf16", inp.layer_seed(8, 9))
    qd, kd, vd = ([x.cuda() for x in t] for t in (q, k, v))
    pol = (1, 1, False)
    need = amskv.amskv_cache_required_bytes(1, H, D, sides, sides, B, BF16, [pol])
    arena = torch.empty(need, dtype=torch.uint8, device="cuda")
    h = amskv.amskv_cache_create(1, H, D, sides, sides, B, BF16, [pol], arena=arena)
    mass = torch.empty(H * amskv.AMSKV_MAX_SCALES + 4, dtype=torch.float32, device="cuda")
    try:
        for s in range(len(sides)):
            amskv.amskv_append_scale(h, 0, s, kd[s], vd[s])
            o = torch.empty_like(qd[s])
            if s < len(sides) - 1:
                amskv.amskv_attend(h, 0, s, qd[s], o)
        s = len(sides) - 1
        o = torch.empty_like(qd[s])
        for bad in (dict(mass=None), dict(mass=mass.data_ptr() + 4), dict(s=s - 1), dict(q=None), dict(o=None)):
            with pytest.raises(amskv.AmskvError) as e:
                amskv.amskv_attend_density(h, 0, bad.get("s", s), bad.get("q", qd[s]), bad.get("o", o), bad.get("mass", mass))
            assert e.value.status == (amskv.AMSKV_ERR_ORDER if "s" in bad else amskv.AMSKV_ERR_INVALID_ARG)
        lens = amskv.amskv_attend_density(h, 0, s, qd[s], o, mass)     # and the well-formed call still goes through
        torch.cuda.synchronize()
        assert lens == [1, 4, 49][-len(lens):] and abs(float(mass[: len(lens)].sum()) - 49.0) < 1e-2
    finally:
        amskv.amskv_cache_destroy(h)
