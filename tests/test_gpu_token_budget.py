"""GPU parity of the token-budget mode (Algorithms 1 and 2 taken literally, Section 4.3): the
HIP path through the C ABI against the oracle's token-list simulation on the same seeded inputs.

Bar: bit-exact for the cached token list, its offsets, the budget in force and the cache
contents; max-abs 1e-4 (fp32) / 2e-2 (bf16) on the attention outputs.  The threshold of each
case sits at least 0.05 away from the score it is compared with, so the fp32 score of the
kernels and the fp64 score of the oracle decide alike.
"""
import numpy as np
import pytest
import torch

import amskv_inputs as inp
import paper_2511_16047_amd as amskv
from oracle import amskv_oracle as orc

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}
DT = {"f32": amskv.AMSKV_DTYPE_F32, "bf16": amskv.AMSKV_DTYPE_BF16}
VAR = (1, 2, 3, 4, 5, 6, 8, 10, 13, 16)


def _bits(t):
    it = torch.int16 if t.dtype == torch.bfloat16 else torch.int32
    return t.contiguous().view(it).cpu().numpy()


def _f64(t):
    return t.detach().to("cpu", torch.float64).numpy()


def _segment_ids(tokens, segs):
    st = orc.scale_starts(tokens)
    ids, at = [], 0
    for scale, first, off, ln in segs:
        if off >= 0:
            assert off == at
            at += ln
        ids += list(range(st[scale] + first, st[scale] + first + ln))
    return ids


def _scores(sides, k):
    """Oracle score of every scale against the one before it: mean over heads of the mean cosine."""
    out = [None]
    for s in range(1, len(sides)):
        cos, _ = orc.interscale_similarity(_f64(k[s]), _f64(k[s - 1]), (sides[s], sides[s]), (sides[s - 1], sides[s - 1]))
        out.append(float(np.mean(cos)))
    return out


def _run(sides, B, H, D, dtype, budget, theta_of, seed, rho=0.8, attend_at=None, softmax_scale=0.0):
    """budget = (c_min, c_max, c_cds); theta_of(scores, asked_step) -> theta.  attend_at: steps whose
    attention is run (None = all); the others are settled by the next append or by settle."""
    tokens = [s * s for s in sides]
    st = orc.scale_starts(tokens)
    c_min, c_max, c_cds = budget
    q, k, v = inp.correlated_qkv(sides, B, H, D, dtype, seed, rho)
    scores = _scores(sides, k)
    # which step would be the first to evaluate the test, were it never to succeed
    asked = []
    orc.alg1_cache_trace(tokens, c_min, c_max, c_cds, lambda i, c: asked.append(i) or False)
    theta = theta_of(scores, asked)

    def below(i, cached):
        prev = set(range(st[i - 1], st[i])) if i > 0 else None
        if c_max == c_min:
            return False                       # nothing to expand to: the library does not evaluate the score
        if not prev or not prev <= set(cached):
            return False                       # the earlier scale is not cached whole: no score
        assert abs(scores[i] - theta) >= 0.05, "threshold too close to the score for a mixed-precision decision"
        return scores[i] < theta

    trace = orc.alg1_cache_trace(tokens, c_min, c_max, c_cds, below)
    allow = orc.alg1_allow_mask(tokens, trace)
    cat = lambda xs: np.concatenate([_f64(x) for x in xs], axis=-2)
    want = orc.masked_attention(cat(q), cat(k), cat(v), allow, softmax_scale or None)
    kb_all = np.concatenate([_bits(x) for x in k], axis=-2)
    vb_all = np.concatenate([_bits(x) for x in v], axis=-2)

    qd, kd, vd = ([x.cuda() for x in t] for t in (q, k, v))
    budgets = [(c_min, c_max, c_cds, theta)]
    need = amskv.amskv_cache_required_bytes(1, H, D, sides, sides, B, DT[dtype], None, softmax_scale, budgets=budgets)
    arena = torch.empty(need, dtype=torch.uint8, device="cuda")
    arena.fill_(0xFF)
    h = amskv.amskv_cache_create(1, H, D, sides, sides, B, DT[dtype], None, softmax_scale, arena=arena, budgets=budgets)

    def check_contents(ids):
        segs = amskv.amskv_cache_segments(h, 0)
        assert _segment_ids(tokens, segs) == ids
        if not ids:
            return
        ko = torch.empty(B, H, len(ids), D, dtype=kd[0].dtype, device="cuda")
        vo = torch.empty_like(ko)
        amskv.amskv_cache_export(h, 0, ko, vo)
        torch.cuda.synchronize()
        assert np.array_equal(_bits(ko), kb_all[..., ids, :]) and np.array_equal(_bits(vo), vb_all[..., ids, :])

    worst = 0.0
    try:
        assert amskv.amskv_cache_capacity_tokens(h, 0) == c_max
        for s in range(len(sides)):
            amskv.amskv_append_scale(h, 0, s, kd[s], vd[s])
            own = list(range(st[s], st[s] + tokens[s]))
            check_contents((trace[s - 1][0] if s else []) + own)      # what the attention of step s reads
            if attend_at is None or s in attend_at:
                o = torch.full_like(qd[s], float("nan"))
                amskv.amskv_attend(h, 0, s, qd[s], o)
                torch.cuda.synchronize()
                got = _f64(o)
                assert np.isfinite(got).all()
                err = float(np.abs(got - want[..., st[s]: st[s] + tokens[s], :]).max())
                worst = max(worst, err)
                assert err <= TOL[dtype], "step %d max-abs %.3e" % (s, err)
                with pytest.raises(amskv.AmskvError):
                    amskv.amskv_attend(h, 0, s, qd[s], o)             # the scale has been rolled in: stale
            elif s % 2:
                amskv.amskv_cache_settle(h, 0)
            else:
                continue                                              # the next append settles it
            check_contents(trace[s][0])
            assert amskv.amskv_cache_budget_tokens(h, 0) == trace[s][1]
            assert amskv.amskv_cache_bytes_held(h, 0) == 2 * (2 if dtype == "bf16" else 4) * B * H * D * len(trace[s][0])
        amskv.amskv_cache_settle(h, 0)
        check_contents(trace[-1][0])
        assert amskv.amskv_cache_budget_tokens(h, 0) == trace[-1][1]
    finally:
        amskv.amskv_cache_destroy(h)
    return trace, worst, scores, asked


def _theta_above(scores, asked):     # cache-demanding at every test: above every score that is compared
    vals = [scores[i] for i in asked if i > 0]
    return max(vals) + 0.1 if vals else 0.0


def _theta_below_all(scores, asked):  # never demanding: below every score that is compared
    vals = [scores[i] for i in asked if i > 0]
    return min(vals) - 0.1 if vals else 0.0


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("theta_of", [_theta_above, _theta_below_all], ids=["demanding", "efficient"])
def test_var_schedule_paper_budgets(dtype, theta_of):
    # Section 5 budgets read as token counts on the 256x256 schedule: condensed = first two scales (5 tokens),
    # C_min = condensed + the 13x13 scale, C_max = condensed + the 10x10 and 13x13 scales
    trace, worst, scores, asked = _run(VAR, 2, 3, 64, dtype, (174, 274, 5), theta_of, inp.layer_seed(7, 0))
    expanded = [b for _, b in trace]
    assert asked[0] == 7
    if theta_of is _theta_above:
        assert expanded == [174] * 7 + [274] * 3
        assert len(trace[-1][0]) == 274        # 5 condensed, 13 tokens of the 13x13 scale, the whole 16x16 scale
    else:
        assert expanded == [174] * 10 and trace[9] == trace[8]
    print("var budgets %s %s worst max-abs %.3e" % (dtype, theta_of.__name__, worst))


@pytest.mark.parametrize("case", [
    dict(sides=(3, 1, 4, 1, 5, 9, 2, 6), budget=(40, 90, 7), D=64),     # condensed cut inside the first scale
    dict(sides=(2, 2, 5, 3, 7), budget=(20, 30, 0), D=128),             # no condensed tokens, head dim 128
    dict(sides=(1, 2, 3, 4, 5, 6), budget=(1, 1, 1), D=64),             # nothing but one token ever cached
    dict(sides=(1, 2, 3, 4, 5, 6), budget=(91, 91, 3), D=64),           # never over budget
    dict(sides=(4, 3, 6, 2, 9, 5), budget=(30, 81, 20), D=64),          # head and tail of one scale kept apart
    dict(sides=(1, 2, 4, 6, 8, 12, 16, 20), budget=(300, 700, 21), D=128),
], ids=lambda c: "x".join(map(str, c["sides"])))
@pytest.mark.parametrize("theta_of", [_theta_above, _theta_below_all], ids=["demanding", "efficient"])
def test_ragged_schedules_and_cuts(case, theta_of):
    _run(case["sides"], 2, 3, case["D"], "bf16", case["budget"], theta_of, inp.layer_seed(7, 1))


@pytest.mark.parametrize("attend_at", [(), (0, 3, 7, 9), (9,)], ids=["never", "some", "last"])
def test_settle_without_attention(attend_at):
    # the iteration of a step whose attention never ran is done by the next append or by settle
    _run(VAR, 2, 2, 64, "bf16", (174, 274, 5), _theta_above, inp.layer_seed(7, 2), attend_at=set(attend_at))


def test_score_unavailable_keeps_the_budget():
    # the 8x8 scale exceeds C_max and is never cached, so the first 5x5 scale overflows C_min without a
    # score and stays in part; the second then finds its predecessor incomplete: again no score.
    # The threshold would expand the budget at once if any score were compared with it.
    sides = (2, 8, 5, 5)
    trace, _, _, asked = _run(sides, 1, 2, 64, "bf16", (27, 60, 4), lambda sc, a: 0.99, inp.layer_seed(7, 3), rho=0.3)
    assert asked == [2, 3] and [b for _, b in trace] == [27] * 4
    assert len(trace[2][0]) == 27 and trace[2][0][4] == 4 + 64 + 2


def test_side_stream_and_softmax_scale():
    st = torch.cuda.Stream()
    with torch.cuda.stream(st):
        _run((2, 3, 5, 7, 11), 1, 5, 64, "f32", (25, 70, 4), _theta_above, inp.layer_seed(7, 4), softmax_scale=0.2)
    st.synchronize()


def test_full_batch_sampled_units():
    """The benchmark's token-budget configuration (VAR-d30 shape, batch 256, budgets 174/274/5): one layer per
    outcome of the Eq. 3 test, 16 sampled (b,h) each against the oracle -- attention within tolerance, cached
    tokens and contents bit for bit."""
    w = inp.config3(batch=256)
    sides, B, H, D = w.sides, w.batch, w.heads, w.head_dim
    tokens = [s * s for s in sides]
    st = orc.scale_starts(tokens)
    c_min, c_max, c_cds = 174, 274, 5
    for layer, grow in ((0, True), (1, False)):
        q, k, v = inp.correlated_qkv(sides, B, H, D, "bf16", inp.layer_seed(3, layer), 0.6, device="cuda")
        budgets = [(c_min, c_max, c_cds, 2.0 if grow else -2.0)]
        need = amskv.amskv_cache_required_bytes(1, H, D, sides, sides, B, DT["bf16"], None, budgets=budgets)
        arena = torch.empty(need, dtype=torch.uint8, device="cuda")
        arena.fill_(0xFF)
        h = amskv.amskv_cache_create(1, H, D, sides, sides, B, DT["bf16"], None, arena=arena, budgets=budgets)
        try:
            outs = []
            for s in range(len(sides)):
                amskv.amskv_append_scale(h, 0, s, k[s], v[s])
                o = torch.full_like(q[s], float("nan"))
                amskv.amskv_attend(h, 0, s, q[s], o)
                outs.append(o)
            torch.cuda.synchronize()
            trace = orc.alg1_cache_trace(tokens, c_min, c_max, c_cds, [grow] * len(sides))
            ids = trace[-1][0]
            assert _segment_ids(tokens, amskv.amskv_cache_segments(h, 0)) == ids
            assert amskv.amskv_cache_budget_tokens(h, 0) == trace[-1][1] == (c_max if grow else c_min)
            ko = torch.empty(B, H, len(ids), D, dtype=torch.bfloat16, device="cuda")
            vo = torch.empty_like(ko)
            amskv.amskv_cache_export(h, 0, ko, vo)
            torch.cuda.synchronize()
            allow = orc.alg1_allow_mask(tokens, trace)
            units = sorted({(b, hh) for (_, b, hh) in inp.sample_units(1, B, H, 16, 91 + layer)})
            worst = 0.0
            for b, hh in units:
                pick = lambda xs: np.concatenate([_f64(x[b:b + 1, hh:hh + 1]) for x in xs], axis=-2)
                want = orc.masked_attention(pick(q), pick(k), pick(v), allow)
                for s in range(len(sides)):
                    got = _f64(outs[s][b:b + 1, hh:hh + 1])
                    assert np.isfinite(got).all()
                    worst = max(worst, float(np.abs(got - want[..., st[s]: st[s] + tokens[s], :]).max()))
                kb = np.concatenate([_bits(x[b:b + 1, hh:hh + 1]) for x in k], axis=-2)[..., ids, :]
                vb = np.concatenate([_bits(x[b:b + 1, hh:hh + 1]) for x in v], axis=-2)[..., ids, :]
                assert np.array_equal(_bits(ko[b:b + 1, hh:hh + 1]), kb) and np.array_equal(_bits(vo[b:b + 1, hh:hh + 1]), vb)
            assert worst <= TOL["bf16"], worst
            print("token-budget full batch, layer %d (expanded: %s): worst max-abs %.3e over %d units" % (layer, grow, worst, len(units)))
        finally:
            amskv.amskv_cache_destroy(h)
            del q, k, v, arena
            torch.cuda.empty_cache()


def test_iterations_left_to_the_next_call_interleaved_layers():
    """The calling pattern of a model: for every step, every layer appends and attends, nothing is queried in
    between.  amskv_attend leaves each trimming iteration (and the reading of its Eq. 3 score) to the layer's next
    append; a reset drops the last one.  Three layers with different outcomes of the test, two images in a row
    through the same cache: outputs of both passes, and the final token list and contents, against the oracle."""
    sides, B, H, D = VAR, 3, 4, 64
    tokens = [s * s for s in sides]
    st = orc.scale_starts(tokens)
    c_min, c_max, c_cds = 174, 274, 5
    data, budgets, traces, wants = [], [], [], []
    for layer, kind in enumerate(("demanding", "efficient", "always")):
        q, k, v = inp.correlated_qkv(sides, B, H, D, "bf16", inp.layer_seed(7, 40 + layer), 0.8)
        scores = _scores(sides, k)
        asked = []
        orc.alg1_cache_trace(tokens, c_min, c_max, c_cds, lambda i, c: asked.append(i) or False)
        theta = {"demanding": _theta_above(scores, asked), "efficient": _theta_below_all(scores, asked), "always": 1.5}[kind]

        def below(i, cached, scores=scores, theta=theta):
            prev = set(range(st[i - 1], st[i])) if i > 0 else None
            if theta > 1.0:
                return True
            if not prev or not prev <= set(cached):
                return False
            assert abs(scores[i] - theta) >= 0.05
            return scores[i] < theta

        trace = orc.alg1_cache_trace(tokens, c_min, c_max, c_cds, below)
        cat = lambda xs: np.concatenate([_f64(x) for x in xs], axis=-2)
        wants.append(orc.masked_attention(cat(q), cat(k), cat(v), orc.alg1_allow_mask(tokens, trace)))
        traces.append(trace)
        budgets.append((c_min, c_max, c_cds, theta))
        data.append(tuple([x.cuda() for x in t] for t in (q, k, v)))
    L = len(data)
    need = amskv.amskv_cache_required_bytes(L, H, D, sides, sides, B, DT["bf16"], None, budgets=budgets)
    arena = torch.empty(need, dtype=torch.uint8, device="cuda")
    h = amskv.amskv_cache_create(L, H, D, sides, sides, B, DT["bf16"], None, arena=arena, budgets=budgets)
    try:
        for image in range(2):
            amskv.amskv_cache_reset(h)
            outs = [[torch.full_like(x, float("nan")) for x in data[l][0]] for l in range(L)]
            for s in range(len(sides)):
                for l in range(L):
                    amskv.amskv_append_scale(h, l, s, data[l][1][s], data[l][2][s])
                    amskv.amskv_attend(h, l, s, data[l][0][s], outs[l][s])
            torch.cuda.synchronize()
            for l in range(L):
                got = np.concatenate([_f64(o) for o in outs[l]], axis=-2)
                assert np.isfinite(got).all()
                assert float(np.abs(got - wants[l]).max()) <= TOL["bf16"], "image %d layer %d" % (image, l)
        for l in range(L):                      # the queries finish the last iteration
            ids = traces[l][-1][0]
            assert amskv.amskv_cache_budget_tokens(h, l) == traces[l][-1][1]
            assert _segment_ids(tokens, amskv.amskv_cache_segments(h, l)) == ids
            ko = torch.empty(B, H, len(ids), D, dtype=torch.bfloat16, device="cuda")
            vo = torch.empty_like(ko)
            amskv.amskv_cache_export(h, l, ko, vo)
            torch.cuda.synchronize()
            kb = np.concatenate([_bits(x) for x in data[l][1]], axis=-2)
            vb = np.concatenate([_bits(x) for x in data[l][2]], axis=-2)
            assert np.array_equal(_bits(ko), kb[..., ids, :]) and np.array_equal(_bits(vo), vb[..., ids, :])
        assert [traces[l][-1][1] for l in range(L)] == [c_max, c_min, c_max]
    finally:
        amskv.amskv_cache_destroy(h)
