"""What bench.py counts -- attention FLOPs, algorithmic bytes per launch, tokens moved and copied -- against the oracle's
kept sets and cached token lists, on plan-only caches (no GPU).  `value` and `roofline.achieved` are these counts
divided by measured time, so a wrong count would be a wrong headline.

Bar: exact (integers and integer-valued floats).
"""
import dataclasses

import numpy as np
import pytest

import amskv_inputs as inp
import bench
import paper_2511_16047_amd as amskv
from oracle import amskv_oracle as orc

EB = 2   # bf16


def _small(w, batch=3):
    return dataclasses.replace(w, batch=batch)


@pytest.mark.parametrize("layout,borrow,fuse", [(amskv.AMSKV_LAYOUT_PLANNED, True, True), (amskv.AMSKV_LAYOUT_COMPACT, False, False),
                                                (amskv.AMSKV_LAYOUT_COMPACT, True, True)], ids=["bench_flags", "compact_copy", "compact_borrow_fuse"])
@pytest.mark.parametrize("make", [inp.config3, inp.config4, inp.config5], ids=["var_d30", "infinity", "var_d24_sweep"])
def test_scale_window_counts(make, layout, borrow, fuse):
    w = _small(make())
    S, tokens = len(w.sides), w.tokens
    pols = list(w.policies) if w.policies else [(2, 2, False)] * w.layers
    pols = pols[:4] + [(0, 0, True), (1, 1, False), (0, 0, False)]
    w = dataclasses.replace(w, layers=len(pols), policies=pols)
    kv_len, moved, copied = bench.plan_trace(amskv, w, pols, None, layout, borrow, fuse)
    unit = w.head_dim * EB * w.batch * w.heads
    for l, pol in enumerate(pols):
        for s in range(S):
            kept = orc.kept_scales(pol, s)
            t_kv = sum(tokens[j] for j in kept)
            assert kv_len[l][s] == t_kv
            stored = orc.stored_scales(pol, s, S) if borrow else kept
            assert copied[l][s] == (tokens[s] if s in stored else 0)
            if layout == amskv.AMSKV_LAYOUT_PLANNED:
                assert moved[l][s] == 0
            else:
                # survivors whose offset among the stored scales changed when the step evicted something below them
                before = orc.stored_scales(pol, s - 1, S) if (borrow and s) else (orc.kept_scales(pol, s - 1) if s else [])
                off_b = {j: sum(tokens[i] for i in before if i < j) for j in before}
                off_a = {j: sum(tokens[i] for i in stored if i < j) for j in stored}
                assert moved[l][s] == sum(tokens[j] for j in stored if j in off_b and off_b[j] != off_a[j])
            fl, by, aby = bench.step_accounting(w, kv_len[l][s], moved[l][s], copied[l][s], s, False, fuse)
            assert fl == 4.0 * w.batch * w.heads * tokens[s] * t_kv * w.head_dim
            read_write = (2 * tokens[s] + 2 * t_kv) * unit                      # Q, O, K~, V~
            if fuse:
                assert by == read_write + 2 * copied[l][s] * unit               # + the write of K_s, V_s by the same launch
                assert aby == 4 * moved[l][s] * unit
            else:
                assert by == read_write
                assert aby == (4 * moved[l][s] + 4 * copied[l][s]) * unit       # read + write, K and V


def test_benchmark_shape_totals():
    """The ten-scale schedule under {0,1} + window 2 and under keep-all: the closed forms of the token counts."""
    w = dataclasses.replace(inp.config3(), layers=2, batch=2)
    pols = [(2, 2, False), (0, 0, True)]
    kv_len, moved, copied = bench.plan_trace(amskv, w, pols, None, amskv.AMSKV_LAYOUT_PLANNED, True, True)
    assert kv_len[0] == [1, 5, 14, 30, 55, 82, 130, 205, 338, 530]
    assert kv_len[1] == [1, 5, 14, 30, 55, 91, 155, 255, 424, 680]
    assert copied[1] == w.tokens[:-1] + [0]            # the last scale is attended in place, never copied
    assert moved == [[0] * 10, [0] * 10]


@pytest.mark.parametrize("budget,theta", [((174, 274, 5), 2.0), ((174, 274, 5), -2.0), ((60, 60, 5), 0.0), ((300, 500, 40), 2.0)])
def test_token_budget_counts(budget, theta):
    w = dataclasses.replace(inp.config3(), layers=1, batch=2)
    tokens, S = w.tokens, len(w.sides)
    c_min, c_max, c_cds = budget
    kv_len, moved, copied = bench.plan_trace(amskv, w, None, [(c_min, c_max, c_cds, theta)], amskv.AMSKV_LAYOUT_COMPACT, False, False)
    trace = orc.alg1_cache_trace(tokens, c_min, c_max, c_cds, [theta > 1.0] * S)
    prev = []
    for s in range(S):
        assert kv_len[0][s] == len(prev) + tokens[s]                  # the cache as the step before left it + the own scale
        now = trace[s][0]
        place_before = {g: i for i, g in enumerate(prev)}
        assert copied[0][s] == sum(1 for g in now if g not in place_before)
        assert moved[0][s] == sum(1 for i, g in enumerate(now) if g in place_before and place_before[g] != i)
        prev = now


@pytest.mark.parametrize("window,n_sink", [(170, 0), (170, 5), (64, 14)])
def test_token_window_counts(window, n_sink):
    w = dataclasses.replace(inp.config3(), layers=1, batch=2)
    tokens, S = w.tokens, len(w.sides)
    kv_len, moved, copied = bench.plan_trace(amskv, w, None, None, amskv.AMSKV_LAYOUT_COMPACT, False, False, windows=[(window, n_sink)])
    cached = orc.token_window_cache(tokens, window, n_sink)
    prev = []
    for s in range(S):
        assert kv_len[0][s] == len(prev) + tokens[s]
        now = list(cached[s])
        place_before = {g: i for i, g in enumerate(prev)}
        assert copied[0][s] == sum(1 for g in now if g not in place_before)
        assert moved[0][s] == sum(1 for i, g in enumerate(now) if g in place_before and place_before[g] != i)
        prev = now
