"""Host logic of the library (policy -> kept set, offsets, eviction lists, bytes held, status
codes) against the oracle, through the C ABI on a plan-only cache: no GPU needed."""
import itertools
import os
import re

import pytest

import paper_2511_16047_amd as amskv
from oracle import amskv_oracle as orc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
VAR = (1, 2, 3, 4, 5, 6, 8, 10, 13, 16)
INF = (1, 2, 4, 6, 8, 12, 16, 20, 24, 32, 40, 48, 64)


def test_library_exports_every_declared_symbol():
    lib = amskv.load_library()
    text = open(os.path.join(ROOT, "include", "amskv.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = set(re.findall(r"\b(amskv_[a-z_]+)\s*\(", text))
    assert names == set(amskv.binding.EXPORTED)
    for n in sorted(names):
        assert hasattr(lib, n), n


def _plan_cache(sides, policies, layout=amskv.AMSKV_LAYOUT_COMPACT, B=2, H=3, D=64, dtype=amskv.AMSKV_DTYPE_BF16):
    return amskv.amskv_cache_create(len(policies), H, D, sides, sides, B, dtype, policies, 0.0, layout)


@pytest.mark.parametrize("sides", [VAR, INF, (1, 2, 3), (2, 2, 5, 3)])
def test_compact_layout_matches_oracle(sides):
    tokens = [s * s for s in sides]
    pols = [(c, w, False) for c, w in itertools.product(range(5), range(5))] + [(0, 0, True), (2, 1, True)]
    B, H, D = 2, 3, 64
    h = _plan_cache(sides, pols, B=B, H=H, D=D)
    try:
        for l, pol in enumerate(pols):
            assert amskv.amskv_cache_capacity_tokens(h, l) == orc.cache_capacity(tokens, pol)
        for s in range(len(sides)):
            for l, pol in enumerate(pols):
                amskv.amskv_append_scale(h, l, s)
                kept = orc.kept_scales(pol, s)
                offs = orc.segment_offsets(tokens, pol, s)
                assert amskv.amskv_cache_layout(h, l) == [(k, o, tokens[k]) for k, o in zip(kept, offs)]
                assert amskv.amskv_cache_last_evicted(h, l) == orc.evicted_scales(pol, s)
                for inc in (True, False):
                    assert amskv.amskv_cache_bytes_held(h, l, inc) == orc.bytes_held(tokens, pol, s, B, H, D, 2, inc)
    finally:
        amskv.amskv_cache_destroy(h)


@pytest.mark.parametrize("sides", [VAR, INF])
def test_planned_layout_is_overlap_free_fixed_and_tight(sides):
    tokens = [s * s for s in sides]
    pols = [(c, w, False) for c, w in itertools.product(range(4), range(5))] + [(0, 0, True)]
    h = _plan_cache(sides, pols, layout=amskv.AMSKV_LAYOUT_PLANNED)
    try:
        slot = [dict() for _ in pols]
        for s in range(len(sides)):
            for l, pol in enumerate(pols):
                amskv.amskv_append_scale(h, l, s)
                lay = amskv.amskv_cache_layout(h, l)
                assert [k for k, _, _ in lay] == orc.kept_scales(pol, s)
                cap = amskv.amskv_cache_capacity_tokens(h, l)
                spans = sorted((o, o + n) for _, o, n in lay)
                for (a0, a1), (b0, b1) in zip(spans, spans[1:]):
                    assert a1 <= b0
                assert spans[-1][1] <= cap
                for k, o, n in lay:
                    assert n == tokens[k]
                    assert slot[l].setdefault(k, o) == o     # a scale never moves
        for l, pol in enumerate(pols):
            # no data movement, and no more memory than the compacting layout needs
            assert amskv.amskv_cache_capacity_tokens(h, l) == orc.cache_capacity(tokens, pol)
    finally:
        amskv.amskv_cache_destroy(h)


@pytest.mark.parametrize("borrow", [False, True])
def test_planned_layout_keeps_reading_order_contiguous_where_it_costs_nothing(borrow):
    """Among the placements of least capacity the one whose steps stream the fewest separate runs is taken: a layer that
    keeps everything holds its scales back to back in ascending order, and under {0,1} + window 2 the scales the last
    step reads form one run."""
    tokens = [s * s for s in VAR]
    st = orc.scale_starts(tokens)
    pols = [(0, 0, True), (2, 2, False)]
    h = amskv.amskv_cache_create(len(pols), 3, 64, VAR, VAR, 2, amskv.AMSKV_DTYPE_BF16, pols, 0.0, amskv.AMSKV_LAYOUT_PLANNED,
                                 borrow_unretained=borrow)
    try:
        for s in range(len(VAR)):
            for l in range(len(pols)):
                amskv.amskv_append_scale(h, l, s)
        keep_all = [x for x in amskv.amskv_cache_layout(h, 0) if x[1] >= 0]
        assert [(k, o) for k, o, _ in keep_all] == [(k, st[k]) for k, _, _ in keep_all]
        window = [x for x in amskv.amskv_cache_layout(h, 1) if x[1] >= 0]
        at = 0
        for k, o, n in window:                      # ascending scale id = reading order
            assert o == at
            at += n
        for l, pol in enumerate(pols):
            want = orc.stored_capacity(tokens, pol) if borrow else orc.cache_capacity(tokens, pol)
            assert amskv.amskv_cache_capacity_tokens(h, l) == want
    finally:
        amskv.amskv_cache_destroy(h)


@pytest.mark.parametrize("layout", [amskv.AMSKV_LAYOUT_COMPACT, amskv.AMSKV_LAYOUT_PLANNED])
def test_borrow_unretained_layout(layout):
    sides = VAR
    tokens = [s * s for s in sides]
    n = len(sides)
    pols = [(c, w, False) for c, w in itertools.product(range(4), range(4))] + [(0, 0, True)]
    B, H, D = 2, 3, 64
    h = amskv.amskv_cache_create(len(pols), H, D, sides, sides, B, amskv.AMSKV_DTYPE_BF16, pols, 0.0, layout,
                                 borrow_unretained=True)
    try:
        for l, pol in enumerate(pols):
            assert amskv.amskv_cache_capacity_tokens(h, l) == orc.stored_capacity(tokens, pol)
        slot = [dict() for _ in pols]
        for s in range(n):
            for l, pol in enumerate(pols):
                amskv.amskv_append_scale(h, l, s)
                lay = amskv.amskv_cache_layout(h, l)
                stored = orc.stored_scales(pol, s, n)
                assert [k for k, _, _ in lay] == orc.kept_scales(pol, s)
                assert [k for k, o, _ in lay if o >= 0] == stored
                assert [k for k, o, _ in lay if o < 0] == [k for k in orc.kept_scales(pol, s) if k not in stored]
                spans = sorted((o, o + ln) for _, o, ln in lay if o >= 0)
                for (a0, a1), (b0, b1) in zip(spans, spans[1:]):
                    assert a1 <= b0
                if spans:
                    assert spans[-1][1] <= amskv.amskv_cache_capacity_tokens(h, l)
                if layout == amskv.AMSKV_LAYOUT_COMPACT:
                    acc = 0
                    for k, o, ln in lay:
                        if o >= 0:
                            assert o == acc
                            acc += ln
                else:
                    for k, o, ln in lay:
                        if o >= 0:
                            assert slot[l].setdefault(k, o) == o
                assert amskv.amskv_cache_last_evicted(h, l) == orc.evicted_scales(pol, s)
                assert amskv.amskv_cache_bytes_held(h, l, True) == orc.bytes_held(tokens, pol, s, B, H, D, 2, True)
                assert amskv.amskv_cache_bytes_held(h, l, False) == orc.bytes_held(tokens, pol, s, B, H, D, 2, False)
    finally:
        amskv.amskv_cache_destroy(h)
    # the arena shrinks: {0,1}+window 2 needs 338 tokens per (b,h) instead of 530
    need_b = amskv.amskv_cache_required_bytes(1, H, D, sides, sides, B, 1, [(2, 2, False)], borrow_unretained=True)
    need = amskv.amskv_cache_required_bytes(1, H, D, sides, sides, B, 1, [(2, 2, False)])
    assert need - need_b >= 2 * B * H * (530 - 338) * D * 2 - 1024


def test_required_bytes_closed_form():
    B, H, D = 4, 5, 64
    pols = [(2, 2, False), (0, 0, True)]
    need = amskv.amskv_cache_required_bytes(2, H, D, VAR, VAR, B, amskv.AMSKV_DTYPE_BF16, pols)
    kv = sum(2 * B * H * cap * D * 2 for cap in (530, 680))
    ws = (2 * B * H * 4 + 2 * 2 * H * 4) * 4                 # similarity: four sums per (tensor, b, h) and per (layer, tensor, h)
    ws += (B * H * ((256 + 31) // 32) + H) * 16 * 4           # density: 16 groups per (b, h, 32-row query block) and per head
    assert kv + ws <= need <= kv + ws + 6 * 256
    need32 = amskv.amskv_cache_required_bytes(2, H, D, VAR, VAR, B, amskv.AMSKV_DTYPE_F32, pols)
    assert need32 >= 2 * kv


def test_status_codes():
    E = amskv.AmskvError
    pol = [(2, 1, False)]
    with pytest.raises(E) as e:
        amskv.amskv_cache_create(1, 4, 48, VAR, VAR, 1, 1, pol)           # head_dim
    assert e.value.status == amskv.AMSKV_ERR_INVALID_ARG
    with pytest.raises(E) as e:
        amskv.amskv_cache_create(2, 4, 64, VAR, VAR, 1, 1, pol)           # layers != n_layers
    assert e.value.status == amskv.AMSKV_ERR_INVALID_ARG
    with pytest.raises(E) as e:
        amskv.amskv_cache_create(1, 4, 64, (1, 0, 3), (1, 2, 3), 1, 1, pol)  # empty scale
    assert e.value.status == amskv.AMSKV_ERR_INVALID_ARG
    with pytest.raises(E) as e:
        amskv.amskv_cache_create(1, 4, 64, VAR, VAR, 1, 7, pol)           # dtype
    assert e.value.status == amskv.AMSKV_ERR_INVALID_ARG
    with pytest.raises(E) as e:
        amskv.amskv_cache_create(1, 4, 64, VAR, VAR, 1, 1, [(-1, 1, False)])
    assert e.value.status == amskv.AMSKV_ERR_INVALID_ARG
    with pytest.raises(E) as e:
        amskv.amskv_cache_create(1, 4, 64, tuple(range(1, 19)), tuple(range(1, 19)), 1, 1, pol)  # > 16 scales
    assert e.value.status == amskv.AMSKV_ERR_INVALID_ARG

    lib = amskv.load_library()
    import ctypes as C
    sc, po, keep = amskv.binding._structs(VAR, VAR, 1, 1, pol, 0.0, 0)
    out = C.c_void_p(None)
    # a non-null (never dereferenced) arena that is too small / misaligned
    assert lib.amskv_cache_create(1, 4, 64, C.byref(sc), C.byref(po), C.c_void_p(4096), 1024, C.byref(out)) == amskv.AMSKV_ERR_ARENA_TOO_SMALL
    assert lib.amskv_cache_create(1, 4, 64, C.byref(sc), C.byref(po), C.c_void_p(4100), 1 << 40, C.byref(out)) == amskv.AMSKV_ERR_INVALID_ARG
    assert out.value is None

    h = amskv.amskv_cache_create(1, 4, 64, VAR, VAR, 1, 1, pol)
    try:
        with pytest.raises(E) as e:
            amskv.amskv_append_scale(h, 0, 1)                              # scale 1 before scale 0
        assert e.value.status == amskv.AMSKV_ERR_ORDER
        with pytest.raises(E) as e:
            amskv.amskv_append_scale(h, 3, 0)                              # no such layer
        assert e.value.status == amskv.AMSKV_ERR_INVALID_ARG
        assert lib.amskv_attend(h, 0, 0, C.c_void_p(256), C.c_void_p(256), None) == amskv.AMSKV_ERR_ORDER  # nothing appended
        for s in range(5):
            amskv.amskv_append_scale(h, 0, s)
        with pytest.raises(E) as e:
            amskv.amskv_append_scale(h, 0, 4)                              # twice
        assert e.value.status == amskv.AMSKV_ERR_ORDER
        assert lib.amskv_attend(h, 0, 3, C.c_void_p(256), C.c_void_p(256), None) == amskv.AMSKV_ERR_ORDER  # stale scale
        assert lib.amskv_attend(h, 0, 4, C.c_void_p(256), C.c_void_p(256), None) == amskv.AMSKV_ERR_NO_DEVICE_MEMORY
        assert lib.amskv_append_scale(h, 0, 5, C.c_void_p(256), C.c_void_p(256), None) == amskv.AMSKV_ERR_NO_DEVICE_MEMORY
        assert lib.amskv_append_scale(h, 0, 5, C.c_void_p(256), None, None) == amskv.AMSKV_ERR_INVALID_ARG
        f = (C.c_float * 4)()
        # window 1 at step 4 holds {0,1,3,4}: scale 2 is gone, scale 5 not there yet
        assert lib.amskv_interscale_similarity(h, 0, 3, f, None, None, None) == amskv.AMSKV_ERR_EVICTED
        assert lib.amskv_interscale_similarity(h, 0, 5, f, None, None, None) == amskv.AMSKV_ERR_ORDER
        assert lib.amskv_interscale_similarity(h, 0, 0, f, None, None, None) == amskv.AMSKV_ERR_INVALID_ARG
        assert lib.amskv_interscale_similarity(h, 0, 4, f, None, None, None) == amskv.AMSKV_ERR_NO_DEVICE_MEMORY
        amskv.amskv_cache_reset(h)
        assert amskv.amskv_cache_layout(h, 0) == []
        amskv.amskv_append_scale(h, 0, 0)
        assert amskv.amskv_cache_layout(h, 0) == [(0, 0, 1)]
    finally:
        amskv.amskv_cache_destroy(h)
    assert amskv.status_string(0) == "ok" and "order" in amskv.status_string(-2)
    assert "host memory" in amskv.status_string(amskv.AMSKV_ERR_NO_HOST_MEMORY)


# ------------------------------------------------------------------ token-budget mode (Algorithms 1 and 2, literal)
def _budget_cache(sides, budgets, B=2, H=3, D=64, dtype=amskv.AMSKV_DTYPE_BF16, **kw):
    return amskv.amskv_cache_create(len(budgets), H, D, sides, sides, B, dtype, None, 0.0,
                                    amskv.AMSKV_LAYOUT_COMPACT, budgets=budgets, **kw)


def _segment_ids(tokens, segs, cached_only=True):
    st = orc.scale_starts(tokens)
    ids, at = [], 0
    for scale, first, off, ln in segs:
        if off < 0:
            if cached_only:
                continue
        else:
            assert off == at, "cached tokens sit back to back from offset 0"
            at += ln
        ids += list(range(st[scale] + first, st[scale] + first + ln))
    return ids


@pytest.mark.parametrize("sides", [VAR, INF, (1, 2, 3), (2, 2, 5, 3), (3, 1, 4, 1, 5, 9, 2, 6)])
def test_token_budget_mode_matches_algorithm_1(sides):
    import random
    tokens = [s * s for s in sides]
    total = sum(tokens)
    rng = random.Random(1234 + len(sides))
    budgets = [(174, 274, 5, 2.0), (174, 274, 5, -2.0), (274, 274, 5, 0.0), (174, 255, 5, 2.0), (174, 300, 5, 2.0),
               (total, total, 0, 0.0), (1, 1, 0, 2.0), (1, 1, 1, 2.0), (7, 7, 7, -2.0)]
    for _ in range(40):
        cds = rng.randint(0, max(tokens))
        cmin = rng.randint(cds, total)
        cmax = rng.randint(max(cmin, 1), total + 3)
        budgets.append((cmin, cmax, cds, rng.choice([2.0, -2.0])))
    B, H, D = 2, 3, 64
    starts, scale_of = orc.scale_starts(tokens), orc.scale_of_token(tokens)
    h = _budget_cache(sides, budgets, B=B, H=H, D=D)
    try:
        traces = [orc.alg1_cache_trace(tokens, a, b, c, [th > 1] * len(tokens)) for a, b, c, th in budgets]
        for l, (a, b, c, th) in enumerate(budgets):
            assert amskv.amskv_cache_capacity_tokens(h, l) == b
            assert amskv.amskv_cache_budget_tokens(h, l) == a
        for s in range(len(sides)):
            for l in range(len(budgets)):
                amskv.amskv_append_scale(h, l, s)
                segs = amskv.amskv_cache_segments(h, l)
                # before the scale's own iteration: the cache of the previous step plus the scale, read in place
                assert segs[-1] == (s, 0, -1, tokens[s])
                assert _segment_ids(tokens, segs) == (traces[l][s - 1][0] if s else [])
                assert amskv.amskv_cache_layout(h, l) == [(a, c, d) for a, _, c, d in segs]
                if s % 2:
                    amskv.amskv_cache_settle(h, l)   # odd steps settle explicitly, even ones at the next append
                    amskv.amskv_cache_settle(h, l)   # and settling twice changes nothing
                    ids, bgt = traces[l][s]
                    assert _segment_ids(tokens, amskv.amskv_cache_segments(h, l), cached_only=False) == ids
                    assert amskv.amskv_cache_budget_tokens(h, l) == bgt
                    held = amskv.amskv_cache_bytes_held(h, l, True)
                    assert held == 2 * 2 * B * H * D * len(ids)
                    # scales that lost cached tokens in this iteration
                    lost = set(traces[l][s - 1][0]) - set(ids)
                    assert amskv.amskv_cache_last_evicted(h, l) == sorted({int(scale_of[g]) for g in lost})
        for l in range(len(budgets)):
            amskv.amskv_cache_settle(h, l)
            ids, bgt = traces[l][-1]
            assert _segment_ids(tokens, amskv.amskv_cache_segments(h, l), cached_only=False) == ids
            assert amskv.amskv_cache_budget_tokens(h, l) == bgt
            assert len(ids) <= bgt
        amskv.amskv_cache_reset(h)
        for l, (a, b, c, th) in enumerate(budgets):
            assert amskv.amskv_cache_segments(h, l) == [] and amskv.amskv_cache_budget_tokens(h, l) == a
    finally:
        amskv.amskv_cache_destroy(h)


def test_token_budget_mode_rejects_bad_configurations():
    sides = (1, 2, 3)
    E = amskv.AMSKV_ERR_INVALID_ARG
    for bad in [(5, 4, 2, 0.0), (1, 4, 2, 0.0), (0, 0, 0, 0.0), (3, 4, -1, 0.0), (3, 4, 1, float("nan"))]:
        with pytest.raises(amskv.AmskvError) as e:
            _budget_cache(sides, [bad])
        assert e.value.status == E
    for kw in [dict(borrow_unretained=True), dict(fuse_append=True)]:
        with pytest.raises(amskv.AmskvError) as e:
            _budget_cache(sides, [(3, 4, 1, 0.0)], **kw)
        assert e.value.status == E
    with pytest.raises(amskv.AmskvError) as e:
        amskv.amskv_cache_create(1, 3, 64, sides, sides, 2, amskv.AMSKV_DTYPE_BF16, None, 0.0,
                                 amskv.AMSKV_LAYOUT_PLANNED, budgets=[(3, 4, 1, 0.0)])
    assert e.value.status == E
    # a threshold inside [-1, 1] needs the keys: a plan-only cache cannot evaluate Eq. 3
    h = _budget_cache(sides, [(4, 9, 1, 0.0)])
    try:
        amskv.amskv_append_scale(h, 0, 0)
        amskv.amskv_append_scale(h, 0, 1)
        amskv.amskv_append_scale(h, 0, 2)      # settles scale 1: 1 + 4 > 4 -> the test is due, scale 0 is cached whole
        assert False, "expected an error"
    except amskv.AmskvError as e:
        assert e.status == amskv.AMSKV_ERR_NO_DEVICE_MEMORY
    finally:
        amskv.amskv_cache_destroy(h)


def test_io_layout_validation_on_plan_only_cache():
    H, D = 3, 64
    h = _plan_cache((1, 2, 3), [(1, 1, False)], H=H, D=D)
    try:
        TM, HM = amskv.AMSKV_IO_TOKEN_MAJOR, amskv.AMSKV_IO_HEAD_MAJOR
        amskv.amskv_cache_set_io_layout(h, TM, 3 * H * D, 3 * H * D + 8, H * D)      # padded strides are fine
        amskv.amskv_cache_set_io_layout(h, HM)
        for bad in [(H * D - 8, H * D, H * D), (H * D, H * D + 1, H * D), (H * D, H * D, 0), (1 << 41, H * D, H * D)]:
            with pytest.raises(amskv.AmskvError) as e:
                amskv.amskv_cache_set_io_layout(h, TM, *bad)
            assert e.value.status == amskv.AMSKV_ERR_INVALID_ARG
        with pytest.raises(amskv.AmskvError) as e:
            amskv.amskv_cache_set_io_layout(h, 2, H * D, H * D, H * D)
        assert e.value.status == amskv.AMSKV_ERR_INVALID_ARG
        amskv.amskv_append_scale(h, 0, 0)
        with pytest.raises(amskv.AmskvError) as e:                                   # a scale is resident
            amskv.amskv_cache_set_io_layout(h, TM, H * D, H * D, H * D)
        assert e.value.status == amskv.AMSKV_ERR_ORDER
        amskv.amskv_cache_reset(h)
        amskv.amskv_cache_set_io_layout(h, TM, H * D, H * D, H * D)
    finally:
        amskv.amskv_cache_destroy(h)


def test_oversized_launches_are_rejected_at_create():
    # units (b, h, 32-row query block) and 16-byte chunks of a scale must fit the 32-bit launch grids
    with pytest.raises(amskv.AmskvError) as e:
        amskv.amskv_cache_required_bytes(1, 4096, 64, (1024,), (1024,), 4096, amskv.AMSKV_DTYPE_BF16, [(0, 0, True)])
    assert e.value.status == amskv.AMSKV_ERR_INVALID_ARG


@pytest.mark.parametrize("sides", [VAR, INF, (1, 2, 3), (2, 2, 5, 3), (3, 1, 4, 1, 5, 9, 2, 6)])
def test_token_window_mode_matches_the_oracle(sides):
    """Sliding window / sink + window at token granularity (the SWA / STA kept sets): the segment list after every
    step is the oracle's window over the flattened token sequence, also where a scale is larger than the window."""
    import random
    tokens = [s * s for s in sides]
    total = sum(tokens)
    rng = random.Random(4321 + len(sides))
    windows = [(170, 0), (170, 5), (total, 0), (total + 5, 3), (1, 0), (1, 1), (7, 7), (max(tokens) - 1, 2)]
    for _ in range(40):
        w = rng.randint(1, total + 3)
        windows.append((w, rng.randint(0, w)))
    B, H, D = 2, 3, 64
    h = amskv.amskv_cache_create(len(windows), H, D, sides, sides, B, amskv.AMSKV_DTYPE_BF16, None, windows=windows)
    try:
        want = [orc.token_window_cache(tokens, w, k) for w, k in windows]
        for s in range(len(sides)):
            for l, (w, k) in enumerate(windows):
                amskv.amskv_append_scale(h, l, s)
                segs = amskv.amskv_cache_segments(h, l)
                assert segs[-1] == (s, 0, -1, tokens[s])
                assert _segment_ids(tokens, segs) == (want[l][s - 1] if s else [])
                amskv.amskv_cache_settle(h, l)
                assert _segment_ids(tokens, amskv.amskv_cache_segments(h, l), cached_only=False) == want[l][s]
                assert amskv.amskv_cache_bytes_held(h, l, True) == 2 * 2 * B * H * D * len(want[l][s])
                assert amskv.amskv_cache_budget_tokens(h, l) == w == amskv.amskv_cache_capacity_tokens(h, l)
    finally:
        amskv.amskv_cache_destroy(h)
    # a window is one budget: two different ones are refused
    with pytest.raises(amskv.AmskvError):
        _two_budget_window(sides, B, H, D)


def _two_budget_window(sides, B, H, D):
    import ctypes as C
    from paper_2511_16047_amd import binding as b
    sc, po, keep = b._structs(sides, sides, B, amskv.AMSKV_DTYPE_BF16, None, 0.0, amskv.AMSKV_LAYOUT_COMPACT,
                              budgets=[(3, 9, 0, 0.0)])
    po.mode = amskv.AMSKV_MODE_TOKEN_WINDOW
    out = C.c_uint64(0)
    b._check(b.load_library().amskv_cache_required_bytes(1, H, D, C.byref(sc), C.byref(po), C.byref(out)), "required_bytes")
