"""GPU parity: the HIP path, through the C ABI, against the CPU oracle on the same seeded inputs.

Bar: bit-exact for slot selection, eviction and cache contents; max-abs 1e-4 (fp32) and
2e-2 (bf16) on attention outputs for unit-variance inputs; 1e-5 abs on the cosine.
"""
import math

import numpy as np
import pytest
import torch

import amskv_inputs as inp
import paper_2511_16047_amd as amskv
from oracle import amskv_oracle as orc

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}
DT = {"f32": amskv.AMSKV_DTYPE_F32, "bf16": amskv.AMSKV_DTYPE_BF16}


def _bits(t: torch.Tensor) -> np.ndarray:
    """Raw element bit patterns as a numpy integer array (host)."""
    it = torch.int16 if t.dtype == torch.bfloat16 else torch.int32
    return t.contiguous().view(it).cpu().numpy()


def _f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to("cpu", torch.float64).numpy()


class Runner:
    """Drives one cache through the ABI and checks every step against the oracle."""

    def __init__(self, sides_h, sides_w, B, H, D, dtype, policies, layout=amskv.AMSKV_LAYOUT_COMPACT,
                 softmax_scale=0.0, borrow=False, fuse=False):
        self.sh, self.sw = list(sides_h), list(sides_w)
        self.tokens = orc.scale_tokens(self.sh, self.sw)
        self.B, self.H, self.D, self.dtype = B, H, D, dtype
        self.policies, self.layout, self.scale, self.borrow, self.fuse = policies, layout, softmax_scale, borrow, fuse
        self.eb = 2 if dtype == "bf16" else 4
        need = amskv.amskv_cache_required_bytes(len(policies), H, D, self.sh, self.sw, B, DT[dtype], policies,
                                                softmax_scale, layout, borrow, fuse)
        self.arena = torch.empty(need, dtype=torch.uint8, device="cuda")
        self.arena.fill_(0xFF)          # every stale or never-written element reads as NaN
        self.h = amskv.amskv_cache_create(len(policies), H, D, self.sh, self.sw, B, DT[dtype], policies,
                                          softmax_scale, layout, arena=self.arena, borrow_unretained=borrow,
                                          fuse_append=fuse)

    def close(self):
        amskv.amskv_cache_destroy(self.h)

    def check_cache(self, layer, s, k_scales, v_scales):
        pol = self.policies[layer]
        kept = orc.kept_scales(pol, s)
        lay = amskv.amskv_cache_layout(self.h, layer)
        assert [x[0] for x in lay] == kept
        assert [x[2] for x in lay] == [self.tokens[k] for k in kept]
        if self.borrow:
            stored = orc.stored_scales(pol, s, len(self.tokens))
            assert [x[0] for x in lay if x[1] >= 0] == stored
            if self.layout == amskv.AMSKV_LAYOUT_COMPACT:
                assert [x[1] for x in lay if x[1] >= 0] == [sum(self.tokens[j] for j in stored[:i]) for i in range(len(stored))]
        elif self.layout == amskv.AMSKV_LAYOUT_COMPACT:
            assert [x[1] for x in lay] == orc.segment_offsets(self.tokens, pol, s)
        assert amskv.amskv_cache_last_evicted(self.h, layer) == orc.evicted_scales(pol, s)
        assert amskv.amskv_cache_bytes_held(self.h, layer) == orc.bytes_held(self.tokens, pol, s, self.B, self.H, self.D, self.eb)
        tk = sum(self.tokens[k] for k in kept)
        ko = torch.empty(self.B, self.H, tk, self.D, dtype=k_scales[0].dtype, device="cuda")
        vo = torch.empty_like(ko)
        amskv.amskv_cache_export(self.h, layer, ko, vo)
        torch.cuda.synchronize()
        want_k = orc.cache_contents([_bits(x) for x in k_scales[: s + 1]], pol, s)
        want_v = orc.cache_contents([_bits(x) for x in v_scales[: s + 1]], pol, s)
        assert np.array_equal(_bits(ko), want_k), "K cache contents differ at layer %d step %d" % (layer, s)
        assert np.array_equal(_bits(vo), want_v), "V cache contents differ at layer %d step %d" % (layer, s)

    def run_layer(self, layer, q, k, v, check_cache=True, units=None):
        """q,k,v: per-scale device tensors.  units: list of (b,h) to compare, None = all."""
        pol = self.policies[layer]
        outs = []
        for s in range(len(self.tokens)):
            amskv.amskv_append_scale(self.h, layer, s, k[s], v[s])
            o = torch.full_like(q[s], float("nan"))
            amskv.amskv_attend(self.h, layer, s, q[s], o)
            outs.append(o)
            if check_cache:
                self.check_cache(layer, s, k, v)
        torch.cuda.synchronize()
        sel = (lambda t: t) if units is None else (lambda t: torch.stack([t[b, h] for b, h in units])[None])
        want = orc.attend_all_steps([_f64(sel(x)) for x in q], [_f64(sel(x)) for x in k], [_f64(sel(x)) for x in v],
                                    self.tokens, pol, self.scale or None)
        worst = 0.0
        for s in range(len(self.tokens)):
            got = _f64(sel(outs[s]))
            assert np.isfinite(got).all(), "non-finite output at layer %d step %d" % (layer, s)
            err = float(np.abs(got - want[s]).max())
            worst = max(worst, err)
            assert err <= TOL[self.dtype], "layer %d step %d max-abs %.3e" % (layer, s, err)
        return outs, worst


def _qkv(sides_h, sides_w, B, H, D, dtype, seed):
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    dt = inp.torch_dtype(dtype)
    mk = lambda: [torch.randn(B, H, a * b, D, generator=g).to(dt).cuda() for a, b in zip(sides_h, sides_w)]
    return mk(), mk(), mk()


# ------------------------------------------------------------------ configuration 1: fp32, one layer
@pytest.mark.parametrize("pol", [(2, 2, False), (0, 0, True)], ids=["c2w2", "vanilla"])
def test_config1_fp32_all_units(pol):
    w = inp.config1()
    q, k, v = inp.iid_qkv(w.sides, w.batch, w.heads, w.head_dim, "f32", inp.layer_seed(1, 0), device="cpu")
    q, k, v = ([x.cuda() for x in t] for t in (q, k, v))
    r = Runner(w.sides, w.sides, w.batch, w.heads, w.head_dim, "f32", [pol])
    try:
        outs, worst = r.run_layer(0, q, k, v)
        assert torch.equal(outs[0], v[0])          # a single key: O = V exactly
        print("config1 %s worst max-abs %.3e" % (pol, worst))
    finally:
        r.close()


# ------------------------------------------------------------------ configuration 2: bf16 stack, B=2 cut
def test_config2_bf16_stack_b2_all_units():
    w = inp.config2(batch=2)
    r = Runner(w.sides, w.sides, w.batch, w.heads, w.head_dim, "bf16", w.policies)
    try:
        for layer in range(w.layers):
            q, k, v = inp.correlated_qkv(w.sides, w.batch, w.heads, w.head_dim, "bf16", inp.layer_seed(2, layer), 0.8)
            q, k, v = ([x.cuda() for x in t] for t in (q, k, v))
            outs, worst = r.run_layer(layer, q, k, v, check_cache=layer in (0, 5, 15))
            assert torch.equal(outs[0], v[0])
    finally:
        r.close()


# ------------------------------------------------------------------ shapes, tails, policies
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("D", [64, 128])
def test_ragged_schedules_and_policies(dtype, D):
    sides_h = (1, 2, 3, 5, 7, 8, 11, 12, 13, 9)       # 121 (one wave short), 144 and 169 (wide path), shrinking last
    sides_w = (1, 3, 3, 4, 7, 8, 11, 12, 13, 9)
    pols = [(2, 2, False), (0, 0, False), (1, 3, False), (3, 0, False), (0, 0, True), (0, 1, False)]
    B, H = 2, 3
    r = Runner(sides_h, sides_w, B, H, D, dtype, pols)
    try:
        for layer in range(len(pols)):
            q, k, v = _qkv(sides_h, sides_w, B, H, D, dtype, 100 + layer)
            r.run_layer(layer, q, k, v)
    finally:
        r.close()


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_planned_layout_matches_oracle(dtype):
    sides = inp.VAR_SIDES
    pols = [(2, 2, False), (1, 1, False), (0, 0, True), (3, 3, False)]
    r = Runner(sides, sides, 2, 2, 64, dtype, pols, layout=amskv.AMSKV_LAYOUT_PLANNED)
    try:
        for layer in range(len(pols)):
            q, k, v = _qkv(sides, sides, 2, 2, 64, dtype, 200 + layer)
            r.run_layer(layer, q, k, v)
    finally:
        r.close()


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("layout", [amskv.AMSKV_LAYOUT_COMPACT, amskv.AMSKV_LAYOUT_PLANNED], ids=["compact", "planned"])
def test_borrowed_unretained_scales(dtype, layout):
    """Scales that no later step reads are used in place from the caller's K/V and never copied."""
    sides = inp.VAR_SIDES
    pols = [(2, 2, False), (0, 0, False), (2, 0, False), (0, 0, True), (1, 3, False)]
    r = Runner(sides, sides, 2, 3, 64, dtype, pols, layout=layout, borrow=True)
    try:
        for layer in range(len(pols)):
            q, k, v = _qkv(sides, sides, 2, 3, 64, dtype, 700 + layer)
            r.run_layer(layer, q, k, v)
    finally:
        r.close()


@pytest.mark.parametrize("dtype,D", [("bf16", 64), ("f32", 64), ("bf16", 128)])
@pytest.mark.parametrize("layout", [amskv.AMSKV_LAYOUT_COMPACT, amskv.AMSKV_LAYOUT_PLANNED], ids=["compact", "planned"])
@pytest.mark.parametrize("borrow", [False, True], ids=["copyall", "borrow"])
def test_fused_append(dtype, D, layout, borrow):
    """fuse_append: the attend call of a step fills the scale's slot; the cache must end up bit-identical."""
    sides_h = (1, 2, 3, 5, 7, 8, 11, 13, 16, 9)
    sides_w = (1, 3, 3, 4, 7, 8, 11, 13, 16, 9)
    pols = [(2, 2, False), (0, 0, False), (2, 0, False), (0, 0, True), (1, 3, False)]
    r = Runner(sides_h, sides_w, 2, 3, D, dtype, pols, layout=layout, borrow=borrow, fuse=True)
    try:
        for layer in range(len(pols)):
            q, k, v = _qkv(sides_h, sides_w, 2, 3, D, dtype, 800 + layer)
            r.run_layer(layer, q, k, v)
    finally:
        r.close()


def test_fused_append_without_attend_is_flushed_by_the_next_append():
    sides = (1, 2, 4, 6, 8, 12)
    tokens = [s * s for s in sides]
    pol = [(1, 2, False)]
    B, H, D = 2, 2, 64
    r = Runner(sides, sides, B, H, D, "bf16", pol, fuse=True)
    try:
        q, k, v = _qkv(sides, sides, B, H, D, "bf16", 900)
        for s in range(len(sides)):
            amskv.amskv_append_scale(r.h, 0, s, k[s], v[s])
            if s % 2 == 0 or s == len(sides) - 1:   # other steps never attend: the next append must copy them
                o = torch.empty_like(q[s])
                amskv.amskv_attend(r.h, 0, s, q[s], o)
            r.check_cache(0, s, k, v)            # export reads pending scales in place
        # after the last append+attend every resident scale must be in the arena itself: clobber the sources
        for s in range(len(sides)):
            k[s].fill_(float("nan"))
            v[s].fill_(float("nan"))
        torch.cuda.synchronize()
        q2, k2, v2 = _qkv(sides, sides, B, H, D, "bf16", 900)
        kept = orc.kept_scales(pol[0], len(sides) - 1)
        tk = sum(tokens[j] for j in kept)
        ko = torch.empty(B, H, tk, D, dtype=torch.bfloat16, device="cuda")
        vo = torch.empty_like(ko)
        amskv.amskv_cache_export(r.h, 0, ko, vo)
        torch.cuda.synchronize()
        assert np.array_equal(_bits(ko), orc.cache_contents([_bits(x) for x in k2], pol[0], len(sides) - 1))
        assert np.array_equal(_bits(vo), orc.cache_contents([_bits(x) for x in v2], pol[0], len(sides) - 1))
    finally:
        r.close()


def test_sixteen_scales_single_scale_and_scale_override():
    sides = tuple(range(1, 17))
    r = Runner(sides, sides, 1, 2, 64, "bf16", [(2, 1, False)], softmax_scale=0.05)
    try:
        q, k, v = _qkv(sides, sides, 1, 2, 64, "bf16", 300)
        r.run_layer(0, q, k, v)
    finally:
        r.close()
    r = Runner((7,), (9,), 3, 1, 128, "f32", [(2, 2, False)], softmax_scale=0.2)
    try:
        q, k, v = _qkv((7,), (9,), 3, 1, 128, "f32", 301)
        r.run_layer(0, q, k, v)
    finally:
        r.close()


def test_reset_reuse_and_side_stream():
    sides = (1, 2, 4, 6, 8)
    r = Runner(sides, sides, 2, 2, 64, "bf16", [(1, 1, False)])
    try:
        st = torch.cuda.Stream()
        for rep in range(2):
            q, k, v = _qkv(sides, sides, 2, 2, 64, "bf16", 400 + rep)
            torch.cuda.synchronize()
            with torch.cuda.stream(st):
                r.run_layer(0, q, k, v)
            st.synchronize()
            amskv.amskv_cache_reset(r.h)
    finally:
        r.close()


def test_large_values_do_not_overflow_softmax():
    sides = (2, 4, 8)
    r = Runner(sides, sides, 1, 2, 64, "bf16", [(0, 0, True)])
    try:
        q, k, v = _qkv(sides, sides, 1, 2, 64, "bf16", 500)
        q = [x * 6 for x in q]          # scores of order +-50: exp must stay finite through the max shift
        k = [x * 6 for x in k]
        r.run_layer(0, q, k, v)
    finally:
        r.close()


@pytest.mark.parametrize("gain", [0.25, 3.0], ids=["jump23bits", "jump270bits"])
@pytest.mark.parametrize("D", [64, 128])
def test_late_dominant_keys_force_the_rescale_path(D, gain):
    """Scores that jump far above the running reference late in the key sequence: one key per scale is aligned with
    every query and scaled up, more so at each later scale, so the lazily updated reference of the online softmax
    has to move (and the accumulators be rescaled) in the last blocks of every kernel variant -- coarse, mid, wide."""
    sides = (1, 2, 3, 4, 5, 6, 8, 10, 13, 16)
    B, H = 1, 3
    q, k, v = inp.iid_qkv(sides, B, H, D, "bf16", inp.layer_seed(6, 70 + D))
    q = [x.abs() for x in q]                                  # every query in the positive orthant ...
    for s, x in enumerate(k):
        x[..., -1, :] = gain * (s + 1)                        # ... so the last key of scale s scores ~ gain*(s+1)*0.8*D above the rest:
                                                              # with gain 3 a reference that failed to move would overflow fp32
    q, k, v = ([x.cuda() for x in t] for t in (q, k, v))
    for pol in [(0, 0, True), (2, 2, False)]:
        r = Runner(sides, sides, B, H, D, "bf16", [pol], layout=amskv.AMSKV_LAYOUT_PLANNED, borrow=True, fuse=True)
        try:
            outs, worst = r.run_layer(0, q, k, v)               # every step against the oracle, cache contents too
            print("late dominant keys, D=%d, gain %g, policy %s: worst max-abs %.3e" % (D, gain, pol, worst))
        finally:
            r.close()


# ------------------------------------------------------------------ Infinity-shaped (D=128, multi-tile queries)
def test_config4_infinity_shape_small_batch():
    w = inp.config4(batch=1)
    H = 2
    pols = [(3, 1, False), (0, 0, True)]
    r = Runner(w.sides, w.sides, 1, H, w.head_dim, "bf16", pols)
    try:
        for layer in range(2):
            q, k, v = _qkv(w.sides, w.sides, 1, H, w.head_dim, "bf16", inp.layer_seed(4, layer))
            r.run_layer(layer, q, k, v, check_cache=(layer == 0))
    finally:
        r.close()


# ------------------------------------------------------------------ similarity
@pytest.mark.parametrize("borrow", [False, True], ids=["copied", "borrowed"])
@pytest.mark.parametrize("dtype,D", [("bf16", 64), ("f32", 64), ("bf16", 128), ("f32", 128)])
def test_interscale_similarity(dtype, D, borrow):
    sides_h = (1, 2, 3, 5, 6, 8, 13, 16)
    sides_w = (1, 2, 4, 5, 6, 9, 13, 16)
    B, H = 3, 5
    pols = [(0, 0, True), (2, 1, False)]
    r = Runner(sides_h, sides_w, B, H, D, dtype, pols, borrow=borrow)
    tokens = r.tokens
    try:
        for layer, rho in enumerate((0.9, 0.4)):
            # correlated across scales so that the cosine is far from zero
            q, k, v = _qkv(sides_h, sides_w, B, H, D, dtype, 600 + layer)
            for s in range(1, len(tokens)):
                up = torch.from_numpy(orc.bilinear_upsample(_f64(k[s - 1]), sides_h[s - 1], sides_w[s - 1], sides_h[s], sides_w[s]))
                k[s] = (rho * up + math.sqrt(1 - rho * rho) * k[s].cpu().double()).to(k[s].dtype).cuda()
            for s in range(len(tokens)):
                amskv.amskv_append_scale(r.h, layer, s, k[s], v[s])
                if s == 0:
                    continue
                ck, cv, sums = amskv.amskv_interscale_similarity(r.h, layer, s, H)
                wk, wsum = orc.interscale_similarity(_f64(k[s]), _f64(k[s - 1]), (sides_h[s], sides_w[s]), (sides_h[s - 1], sides_w[s - 1]))
                wv, _ = orc.interscale_similarity(_f64(v[s]), _f64(v[s - 1]), (sides_h[s], sides_w[s]), (sides_h[s - 1], sides_w[s - 1]))
                np.testing.assert_allclose(np.array(ck), wk, rtol=0, atol=1e-5)
                np.testing.assert_allclose(np.array(cv), wv, rtol=0, atol=1e-5)
                np.testing.assert_allclose(np.array(sums), wsum, rtol=2e-5, atol=1e-3)
                ck2, none_v, none_s = amskv.amskv_interscale_similarity(r.h, layer, s, H, want_v=False, want_sums=False)
                assert ck2 == ck and none_v is None and none_s is None       # deterministic
                l2 = orc.neg_l2_from_sums(np.array(sums))
                np.testing.assert_allclose(l2, orc.neg_l2_from_sums(wsum), rtol=1e-3)
        # an evicted neighbour is an error, not garbage: layer 1 (window 1) at the last step holds s-1 only
        with pytest.raises(amskv.AmskvError) as e:
            amskv.amskv_interscale_similarity(r.h, 1, len(tokens) - 2, H)
        assert e.value.status == amskv.AMSKV_ERR_EVICTED
    finally:
        r.close()


# ------------------------------------------------------------------ full-size launches, sampled units
def _full_size_layers(w, layers, n_units, gen, policies_of, **flags):
    r = Runner(w.sides, w.sides, w.batch, w.heads, w.head_dim, w.dtype, policies_of, **flags)
    try:
        for li, layer in enumerate(layers):
            q, k, v = gen(layer)
            units = sorted({(b, h) for (_, b, h) in inp.sample_units(1, w.batch, w.heads, n_units, 77 + layer)})
            outs, worst = r.run_layer(li, q, k, v, check_cache=False, units=units)
            # bit-exact cache contents on the sampled units at the last step
            lay = amskv.amskv_cache_layout(r.h, li)
            tk = sum(x[2] for x in lay)
            ko = torch.empty(w.batch, w.heads, tk, w.head_dim, dtype=k[0].dtype, device="cuda")
            vo = torch.empty_like(ko)
            amskv.amskv_cache_export(r.h, li, ko, vo)
            torch.cuda.synchronize()
            s = len(w.sides) - 1
            for b, h in units:
                wk = orc.cache_contents([_bits(x[b:b + 1, h:h + 1]) for x in k], policies_of[li], s)
                wv = orc.cache_contents([_bits(x[b:b + 1, h:h + 1]) for x in v], policies_of[li], s)
                assert np.array_equal(_bits(ko[b:b + 1, h:h + 1]), wk) and np.array_equal(_bits(vo[b:b + 1, h:h + 1]), wv)
            print("layer %d policy %s worst max-abs %.3e over %d units" % (layer, policies_of[li], worst, len(units)))
            del q, k, v, outs, ko, vo
    finally:
        r.close()
        torch.cuda.empty_cache()


def test_config3_full_batch_sampled_units():
    """VAR-d30 shape at batch 256 (the launch configuration the benchmark times): three layers,
    one per policy class, 24 sampled (b,h) each against the oracle."""
    w = inp.config3(batch=256)
    rhos = inp.layer_rhos(w.layers, inp.layer_seed(3, 999))
    layers = [0, 14, 29]
    pols = [(2, 2, False), (0, 0, True), (2, 1, False)]

    def gen(layer):
        return inp.correlated_qkv(w.sides, w.batch, w.heads, w.head_dim, "bf16", inp.layer_seed(3, layer), rhos[layer], device="cuda")

    _full_size_layers(w, layers, 24, gen, pols)


def test_config3_full_batch_bench_flags_sampled_units():
    """The same launches with the flags the benchmark runs with (borrowed final scale, fused append)."""
    w = inp.config3(batch=256)
    rhos = inp.layer_rhos(w.layers, inp.layer_seed(3, 999))
    layers = [1, 7]
    pols = [(2, 2, False), (0, 0, True)]

    def gen(layer):
        return inp.correlated_qkv(w.sides, w.batch, w.heads, w.head_dim, "bf16", inp.layer_seed(3, layer), rhos[layer], device="cuda")

    _full_size_layers(w, layers, 24, gen, pols, borrow=True, fuse=True)


def test_config5_policy_sweep_sampled_units():
    w = inp.config5(batch=64)
    layers = [0, 7, 13, 23]
    pols = [w.policies[l] for l in layers]

    def gen(layer):
        return inp.iid_qkv(w.sides, w.batch, w.heads, w.head_dim, "bf16", inp.layer_seed(5, layer), device="cuda")

    _full_size_layers(w, layers, 16, gen, pols)


# ------------------------------------------------------------------ run-to-run reproducibility
@pytest.mark.parametrize("D", [64, 128])
def test_attend_bf16_is_bit_reproducible(D):
    """Same inputs, same bits, launch after launch, for every kernel variant of the schedule (coarse, mid and
    wide scales).  A read of a matrix-instruction result before the instruction has finished writing it shows
    up here as last-bit differences between runs long before it exceeds the parity tolerance."""
    sides = (1, 2, 3, 4, 5, 6, 8, 10, 13, 16)
    B, H = 2, 5
    q, k, v = inp.iid_qkv(sides, B, H, D, "bf16", inp.layer_seed(6, D))
    q, k, v = ([x.cuda() for x in t] for t in (q, k, v))
    runs = []
    for rep in range(3):
        r = Runner(sides, sides, B, H, D, "bf16", [(0, 0, True)], layout=amskv.AMSKV_LAYOUT_PLANNED, borrow=True, fuse=True)
        try:
            outs = []
            for s in range(len(sides)):
                amskv.amskv_append_scale(r.h, 0, s, k[s], v[s])
                o = torch.full_like(q[s], float("nan"))
                amskv.amskv_attend(r.h, 0, s, q[s], o)
                outs.append(o)
            torch.cuda.synchronize()
            runs.append([_bits(o) for o in outs])
        finally:
            r.close()
    for s in range(len(sides)):
        assert np.array_equal(runs[0][s], runs[1][s]) and np.array_equal(runs[0][s], runs[2][s]), "scale %d" % s


# ------------------------------------------------------------------ similarity without the per-call wait
def test_similarity_enqueue_collect_matches_the_waiting_call():
    sides = (2, 3, 5, 8, 6)
    B, H, D, L = 2, 3, 64, 4
    pols = [(1, 2, False), (0, 0, True), (2, 1, False), (0, 1, False)]
    r = Runner(sides, sides, B, H, D, "bf16", pols, layout=amskv.AMSKV_LAYOUT_PLANNED, borrow=True, fuse=True)
    try:
        data = [inp.correlated_qkv(sides, B, H, D, "bf16", inp.layer_seed(6, 50 + l), 0.3 + 0.2 * l) for l in range(L)]
        dev = [[[x.cuda() for x in t] for t in d] for d in data]
        nan = lambda rows: all(all(math.isnan(x) for x in row) for row in rows)
        ck, cv, sm = amskv.amskv_interscale_similarity_collect(r.h, L, H)
        assert nan(ck) and nan(cv)                                    # nothing enqueued yet
        want = {}
        for s in range(len(sides)):
            for l in range(L):
                amskv.amskv_append_scale(r.h, l, s, dev[l][1][s], dev[l][2][s])
            if s == 3:
                for l in range(L):
                    want[l] = amskv.amskv_interscale_similarity(r.h, l, s, H)          # waits every time
                for l in range(L):
                    amskv.amskv_interscale_similarity_enqueue(r.h, l, s, want_v=(l != 2))
                ck, cv, sm = amskv.amskv_interscale_similarity_collect(r.h, L, H)       # one wait for all
                for l in range(L):
                    assert ck[l] == want[l][0] and sm[l] == want[l][2]
                    if l != 2:
                        assert cv[l] == want[l][1]
                    else:
                        assert all(math.isnan(x) for x in cv[l])                        # enqueued without the values
                    wk, _ = orc.interscale_similarity(_f64(data[l][1][s]), _f64(data[l][1][s - 1]), (sides[s],) * 2, (sides[s - 1],) * 2)
                    assert np.abs(np.array(ck[l]) - wk).max() < 1e-5
            for l in range(L):
                o = torch.empty_like(dev[l][0][s])
                amskv.amskv_attend(r.h, l, s, dev[l][0][s], o)
        with pytest.raises(amskv.AmskvError) as e:                     # policy (0,1): scale 2 is gone at step 4
            amskv.amskv_interscale_similarity_enqueue(r.h, 3, 3)
        assert e.value.status == amskv.AMSKV_ERR_EVICTED
        amskv.amskv_cache_reset(r.h)
        ck, _, _ = amskv.amskv_interscale_similarity_collect(r.h, L, H)
        assert nan(ck)
    finally:
        r.close()


@pytest.mark.parametrize("flags", [dict(), dict(fuse=True), dict(layout=amskv.AMSKV_LAYOUT_PLANNED, borrow=True, fuse=True)],
                         ids=["copy", "fuse", "planned_borrow_fuse"])
@pytest.mark.parametrize("dtype,D", [("bf16", 64), ("bf16", 128), ("f32", 64)])
def test_several_attend_calls_within_one_step(dtype, D, flags):
    """A step may be attended more than once (two sets of queries against the same keys): with fuse_append the first
    call fills the slot and the later ones read it from the cache; every call must match the oracle, the same queries
    must give the same bits, and the cache must end up as after a single call."""
    sides = (1, 2, 4, 7, 10, 13)
    pols = [(1, 2, False), (0, 0, True)]
    B, H = 2, 3
    r = Runner(sides, sides, B, H, D, dtype, pols, **flags)
    try:
        for layer, pol in enumerate(pols):
            q, k, v = _qkv(sides, sides, B, H, D, dtype, 1500 + layer)
            q2, _, _ = _qkv(sides, sides, B, H, D, dtype, 1600 + layer)
            want = orc.attend_all_steps([_f64(x) for x in q], [_f64(x) for x in k], [_f64(x) for x in v], r.tokens, pol, None)
            want2 = orc.attend_all_steps([_f64(x) for x in q2], [_f64(x) for x in k], [_f64(x) for x in v], r.tokens, pol, None)
            for s in range(len(sides)):
                amskv.amskv_append_scale(r.h, layer, s, k[s], v[s])
                o = [torch.full_like(q[s], float("nan")) for _ in range(3)]
                amskv.amskv_attend(r.h, layer, s, q[s], o[0])
                amskv.amskv_attend(r.h, layer, s, q2[s], o[1])
                amskv.amskv_attend(r.h, layer, s, q[s], o[2])
                torch.cuda.synchronize()
                assert np.abs(_f64(o[0]) - want[s]).max() <= TOL[dtype]
                assert np.abs(_f64(o[1]) - want2[s]).max() <= TOL[dtype]
                assert np.array_equal(_bits(o[0]), _bits(o[2])), (layer, s)
                r.check_cache(layer, s, k, v)
    finally:
        r.close()
