"""GPU parity at the full shapes of the benchmark configurations, on sampled (b, h) units the oracle can
compute one by one: the inter-scale similarity (Eq. 3) at batch 256 x 30 heads on the full batch, the
1024x1024 schedule (head dim 128) at batch 8 x 16 heads, and the 256x256 schedule at batch 128.

Bar as everywhere: bit-exact cache contents, max-abs 2e-2 on bf16 attention outputs, 1e-5 abs on the cosine."""
import numpy as np
import pytest
import torch

import amskv_inputs as inp
import paper_2511_16047_amd as amskv
from oracle import amskv_oracle as orc

pytestmark = pytest.mark.gpu

BF16 = amskv.AMSKV_DTYPE_BF16
TOL = 2e-2


def _f64(t):
    return t.detach().to("cpu", torch.float64).numpy()


def _bits(t):
    return t.contiguous().view(torch.int16).cpu().numpy()


# ------------------------------------------------------------------ Eq. 3 at the benchmark's launch size
def test_similarity_full_batch_decides_the_benchmark_policy():
    """Batch 256 x 30 heads x head dim 64 on the correlated generator of the VAR-d30 configuration: the probe
    scale (5) of six layers spread over the rho range and the last cached pair (8 -> 9) of one of them, through
    the waiting call and through enqueue/collect, against the oracle on the FULL batch; the set of layers the
    benchmark would flag (mean cosine < 0.5) must be the oracle's."""
    w = inp.config3(batch=256)
    B, H, D = w.batch, w.heads, w.head_dim
    probe = 5
    rhos = inp.layer_rhos(w.layers, inp.layer_seed(3, 999))
    layers = [0, 1, 7, 14, 22, 29]
    pols = [(0, 0, True)] * len(layers)
    need = amskv.amskv_cache_required_bytes(len(layers), H, D, w.sides, w.sides, B, BF16, pols)
    arena = torch.empty(need, dtype=torch.uint8, device="cuda")
    h = amskv.amskv_cache_create(len(layers), H, D, w.sides, w.sides, B, BF16, pols, arena=arena)
    side = lambda s: (w.sides[s], w.sides[s])
    try:
        got_wait, want = [], []
        for li, layer in enumerate(layers):
            _, k, v = inp.correlated_qkv(w.sides, B, H, D, "bf16", inp.layer_seed(3, layer), rhos[layer], device="cuda")
            last = len(w.sides) - 1 if li == 2 else probe
            for s in range(last + 1):
                amskv.amskv_append_scale(h, li, s, k[s], v[s])
                if s == probe:
                    ck, _, sums = amskv.amskv_interscale_similarity(h, li, s, H, want_v=False)
                    wk, wsum = orc.interscale_similarity(_f64(k[s]), _f64(k[s - 1]), side(s), side(s - 1))
                    np.testing.assert_allclose(np.array(ck), wk, rtol=0, atol=1e-5)
                    np.testing.assert_allclose(np.array(sums), wsum, rtol=2e-5, atol=1e-2)
                    got_wait.append(ck)
                    want.append(wk)
            if li == 2:
                # the last cached pair, largest reduction of the schedule: sampled heads, full batch
                s = last
                ck, cv, sums = amskv.amskv_interscale_similarity(h, li, s, H)
                for hd in (0, 11, 29):
                    wk, wsum = orc.interscale_similarity(_f64(k[s][:, hd:hd + 1]), _f64(k[s - 1][:, hd:hd + 1]), side(s), side(s - 1))
                    wv, _ = orc.interscale_similarity(_f64(v[s][:, hd:hd + 1]), _f64(v[s - 1][:, hd:hd + 1]), side(s), side(s - 1))
                    assert abs(ck[hd] - wk[0]) <= 1e-5 and abs(cv[hd] - wv[0]) <= 1e-5
                    np.testing.assert_allclose(np.array(sums[hd]), wsum[0], rtol=2e-5, atol=1e-2)
            del k, v
        # the same scores without a wait per layer: enqueue everything, collect once.  Layer 2 went on to scale 9,
        # so its enqueue is for that pair; the others repeat the probe scale.
        for li in range(len(layers)):
            amskv.amskv_interscale_similarity_enqueue(h, li, len(w.sides) - 1 if li == 2 else probe, want_v=False)
        ck_all, _, _ = amskv.amskv_interscale_similarity_collect(h, len(layers), H, want_v=False, want_sums=False)
        for li in range(len(layers)):
            if li != 2:
                assert ck_all[li] == got_wait[li]            # same kernels, same order: same bits
        flagged = [l for l, ck in zip(layers, got_wait) if sum(ck) / H < 0.5]
        assert flagged == [l for l, wk in zip(layers, want) if wk.mean() < 0.5]
        assert 0 < len(flagged) < len(layers)                 # the sample holds both kinds of layer
        torch.cuda.synchronize()
    finally:
        amskv.amskv_cache_destroy(h)
        del arena
        torch.cuda.empty_cache()


# ------------------------------------------------------------------ full-size launches, sampled units
def _run_sampled(w, pol, q, k, v, units, chunk, **flags):
    """One layer through every step; outputs of the sampled units against the oracle (`chunk` units at a time:
    the oracle materialises the whole T x T score matrix per unit), cache contents of those units bit for bit."""
    B, H, D = w.batch, w.heads, w.head_dim
    layout = flags.pop("layout", amskv.AMSKV_LAYOUT_COMPACT)
    need = amskv.amskv_cache_required_bytes(1, H, D, w.sides, w.sides, B, BF16, [pol], 0.0, layout, **flags)
    arena = torch.empty(need, dtype=torch.uint8, device="cuda")
    arena.fill_(0xFF)
    h = amskv.amskv_cache_create(1, H, D, w.sides, w.sides, B, BF16, [pol], 0.0, layout, arena=arena, **flags)
    S = len(w.sides)
    try:
        outs = []
        for s in range(S):
            amskv.amskv_append_scale(h, 0, s, k[s], v[s])
            o = torch.full_like(q[s], float("nan"))
            amskv.amskv_attend(h, 0, s, q[s], o)
            outs.append(o)
            lay = amskv.amskv_cache_layout(h, 0)
            assert [x[0] for x in lay] == orc.kept_scales(pol, s)
        torch.cuda.synchronize()
        worst = 0.0
        for i in range(0, len(units), chunk):
            part = units[i:i + chunk]
            sel = lambda t: torch.stack([t[b, hh] for b, hh in part])[None]
            want = orc.attend_all_steps([_f64(sel(x)) for x in q], [_f64(sel(x)) for x in k], [_f64(sel(x)) for x in v],
                                        w.tokens, pol)
            for s in range(S):
                got = _f64(sel(outs[s]))
                assert np.isfinite(got).all()
                err = float(np.abs(got - want[s]).max())
                worst = max(worst, err)
                assert err <= TOL, "step %d units %s max-abs %.3e" % (s, part, err)
        tk = sum(x[2] for x in amskv.amskv_cache_layout(h, 0))
        ko = torch.empty(B, H, tk, D, dtype=torch.bfloat16, device="cuda")
        vo = torch.empty_like(ko)
        amskv.amskv_cache_export(h, 0, ko, vo)
        torch.cuda.synchronize()
        for b, hh in units:
            wk = orc.cache_contents([_bits(x[b:b + 1, hh:hh + 1]) for x in k], pol, S - 1)
            wv = orc.cache_contents([_bits(x[b:b + 1, hh:hh + 1]) for x in v], pol, S - 1)
            assert np.array_equal(_bits(ko[b:b + 1, hh:hh + 1]), wk) and np.array_equal(_bits(vo[b:b + 1, hh:hh + 1]), wv)
        assert amskv.amskv_cache_bytes_held(h, 0) == orc.bytes_held(w.tokens, pol, S - 1, B, H, D, 2)
        return worst
    finally:
        amskv.amskv_cache_destroy(h)
        del arena


BENCH_FLAGS = dict(layout=amskv.AMSKV_LAYOUT_PLANNED, borrow_unretained=True, fuse_append=True)


@pytest.mark.parametrize("flags", [dict(), BENCH_FLAGS], ids=["compact", "bench_flags"])
@pytest.mark.parametrize("pol", [(3, 1, False), (0, 0, True)], ids=["c3w1", "vanilla"])
def test_config4_full_shape_sampled_units(pol, flags):
    """1024x1024 schedule (13 scales, 10521 tokens), 16 heads x head dim 128, batch 8: the grids the benchmark's
    Infinity-shaped workload launches (several query blocks per (b,h), 128 units), 16 sampled units."""
    w = inp.config4()
    assert (w.batch, w.heads, w.head_dim) == (8, 16, 128)
    q, k, v = inp.iid_qkv(w.sides, w.batch, w.heads, w.head_dim, "bf16", inp.layer_seed(4, 3), device="cuda")
    units = sorted({(b, hh) for (_, b, hh) in inp.sample_units(1, w.batch, w.heads, 16, 404)})
    assert len(units) >= 16
    worst = _run_sampled(w, pol, q, k, v, units, 2, **dict(flags))
    print("config 4 full shape, policy %s, %s: worst max-abs %.3e over %d units" % (pol, "bench flags" if flags else "compact", worst, len(units)))
    del q, k, v
    torch.cuda.empty_cache()


def test_config3_batch128_sampled_units():
    """VAR-d30 shape at batch 128 (the other batch size the configuration names): one layer per policy class."""
    w = inp.config3(batch=128)
    rhos = inp.layer_rhos(w.layers, inp.layer_seed(3, 999))
    for layer, pol, flags in [(0, (2, 2, False), BENCH_FLAGS), (14, (0, 0, True), BENCH_FLAGS), (29, (2, 1, False), dict())]:
        q, k, v = inp.correlated_qkv(w.sides, w.batch, w.heads, w.head_dim, "bf16", inp.layer_seed(3, layer), rhos[layer], device="cuda")
        units = sorted({(b, hh) for (_, b, hh) in inp.sample_units(1, w.batch, w.heads, 16, 128 + layer)})
        worst = _run_sampled(w, pol, q, k, v, units, 16, **dict(flags))
        print("config 3 batch 128, layer %d policy %s: worst max-abs %.3e over %d units" % (layer, pol, worst, len(units)))
        del q, k, v
        torch.cuda.empty_cache()
