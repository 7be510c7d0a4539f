"""The entry point that allocates nothing (for callers that cannot call hipMalloc): the similarity kernels with
their partial sums in the library's static device array, against the arena-workspace entry point."""
import numpy as np
import pytest
import torch

import amskv_inputs as inp
import paper_2511_16047_amd as amskv

pytestmark = pytest.mark.gpu

BF16 = amskv.AMSKV_DTYPE_BF16


def _cache(sides, B, H, D, pol):
    need = amskv.amskv_cache_required_bytes(1, H, D, sides, sides, B, BF16, [pol])
    arena = torch.empty(need, dtype=torch.uint8, device="cuda")
    return amskv.amskv_cache_create(1, H, D, sides, sides, B, BF16, [pol], arena=arena), arena


def _compare(h, s, B, H, T, want_v):
    """Static-workspace call against the waiting call of the existing entry point, same cache, same scale."""
    ck, cv, sums = amskv.amskv_interscale_similarity(h, 0, s, H, want_v=want_v)
    out = torch.full(((2 if want_v else 1) * H * 4,), float("nan"), dtype=torch.float32, device="cuda")
    amskv.amskv_interscale_similarity_enqueue_static(h, 0, s, want_v, out)
    torch.cuda.synchronize()
    got = out.cpu().numpy().reshape(-1, H, 4)
    n_tok = float(B * T)
    # same kernels, same reduction order: the bar is the similarity's (1e-5 on the cosine), the bits are equal
    cos_k = (got[0, :, 0].astype(np.float64) / n_tok).astype(np.float32)
    assert np.abs(cos_k - np.array(ck, dtype=np.float32)).max() <= 1e-5
    assert np.array_equal(cos_k, np.array(ck, dtype=np.float32))
    assert np.array_equal(got[0, :, 1:], np.array(sums, dtype=np.float32))
    if want_v:
        cos_v = (got[1, :, 0].astype(np.float64) / n_tok).astype(np.float32)
        assert np.array_equal(cos_v, np.array(cv, dtype=np.float32))
    assert np.isfinite(got).all()


def test_static_workspace_matches_arena_workspace_twice_second_smaller():
    sides = (2, 3, 5, 8, 13)
    D = 64
    big = dict(B=6, H=7)
    small = dict(B=2, H=3)
    caches = []
    try:
        for cfg, rho, seed in ((big, 0.7, 1), (small, 0.3, 2)):       # two calls in a row, the second on a smaller input
            B, H = cfg["B"], cfg["H"]
            h, arena = _cache(sides, B, H, D, (0, 0, True))
            caches.append((h, arena))
            _, k, v = inp.correlated_qkv(sides, B, H, D, "bf16", inp.layer_seed(10, seed), rho, device="cuda")
            for s in range(len(sides)):
                amskv.amskv_append_scale(h, 0, s, k[s], v[s])
            _compare(h, len(sides) - 1, B, H, sides[-1] ** 2, want_v=True)
            _compare(h, 2, B, H, sides[2] ** 2, want_v=False)           # and a smaller scale of the same cache
    finally:
        for h, _ in caches:
            amskv.amskv_cache_destroy(h)


def test_static_workspace_limit_and_argument_checks():
    sides = (1, 2)
    B, H, D = 1, 2, 64
    h, arena = _cache(sides, B, H, D, (0, 0, True))
    try:
        x = torch.zeros(B, H, 4, D, dtype=torch.bfloat16, device="cuda")
        amskv.amskv_append_scale(h, 0, 0, x[:, :, :1].contiguous(), x[:, :, :1].contiguous())
        amskv.amskv_append_scale(h, 0, 1, x, x)
        out = torch.zeros(2 * H * 4, dtype=torch.float32, device="cuda")
        with pytest.raises(amskv.AmskvError) as e:
            amskv.amskv_interscale_similarity_enqueue_static(h, 0, 1, True, None)
        assert e.value.status == amskv.AMSKV_ERR_INVALID_ARG
        with pytest.raises(amskv.AmskvError) as e:
            amskv.amskv_interscale_similarity_enqueue_static(h, 0, 1, True, out.data_ptr() + 4)     # not 16-byte aligned
        assert e.value.status == amskv.AMSKV_ERR_INVALID_ARG
        with pytest.raises(amskv.AmskvError) as e:
            amskv.amskv_interscale_similarity_enqueue_static(h, 0, 0, True, out)                     # s >= 1
        assert e.value.status == amskv.AMSKV_ERR_INVALID_ARG
    finally:
        amskv.amskv_cache_destroy(h)
    # batch * heads beyond the static array: refused before anything is launched (a plan-only cache is enough to
    # ask, but the residency checks come first, so give it an arena-less schedule that reaches the size test)
    Bx, Hx = 129, 128                                                # 16512 > AMSKV_STATIC_MAX_UNITS
    assert Bx * Hx > amskv.AMSKV_STATIC_MAX_UNITS
    need = amskv.amskv_cache_required_bytes(1, Hx, D, sides, sides, Bx, BF16, [(0, 0, True)])
    arena = torch.empty(need, dtype=torch.uint8, device="cuda")
    h = amskv.amskv_cache_create(1, Hx, D, sides, sides, Bx, BF16, [(0, 0, True)], arena=arena)
    try:
        k0 = torch.zeros(Bx, Hx, 1, D, dtype=torch.bfloat16, device="cuda")
        k1 = torch.zeros(Bx, Hx, 4, D, dtype=torch.bfloat16, device="cuda")
        amskv.amskv_append_scale(h, 0, 0, k0, k0)
        amskv.amskv_append_scale(h, 0, 1, k1, k1)
        out = torch.zeros(2 * Hx * 4, dtype=torch.float32, device="cuda")
        with pytest.raises(amskv.AmskvError) as e:
            amskv.amskv_interscale_similarity_enqueue_static(h, 0, 1, True, out)
        assert e.value.status == amskv.AMSKV_ERR_STATIC_LIMIT
        amskv.amskv_interscale_similarity(h, 0, 1, Hx)                # the arena-workspace entry point takes it
    finally:
        amskv.amskv_cache_destroy(h)
