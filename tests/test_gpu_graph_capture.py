"""A whole image's worth of steps (append + attend for every scale and layer, scale-window mode, plus the
enqueued inter-scale similarity) captured into a HIP graph through the C ABI and replayed: these calls enqueue
kernels only, so a serving loop can record them once and replay the device work, with new inputs written into
the same buffers.  Every replay is checked against the eager calls on the same inputs (bit for bit) and one of
them against the oracle, with eager work and synchronisations between the replays.

Bar: bit-exact between replay and eager run; max-abs 2e-2 (bf16) against the oracle.
"""
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


@pytest.mark.parametrize("flags", [dict(), dict(layout=amskv.AMSKV_LAYOUT_PLANNED, borrow_unretained=True, fuse_append=True)],
                         ids=["compact_copy", "planned_borrow_fuse"])
def test_captured_steps_replay_like_the_eager_calls(flags):
    B, H, D = 2, 3, 64
    tokens = [x * x for x in VAR]
    S = len(VAR)
    pols = [(2, 2, False), (0, 0, True), (1, 1, False)]
    L = len(pols)
    kw = dict(flags)
    layout = kw.pop("layout", amskv.AMSKV_LAYOUT_COMPACT)
    need = amskv.amskv_cache_required_bytes(L, H, D, VAR, VAR, B, BF16, pols, 0.0, layout, **kw)

    def new_cache():
        arena = torch.empty(need, dtype=torch.uint8, device="cuda")
        arena.fill_(0xFF)
        return arena, amskv.amskv_cache_create(L, H, D, VAR, VAR, B, BF16, pols, 0.0, layout, arena=arena, **kw)

    def draw(seed):
        return [inp.correlated_qkv(VAR, B, H, D, "bf16", inp.layer_seed(11, 10 * seed + l), 0.7) for l in range(L)]

    # static buffers: what a replay reads and writes
    first = draw(0)
    Q = [[first[l][0][s].cuda() for s in range(S)] for l in range(L)]
    K = [[first[l][1][s].cuda() for s in range(S)] for l in range(L)]
    V = [[first[l][2][s].cuda() for s in range(S)] for l in range(L)]
    O = [[torch.full_like(Q[l][s], float("nan")) for s in range(S)] for l in range(L)]
    sums = torch.full((L, H * 4), float("nan"), dtype=torch.float32, device="cuda")
    O_eager = [[torch.empty_like(Q[l][s]) for s in range(S)] for l in range(L)]
    sums_eager = torch.empty_like(sums)
    # attention density of layer 0 at a coarse step (stand-alone kernels inside the call) and at a later one (by-product)
    mass = torch.full((S, H * amskv.AMSKV_MAX_SCALES), float("nan"), dtype=torch.float32, device="cuda")
    mass_eager = torch.empty_like(mass)

    def load(data):
        for l in range(L):
            for s in range(S):
                Q[l][s].copy_(data[l][0][s])
                K[l][s].copy_(data[l][1][s])
                V[l][s].copy_(data[l][2][s])

    def steps(cache, out, sm, ms, stream):
        amskv.amskv_cache_reset(cache)
        for s in range(S):
            for l in range(L):
                amskv.amskv_append_scale(cache, l, s, K[l][s], V[l][s], stream)
                if l == 0 and s in (2, 7):
                    amskv.amskv_attend_density(cache, l, s, Q[l][s], out[l][s], ms[s], stream)
                else:
                    amskv.amskv_attend(cache, l, s, Q[l][s], out[l][s], stream)
                if s == 5:   # Eq. 3 between scales 5 and 4, partial sums in the library's static array, result in sm
                    amskv.amskv_interscale_similarity_enqueue_static(cache, l, s, False, sm[l], stream)

    arena_g, cache_g = new_cache()
    arena_e, cache_e = new_cache()
    side = torch.cuda.Stream()
    try:
        # warm the path once outside the capture (first-call work such as the static array's address lookup)
        with torch.cuda.stream(side):
            steps(cache_g, O, sums, mass, side.cuda_stream)
        side.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            steps(cache_g, O, sums, mass, torch.cuda.current_stream().cuda_stream)
        for rep in range(3):
            data = draw(rep + 1)
            load(data)
            for l in range(L):
                for s in range(S):
                    O[l][s].fill_(float("nan"))
            sums.fill_(float("nan"))
            mass.fill_(float("nan"))
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            # eager calls on a twin cache, same inputs (the program's own work between the replays)
            steps(cache_e, O_eager, sums_eager, mass_eager, None)
            torch.cuda.synchronize()
            for l in range(L):
                for s in range(S):
                    assert torch.equal(O[l][s].view(torch.int16), O_eager[l][s].view(torch.int16)), (rep, l, s)
            assert torch.equal(sums.view(torch.int32), sums_eager.view(torch.int32)), rep
            for s in (2, 7):
                assert torch.equal(mass[s].view(torch.int32), mass_eager[s].view(torch.int32)), (rep, s)
                n = len(orc.kept_scales(pols[0], s))
                assert abs(float(mass[s].view(H, -1)[0, :n].sum()) - tokens[s]) <= 1e-3 * tokens[s]
            if rep == 1:
                for l, pol in enumerate(pols):
                    want = orc.attend_all_steps([_f64(x) for x in data[l][0]], [_f64(x) for x in data[l][1]],
                                                [_f64(x) for x in data[l][2]], tokens, pol, None)
                    for s in range(S):
                        assert np.abs(_f64(O[l][s]) - want[s]).max() <= 2e-2
                    cos, _ = orc.interscale_similarity(_f64(data[l][1][5]), _f64(data[l][1][4]), (VAR[5], VAR[5]), (VAR[4], VAR[4]))
                    got = sums[l].cpu().numpy().reshape(H, 4)[:, 0] / (B * tokens[5])
                    assert np.abs(got - cos).max() <= 1e-5
            # the caches hold the same scales, bit for bit
            for l, pol in enumerate(pols):
                tk = sum(tokens[j] for j in orc.kept_scales(pol, S - 1))
                ex = [torch.empty(B, H, tk, D, dtype=torch.bfloat16, device="cuda") for _ in range(4)]
                amskv.amskv_cache_export(cache_g, l, ex[0], ex[1])
                amskv.amskv_cache_export(cache_e, l, ex[2], ex[3])
                torch.cuda.synchronize()
                assert torch.equal(ex[0], ex[2]) and torch.equal(ex[1], ex[3])
    finally:
        amskv.amskv_cache_destroy(cache_g)
        amskv.amskv_cache_destroy(cache_e)
