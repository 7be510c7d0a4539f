"""Token-major caller tensors (a fused QKV projection output [B][T][3][H][D] read in place, O written
as [B][T][H*D]) against the oracle, and bit for bit against the head-major path on the same values."""
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


def _f64(t):
    return t.detach().to("cpu", torch.float64).numpy()


def _bits(t):
    it = torch.int16 if t.dtype == torch.bfloat16 else torch.int32
    return t.contiguous().view(it).cpu().numpy()


def _pack(q, k, v, pad):
    """[B][H][T][D] x3 -> one [B][T][3*H*D + pad] tensor (the last `pad` elements of a token are filler)."""
    B, H, T, D = q.shape
    x = torch.full((B, T, 3 * H * D + pad), float("nan"), dtype=q.dtype)
    for i, t in enumerate((q, k, v)):
        x[:, :, i * H * D:(i + 1) * H * D] = t.permute(0, 2, 1, 3).reshape(B, T, H * D)
    return x.cuda()


def _run(sides, B, H, D, dtype, token_major, pad=0, policies=None, budgets=None, **flags):
    tokens = [s * s for s in sides]
    q, k, v = inp.correlated_qkv(sides, B, H, D, dtype, inp.layer_seed(9, D), 0.7)
    n_layers = len(budgets) if budgets is not None else len(policies)
    layout = flags.pop("layout", amskv.AMSKV_LAYOUT_COMPACT)
    need = amskv.amskv_cache_required_bytes(n_layers, H, D, sides, sides, B, DT[dtype], policies, 0.0, layout, budgets=budgets, **flags)
    arena = torch.empty(need, dtype=torch.uint8, device="cuda")
    arena.fill_(0xFF)
    h = amskv.amskv_cache_create(n_layers, H, D, sides, sides, B, DT[dtype], policies, 0.0, layout, arena=arena,
                                 budgets=budgets, **flags)
    tok = 3 * H * D + pad
    if token_major:
        amskv.amskv_cache_set_io_layout(h, amskv.AMSKV_IO_TOKEN_MAJOR, tok, tok, H * D)
    outs, exports, sims, dens = [], [], [], []
    keep = []
    eb = 2 if dtype == "bf16" else 4
    try:
        for s in range(len(sides)):
            if token_major:
                x = _pack(q[s], k[s], v[s], pad)
                keep.append(x)
                qp, kp, vp = x.data_ptr(), x.data_ptr() + H * D * eb, x.data_ptr() + 2 * H * D * eb
                o = torch.full((B, tokens[s], H * D), float("nan"), dtype=q[s].dtype, device="cuda")
            else:
                qd, kd, vd = q[s].cuda(), k[s].cuda(), v[s].cuda()
                keep += [qd, kd, vd]
                qp, kp, vp = qd.data_ptr(), kd.data_ptr(), vd.data_ptr()
                o = torch.full((B, H, tokens[s], D), float("nan"), dtype=q[s].dtype, device="cuda")
            for l in range(n_layers):
                amskv.amskv_append_scale(h, l, s, kp, vp)
                if dtype == "bf16" and l == 0 and s in (3, len(sides) - 1):
                    dens.append(amskv.amskv_attention_density(h, l, s, qp, H)[1])
                amskv.amskv_attend(h, l, s, qp, o.data_ptr())
                torch.cuda.synchronize()
                outs.append(o.view(B, tokens[s], H, D).permute(0, 2, 1, 3).contiguous().cpu() if token_major else o.cpu())
                if budgets is None and s >= 1 and l == 0:
                    try:
                        sims.append(amskv.amskv_interscale_similarity(h, l, s, H))
                    except amskv.AmskvError as e:
                        assert e.status == amskv.AMSKV_ERR_EVICTED
                        sims.append(None)
                n_tok = sum(x[3] for x in amskv.amskv_cache_segments(h, l))
                ko = torch.empty(B, H, n_tok, D, dtype=q[s].dtype, device="cuda")
                vo = torch.empty_like(ko)
                amskv.amskv_cache_export(h, l, ko, vo)
                torch.cuda.synchronize()
                exports.append((_bits(ko), _bits(vo)))
    finally:
        amskv.amskv_cache_destroy(h)
    return (q, k, v), outs, exports, sims, dens


CASES = [
    dict(dtype="bf16", D=64, policies=[(2, 1, False), (0, 0, True)]),
    dict(dtype="bf16", D=128, policies=[(2, 2, False), (1, 0, False)], layout=amskv.AMSKV_LAYOUT_PLANNED,
         borrow_unretained=True, fuse_append=True),
    dict(dtype="bf16", D=64, policies=[(2, 1, False)], fuse_append=True, pad=24),
    dict(dtype="f32", D=64, policies=[(1, 1, False), (0, 0, True)], borrow_unretained=True, fuse_append=True, pad=4),
    dict(dtype="bf16", D=64, budgets=[(174, 274, 5, 2.0), (60, 60, 5, -2.0)]),
]


@pytest.mark.parametrize("case", CASES, ids=lambda c: "%s-D%d-%s" % (c["dtype"], c["D"], "budget" if "budgets" in c else "window"))
def test_token_major_matches_oracle_and_head_major(case):
    case = dict(case)
    dtype, D = case.pop("dtype"), case.pop("D")
    B, H = 2, 3
    (q, k, v), o_tm, ex_tm, sim_tm, dens_tm = _run(VAR, B, H, D, dtype, True, **dict(case))
    case.pop("pad", None)
    _, o_hm, ex_hm, sim_hm, dens_hm = _run(VAR, B, H, D, dtype, False, **dict(case))
    # same kernels, same arithmetic order: the two layouts agree bit for bit
    assert len(o_tm) == len(o_hm)
    for a, b in zip(o_tm, o_hm):
        assert torch.equal(a, b)
    for (ka, va), (kb, vb) in zip(ex_tm, ex_hm):
        assert np.array_equal(ka, kb) and np.array_equal(va, vb)
    assert sim_tm == sim_hm and dens_tm == dens_hm
    # and the token-major outputs against the oracle, in both policy modes
    tokens = [s * s for s in VAR]
    st = orc.scale_starts(tokens)
    f64s = lambda xs: [_f64(x) for x in xs]
    if "policies" in case:
        n_layers = len(case["policies"])
        wants = [orc.attend_all_steps(f64s(q), f64s(k), f64s(v), tokens, pol) for pol in case["policies"]]
    else:
        n_layers = len(case["budgets"])
        cat = lambda xs: np.concatenate(f64s(xs), axis=-2)
        wants = []
        for c_min, c_max, c_cds, theta in case["budgets"]:
            trace = orc.alg1_cache_trace(tokens, c_min, c_max, c_cds, [theta > 1.0] * len(VAR))
            o = orc.masked_attention(cat(q), cat(k), cat(v), orc.alg1_allow_mask(tokens, trace))
            wants.append([o[..., st[s]: st[s] + tokens[s], :] for s in range(len(VAR))])
    for l in range(n_layers):
        for s in range(len(VAR)):
            err = float(np.abs(_f64(o_tm[s * n_layers + l]) - wants[l][s]).max())
            assert err <= TOL[dtype], (l, s, err)
    # Eq. 3 on token-major tensors against the oracle (layer 0, every step whose neighbour is still cached)
    if "policies" in case:
        for s in range(1, len(VAR)):
            got = sim_tm[s - 1]
            if got is None:
                continue
            wk, wsum = orc.interscale_similarity(_f64(k[s]), _f64(k[s - 1]), (VAR[s],) * 2, (VAR[s - 1],) * 2)
            wv, _ = orc.interscale_similarity(_f64(v[s]), _f64(v[s - 1]), (VAR[s],) * 2, (VAR[s - 1],) * 2)
            np.testing.assert_allclose(np.array(got[0]), wk, rtol=0, atol=1e-5)
            np.testing.assert_allclose(np.array(got[1]), wv, rtol=0, atol=1e-5)
            np.testing.assert_allclose(np.array(got[2]), wsum, rtol=2e-5, atol=1e-3)
    # attention density (mass per group of keys) on token-major queries against the oracle, layer 0
    if dens_tm:
        k_all = np.concatenate(f64s(k), axis=-2)
        for got_m, s in zip(dens_tm, (3, len(VAR) - 1)):
            if "policies" in case:
                pol = case["policies"][0]
                pieces = [(st[j], tokens[j]) for j in orc.kept_scales(pol, s)]
                rows = orc.allow_mask(tokens, pol)[st[s]: st[s] + tokens[s]]
            else:
                c_min, c_max, c_cds, theta = case["budgets"][0]
                trace = orc.alg1_cache_trace(tokens, c_min, c_max, c_cds, [theta > 1.0] * len(VAR))
                rows = orc.alg1_allow_mask(tokens, trace)[st[s]: st[s] + tokens[s]]
                ids = np.flatnonzero(rows[0]).tolist()
                scale_of = orc.scale_of_token(tokens)
                pieces = []
                for g in ids:
                    if pieces and pieces[-1][0] + pieces[-1][1] == g and scale_of[g] == scale_of[pieces[-1][0]]:
                        pieces[-1][1] += 1
                    else:
                        pieces.append([g, 1])
                pieces = [tuple(x) for x in pieces]
            _, want_m = orc.attention_density(_f64(q[s]), k_all, rows, pieces)
            assert np.allclose(np.asarray(got_m)[:, : len(pieces)], want_m, rtol=2e-4, atol=1e-5)


def test_io_layout_argument_checks():
    B, H, D = 1, 2, 64
    sides = (1, 2)
    need = amskv.amskv_cache_required_bytes(1, H, D, sides, sides, B, DT["bf16"], [(1, 1, False)])
    arena = torch.empty(need, dtype=torch.uint8, device="cuda")
    h = amskv.amskv_cache_create(1, H, D, sides, sides, B, DT["bf16"], [(1, 1, False)], arena=arena)
    try:
        TM, E = amskv.AMSKV_IO_TOKEN_MAJOR, amskv.AMSKV_ERR_INVALID_ARG
        for bad in [(H * D - 8, H * D, H * D), (H * D, H * D + 4, H * D), (H * D, H * D, 0)]:
            with pytest.raises(amskv.AmskvError) as e:
                amskv.amskv_cache_set_io_layout(h, TM, *bad)
            assert e.value.status == E
        with pytest.raises(amskv.AmskvError) as e:
            amskv.amskv_cache_set_io_layout(h, 7, H * D, H * D, H * D)
        assert e.value.status == E
        amskv.amskv_cache_set_io_layout(h, TM, 3 * H * D, 3 * H * D, H * D)
        x = torch.zeros(B, 1, 3 * H * D, dtype=torch.bfloat16, device="cuda")
        with pytest.raises(amskv.AmskvError) as e:          # a pointer that is not 16-byte aligned
            amskv.amskv_append_scale(h, 0, 0, x.data_ptr() + 2, x.data_ptr() + 2 * H * D * 2)
        assert e.value.status == E
        amskv.amskv_append_scale(h, 0, 0, x.data_ptr() + H * D * 2, x.data_ptr() + 2 * H * D * 2)
        with pytest.raises(amskv.AmskvError) as e:          # not while a scale is resident
            amskv.amskv_cache_set_io_layout(h, amskv.AMSKV_IO_HEAD_MAJOR)
        assert e.value.status == amskv.AMSKV_ERR_ORDER
        amskv.amskv_cache_reset(h)
        amskv.amskv_cache_set_io_layout(h, amskv.AMSKV_IO_HEAD_MAJOR)
    finally:
        amskv.amskv_cache_destroy(h)
