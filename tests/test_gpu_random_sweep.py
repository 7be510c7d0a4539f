"""Seeded random sweep over the three policy modes: schedules with arbitrary (also shrinking) sides, batch, heads,
head dim, dtype, layouts and flags drawn together, every case driven through the C ABI and compared with the oracle
by the same runners the hand-picked cases use -- kept sets, offsets, eviction lists, bytes held and cache contents
bit for bit, attention within the tolerance.  The hand-picked cases fix one thing at a time; this one looks for
interactions between them.

Bar: as in the runners (bit-exact bookkeeping and contents; max-abs 1e-4 fp32 / 2e-2 bf16 on attention outputs).
"""
import numpy as np
import pytest

import paper_2511_16047_amd as amskv
import test_gpu_parity as sw
import test_gpu_token_budget as tb
import test_gpu_token_window as tw

pytestmark = pytest.mark.gpu

MAX_TOKENS = 700      # per schedule: the oracle's T x T mask stays small


def _schedule(rng, max_side=16):
    n = int(rng.integers(2, 10))
    while True:
        sides = [int(rng.integers(1, max_side + 1)) for _ in range(n)]
        if rng.random() < 0.6:
            sides.sort()                     # the usual coarse-to-fine order; otherwise any order, shrinking included
        if sum(s * s for s in sides) <= MAX_TOKENS:
            return tuple(sides)


def _scale_window_cases():
    rng = np.random.default_rng(2511_16047_1)
    cases = []
    for i in range(40):
        sides = _schedule(rng)
        n = len(sides)
        pols = []
        for _ in range(int(rng.integers(1, 4))):
            pols.append((int(rng.integers(0, n + 1)), int(rng.integers(0, n + 1)), bool(rng.random() < 0.2)))
        cases.append(dict(sides=sides, B=int(rng.integers(1, 4)), H=int(rng.integers(1, 5)), D=int(rng.choice([64, 128])),
                          dtype=str(rng.choice(["bf16", "bf16", "f32"])), pols=pols,
                          layout=int(rng.choice([amskv.AMSKV_LAYOUT_COMPACT, amskv.AMSKV_LAYOUT_PLANNED])),
                          borrow=bool(rng.random() < 0.5), fuse=bool(rng.random() < 0.5),
                          scale=float(rng.choice([0.0, 0.0, 0.07])), seed=5000 + i))
    return cases


def _case_id(c):
    return "-".join("%s" % v if not isinstance(v, (list, tuple)) else "x".join(map(str, v)) for k, v in c.items()
                    if k in ("sides", "B", "H", "D", "dtype"))


@pytest.mark.parametrize("c", _scale_window_cases(), ids=_case_id)
def test_scale_window_mode(c):
    r = sw.Runner(c["sides"], c["sides"], c["B"], c["H"], c["D"], c["dtype"], c["pols"], layout=c["layout"],
                  softmax_scale=c["scale"], borrow=c["borrow"], fuse=c["fuse"])
    try:
        for layer in range(len(c["pols"])):
            q, k, v = sw._qkv(c["sides"], c["sides"], c["B"], c["H"], c["D"], c["dtype"], c["seed"] + 17 * layer)
            r.run_layer(layer, q, k, v)
    finally:
        r.close()


def _theta_between(scores, asked):
    """Above some of the compared scores and below the others where they are far enough apart (the expansion then
    happens at a later test than the first); otherwise above all of them."""
    vals = sorted(scores[i] for i in asked if i > 0)
    gaps = [(b - a, (a + b) / 2) for a, b in zip(vals, vals[1:]) if b - a >= 0.12]
    return max(gaps)[1] if gaps else tb._theta_above(scores, asked)


def _token_budget_cases():
    rng = np.random.default_rng(2511_16047_2)
    cases = []
    for i in range(30):
        sides = _schedule(rng, 14)
        total = sum(s * s for s in sides)
        c_min = int(rng.integers(1, total + 1))
        c_max = int(rng.integers(c_min, total + 1)) if rng.random() < 0.8 else c_min
        c_cds = int(rng.integers(0, c_min + 1)) if rng.random() < 0.8 else 0
        steps = [s for s in range(len(sides)) if rng.random() < 0.7]
        cases.append(dict(sides=sides, B=int(rng.integers(1, 3)), H=int(rng.integers(1, 4)), D=int(rng.choice([64, 128])),
                          dtype=str(rng.choice(["bf16", "bf16", "f32"])), budget=(c_min, c_max, c_cds),
                          theta=int(rng.integers(0, 3)), attend_at=None if rng.random() < 0.6 else tuple(steps),
                          rho=float(rng.choice([0.3, 0.8])), seed=6000 + i))
    return cases


@pytest.mark.parametrize("c", _token_budget_cases(), ids=lambda c: _case_id(c) + "-" + "_".join(map(str, c["budget"])))
def test_token_budget_mode(c):
    theta_of = (tb._theta_above, tb._theta_below_all, _theta_between)[c["theta"]]
    tb._run(c["sides"], c["B"], c["H"], c["D"], c["dtype"], c["budget"], theta_of, c["seed"], rho=c["rho"],
            attend_at=c["attend_at"])


def _token_window_cases():
    rng = np.random.default_rng(2511_16047_3)
    cases = []
    for i in range(30):
        sides = _schedule(rng, 14)
        total = sum(s * s for s in sides)
        window = int(rng.integers(1, total + 1))
        n_sink = int(rng.integers(0, window + 1)) if rng.random() < 0.6 else 0
        cases.append(dict(sides=sides, B=int(rng.integers(1, 3)), H=int(rng.integers(1, 4)), D=int(rng.choice([64, 128])),
                          dtype=str(rng.choice(["bf16", "bf16", "f32"])), window=window, n_sink=n_sink,
                          between=bool(rng.random() < 0.75), seed=7000 + i))
    return cases


@pytest.mark.parametrize("c", _token_window_cases(), ids=lambda c: _case_id(c) + "-w%d_s%d" % (c["window"], c["n_sink"]))
def test_token_window_mode(c):
    tw._run(c["sides"], c["B"], c["H"], c["D"], c["dtype"], c["window"], c["n_sink"], c["seed"], query_between=c["between"])
