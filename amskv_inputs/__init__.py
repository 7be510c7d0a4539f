"""Seeded synthetic inputs for the AMS-KV hot path.

Serves both the CPU oracle's tests and the GPU library's tests/benchmark, and holds none
of the method's arithmetic: it only draws random tensors of the shapes the paper's
workloads have (Section 5 set-up: VAR-d16/d24/d30 at 256x256 with ten scales of side
1,2,3,4,5,6,8,10,13,16; an Infinity-2B-like 13-scale 1024x1024 schedule) and rounds them
to the run dtype.  The pretrained weights and the image/prompt sets the paper evaluates on
are not available, so these stand in for the Q/K/V the transformer would produce.

The correlated recipe (K_s = rho * resize(K_{s-1}) + sqrt(1-rho^2) * noise) uses the
library resize torch.nn.functional.interpolate; the oracle and the HIP kernels each carry
their own resize and neither is used here.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Sequence, Tuple

import torch
import torch.nn.functional as F

SEED_BASE = 251116000

VAR_SIDES = (1, 2, 3, 4, 5, 6, 8, 10, 13, 16)                      # 680 tokens
INFINITY_SIDES = (1, 2, 4, 6, 8, 12, 16, 20, 24, 32, 40, 48, 64)    # 10521 tokens


@dataclass
class Workload:
    """Shape of one benchmark/parity configuration."""
    name: str
    sides: Tuple[int, ...]
    layers: int
    batch: int
    heads: int
    head_dim: int
    dtype: str                      # "f32" | "bf16"
    config_id: int
    policies: List[Tuple[int, int, bool]] = field(default_factory=list)  # per layer (c, w, keep_all)

    @property
    def tokens(self) -> List[int]:
        return [s * s for s in self.sides]


def torch_dtype(name: str) -> torch.dtype:
    return {"f32": torch.float32, "bf16": torch.bfloat16}[name]


def layer_seed(config_id: int, layer: int) -> int:
    return SEED_BASE + 1000 * config_id + layer


def _gen(device, seed):
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


def iid_qkv(sides: Sequence[int], batch: int, heads: int, head_dim: int, dtype: str,
            seed: int, device="cpu"):
    """Q, K, V per scale, each [B, H, T_s, D], iid N(0,1) rounded to `dtype`."""
    g = _gen(device, seed)
    dt = torch_dtype(dtype)
    q, k, v = [], [], []
    for s in sides:
        t = s * s
        for lst in (q, k, v):
            lst.append(torch.randn(batch, heads, t, head_dim, generator=g, device=device,
                                   dtype=torch.float32).to(dt))
    return q, k, v


def _resize(x: torch.Tensor, side_in: int, side_out: int) -> torch.Tensor:
    """[B,H,T_in,D] -> [B,H,T_out,D] with the library bilinear resize (fp32)."""
    b, h, t, d = x.shape
    g = x.float().reshape(b * h, side_in, side_in, d).permute(0, 3, 1, 2)
    g = F.interpolate(g, size=(side_out, side_out), mode="bilinear", align_corners=False)
    return g.permute(0, 2, 3, 1).reshape(b, h, side_out * side_out, d)


def correlated_qkv(sides: Sequence[int], batch: int, heads: int, head_dim: int, dtype: str,
                   seed: int, rho: float, device="cpu"):
    """Q iid N(0,1); K_0, V_0 ~ N(0,1); X_s = rho*resize(X_{s-1}) + sqrt(1-rho^2)*N(0,1).

    The recursion runs on the unrounded fp32 tensors; each scale is rounded to `dtype`
    when emitted.  rho=0.8 gives the 0.8/0.6 mix of the VAR-d16 stack configuration.
    """
    g = _gen(device, seed)
    dt = torch_dtype(dtype)
    noise = math.sqrt(max(0.0, 1.0 - rho * rho))
    q, k, v = [], [], []
    pk = pv = None
    for i, s in enumerate(sides):
        t = s * s
        shape = (batch, heads, t, head_dim)
        q.append(torch.randn(shape, generator=g, device=device, dtype=torch.float32).to(dt))
        nk = torch.randn(shape, generator=g, device=device, dtype=torch.float32)
        nv = torch.randn(shape, generator=g, device=device, dtype=torch.float32)
        if i == 0:
            ck, cv = nk, nv
        else:
            ck = rho * _resize(pk, sides[i - 1], s) + noise * nk
            cv = rho * _resize(pv, sides[i - 1], s) + noise * nv
        k.append(ck.to(dt))
        v.append(cv.to(dt))
        pk, pv = ck, cv
    return q, k, v


def layer_rhos(n_layers: int, seed: int, lo: float = 0.2, hi: float = 0.95) -> List[float]:
    """Per-layer correlation strengths, uniform in [lo, hi] (VAR-d30 configuration)."""
    g = _gen("cpu", seed)
    u = torch.rand(n_layers, generator=g, dtype=torch.float64)
    return [float(lo + (hi - lo) * x) for x in u]


def policy_sweep(n_layers: int, seed: int, windows=(1, 2, 3, 4), condensed=(1, 2, 3)):
    """Per-layer (c, w, False) drawn from the seed (policy-sweep configuration)."""
    g = _gen("cpu", seed)
    wi = torch.randint(0, len(windows), (n_layers,), generator=g)
    ci = torch.randint(0, len(condensed), (n_layers,), generator=g)
    return [(int(condensed[int(c)]), int(windows[int(w)]), False) for c, w in zip(ci, wi)]


def sample_units(layers: int, batch: int, heads: int, n: int, seed: int):
    """Seeded sample of (layer, b, h) triples that always contains the corner units."""
    g = _gen("cpu", seed)
    units = {(l, b, h) for l in (0, layers - 1) for b in (0, batch - 1) for h in (0, heads - 1)}
    while len(units) < min(n, layers * batch * heads):
        l = int(torch.randint(0, layers, (1,), generator=g))
        b = int(torch.randint(0, batch, (1,), generator=g))
        h = int(torch.randint(0, heads, (1,), generator=g))
        units.add((l, b, h))
    return sorted(units)


# ---- the five configurations of the benchmark contract -------------------------------
def config1() -> Workload:
    return Workload("var_d16_single_layer_f32", VAR_SIDES, 1, 1, 16, 64, "f32", 1, [(2, 2, False)])


def config2(batch: int = 32) -> Workload:
    pol = [(2, 2, True) if (l < 4 or l >= 12) else (2, 2, False) for l in range(16)]
    return Workload("var_d16_stack_bf16", VAR_SIDES, 16, batch, 16, 64, "bf16", 2, pol)


def config3(batch: int = 256) -> Workload:
    return Workload("var_d30_bf16_b%d" % batch, VAR_SIDES, 30, batch, 30, 64, "bf16", 3,
                    [(2, 2, False)] * 30)


def config4(batch: int = 8) -> Workload:
    return Workload("infinity_2b_1024_bf16", INFINITY_SIDES, 32, batch, 16, 128, "bf16", 4,
                    [(3, 1, False)] * 32)


def config5(batch: int = 64) -> Workload:
    return Workload("var_d24_policy_sweep_bf16", VAR_SIDES, 24, batch, 24, 64, "bf16", 5,
                    policy_sweep(24, layer_seed(5, 0)))
