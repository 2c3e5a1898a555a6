"""Seeded synthetic inputs shaped like the paper's video-latent workloads.

This module only draws random tensors (shapes, dtypes, value distributions).
It holds none of the method's arithmetic: no scoring, no selection, no
attention.  Both the HIP path and the CPU oracle are fed the tensors made
here, so the two sides always see identical bits.

Workload shapes follow the five benchmark configurations: a 24-head,
128-wide-head video DiT layer over 13x30x45 (480p-like) or 33x45x80
(720p-like) latent tokens, plus two smaller layers for full-oracle checks.
The paper's own models and prompts are not used; these tensors stand in for
the Q/K/V, token features and cached outputs of one attention block
(Algorithm 1 "Require" list in the paper's supplementary).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Tuple

import torch


@dataclass(frozen=True)
class Workload:
    """Shape and recipe of one benchmark configuration."""

    name: str
    dtype: str                      # "f32" or "bf16"
    N: int                          # tokens
    H: int                          # heads
    D: int                          # head dim
    C: int                          # width of the token feature used for scoring
    budgets_pct: Tuple[int, ...]    # token budgets in percent
    feature_recipe: str             # "independent" | "drift"
    key_bias_std: float = 0.0       # shared per-head bias added to K (0 = none)
    latent: Tuple[int, int, int] = (0, 0, 0)

    @property
    def torch_dtype(self) -> torch.dtype:
        return torch.float32 if self.dtype == "f32" else torch.bfloat16

    @property
    def row_elems(self) -> int:
        return self.H * self.D


WORKLOADS: Dict[str, Workload] = {
    # config 0: small fp32 layer the oracle finishes in seconds
    "cfg0": Workload("cfg0", "f32", 4096, 8, 64, 512, (50,), "independent", latent=(16, 16, 16)),
    # config 1: bf16 layer with correlated keys (shared per-head bias on K)
    "cfg1": Workload("cfg1", "bf16", 16384, 24, 128, 512, (25, 50, 75), "independent",
                     key_bias_std=0.5, latent=(16, 32, 32)),
    # config 2: 480p-shaped layer
    "cfg2": Workload("cfg2", "bf16", 17550, 24, 128, 3072, (40,), "drift", latent=(13, 30, 45)),
    # config 3: 720p-shaped layer (headline)
    "cfg3": Workload("cfg3", "bf16", 118800, 24, 128, 3072, (30,), "drift", latent=(33, 45, 80)),
    # config 4: budget sweep at the 720p shape; budgets are drawn by budget_schedule()
    "cfg4": Workload("cfg4", "bf16", 118800, 24, 128, 3072, tuple(range(10, 101, 10)), "drift",
                     latent=(33, 45, 80)),
}


def _gen(seed: int, slot: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed) * 1000 + int(slot))
    return g


def _randn(shape, seed, slot, device, dtype, std=1.0, chunk_rows=1 << 15) -> torch.Tensor:
    """N(0, std^2) drawn in fp32 then rounded once (RNE) to `dtype`.

    Large tensors are drawn in row chunks so the fp32 staging copy stays small.
    """
    g = _gen(seed, slot, device)
    out = torch.empty(shape, device=device, dtype=dtype)
    flat = out.view(shape[0], -1) if len(shape) > 1 else out.view(-1, 1)
    for r0 in range(0, flat.shape[0], chunk_rows):
        r1 = min(flat.shape[0], r0 + chunk_rows)
        t = torch.randn((r1 - r0, flat.shape[1]), generator=g, device=device, dtype=torch.float32)
        if std != 1.0:
            t.mul_(std)
        flat[r0:r1].copy_(t)
    return out


def make_layer_inputs(w: Workload, seed: int = 0, device="cpu", step: int = 0,
                      N: int | None = None) -> Dict[str, torch.Tensor]:
    """Draw every tensor one layer-step consumes.

    Returns a dict with
      x_prev, x_cur : [N, C]     token features of the previous / current step
      q             : [N, H, D]  queries of all tokens (the path gathers rows)
      k_new, v_new  : [N, H, D]  this step's keys / values (only selected rows are used)
      k_cache, v_cache : [N, H, D] persistent K/V holding earlier steps' rows
      out_cache     : [N, H*D]   cached per-token attention outputs
    `N` overrides the token count (for reduced-size test cases of the same recipe).
    `step` shifts the generator slots so a sweep can draw fresh tensors per step.
    """
    n = int(N if N is not None else w.N)
    dt = w.torch_dtype
    base = 100 * int(step)
    t: Dict[str, torch.Tensor] = {}
    if w.feature_recipe == "independent":
        t["x_prev"] = _randn((n, w.C), seed, base + 0, device, dt)
        t["x_cur"] = _randn((n, w.C), seed, base + 1, device, dt)
    elif w.feature_recipe == "drift":
        # cur = prev + 0.1 * N(0,1), formed in fp32 and rounded once
        prev32 = _randn((n, w.C), seed, base + 0, device, torch.float32)
        noise = _randn((n, w.C), seed, base + 1, device, torch.float32, std=0.1)
        t["x_prev"] = prev32.to(dt)
        t["x_cur"] = (prev32 + noise).to(dt)
        del prev32, noise
    else:
        raise ValueError(w.feature_recipe)
    for slot, name in ((2, "q"), (3, "k_new"), (4, "v_new"), (5, "k_cache"), (6, "v_cache")):
        if w.key_bias_std > 0.0 and name in ("k_new", "k_cache"):
            x = _randn((n, w.H, w.D), seed, base + slot, device, torch.float32)
            # one shared bias vector per head, the same for fresh and cached keys
            b = torch.randn((1, w.H, w.D), generator=_gen(seed, 9, device), device=device,
                            dtype=torch.float32) * w.key_bias_std
            t[name] = (x + b).to(dt)
            del x
        else:
            t[name] = _randn((n, w.H, w.D), seed, base + slot, device, dt)
    t["out_cache"] = _randn((n, w.H * w.D), seed, base + 7, device, dt)
    return t


def budget_schedule(seed: int, steps: int = 50) -> List[int]:
    """Per-timestep budgets, uniform over {10, 20, ..., 100} percent (config 4)."""
    g = torch.Generator(device="cpu")
    g.manual_seed(int(seed) * 1000 + 999)
    draws = torch.randint(1, 11, (steps,), generator=g)
    return [int(v) * 10 for v in draws]


def random_scores(n: int, seed: int, kind: str = "normal", device="cpu") -> torch.Tensor:
    """Score arrays for selection tests: distinct, heavy-tailed, or massively tied."""
    g = _gen(seed, 500, device)
    if kind == "normal":
        return torch.randn(n, generator=g, device=device)
    if kind == "lognormal":
        return torch.exp(2.0 * torch.randn(n, generator=g, device=device))
    if kind == "tied":
        return torch.randint(0, 7, (n,), generator=g, device=device).to(torch.float32)
    if kind == "narrow":
        # values crowded in a narrow band sharing their high bits, many exact ties
        return 5.5 + torch.randint(0, 4096, (n,), generator=g, device=device).to(torch.float32) * (2.0 ** -18)
    if kind == "signed_tied":
        return (torch.randint(-3, 4, (n,), generator=g, device=device)).to(torch.float32) * 0.5
    raise ValueError(kind)
