"""One layer-step of the token-wise attention path, as a chain of C-ABI calls.

Order of the calls (paper, supplementary Algorithm 1; Sec. 3.2 execution flow):
score -> select top-k -> refresh the cached K/V rows of the selected tokens ->
attention of the selected queries over the full-length K/V (queries gathered
in-kernel) -> scatter of the fresh outputs into the cached output buffer.

Host logic only: buffers are allocated once, k comes from the budget on the
host, nothing is read back from the device between calls.
"""
from __future__ import annotations

import math
from typing import Dict, Optional

import torch

from . import binding as ab


class LayerStep:
    """Pre-allocated buffers plus the call chain for one (N, H, D) layer."""

    def __init__(self, N: int, H: int, D: int, dtype: torch.dtype, device="cuda"):
        self.N, self.H, self.D, self.dtype = N, H, D, dtype
        self.score = torch.empty(N, dtype=torch.float32, device=device)
        self.idx_sel = torch.empty(max(N, 1), dtype=torch.int32, device=device)
        self.o_sel = torch.empty((N, H, D), dtype=dtype, device=device)
        self.topk_ws = torch.empty(ab.workspace_bytes(ab.OP_SELECT_TOPK, N), dtype=torch.uint8, device=device)
        wsb = ab.workspace_bytes(ab.OP_SPARSE_ATTN, N, N, H, D)
        self.attn_ws = torch.empty(wsb, dtype=torch.uint8, device=device) if wsb else None
        self.scale = 1.0 / math.sqrt(D)

    def budget_to_k(self, budget_pct: int) -> int:
        return ab.astraea_budget_to_k(self.N, budget_pct)

    # individual steps, so a benchmark can time them apart -----------------
    def step_score(self, t: Dict[str, torch.Tensor]) -> None:
        ab.astraea_score(t["x_cur"], t["x_prev"], self.score)

    def step_select(self, k: int) -> None:
        ab.astraea_select_topk(self.score, k, self.idx_sel, self.topk_ws)

    def step_kv_refresh(self, t: Dict[str, torch.Tensor], k: int) -> None:
        N, E = self.N, self.H * self.D
        ab.astraea_scatter_update(t["k_cache"].view(N, E), t["k_new"].view(N, E), self.idx_sel, k, src_is_full=True)
        ab.astraea_scatter_update(t["v_cache"].view(N, E), t["v_new"].view(N, E), self.idx_sel, k, src_is_full=True)

    def step_attn(self, t: Dict[str, torch.Tensor], k: int, lse: Optional[torch.Tensor] = None) -> None:
        ab.astraea_sparse_attn_fwd(t["q"], t["k_cache"], t["v_cache"], self.idx_sel, k, self.o_sel[:max(k, 1)],
                                   self.scale, q_is_compact=False, lse_sel=lse, workspace=self.attn_ws)

    def step_scatter(self, t: Dict[str, torch.Tensor], k: int) -> None:
        E = self.H * self.D
        ab.astraea_scatter_update(t["out_cache"], self.o_sel.view(self.N, E), self.idx_sel, k, src_is_full=False)

    def run(self, t: Dict[str, torch.Tensor], k: int) -> None:
        """The whole hot path for one batch of inputs; updates k_cache, v_cache and out_cache in place."""
        self.step_score(t)
        self.step_select(k)
        self.step_kv_refresh(t, k)
        self.step_attn(t, k)
        self.step_scatter(t, k)
