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

    def __init__(self, N: int, H: int, D: int, dtype: torch.dtype, device="cuda", fused_update: bool = False):
        self.N, self.H, self.D, self.dtype = N, H, D, dtype
        # fused_update: the attention writes its rows straight into the cached output buffer
        # (astraea_sparse_attn_update_fwd) instead of into o_sel followed by a scatter
        self.fused_update = fused_update
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
        ab.astraea_kv_refresh(t["k_cache"].view(N, E), t["v_cache"].view(N, E), t["k_new"].view(N, E),
                              t["v_new"].view(N, E), self.idx_sel, k)

    def step_attn(self, t: Dict[str, torch.Tensor], k: int, lse: Optional[torch.Tensor] = None) -> None:
        ab.astraea_sparse_attn_fwd(t["q"], t["k_cache"], t["v_cache"], self.idx_sel, k, self.o_sel[:max(k, 1)],
                                   self.scale, q_is_compact=False, lse_sel=lse, workspace=self.attn_ws)

    def step_attn_update(self, t: Dict[str, torch.Tensor], k: int, lse: Optional[torch.Tensor] = None) -> None:
        ab.astraea_sparse_attn_update_fwd(t["q"], t["k_cache"], t["v_cache"], self.idx_sel, k, t["out_cache"],
                                          self.scale, q_is_compact=False, lse_sel=lse, workspace=self.attn_ws)

    def step_scatter(self, t: Dict[str, torch.Tensor], k: int) -> None:
        E = self.H * self.D
        ab.astraea_scatter_update(t["out_cache"], self.o_sel.view(self.N, E), self.idx_sel, k, src_is_full=False)

    def run(self, t: Dict[str, torch.Tensor], k: int) -> None:
        """The whole hot path for one batch of inputs; updates k_cache, v_cache and out_cache in place."""
        self.step_score(t)
        self.step_select(k)
        self.step_kv_refresh(t, k)
        if self.fused_update:
            self.step_attn_update(t, k)
        else:
            self.step_attn(t, k)
            self.step_scatter(t, k)


class StatefulLayer(LayerStep):
    """The layer-step with the state the full selection metric carries from one timestep to the next
    (paper Sec. 3.2 "Selection Metric"): the features of the last step each token was computed in
    (`x_ref`), the per-token softmax by-product S_LSE (`lse_weight`) and the count of consecutive
    non-selections n_i (`skip_count`), whose penalty e^{n_i} comes from a table built by the caller."""

    def __init__(self, N: int, H: int, D: int, C: int, dtype: torch.dtype, penalty_table: torch.Tensor,
                 w_alpha: float = 1.0, w_beta: float = 0.0, device="cuda", fused_update: bool = False):
        super().__init__(N, H, D, dtype, device, fused_update)
        self.x_ref = torch.zeros((N, C), dtype=dtype, device=device)
        self.lse_weight = torch.ones(N, dtype=torch.float32, device=device)
        self.skip_count = torch.zeros(N, dtype=torch.int32, device=device)
        self.lse_sel = torch.empty((N, H), dtype=torch.float32, device=device)
        self.penalty_table = penalty_table.to(device=device, dtype=torch.float32)
        self.w_alpha, self.w_beta = w_alpha, w_beta

    def step_score(self, t: Dict[str, torch.Tensor]) -> None:
        ab.astraea_score(t["x_cur"], self.x_ref, self.score, lse_weight=self.lse_weight, skip_count=self.skip_count,
                         penalty_table=self.penalty_table, w_alpha=self.w_alpha, w_beta=self.w_beta)

    def step_select(self, k: int) -> None:
        ab.astraea_select_topk(self.score, k, self.idx_sel, self.topk_ws, skip_count=self.skip_count)

    def step_state(self, t: Dict[str, torch.Tensor], k: int) -> None:
        """After the attention: selected tokens were computed at this step, so their reference features and
        their S_LSE are refreshed; the others keep what they had."""
        ab.astraea_scatter_update(self.x_ref, t["x_cur"], self.idx_sel, k, src_is_full=True)
        ab.astraea_lse_weight_update(self.lse_sel[:max(k, 1)], self.idx_sel, k, self.lse_weight)

    def run(self, t: Dict[str, torch.Tensor], k: int) -> None:
        self.step_score(t)
        self.step_select(k)
        self.step_kv_refresh(t, k)
        if self.fused_update:
            self.step_attn_update(t, k, lse=self.lse_sel[:max(k, 1)])
            self.step_state(t, k)
        else:
            self.step_attn(t, k, lse=self.lse_sel[:max(k, 1)])
            self.step_state(t, k)
            self.step_scatter(t, k)


class TokenSparseBlock(LayerStep):
    """A whole token-wise block on the selected tokens (paper Sec. 3.2: "each token is processed
    independently" in every layer but the attention, so all of them are computed for the selected tokens only
    and the block's cached output serves the rest; Algorithm 1 steps 4-7; FLOPs appendix: Q/K/V projection,
    attention, output projection, two MLP layers).  Layer norms, modulation and residual sums of a real DiT
    block are not part of the paper's algorithm and are left out.

    Weights are [c_out, c_in] tensors of the block's dtype (bf16, or fp32 for the fp32 configuration) supplied by
    the caller (synthetic in the tests and the benchmark).
    K and V of the selected tokens are written straight into the cached K/V by the projection (the cache
    refresh fused into its producer), the MLP's second layer writes straight into the cached block output.
    With a packed cache t["qkv_cache"] [N, 3, H, D] and a stacked weight "wqkv" [3E, E] the three projections
    are one call, and the attention reads Q, K and V through strides.
    """

    def __init__(self, N: int, H: int, D: int, weights: Dict[str, torch.Tensor], device="cuda", mlp_ratio: int = 4,
                 dtype: torch.dtype = torch.bfloat16):
        super().__init__(N, H, D, dtype, device)
        E = H * D
        self.E, self.hidden = E, mlp_ratio * E
        self.w = weights            # wq wk wv wo [E, E]; w1 [hidden, E]; w2 [E, hidden]; optional b* biases
        bf = dict(dtype=dtype, device=device)
        self.q_sel = torch.empty((N, H, D), **bf)
        self.h_sel = torch.empty((N, E), **bf)           # output projection result
        self.m_sel = torch.empty((N, self.hidden), **bf)  # MLP hidden activations

    def _b(self, name):
        return self.w.get(name)

    def flops(self, k: int) -> Dict[str, float]:
        """Multiply-add counts of one block step at k selected tokens, by the formulas of the paper's FLOPs
        appendix with the token count N replaced by k where a layer runs on the selected tokens only (E = H*D,
        batch 1): Q/K/V projection 6kE^2, attention scores and output 4kNE, output projection 2kE^2, the two
        MLP layers 2 * 2kE*hidden (16kE^2 at hidden = 4E)."""
        E, hid, N = float(self.E), float(self.hidden), float(self.N)
        return {"qkv_proj": 6.0 * k * E * E, "attn": 4.0 * k * N * E, "out_proj": 2.0 * k * E * E,
                "mlp": 4.0 * k * E * hid}

    def step_qkv(self, t: Dict[str, torch.Tensor], k: int) -> None:
        N, E, idx = self.N, self.E, self.idx_sel
        x = t["x_in"]
        if "qkv_cache" in t:
            # packed form: one projection with the stacked weight [3E, E] writes Q, K and V of the selected
            # tokens side by side into their rows of one cached [N, 3, H, D] buffer (one launch instead of
            # three: 20 rounds of tiles instead of 3 x 7 at the headline size)
            ab.astraea_sparse_linear(x, self.w["wqkv"], self._b("bqkv"), idx, k, t["qkv_cache"].view(N, 3 * E),
                                     y_is_compact=False)
            return
        ab.astraea_sparse_linear(x, self.w["wq"], self._b("bq"), idx, k, self.q_sel.view(N, E)[:max(k, 1)])
        ab.astraea_sparse_linear(x, self.w["wk"], self._b("bk"), idx, k, t["k_cache"].view(N, E), y_is_compact=False)
        ab.astraea_sparse_linear(x, self.w["wv"], self._b("bv"), idx, k, t["v_cache"].view(N, E), y_is_compact=False)

    def step_attn(self, t: Dict[str, torch.Tensor], k: int, lse: Optional[torch.Tensor] = None) -> None:
        if "qkv_cache" in t:
            c = t["qkv_cache"]          # queries gathered by index from the packed rows, K and V read through strides
            ab.astraea_sparse_attn_fwd(c[:, 0], c[:, 1], c[:, 2], self.idx_sel, k, self.o_sel[:max(k, 1)], self.scale,
                                       q_is_compact=False, lse_sel=lse, workspace=self.attn_ws)
            return
        ab.astraea_sparse_attn_fwd(self.q_sel[:max(k, 1)], t["k_cache"], t["v_cache"], self.idx_sel, k,
                                   self.o_sel[:max(k, 1)], self.scale, q_is_compact=True, lse_sel=lse,
                                   workspace=self.attn_ws)

    def step_proj_mlp(self, t: Dict[str, torch.Tensor], k: int) -> None:
        N, E, kk = self.N, self.E, max(k, 1)
        ab.astraea_sparse_linear(self.o_sel.view(N, E)[:kk], self.w["wo"], self._b("bo"), None, k, self.h_sel[:kk],
                                 x_is_compact=True)
        ab.astraea_sparse_linear(self.h_sel[:kk], self.w["w1"], self._b("b1"), None, k, self.m_sel[:kk],
                                 act=ab.ACT_GELU_TANH, x_is_compact=True)
        ab.astraea_sparse_linear(self.m_sel[:kk], self.w["w2"], self._b("b2"), self.idx_sel, k, t["out_cache"],
                                 x_is_compact=True, y_is_compact=False, N=N)

    def run(self, t: Dict[str, torch.Tensor], k: int) -> None:
        """score -> top-k -> Q/K/V projections of the selected rows (K/V into the caches) -> attention ->
        output projection -> MLP, whose last layer updates the cached block output in place."""
        ab.astraea_score(t["x_in"], t["x_prev"], self.score)
        self.step_select(k)
        self.step_qkv(t, k)
        self.step_attn(t, k)
        self.step_proj_mlp(t, k)


class GraphedStep:
    """A call chain recorded once as a HIP graph and replayed with one launch.

    Every entry point of the library only enqueues kernels on the caller's stream: it allocates nothing,
    never waits for the device and records no memset, and k is a host number, so a whole layer-step at a fixed
    k can be captured.  That pays where the step is short against the cost of launching its seven to ten
    kernels one by one (small token counts, small budgets); the 50-step schedule of a denoising run needs one
    graph per distinct budget, at most ten.

    `fn` is any callable that makes the calls (e.g. ``lambda: layer.run(t, k)``); the tensors it touches must
    stay alive and in place, new inputs are copied into them before a replay.  With `warm` the chain is run
    once for real before the capture, so that code objects are loaded outside it; that run changes the caches
    and counters like any step, so pass ``warm=False`` when the same chain has already run in this process
    and its state must not advance.  Capture and replay use torch's HIP-graph wrapper, on streams of default
    priority.
    """

    def __init__(self, fn, warm: bool = True):
        if warm:
            fn()
        torch.cuda.synchronize()
        self.graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(self.graph):
            fn()

    def replay(self) -> None:
        self.graph.replay()
