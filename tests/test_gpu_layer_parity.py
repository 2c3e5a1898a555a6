"""End-to-end layer-step parity at the benchmark configurations, through the C ABI, in the launch
configuration bench.py times (paper_2506_05096_amd.layer.LayerStep).

Config 0 is checked in full.  At the larger configurations the oracle recomputes every score, every
selected index, every refreshed K/V row and every untouched cache row, and the attention output on a
sample of selected rows (rows are independent: each is an exact softmax row over all N keys), always
including the first and last selected token and rows of the last, partially filled query tile.
"""
import numpy as np
import pytest
import torch

import oracle
from conftest import bf16_bits_to_f64, to_np
from paper_2506_05096_amd import synth
from paper_2506_05096_amd.layer import LayerStep

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _f64(a):
    return bf16_bits_to_f64(a) if a.dtype == np.uint16 else a.astype(np.float64)


def _sample_rows(k, n_rows, seed):
    """Positions in the selected list: ends, the ragged tail of the last 256-query tile, and random ones."""
    rng = np.random.default_rng(seed)
    fixed = {0, 1, k - 1, k - 2, (k // 256) * 256 - 1, (k // 256) * 256, min(k - 1, (k // 256) * 256 + 1)}
    fixed = {r for r in fixed if 0 <= r < k}
    extra = rng.choice(k, size=min(k, max(0, n_rows - len(fixed))), replace=False)
    return np.array(sorted(fixed | set(int(e) for e in extra)), dtype=np.int64)


def _check_step(w, t, host, layer, budget_pct, n_rows, tag, out_known=None):
    """Runs one layer step on the GPU and checks it against the oracle.  `host` holds numpy copies of the
    inputs as they were before the step (all drawn by the seeded generators or computed by the oracle);
    `out_known` marks the rows of host["out_cache"] whose value is known that way (None: all of them).
    Returns the oracle's K and V caches after the step and the selected indices."""
    n, H, D, E = w.N, w.H, w.D, w.H * w.D
    k = layer.budget_to_k(budget_pct)
    assert k == oracle.budget_to_k(n, budget_pct)
    before = to_np(t["out_cache"]).copy()          # only for the property check "unselected rows do not move"
    layer.run(t, k)
    torch.cuda.synchronize()

    # score and selection: bit-exact
    e_score = oracle.score(host["x_cur"], host["x_prev"])
    assert np.array_equal(layer.score.cpu().numpy().view(np.uint32), e_score.view(np.uint32)), f"{tag}: scores"
    e_idx, e_rem, _ = oracle.topk(e_score, k)
    assert np.array_equal(layer.idx_sel[:k].cpu().numpy(), e_idx), f"{tag}: selected indices"

    # K/V caches: selected rows refreshed, the rest untouched (bit-exact, full comparison)
    kc, vc = host["k_cache"].reshape(n, E).copy(), host["v_cache"].reshape(n, E).copy()
    oracle.scatter(kc, host["k_new"].reshape(n, E), e_idx, src_is_full=True)
    oracle.scatter(vc, host["v_new"].reshape(n, E), e_idx, src_is_full=True)
    assert np.array_equal(to_np(t["k_cache"]).reshape(n, E), kc), f"{tag}: K cache"
    assert np.array_equal(to_np(t["v_cache"]).reshape(n, E), vc), f"{tag}: V cache"

    # output cache: unselected rows keep the cached value, bit for bit
    got = to_np(t["out_cache"])
    rem_known = e_rem if out_known is None else e_rem[out_known[e_rem]]
    assert np.array_equal(got[rem_known], host["out_cache"][rem_known]), f"{tag}: unselected cache rows changed"
    assert np.array_equal(got[e_rem], before[e_rem]), f"{tag}: a row outside the selection moved"
    # scatter positions: cache row idx[r] holds exactly row r of the compact attention output
    if not layer.fused_update:      # the fused path has no compact result to compare positions with
        assert np.array_equal(got[e_idx], to_np(layer.o_sel[:k]).reshape(k, E)), f"{tag}: scatter positions"

    # attention on the sampled rows against the oracle
    rows = np.arange(k) if n_rows >= k else _sample_rows(k, n_rows, seed=n + k)
    o64, _ = oracle.sparse_attn(host["q"], kc.reshape(n, H, D), vc.reshape(n, H, D), e_idx[rows], layer.scale)
    g64 = _f64(got[e_idx[rows]]).reshape(len(rows), H, D)
    assert np.all(np.isfinite(g64))
    if w.dtype == "f32":
        err = float(np.max(np.abs(g64 - o64)))
        assert err <= 1e-4, f"{tag}: max abs error {err}"
    else:
        err = float(np.linalg.norm((g64 - o64).ravel()) / np.linalg.norm(o64.ravel()))
        assert err <= 1e-2, f"{tag}: relative L2 error {err}"
        worst = np.max(np.linalg.norm((g64 - o64).reshape(len(rows), -1), axis=1) /
                       np.linalg.norm(o64.reshape(len(rows), -1), axis=1))
        assert worst <= 2e-2, f"{tag}: worst row relative L2 {worst}"
    print(f"{tag}: N={n} k={k} rows checked={len(rows)} err={err:.3g}", flush=True)
    return kc, vc, e_idx


def _host(t):
    return {name: to_np(v) for name, v in t.items()}


def test_config0_fp32_full():
    w = synth.WORKLOADS["cfg0"]
    t = synth.make_layer_inputs(w, seed=0, device=DEV)
    layer = LayerStep(w.N, w.H, w.D, w.torch_dtype, device=DEV)
    _check_step(w, t, _host(t), layer, 50, n_rows=10**9, tag="cfg0")


@pytest.mark.parametrize("budget", [25, 50, 75])
def test_config1_bf16_key_bias(budget):
    w = synth.WORKLOADS["cfg1"]
    t = synth.make_layer_inputs(w, seed=0, device=DEV)
    layer = LayerStep(w.N, w.H, w.D, w.torch_dtype, device=DEV)
    _check_step(w, t, _host(t), layer, budget, n_rows=48, tag=f"cfg1@{budget}%")


@pytest.mark.parametrize("fused", [False, True])
def test_config2_480p(fused):
    w = synth.WORKLOADS["cfg2"]
    t = synth.make_layer_inputs(w, seed=0, device=DEV)
    layer = LayerStep(w.N, w.H, w.D, w.torch_dtype, device=DEV, fused_update=fused)
    _check_step(w, t, _host(t), layer, 40, n_rows=48, tag="cfg2" + ("/fused" if fused else ""))


@pytest.mark.parametrize("fused", [False, True])
def test_config3_720p_headline(fused):
    w = synth.WORKLOADS["cfg3"]
    t = synth.make_layer_inputs(w, seed=0, device=DEV)
    layer = LayerStep(w.N, w.H, w.D, w.torch_dtype, device=DEV, fused_update=fused)
    _check_step(w, t, _host(t), layer, 30, n_rows=24, tag="cfg3" + ("/fused" if fused else ""))


@pytest.mark.parametrize("budget", [10, 100])
def test_config3_at_the_ends_of_the_budget_range(budget):
    """The headline shape at the smallest budget of the schedule (the launch plan with the largest share of split
    work items) and at 100 % (dense attention for every token)."""
    w = synth.WORKLOADS["cfg3"]
    t = synth.make_layer_inputs(w, seed=0, device=DEV)
    layer = LayerStep(w.N, w.H, w.D, w.torch_dtype, device=DEV)
    _check_step(w, t, _host(t), layer, budget, n_rows=16, tag=f"cfg3@{budget}%")


def test_config4_sweep_three_steps_with_carried_caches():
    """Budgets from the drawn schedule, fresh features / Q / K / V rows per step, caches carried over."""
    w = synth.WORKLOADS["cfg4"]
    sched = synth.budget_schedule(0, 50)[:3]
    layer = LayerStep(w.N, w.H, w.D, w.torch_dtype, device=DEV)
    t = synth.make_layer_inputs(w, seed=0, device=DEV, step=0)
    host = _host(t)
    never_selected = np.ones(w.N, dtype=bool)       # rows whose cached output is still the seeded draw
    for s, pct in enumerate(sched):
        if s > 0:
            fresh = synth.make_layer_inputs(w, seed=0, device=DEV, step=s)
            for name in ("x_prev", "x_cur", "q", "k_new", "v_new"):
                t[name] = fresh[name]
                host[name] = to_np(fresh[name])
            del fresh
        kc, vc, e_idx = _check_step(w, t, host, layer, pct, n_rows=8, tag=f"cfg4 step {s} ({pct}%)",
                                    out_known=never_selected)
        # carry the oracle's own K/V caches; output rows selected once are no longer known to the oracle
        # in full (it recomputes samples only), so later steps compare them as "must not move" only
        host["k_cache"], host["v_cache"] = kc.reshape(w.N, w.H, w.D), vc.reshape(w.N, w.H, w.D)
        never_selected[e_idx] = False


def test_budget_zero_and_full():
    """Budget 0% leaves every cache unchanged; budget 100% is dense attention for every token."""
    w0 = synth.WORKLOADS["cfg2"]
    w = synth.Workload("small", "bf16", 1000, 4, 128, 512, (0, 100), "drift")
    t = synth.make_layer_inputs(w, seed=1, device=DEV)
    host = _host(t)
    layer = LayerStep(w.N, w.H, w.D, w.torch_dtype, device=DEV)
    layer.run(t, 0)
    torch.cuda.synchronize()
    for name in ("k_cache", "v_cache", "out_cache"):
        assert np.array_equal(to_np(t[name]), host[name]), name
    _check_step(w, t, host, layer, 100, n_rows=10**9, tag="budget100")
    assert w0.N == 17550
