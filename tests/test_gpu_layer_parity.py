"""End-to-end layer-step parity at the benchmark configurations, through the C ABI, in the launch
configuration bench.py times (paper_2506_05096_amd.layer.LayerStep).

Config 0 is checked in full.  At the larger configurations the oracle recomputes every score, every
selected index, every refreshed K/V row and every untouched cache row, and the attention output on a
sample of selected rows (rows are independent: each is an exact softmax row over all N keys): the first and
last selected token, both sides of the last query-tile edges (the last tile is partly filled), rows of
work items that the budget-aware launch cuts into key ranges, and random ones.  bf16 results must be within
relative L2 1e-2 of the oracle over the whole sample and for every (row, head) by itself.
"""
import numpy as np
import pytest
import torch

import oracle
from conftest import assert_rel_l2, bf16_bits_to_f64, to_np
from paper_2506_05096_amd import binding as ab
from paper_2506_05096_amd import synth
from paper_2506_05096_amd.layer import LayerStep

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _f64(a):
    return bf16_bits_to_f64(a) if a.dtype == np.uint16 else a.astype(np.float64)


Q_TILE = 256        # selected queries per work item of the bf16 attention launch


def _split_item_rows(n, H, k):
    """Positions (in the selected list) whose query tile belongs, for at least one head, to a work item that the
    launch plan cuts into key ranges: work items are (head, query tile) pairs, head-major, XCD x owns items
    [x * items_per_xcd, (x + 1) * items_per_xcd) and the items past the first full_items of each XCD are cut."""
    plan = ab.astraea_attn_plan(n, H, k)
    rows = set()
    if plan["splits"] > 1:
        for xcd in range(8):
            for item in range(xcd * plan["items_per_xcd"] + plan["full_items"], (xcd + 1) * plan["items_per_xcd"]):
                if item < H * plan["q_tiles"]:
                    qt = item % plan["q_tiles"]
                    rows.update(r for r in (qt * Q_TILE, qt * Q_TILE + 97, qt * Q_TILE + Q_TILE - 1) if r < k)
    return sorted(rows)


def _sample_rows(n, H, k, n_rows, seed, bf16):
    """Positions in the selected list: the ends, both sides of the last three query-tile edges, a few rows of the
    work items the launch cuts along the keys, and random ones up to n_rows."""
    rng = np.random.default_rng(seed)
    fixed = {0, 1, k - 2, k - 1}
    last_edge = (k // Q_TILE) * Q_TILE
    for e in (last_edge, last_edge - Q_TILE, last_edge - 2 * Q_TILE):
        fixed.update((e - 1, e, e + 1))
    if bf16:
        split = _split_item_rows(n, H, k)
        if split:
            fixed.update(int(r) for r in rng.choice(split, size=min(len(split), 12), replace=False))
    fixed = {r for r in fixed if 0 <= r < k}
    pool = np.setdiff1d(np.arange(k), np.fromiter(fixed, dtype=np.int64), assume_unique=False)
    extra = rng.choice(pool, size=min(len(pool), max(0, n_rows - len(fixed))), replace=False)
    return np.array(sorted(fixed | set(int(e) for e in extra)), dtype=np.int64)


# oracle attention rows already computed in this session, for cases that run the same inputs twice
# (the fused and the unfused step): keyed by the caller, checked against the indices before reuse
_ORACLE_ROWS = {}


def _check_step(w, t, host, layer, budget_pct, n_rows, tag, out_known=None, reuse_key=None):
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
    rows = np.arange(k) if n_rows >= k else _sample_rows(n, H, k, n_rows, seed=n + k, bf16=w.dtype == "bf16")
    cached = _ORACLE_ROWS.get(reuse_key) if reuse_key else None
    if cached is not None and np.array_equal(cached[0], e_idx[rows]):
        o64 = cached[1]        # same inputs, same indices (all checked bit for bit above): the same oracle rows
    else:
        o64, _ = oracle.sparse_attn(host["q"], kc.reshape(n, H, D), vc.reshape(n, H, D), e_idx[rows], layer.scale)
        if reuse_key:
            _ORACLE_ROWS[reuse_key] = (e_idx[rows].copy(), o64)
    g64 = _f64(got[e_idx[rows]]).reshape(len(rows), H, D)
    assert np.all(np.isfinite(g64))
    if w.dtype == "f32":
        err = float(np.max(np.abs(g64 - o64)))
        assert err <= 1e-4, f"{tag}: max abs error {err}"
    else:
        err, worst = assert_rel_l2(g64, o64, tag=tag)       # whole sample, and every (row, head) by itself
        print(f"{tag}: worst (row, head) relative L2 {worst:.3g}", flush=True)
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
    _check_step(w, t, _host(t), layer, budget, n_rows=256, tag=f"cfg1@{budget}%")


@pytest.mark.parametrize("fused", [False, True])
def test_config2_480p(fused):
    w = synth.WORKLOADS["cfg2"]
    t = synth.make_layer_inputs(w, seed=0, device=DEV)
    layer = LayerStep(w.N, w.H, w.D, w.torch_dtype, device=DEV, fused_update=fused)
    _check_step(w, t, _host(t), layer, 40, n_rows=256, tag="cfg2" + ("/fused" if fused else ""),
                reuse_key=("cfg2", 0, 40))


@pytest.mark.parametrize("fused", [False, True])
def test_config3_720p_headline(fused):
    w = synth.WORKLOADS["cfg3"]
    t = synth.make_layer_inputs(w, seed=0, device=DEV)
    layer = LayerStep(w.N, w.H, w.D, w.torch_dtype, device=DEV, fused_update=fused)
    _check_step(w, t, _host(t), layer, 30, n_rows=256, tag="cfg3" + ("/fused" if fused else ""),
                reuse_key=("cfg3", 0, 30))


@pytest.mark.parametrize("budget", [10, 100])
def test_config3_at_the_ends_of_the_budget_range(budget):
    """The headline shape at the smallest budget of the schedule (the launch plan with the largest share of split
    work items) and at 100 % (dense attention for every token)."""
    w = synth.WORKLOADS["cfg3"]
    t = synth.make_layer_inputs(w, seed=0, device=DEV)
    layer = LayerStep(w.N, w.H, w.D, w.torch_dtype, device=DEV)
    _check_step(w, t, _host(t), layer, budget, n_rows=256, tag=f"cfg3@{budget}%")


def _first_visit_order(schedule):
    """The budget levels in the order the drawn schedule first reaches them."""
    seen = []
    for pct in schedule:
        if pct not in seen:
            seen.append(pct)
    return seen


CFG4_LEVELS = _first_visit_order(synth.budget_schedule(0, 50))


class _Sweep:
    """State of the config-4 run carried from one parametrised case to the next: the layer, the device tensors,
    their host copies as the oracle sees them, and which cached output rows are still the seeded draw."""
    layer = None
    t = None
    host = None
    never_selected = None
    step = 0


@pytest.mark.parametrize("budget", CFG4_LEVELS)
def test_config4_every_budget_level_with_carried_caches(budget):
    """Config 4 at full size: one step per budget level 10 %, 20 %, ..., 100 % (in the order the drawn 50-step
    schedule first reaches them), fresh features / Q / K / V rows per step, the K/V and output caches carried
    from step to step on both sides.  Every level has its own launch plan (items per XCD, how many are cut
    into key ranges, how many ranges), so every level is checked: scores, indices, K/V caches and untouched
    rows in full and bit for bit, the attention on 64 sampled rows including rows of cut work items."""
    w = synth.WORKLOADS["cfg4"]
    assert sorted(CFG4_LEVELS) == list(range(10, 101, 10))
    sw = _Sweep
    if sw.layer is None:
        sw.layer = LayerStep(w.N, w.H, w.D, w.torch_dtype, device=DEV)
        sw.t = synth.make_layer_inputs(w, seed=0, device=DEV, step=0)
        sw.host = _host(sw.t)
        sw.never_selected = np.ones(w.N, dtype=bool)      # rows whose cached output is still the seeded draw
    else:
        fresh = synth.make_layer_inputs(w, seed=0, device=DEV, step=sw.step)
        for name in ("x_prev", "x_cur", "q", "k_new", "v_new"):
            sw.t[name] = fresh[name]
            sw.host[name] = to_np(fresh[name])
        del fresh
    kc, vc, e_idx = _check_step(w, sw.t, sw.host, sw.layer, budget, n_rows=64,
                                tag=f"cfg4 step {sw.step} ({budget}%)", out_known=sw.never_selected)
    # carry the oracle's own K/V caches; output rows selected once are no longer known to the oracle
    # in full (it recomputes samples only), so later steps compare them as "must not move" only
    sw.host["k_cache"], sw.host["v_cache"] = kc.reshape(w.N, w.H, w.D), vc.reshape(w.N, w.H, w.D)
    sw.never_selected[e_idx] = False
    sw.step += 1
    if sw.step == len(CFG4_LEVELS):                       # release 12 GB of device and host memory
        sw.layer = sw.t = sw.host = sw.never_selected = None
        sw.step = 0
        torch.cuda.empty_cache()


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
