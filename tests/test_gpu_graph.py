"""A layer-step recorded as a HIP graph gives, on every replay, the bits the same calls give when launched one
by one: replays are interleaved with eager work and device synchronisations, each with new inputs copied into
the captured tensors, and each is compared with an eager run on separate buffers holding the same inputs."""
import numpy as np
import pytest
import torch

from conftest import to_np
from paper_2506_05096_amd import binding as ab
from paper_2506_05096_amd.layer import GraphedStep, LayerStep, StatefulLayer

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _inputs(n, h, d, c, dtype, seed):
    g = torch.Generator().manual_seed(seed)
    r = lambda *s: torch.randn(*s, generator=g).to(dtype).to(DEV)
    x_prev = r(n, c)
    return {"x_prev": x_prev, "x_cur": (x_prev.float() + 0.1 * r(n, c).float()).to(dtype),
            "q": r(n, h, d), "k_new": r(n, h, d), "v_new": r(n, h, d),
            "k_cache": r(n, h, d), "v_cache": r(n, h, d), "out_cache": r(n, h * d)}


@pytest.mark.parametrize("dtype,n,h,d,c,pct,fused", [
    (torch.bfloat16, 4100, 4, 128, 512, 30, False),     # ragged N, split work items in the attention
    (torch.bfloat16, 4100, 4, 128, 512, 70, True),
    (torch.float32, 1500, 2, 64, 256, 50, False),
])
def test_graph_replays_equal_eager_steps(dtype, n, h, d, c, pct, fused):
    lg = LayerStep(n, h, d, dtype, DEV, fused_update=fused)
    le = LayerStep(n, h, d, dtype, DEV, fused_update=fused)
    k = lg.budget_to_k(pct)
    tg = _inputs(n, h, d, c, dtype, seed=1)
    step = GraphedStep(lambda: lg.run(tg, k))           # the warm-up run advanced tg's caches once
    for rep in range(4):
        fresh = _inputs(n, h, d, c, dtype, seed=10 + rep)
        te = {name: v.clone() for name, v in fresh.items()}
        for name, v in fresh.items():
            tg[name].copy_(v)                            # same storage the graph recorded
        le.run(te, k)                                    # eager work between the replays
        torch.cuda.synchronize()
        step.replay()
        torch.cuda.synchronize()
        assert np.array_equal(lg.idx_sel[:k].cpu().numpy(), le.idx_sel[:k].cpu().numpy()), rep
        for name in ("k_cache", "v_cache", "out_cache"):
            assert np.array_equal(to_np(tg[name]), to_np(te[name])), (rep, name)


def test_graph_of_the_stateful_step_carries_its_state():
    """Counters, S_LSE weights and reference features live in the layer's own tensors, so consecutive replays
    advance them exactly like consecutive eager steps."""
    n, h, d, c, dtype = 3000, 2, 128, 256, torch.bfloat16
    table = torch.tensor([float(np.float32(np.exp(float(i)))) for i in range(16)])
    mk = lambda: StatefulLayer(n, h, d, c, dtype, table, w_alpha=1.0, w_beta=0.01, device=DEV)
    lg, le = mk(), mk()
    k = lg.budget_to_k(40)
    tg = _inputs(n, h, d, c, dtype, seed=2)
    te = {name: v.clone() for name, v in tg.items()}
    le.run(te, k)                                        # eager step 1 == the graph's warm-up run
    step = GraphedStep(lambda: lg.run(tg, k))
    for rep in range(3):
        fresh = _inputs(n, h, d, c, dtype, seed=20 + rep)
        for name in ("x_cur", "q", "k_new", "v_new"):
            tg[name].copy_(fresh[name])
            te[name].copy_(fresh[name])
        le.run(te, k)
        torch.cuda.synchronize()
        step.replay()
        torch.cuda.synchronize()
        assert np.array_equal(lg.idx_sel[:k].cpu().numpy(), le.idx_sel[:k].cpu().numpy()), rep
        assert np.array_equal(lg.skip_count.cpu().numpy(), le.skip_count.cpu().numpy()), rep
        assert np.array_equal(lg.lse_weight.cpu().numpy(), le.lse_weight.cpu().numpy()), rep
        assert np.array_equal(to_np(lg.x_ref), to_np(le.x_ref)), rep
        assert np.array_equal(to_np(tg["out_cache"]), to_np(te["out_cache"])), rep


def test_kernel_timer_skips_launches_made_under_capture():
    """Event records inside a capture would become graph nodes without a time of their own: with the timer on,
    a captured launch is not counted, the eager launch after it is."""
    n, h, d, c, dtype = 1500, 2, 128, 256, torch.bfloat16
    layer = LayerStep(n, h, d, dtype, DEV)
    k = layer.budget_to_k(50)
    t = _inputs(n, h, d, c, dtype, seed=3)
    layer.run(t, k)
    torch.cuda.synchronize()
    ab.kernel_timer(True)
    try:
        step = GraphedStep(lambda: layer.run(t, k), warm=False)
        assert ab.kernel_times_ms() == []
        step.replay()
        torch.cuda.synchronize()
        assert ab.kernel_times_ms() == []
        layer.run(t, k)
        torch.cuda.synchronize()
        ms = ab.kernel_times_ms()
        assert len(ms) == 1 and ms[0] > 0.0
    finally:
        ab.kernel_timer(False)
