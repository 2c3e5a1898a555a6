"""The whole token-wise block on the selected tokens (paper Sec. 3.2; Algorithm 1 steps 1-7 with the per-token
layers of the FLOPs appendix) against the oracle, stage by stage: every stage of the oracle starts from the bf16
values the GPU produced for the stage before it, so each comparison isolates one kernel."""
import math

import numpy as np
import pytest
import torch

import oracle
from conftest import assert_rel_l2, bf16_bits_to_f64, to_np
from paper_2506_05096_amd import binding as ab
from paper_2506_05096_amd.layer import TokenSparseBlock

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _close(got64, ref64, tag, heads=None):
    """relative L2 <= 1e-2 over the whole stage and for every row by itself (every (row, head) for the attention)."""
    if heads:
        got64, ref64 = got64.reshape(got64.shape[0], heads, -1), ref64.reshape(ref64.shape[0], heads, -1)
    assert_rel_l2(got64, ref64, tag=tag)


def test_block_matches_oracle_stage_by_stage():
    n, H, D, budget = 1300, 2, 128, 35
    E, hid = H * D, 4 * H * D
    g = torch.Generator().manual_seed(13)
    rnd = lambda *s, sc=1.0: (torch.randn(*s, generator=g) * sc).bfloat16()
    w = {"wq": rnd(E, E, sc=E ** -0.5), "wk": rnd(E, E, sc=E ** -0.5), "wv": rnd(E, E, sc=E ** -0.5),
         "wo": rnd(E, E, sc=E ** -0.5), "w1": rnd(hid, E, sc=E ** -0.5), "w2": rnd(E, hid, sc=hid ** -0.5),
         "bq": rnd(E, sc=0.1), "b1": rnd(hid, sc=0.1), "b2": rnd(E, sc=0.1)}
    t = {"x_prev": rnd(n, E), "k_cache": rnd(n, H, D), "v_cache": rnd(n, H, D), "out_cache": rnd(n, E)}
    t["x_in"] = (t["x_prev"].float() + 0.1 * torch.randn(n, E, generator=g)).bfloat16()
    host = {k_: to_np(v) for k_, v in t.items()}
    hw = {k_: to_np(v) for k_, v in w.items()}
    t = {k_: v.to(DEV) for k_, v in t.items()}
    blk = TokenSparseBlock(n, H, D, {k_: v.to(DEV) for k_, v in w.items()}, device=DEV)
    k = blk.budget_to_k(budget)
    blk.run(t, k)
    torch.cuda.synchronize()

    # selection: bit-exact
    so = oracle.score(host["x_in"], host["x_prev"], oracle.DELTA_L2)
    e_idx, e_rem, _ = oracle.topk(so, k)
    assert np.array_equal(blk.idx_sel[:k].cpu().numpy(), e_idx)
    # projections of the selected rows
    q_gpu = to_np(blk.q_sel.view(n, E)[:k])
    _close(bf16_bits_to_f64(q_gpu), oracle.sparse_linear(host["x_in"], hw["wq"], e_idx, bias=hw["bq"]), "Q projection")
    kc, vc = to_np(t["k_cache"]).reshape(n, E), to_np(t["v_cache"]).reshape(n, E)
    for got, name, wn in ((kc, "k_cache", "wk"), (vc, "v_cache", "wv")):
        ref = oracle.sparse_linear(host["x_in"], hw[wn], e_idx)
        _close(bf16_bits_to_f64(got[e_idx]), ref, "K/V projection into the cache")
        assert np.array_equal(got[e_rem], host[name].reshape(n, E)[e_rem])          # cached rows of the others kept
    # attention on the GPU's own Q and refreshed K/V
    o64, _ = oracle.sparse_attn(q_gpu.reshape(k, H, D), kc.reshape(n, H, D), vc.reshape(n, H, D), None,
                                1.0 / math.sqrt(D), q_is_compact=True)
    o_gpu = to_np(blk.o_sel.view(n, E)[:k])
    _close(bf16_bits_to_f64(o_gpu), o64.reshape(k, E), "attention", heads=H)
    # output projection, MLP
    h_gpu = to_np(blk.h_sel[:k])
    _close(bf16_bits_to_f64(h_gpu), oracle.sparse_linear(o_gpu, hw["wo"], None, x_is_compact=True), "output projection")
    m_gpu = to_np(blk.m_sel[:k])
    ref = oracle.sparse_linear(h_gpu, hw["w1"], None, bias=hw["b1"], act=oracle.ACT_GELU_TANH, x_is_compact=True)
    _close(bf16_bits_to_f64(m_gpu), ref, "MLP layer 1 (GELU)")
    out = to_np(t["out_cache"])
    ref = oracle.sparse_linear(m_gpu, hw["w2"], None, bias=hw["b2"], x_is_compact=True)
    _close(bf16_bits_to_f64(out[e_idx]), ref, "MLP layer 2 into the cached output")
    assert np.array_equal(out[e_rem], host["out_cache"][e_rem])                      # block output of the others reused


def test_block_budget_zero_changes_nothing():
    n, H, D = 300, 1, 128
    E = H * D
    g = torch.Generator().manual_seed(1)
    rnd = lambda *s: torch.randn(*s, generator=g).bfloat16().to(DEV)
    w = {"wq": rnd(E, E), "wk": rnd(E, E), "wv": rnd(E, E), "wo": rnd(E, E), "w1": rnd(4 * E, E), "w2": rnd(E, 4 * E)}
    t = {"x_prev": rnd(n, E), "x_in": rnd(n, E), "k_cache": rnd(n, H, D), "v_cache": rnd(n, H, D), "out_cache": rnd(n, E)}
    before = {k_: v.clone() for k_, v in t.items()}
    TokenSparseBlock(n, H, D, w, device=DEV).run(t, 0)
    torch.cuda.synchronize()
    for k_ in t:
        assert torch.equal(t[k_], before[k_]), k_


def test_block_at_the_headline_size_on_sampled_rows():
    """The block as bench.py runs it: N=118800, H=24, d=128, 30 % budget (k=35640), feature width 3072, MLP width
    12288.  The oracle cannot recompute all of it, but rows are independent: selection is checked in full and bit for
    bit, every stage on a sample of selected rows (first and last rows, rows on both sides of tile edges, random
    ones), each stage from the GPU's own output of the stage before."""
    from paper_2506_05096_amd import synth
    w = synth.WORKLOADS["cfg3"]
    n, H, D, E, hid = w.N, w.H, w.D, w.H * w.D, 4 * w.H * w.D
    t = synth.make_layer_inputs(w, seed=0, device=DEV)
    g = torch.Generator(device=DEV).manual_seed(77)
    mk = lambda o, i: (torch.randn(o, i, device=DEV, generator=g) * i ** -0.5).bfloat16()
    wts = {"wq": mk(E, E), "wk": mk(E, E), "wv": mk(E, E), "wo": mk(E, E), "w1": mk(hid, E), "w2": mk(E, hid),
           "bq": (torch.randn(E, device=DEV, generator=g) * 0.1).bfloat16(),
           "b1": (torch.randn(hid, device=DEV, generator=g) * 0.1).bfloat16()}
    tt = {"x_in": t["x_cur"], "x_prev": t["x_prev"], "k_cache": t["k_cache"], "v_cache": t["v_cache"],
          "out_cache": t["out_cache"]}
    before = {k_: to_np(tt[k_]).reshape(n, E).copy() for k_ in ("k_cache", "v_cache", "out_cache")}
    x_in, x_prev = to_np(tt["x_in"]), to_np(tt["x_prev"])
    hw = {k_: to_np(v) for k_, v in wts.items()}
    blk = TokenSparseBlock(n, H, D, wts, device=DEV)
    k = blk.budget_to_k(30)
    blk.run(tt, k)
    torch.cuda.synchronize()

    e_idx, e_rem, _ = oracle.topk(oracle.score(x_in, x_prev, oracle.DELTA_L2), k)
    assert np.array_equal(blk.idx_sel[:k].cpu().numpy(), e_idx)
    rng = np.random.default_rng(0)
    rows = np.unique(np.concatenate([[0, 1, 63, 64, 255, 256, 257, k - 257, k - 256, k - 2, k - 1],
                                     rng.integers(0, k, 13)]))
    tok = e_idx[rows]
    kc, vc, out = (to_np(tt[k_]).reshape(n, E) for k_ in ("k_cache", "v_cache", "out_cache"))
    for name, arr in (("k_cache", kc), ("v_cache", vc), ("out_cache", out)):
        assert np.array_equal(arr[e_rem], before[name][e_rem]), name                 # the others keep their cached rows
    xs = x_in[tok]
    q_gpu = to_np(blk.q_sel.view(n, E)[:k])[rows]
    _close(bf16_bits_to_f64(q_gpu), oracle.sparse_linear(xs, hw["wq"], None, bias=hw["bq"], x_is_compact=True), "Q projection")
    _close(bf16_bits_to_f64(kc[tok]), oracle.sparse_linear(xs, hw["wk"], None, x_is_compact=True), "K projection into the cache")
    _close(bf16_bits_to_f64(vc[tok]), oracle.sparse_linear(xs, hw["wv"], None, x_is_compact=True), "V projection into the cache")
    o64, _ = oracle.sparse_attn(q_gpu.reshape(len(rows), H, D), kc.reshape(n, H, D), vc.reshape(n, H, D), None,
                                1.0 / math.sqrt(D), q_is_compact=True)
    o_gpu = to_np(blk.o_sel.view(n, E)[:k])[rows]
    _close(bf16_bits_to_f64(o_gpu), o64.reshape(len(rows), E), "attention", heads=H)
    h_gpu = to_np(blk.h_sel[:k])[rows]
    _close(bf16_bits_to_f64(h_gpu), oracle.sparse_linear(o_gpu, hw["wo"], None, x_is_compact=True), "output projection")
    m_gpu = to_np(blk.m_sel[:k])[rows]
    ref = oracle.sparse_linear(h_gpu, hw["w1"], None, bias=hw["b1"], act=oracle.ACT_GELU_TANH, x_is_compact=True)
    _close(bf16_bits_to_f64(m_gpu), ref, "MLP layer 1 (GELU)")
    _close(bf16_bits_to_f64(out[tok]), oracle.sparse_linear(m_gpu, hw["w2"], None, x_is_compact=True), "MLP layer 2 into the cached output")


def test_block_with_packed_qkv_cache_equals_the_three_projection_form():
    """One stacked projection into a packed [N, 3, H, D] cache must give the bits of the three separate ones."""
    n, H, D = 1100, 2, 128
    E, hid = H * D, 4 * H * D
    g = torch.Generator().manual_seed(5)
    rnd = lambda *s, sc=1.0: (torch.randn(*s, generator=g) * sc).bfloat16().to(DEV)
    w = {"wq": rnd(E, E, sc=E ** -0.5), "wk": rnd(E, E, sc=E ** -0.5), "wv": rnd(E, E, sc=E ** -0.5),
         "wo": rnd(E, E, sc=E ** -0.5), "w1": rnd(hid, E, sc=E ** -0.5), "w2": rnd(E, hid, sc=hid ** -0.5)}
    x_prev = rnd(n, E)
    base = {"x_prev": x_prev, "x_in": (x_prev.float() + 0.1 * torch.randn(n, E, generator=g).to(DEV)).bfloat16(),
            "k_cache": rnd(n, H, D), "v_cache": rnd(n, H, D), "out_cache": rnd(n, E)}
    ta = {k_: v.clone() for k_, v in base.items()}
    blk = TokenSparseBlock(n, H, D, w, device=DEV)
    k = blk.budget_to_k(40)
    blk.run(ta, k)
    wp = dict(w, wqkv=torch.cat([w["wq"], w["wk"], w["wv"]], dim=0).contiguous())
    q_old = rnd(n, H, D)
    tb = {k_: v.clone() for k_, v in base.items() if k_ not in ("k_cache", "v_cache")}
    tb["qkv_cache"] = torch.stack([q_old, base["k_cache"], base["v_cache"]], dim=1).contiguous()
    blk2 = TokenSparseBlock(n, H, D, wp, device=DEV)
    blk2.run(tb, k)
    torch.cuda.synchronize()
    idx = blk.idx_sel[:k].long()
    assert torch.equal(blk.idx_sel[:k], blk2.idx_sel[:k])
    assert torch.equal(tb["qkv_cache"][:, 1], ta["k_cache"]) and torch.equal(tb["qkv_cache"][:, 2], ta["v_cache"])
    assert torch.equal(tb["qkv_cache"][idx, 0], blk.q_sel[:k])                 # fresh Q of the selected tokens
    rest = torch.ones(n, dtype=torch.bool, device=DEV)
    rest[idx] = False
    assert torch.equal(tb["qkv_cache"][rest, 0], q_old[rest])                  # the others keep what they had
    assert torch.equal(tb["out_cache"], ta["out_cache"])


def test_block_fp32_at_the_fp32_configuration():
    """The fp32 configuration (N=4096, 8 heads of 64, feature width 512, budget 50 %): the same chain in fp32,
    each stage from the GPU's own output of the stage before, max-abs <= 1e-4 per stage."""
    from paper_2506_05096_amd import synth
    wl = synth.WORKLOADS["cfg0"]
    n, H, D, E, hid = wl.N, wl.H, wl.D, wl.H * wl.D, 4 * wl.H * wl.D
    t = synth.make_layer_inputs(wl, seed=0, device=DEV)
    g = torch.Generator(device=DEV).manual_seed(5)
    mk = lambda o, i: torch.randn(o, i, device=DEV, generator=g) * i ** -0.5
    wts = {"wq": mk(E, E), "wk": mk(E, E), "wv": mk(E, E), "wo": mk(E, E), "w1": mk(hid, E), "w2": mk(E, hid),
           "bq": torch.randn(E, device=DEV, generator=g) * 0.1, "b1": torch.randn(hid, device=DEV, generator=g) * 0.1}
    tt = {"x_in": t["x_cur"], "x_prev": t["x_prev"], "k_cache": t["k_cache"], "v_cache": t["v_cache"],
          "out_cache": t["out_cache"]}
    before = {k_: to_np(tt[k_]).reshape(n, E).copy() for k_ in ("k_cache", "v_cache", "out_cache")}
    x_in, x_prev = to_np(tt["x_in"]), to_np(tt["x_prev"])
    hw = {k_: to_np(v) for k_, v in wts.items()}
    blk = TokenSparseBlock(n, H, D, wts, device=DEV, dtype=torch.float32)
    k = blk.budget_to_k(50)
    blk.run(tt, k)
    torch.cuda.synchronize()
    err = lambda got, ref: float(np.max(np.abs(got.astype(np.float64) - ref)))

    e_idx, e_rem, _ = oracle.topk(oracle.score(x_in, x_prev, oracle.DELTA_L2), k)
    assert np.array_equal(blk.idx_sel[:k].cpu().numpy(), e_idx)
    kc, vc, out = (to_np(tt[k_]).reshape(n, E) for k_ in ("k_cache", "v_cache", "out_cache"))
    for name, arr in (("k_cache", kc), ("v_cache", vc), ("out_cache", out)):
        assert np.array_equal(arr[e_rem], before[name][e_rem]), name
    q_gpu = to_np(blk.q_sel.view(n, E)[:k])
    assert err(q_gpu, oracle.sparse_linear(x_in, hw["wq"], e_idx, bias=hw["bq"])) <= 1e-4
    assert err(kc[e_idx], oracle.sparse_linear(x_in, hw["wk"], e_idx)) <= 1e-4
    assert err(vc[e_idx], oracle.sparse_linear(x_in, hw["wv"], e_idx)) <= 1e-4
    rows = np.unique(np.concatenate([[0, 1, 127, 128, k - 2, k - 1], np.random.default_rng(0).integers(0, k, 58)]))
    o64, _ = oracle.sparse_attn(q_gpu[rows].reshape(len(rows), H, D), kc.reshape(n, H, D), vc.reshape(n, H, D), None,
                                1.0 / math.sqrt(D), q_is_compact=True)
    o_gpu = to_np(blk.o_sel.view(n, E)[:k])
    assert err(o_gpu[rows], o64.reshape(len(rows), E)) <= 1e-4
    h_gpu = to_np(blk.h_sel[:k])
    assert err(h_gpu, oracle.sparse_linear(o_gpu, hw["wo"], None, x_is_compact=True)) <= 1e-4
    m_gpu = to_np(blk.m_sel[:k])
    ref = oracle.sparse_linear(h_gpu, hw["w1"], None, bias=hw["b1"], act=oracle.ACT_GELU_TANH, x_is_compact=True)
    assert err(m_gpu, ref) <= 1e-4
    assert err(out[e_idx], oracle.sparse_linear(m_gpu, hw["w2"], None, x_is_compact=True)) <= 1e-4
