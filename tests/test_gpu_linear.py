"""GPU parity of astraea_sparse_linear (per-token layers on the selected rows; paper Algorithm 1, query
projection step, and the projection / MLP terms of the FLOPs appendix) against the fp64 oracle.

Bar: the kernel accumulates bf16 products in fp32 and rounds once to bf16, so every output must lie within
one bf16 rounding (2^-8 relative) of the fp64 value plus the fp32 accumulation error; relative L2 <= 1e-2 as
for the attention.  Rows that are not selected, and columns past c_out in a wider row, keep their bits.
"""
import numpy as np
import pytest
import torch

import oracle
from conftest import assert_rel_l2, bf16_bits_to_f64, to_np
from paper_2506_05096_amd import binding as ab

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _case(n, cin, cout, k_sel, seed, scale_w=None):
    g = torch.Generator().manual_seed(seed)
    x = torch.randn(n, cin, generator=g).bfloat16()
    w = (torch.randn(cout, cin, generator=g) * (scale_w or cin ** -0.5)).bfloat16()
    b = torch.randn(cout, generator=g).bfloat16()
    idx = torch.randperm(n, generator=g)[:k_sel].sort().values.to(torch.int32)
    return x, w, b, idx


def _check(got_bits, ref64, cin):
    got = bf16_bits_to_f64(got_bits)
    rel, _ = assert_rel_l2(got, ref64, tag="sparse linear")        # whole result, and every row by itself
    # element-wise: half an ulp of bf16 (2^-9 relative) for the one rounding, doubled for slack, plus fp32 accumulation
    tol = 2.0 ** -8 * np.abs(ref64) + 1e-6 * cin
    assert np.all(np.abs(got - ref64) <= tol), float(np.max(np.abs(got - ref64) - tol))
    return rel


@pytest.mark.parametrize("n,cin,cout,k_sel", [
    (1000, 128, 264, 333),      # ragged in both tile directions
    (700, 3072, 512, 700),      # the path's feature width, every token selected
    (5000, 256, 1024, 1500),    # several token tiles x several feature tiles
    (64, 64, 8, 1),             # smallest legal shape
    (300, 192, 256, 257),       # one row past a token tile
])
@pytest.mark.parametrize("act", [ab.ACT_NONE, ab.ACT_GELU_TANH])
def test_sparse_linear_gathered_input_compact_output(n, cin, cout, k_sel, act):
    x, w, b, idx = _case(n, cin, cout, k_sel, seed=n + cin)
    ref = oracle.sparse_linear(to_np(x), to_np(w), idx.numpy(), bias=to_np(b), act=act)
    y = torch.full((k_sel, cout), float("nan"), dtype=torch.bfloat16, device=DEV)
    ab.astraea_sparse_linear(x.to(DEV), w.to(DEV), b.to(DEV), idx.to(DEV), k_sel, y, act=act)
    torch.cuda.synchronize()
    _check(to_np(y), ref, cin)


def test_sparse_linear_all_row_modes_agree_bit_for_bit():
    n, cin, cout, k_sel, pad = 2100, 512, 384, 777, 40
    x, w, b, idx = _case(n, cin, cout, k_sel, seed=9)
    dx, dw, db, di = x.to(DEV), w.to(DEV), b.to(DEV), idx.to(DEV)
    ref = oracle.sparse_linear(to_np(x), to_np(w), idx.numpy(), bias=to_np(b))
    # gathered in, compact out
    y0 = torch.empty(k_sel, cout, dtype=torch.bfloat16, device=DEV)
    ab.astraea_sparse_linear(dx, dw, db, di, k_sel, y0)
    # compact in, compact out, no index list at all
    y1 = torch.empty(k_sel, cout, dtype=torch.bfloat16, device=DEV)
    ab.astraea_sparse_linear(dx[di.long()].contiguous(), dw, db, None, k_sel, y1, x_is_compact=True)
    # gathered in, scattered out into a wider cached buffer (the projection fused with the cache refresh)
    g = torch.Generator().manual_seed(1)
    cache0 = torch.randn(n, cout + pad, generator=g).bfloat16()
    cache = cache0.to(DEV)
    ab.astraea_sparse_linear(dx, dw, db, di, k_sel, cache[:, :cout], y_is_compact=False)
    # compact in, scattered out
    cache2 = cache0.to(DEV)
    ab.astraea_sparse_linear(dx[di.long()].contiguous(), dw, db, di, k_sel, cache2[:, :cout], x_is_compact=True,
                             y_is_compact=False, N=n)
    torch.cuda.synchronize()
    _check(to_np(y0), ref, cin)
    a0 = to_np(y0)
    assert np.array_equal(a0, to_np(y1))
    c, c2 = to_np(cache), to_np(cache2)
    assert np.array_equal(c[idx.numpy()][:, :cout], a0) and np.array_equal(c, c2)
    rest = np.setdiff1d(np.arange(n), idx.numpy())
    assert np.array_equal(c[rest], to_np(cache0)[rest])                    # unselected rows untouched
    assert np.array_equal(c[:, cout:], to_np(cache0)[:, cout:])            # padding columns untouched
    # no bias is the same as a zero bias
    y2 = torch.empty(k_sel, cout, dtype=torch.bfloat16, device=DEV)
    y3 = torch.empty(k_sel, cout, dtype=torch.bfloat16, device=DEV)
    ab.astraea_sparse_linear(dx, dw, None, di, k_sel, y2)
    ab.astraea_sparse_linear(dx, dw, torch.zeros_like(db), di, k_sel, y3)
    torch.cuda.synchronize()
    assert np.array_equal(to_np(y2), to_np(y3))


@pytest.mark.parametrize("n,cin,cout,k_sel,act", [
    (9000, 256, 4104, 8200, ab.ACT_GELU_TANH),     # 33 x 17 tiles, both ragged, a short contraction
    (70000, 384, 3072, 33000, ab.ACT_NONE),        # 129 x 12 tiles: the super-block rows end in a partly filled one
])
def test_sparse_linear_many_tiles_per_compute_unit(n, cin, cout, k_sel, act):
    """Shapes with several tiles per compute unit (several rounds of workgroups, super-block rows that end in a
    partly filled one): gathered input, rows scattered into a wider cached buffer, ragged last tiles in both
    directions.  Checked against the oracle on sampled rows (all features), for untouched rows and padding in
    full, and against the compact form bit for bit."""
    x, w, b, idx = _case(n, cin, cout, k_sel, seed=n + cout)
    pad = 24
    g = torch.Generator().manual_seed(5)
    cache0 = torch.randn(n, cout + pad, generator=g).bfloat16()
    cache = cache0.to(DEV)
    dx, dw, db, di = x.to(DEV), w.to(DEV), b.to(DEV), idx.to(DEV)
    ab.astraea_sparse_linear(dx, dw, db, di, k_sel, cache[:, :cout], act=act, y_is_compact=False)
    y = torch.full((k_sel, cout), float("nan"), dtype=torch.bfloat16, device=DEV)
    ab.astraea_sparse_linear(dx, dw, db, di, k_sel, y, act=act)
    torch.cuda.synchronize()
    c, yc = to_np(cache), to_np(y)
    assert np.array_equal(c[idx.numpy()][:, :cout], yc)
    rest = np.setdiff1d(np.arange(n), idx.numpy())
    assert np.array_equal(c[rest], to_np(cache0)[rest]) and np.array_equal(c[:, cout:], to_np(cache0)[:, cout:])
    rng = np.random.default_rng(1)
    rows = np.unique(np.concatenate([[0, 1, 255, 256, 257, k_sel - 257, k_sel - 256, k_sel - 2, k_sel - 1],
                                     (k_sel // 256) * 256 + np.array([-1, 0, 1]), rng.integers(0, k_sel, 300)]))
    rows = rows[(rows >= 0) & (rows < k_sel)]
    ref = oracle.sparse_linear(to_np(x)[idx.numpy()[rows]], to_np(w), None, bias=to_np(b), act=act, x_is_compact=True)
    _check(yc[rows], ref, cin)


def test_sparse_linear_closed_forms_on_gpu():
    n, c = 500, 256
    g = torch.Generator().manual_seed(3)
    x = torch.randn(n, c, generator=g).bfloat16()
    idx = torch.arange(3, n, 7, dtype=torch.int32)
    k_sel = idx.numel()
    # identity weight: the layer is a gather, exactly
    y = torch.empty(k_sel, c, dtype=torch.bfloat16, device=DEV)
    ab.astraea_sparse_linear(x.to(DEV), torch.eye(c).bfloat16().to(DEV), None, idx.to(DEV), k_sel, y)
    torch.cuda.synchronize()
    assert np.array_equal(to_np(y), to_np(x)[idx.numpy()])
    # a weight row that is a unit vector picks one input column (catches a transposed or mis-swizzled operand)
    w = torch.zeros(c, c)
    perm = torch.randperm(c, generator=g)
    w[torch.arange(c), perm] = 1.0
    ab.astraea_sparse_linear(x.to(DEV), w.bfloat16().to(DEV), None, idx.to(DEV), k_sel, y)
    torch.cuda.synchronize()
    assert np.array_equal(to_np(y), to_np(x)[idx.numpy()][:, perm.numpy()])
    # k_sel = 0 writes nothing
    y.fill_(7.0)
    ab.astraea_sparse_linear(x.to(DEV), w.bfloat16().to(DEV), None, idx.to(DEV), 0, y)
    torch.cuda.synchronize()
    assert torch.all(y == 7.0)


def test_sparse_linear_rejects_what_it_cannot_do():
    x = torch.zeros(64, 96, dtype=torch.bfloat16, device=DEV)
    w = torch.zeros(8, 96, dtype=torch.bfloat16, device=DEV)
    y = torch.zeros(64, 8, dtype=torch.bfloat16, device=DEV)
    with pytest.raises(ab.AstraeaError) as e:
        ab.astraea_sparse_linear(x, w, None, None, 64, y, x_is_compact=True)       # c_in not a multiple of 64
    assert e.value.status == ab.ERR_UNSUPPORTED
    xf = torch.zeros(64, 96, device=DEV)
    with pytest.raises(ab.AstraeaError) as e:
        ab.astraea_sparse_linear(xf, torch.zeros(8, 96, device=DEV), None, None, 64, torch.zeros(64, 8, device=DEV),
                                 x_is_compact=True)                                 # the same rule in fp32
    assert e.value.status == ab.ERR_UNSUPPORTED


# ------------------------------------------------------------------- fp32 mode --

@pytest.mark.parametrize("n,cin,cout,k_sel", [
    (4096, 512, 512, 2048),     # the fp32 configuration's width and budget
    (1000, 128, 264, 333),      # ragged in both tile directions
    (300, 192, 1536, 257),      # one row past a token tile, several feature tiles
    (64, 64, 8, 1),             # smallest legal shape
    (700, 3072, 128, 130),      # long contraction
])
@pytest.mark.parametrize("act", [ab.ACT_NONE, ab.ACT_GELU_TANH])
def test_sparse_linear_fp32_matches_oracle(n, cin, cout, k_sel, act):
    """fp32 in, fp32 accumulation on the fp32 matrix instruction, fp32 out: max-abs <= 1e-4 against the fp64
    oracle for outputs of order one (the bar of the fp32 attention)."""
    g = torch.Generator().manual_seed(n + cout)
    x = torch.randn(n, cin, generator=g)
    w = torch.randn(cout, cin, generator=g) * cin ** -0.5
    b = torch.randn(cout, generator=g)
    idx = torch.randperm(n, generator=g)[:k_sel].sort().values.to(torch.int32)
    ref = oracle.sparse_linear(x.numpy(), w.numpy(), idx.numpy(), bias=b.numpy(), act=act)
    y = torch.full((k_sel, cout), float("nan"), device=DEV)
    ab.astraea_sparse_linear(x.to(DEV), w.to(DEV), b.to(DEV), idx.to(DEV), k_sel, y, act=act)
    torch.cuda.synchronize()
    got = y.cpu().numpy().astype(np.float64)
    assert np.all(np.isfinite(got))
    assert np.max(np.abs(got - ref)) <= 1e-4, float(np.max(np.abs(got - ref)))


def test_sparse_linear_fp32_row_modes_agree_and_leave_other_rows_alone():
    n, cin, cout, k_sel, pad = 1300, 256, 200, 500, 24
    g = torch.Generator().manual_seed(4)
    x = torch.randn(n, cin, generator=g)
    w = torch.randn(cout, cin, generator=g) / 16.0
    idx = torch.randperm(n, generator=g)[:k_sel].sort().values.to(torch.int32)
    dx, dw, di = x.to(DEV), w.to(DEV), idx.to(DEV)
    y0 = torch.empty(k_sel, cout, device=DEV)
    ab.astraea_sparse_linear(dx, dw, None, di, k_sel, y0)
    y1 = torch.empty(k_sel, cout, device=DEV)
    ab.astraea_sparse_linear(dx[di.long()].contiguous(), dw, None, None, k_sel, y1, x_is_compact=True)
    cache0 = torch.randn(n, cout + pad, generator=g)
    cache = cache0.to(DEV)
    ab.astraea_sparse_linear(dx, dw, None, di, k_sel, cache[:, :cout], y_is_compact=False)
    ab.astraea_sparse_linear(dx, dw, None, di, 0, cache[:, :cout], y_is_compact=False)      # budget 0: nothing moves
    torch.cuda.synchronize()
    ref = oracle.sparse_linear(x.numpy(), w.numpy(), idx.numpy())
    assert np.max(np.abs(y0.cpu().numpy() - ref)) <= 1e-4
    assert np.array_equal(y0.cpu().numpy(), y1.cpu().numpy())
    got = cache.cpu().numpy()
    assert np.array_equal(got[idx.numpy()][:, :cout], y0.cpu().numpy())
    rest = np.setdiff1d(np.arange(n), idx.numpy())
    assert np.array_equal(got[rest], cache0.numpy()[rest])
    assert np.array_equal(got[:, cout:], cache0.numpy()[:, cout:])
