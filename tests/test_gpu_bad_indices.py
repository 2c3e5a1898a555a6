"""Indices outside [0, N) in idx_sel are a caller's mistake, but they must never become an access outside the
buffers: a row read through such an index reads some valid row, a row written through one is dropped.  Every
indexed buffer here is a view into the middle of a larger allocation, so a write that slipped through would land
in the guard rows around it and show up as a changed bit (the bad indices are kept within the guard rows'
reach for that reason).  Rows with valid indices are checked against the oracle as usual."""
import math

import numpy as np
import pytest
import torch

import oracle
from conftest import assert_rel_l2, bf16_bits_to_f64, to_np
from paper_2506_05096_amd import binding as ab

pytestmark = pytest.mark.gpu
DEV = "cuda"
G = 4                                                   # guard rows on either side


def _f64(a):
    return bf16_bits_to_f64(a) if a.dtype == np.uint16 else a.astype(np.float64)


def _guarded(n, cols, dtype, gen):
    """[n + 2G, cols] on the device, its host copy, and the [n, cols] view in the middle."""
    big = torch.randn(n + 2 * G, cols, generator=gen).to(dtype)
    dev = big.to(DEV)
    return dev, to_np(big).copy(), dev[G:G + n]


def _indices(n, k, seed):
    """k entries: ascending valid indices with a few bad ones planted at the ends and in the middle."""
    rng = np.random.default_rng(seed)
    idx = np.sort(rng.choice(n, size=k, replace=False)).astype(np.int32)
    bad_pos = np.array([0, 1, k // 2, k - 2, k - 1])
    idx[bad_pos] = np.array([-1, -G, n, n + 1, n + G - 1], dtype=np.int32)
    good = np.ones(k, dtype=bool)
    good[bad_pos] = False
    return idx, good


def _guards_untouched(dev_big, host_big, n):
    got = to_np(dev_big)
    return np.array_equal(got[:G], host_big[:G]) and np.array_equal(got[G + n:], host_big[G + n:])


@pytest.mark.parametrize("dtype,e", [(torch.bfloat16, 512), (torch.float32, 100), (torch.bfloat16, 5)])
def test_row_movers_drop_rows_with_bad_indices(dtype, e):
    n, k = 300, 90
    g = torch.Generator().manual_seed(e)
    idx, good = _indices(n, k, seed=e)
    didx = torch.from_numpy(idx).to(DEV)
    # scatter of compact rows
    cbig, chost, cache = _guarded(n, e, dtype, g)
    src = torch.randn(k, e, generator=g).to(dtype)
    ab.astraea_scatter_update(cache, src.to(DEV), didx, k, src_is_full=False)
    torch.cuda.synchronize()
    exp = chost[G:G + n].copy()
    exp[idx[good]] = to_np(src)[good]
    assert np.array_equal(to_np(cache), exp) and _guards_untouched(cbig, chost, n)
    # scatter of rows of a full-length source
    cbig, chost, cache = _guarded(n, e, dtype, g)
    sbig, shost, full = _guarded(n, e, dtype, g)
    ab.astraea_scatter_update(cache, full, didx, k, src_is_full=True)
    torch.cuda.synchronize()
    exp = chost[G:G + n].copy()
    exp[idx[good]] = shost[G:G + n][idx[good]]
    assert np.array_equal(to_np(cache), exp) and _guards_untouched(cbig, chost, n)
    # gather: rows of bad indices keep what the destination held
    dst0 = torch.randn(k, e, generator=g).to(dtype)
    dst = dst0.to(DEV)
    ab.astraea_gather_rows(full, dst, didx, k)
    torch.cuda.synchronize()
    exp = to_np(dst0).copy()
    exp[good] = shost[G:G + n][idx[good]]
    assert np.array_equal(to_np(dst), exp)


def test_lse_weight_update_drops_bad_indices():
    n, k, h = 200, 40, 3
    g = torch.Generator().manual_seed(5)
    idx, good = _indices(n, k, seed=5)
    wbig = torch.rand(n + 2 * G, generator=g)
    whost = wbig.numpy().copy()
    wdev = wbig.to(DEV)
    lse = torch.randn(k, h, generator=g) + math.log(n)
    ab.astraea_lse_weight_update(lse.to(DEV), torch.from_numpy(idx).to(DEV), k, wdev[G:G + n])
    torch.cuda.synchronize()
    want = whost[G:G + n].copy()
    oracle.lse_weight_update(want, lse.numpy()[good], idx[good])
    got = wdev.cpu().numpy()
    assert np.array_equal(got[:G], whost[:G]) and np.array_equal(got[G + n:], whost[G + n:])
    rest = np.setdiff1d(np.arange(n), idx[good])
    assert np.array_equal(got[G:G + n][rest], want[rest])
    assert np.allclose(got[G:G + n][idx[good]], want[idx[good]], rtol=1e-5, atol=0.0)


@pytest.mark.parametrize("dtype,d", [(torch.bfloat16, 128), (torch.float32, 64)])
def test_attention_reads_and_writes_stay_inside_the_buffers(dtype, d):
    n, h, k = 700, 2, 300
    e = h * d
    g = torch.Generator().manual_seed(d)
    idx, good = _indices(n, k, seed=d)
    didx = torch.from_numpy(idx).to(DEV)
    qbig, qhost, q = _guarded(n, e, dtype, g)
    kk = torch.randn(n, h, d, generator=g).to(dtype)
    vv = torch.randn(n, h, d, generator=g).to(dtype)
    scale = 1.0 / math.sqrt(d)
    wsb = ab.workspace_bytes(ab.OP_SPARSE_ATTN, n, k, h, d)
    ws = torch.empty(max(wsb, 1), dtype=torch.uint8, device=DEV) if wsb else None
    eo, _ = oracle.sparse_attn(qhost[G:G + n].reshape(n, h, d), to_np(kk), to_np(vv), idx[good], scale)

    def close(got):
        got = _f64(got).reshape(-1, h, d)
        if dtype == torch.float32:
            return np.max(np.abs(got - eo)) <= 1e-4
        assert_rel_l2(got, eo, tag="rows of valid indices")       # whole result and every (row, head)
        return True

    # gathered queries, compact output: rows of valid indices are right, the others hold finite numbers
    o = torch.zeros(k, h, d, dtype=dtype, device=DEV)
    ab.astraea_sparse_attn_fwd(q.view(n, h, d), kk.to(DEV), vv.to(DEV), didx, k, o, scale, workspace=ws)
    torch.cuda.synchronize()
    got = to_np(o)
    assert close(got[good]) and np.all(np.isfinite(_f64(got)))
    # straight into the cached output: rows of bad indices are written nowhere
    cbig, chost, cache = _guarded(n, e, dtype, g)
    ab.astraea_sparse_attn_update_fwd(q.view(n, h, d), kk.to(DEV), vv.to(DEV), didx, k, cache, scale, workspace=ws)
    torch.cuda.synchronize()
    assert _guards_untouched(cbig, chost, n)
    got = to_np(cache)
    rest = np.setdiff1d(np.arange(n), idx[good])
    assert np.array_equal(got[rest], chost[G:G + n][rest])
    assert close(got[idx[good]])


def test_sparse_linear_reads_and_writes_stay_inside_the_buffers():
    n, k, c_in, c_out = 500, 300, 128, 264
    g = torch.Generator().manual_seed(9)
    idx, good = _indices(n, k, seed=9)
    didx = torch.from_numpy(idx).to(DEV)
    xbig, xhost, x = _guarded(n, c_in, torch.bfloat16, g)
    w = (torch.randn(c_out, c_in, generator=g) / math.sqrt(c_in)).to(torch.bfloat16)
    want = oracle.sparse_linear(xhost[G:G + n], to_np(w), idx[good])

    def close(got):
        got = _f64(got)
        assert_rel_l2(got, want, tag="rows of valid indices")     # whole result and every row
        return True

    y = torch.zeros(k, c_out, dtype=torch.bfloat16, device=DEV)
    ab.astraea_sparse_linear(x, w.to(DEV), None, didx, k, y)
    torch.cuda.synchronize()
    assert close(to_np(y)[good]) and np.all(np.isfinite(_f64(to_np(y))))
    ybig, yhost, yc = _guarded(n, c_out, torch.bfloat16, g)
    ab.astraea_sparse_linear(x, w.to(DEV), None, didx, k, yc, y_is_compact=False)
    torch.cuda.synchronize()
    assert _guards_untouched(ybig, yhost, n)
    got = to_np(yc)
    rest = np.setdiff1d(np.arange(n), idx[good])
    assert np.array_equal(got[rest], yhost[G:G + n][rest])
    assert close(got[idx[good]])


def test_check_indices_counts_what_breaks_the_contract():
    n = 5000
    counts = torch.full((2,), -7, dtype=torch.int32, device=DEV)
    good = torch.arange(0, n, 3, dtype=torch.int32)
    ab.astraea_check_indices(good.to(DEV), good.numel(), n, counts)
    assert counts.cpu().tolist() == [0, 0]
    bad = good.clone()
    bad[10], bad[11], bad[500], bad[700] = -1, n, bad[499], bad[650]       # 2 out of range; 4 order breaks, see below
    ab.astraea_check_indices(bad.to(DEV), bad.numel(), n, counts)
    b = bad.numpy().astype(np.int64)
    assert counts.cpu().tolist() == [int(((b < 0) | (b >= n)).sum()), int((b[1:] <= b[:-1]).sum())]
    assert counts.cpu().tolist()[0] == 2 and counts.cpu().tolist()[1] >= 3
    # what astraea_select_topk emits passes
    score = torch.rand(n, generator=torch.Generator().manual_seed(1)).to(DEV)
    idx = torch.empty(n, dtype=torch.int32, device=DEV)
    ws = torch.empty(ab.workspace_bytes(ab.OP_SELECT_TOPK, n), dtype=torch.uint8, device=DEV)
    ab.astraea_select_topk(score, 1234, idx, ws)
    ab.astraea_check_indices(idx, 1234, n, counts)
    assert counts.cpu().tolist() == [0, 0]
    ab.astraea_check_indices(None, 0, n, counts)                             # empty list: counts cleared
    assert counts.cpu().tolist() == [0, 0]
