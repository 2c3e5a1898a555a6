"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, and rejects bad arguments before any HIP call (so nothing is enqueued)."""
import ctypes as C
import re
from pathlib import Path

import pytest

from paper_2506_05096_amd import binding as ab
from paper_2506_05096_amd.build import ensure_built

ROOT = Path(__file__).resolve().parents[1]


@pytest.fixture(scope="module")
def L():
    ensure_built()
    return ab.lib()


def test_library_exports_every_declared_symbol(L):
    header = (ROOT / "include" / "astraea.h").read_text()
    declared = set(re.findall(r"\b(astraea_[a-z_0-9]+)\s*\(", header))
    assert declared == set(ab.EXPORTS), declared ^ set(ab.EXPORTS)
    for name in declared:
        assert getattr(L, name) is not None


def test_status_strings(L):
    assert L.astraea_status_string(0) == b"ok"
    for code in (-1, -2, -3, -4):
        assert len(L.astraea_status_string(code)) > 3
    assert L.astraea_status_string(-99) == b"unknown status"


def test_budget_to_k_and_flops(L):
    assert ab.astraea_budget_to_k(118800, 30) == 35640
    assert ab.astraea_budget_to_k(17550, 40) == 7020
    assert ab.astraea_budget_to_k(7, 50) == 4
    assert ab.astraea_budget_to_k(10, 0) == 0 and ab.astraea_budget_to_k(10, 100) == 10
    assert ab.astraea_budget_to_k(10, 101) == -1 and ab.astraea_budget_to_k(-1, 10) == -1
    # 4*k*N*D*H: the QK^T and AV terms of the paper's FLOPs appendix with one N replaced by k
    assert ab.astraea_attn_flops(118800, 35640, 24, 128) == 4.0 * 35640 * 118800 * 128 * 24
    # ratio to dense attention is the budget, as in the paper's FLOPs tables
    assert ab.astraea_attn_flops(1000, 400, 8, 64) / ab.astraea_attn_flops(1000, 1000, 8, 64) == 0.4


def test_workspace_sizes(L):
    w = ab.workspace_bytes(ab.OP_SELECT_TOPK, 118800)
    assert w % 256 == 0 and 8 * 1024 < w < 64 * 1024           # O(N / 2048) counters + a fixed histogram
    assert ab.workspace_bytes(ab.OP_SELECT_TOPK, 1) >= 8 * 1024
    assert ab.workspace_bytes(99, 1000) == 0
    # attention workspace is linear in N (a re-tiled copy of V plus a fixed area for split items): no N x N buffer
    wa = ab.workspace_bytes(ab.OP_SPARSE_ATTN, 118800, 35640, 24, 128)
    assert 118800 * 24 * 128 * 2 <= wa <= 118800 * 24 * 128 * 2 + (80 << 20)
    # fp32 path: partial results only when a small selection is cut along the keys (4 shares at the fp32
    # configuration: 4 x k x H x (D + 4) floats).  A selection that fills the chip by itself is not cut, but
    # the size named for k_sel also serves every smaller selection (which may be cut into more shares), so a
    # buffer sized once for the largest budget works at all of them: it never shrinks as k_sel grows, and
    # it stays a few MB (at most 2048 waves' worth of partial rows)
    assert ab.workspace_bytes(ab.OP_SPARSE_ATTN, 4096, 2048, 8, 64) == 4 * 2048 * 8 * 68 * 4
    for n, h, d in ((4096, 8, 64), (8192, 8, 64), (118800, 24, 64), (700, 3, 128)):
        sizes = [ab.workspace_bytes(ab.OP_SPARSE_ATTN, n, k, h, d) for k in range(1, n + 1, max(1, n // 97))]
        assert all(a <= b for a, b in zip(sizes, sizes[1:])), (n, h, d)
        assert sizes[-1] <= 8 * 65536 * (d + 4) * 4, (n, h, d)
    assert ab.workspace_bytes(ab.OP_SPARSE_ATTN, 118800, 35640, 24, 64) == 7 * 384 * 24 * 68 * 4     # 3 query tiles x 7 shares


FAKE = 0x10000   # a non-NULL, 256-byte aligned address; rejected calls must never touch it


def _err(L):
    return L.astraea_last_error().decode()


def test_score_rejects_bad_arguments(L):
    f = L.astraea_score
    assert f(FAKE, FAKE, 7, 10, 8, 8, 0, None, None, None, 0, 1.0, 0.0, FAKE, None) == ab.ERR_UNSUPPORTED
    assert f(FAKE, FAKE, ab.F32, 10, 8, 8, 5, None, None, None, 0, 1.0, 0.0, FAKE, None) == ab.ERR_INVALID
    assert f(FAKE, FAKE, ab.F32, -1, 8, 8, 0, None, None, None, 0, 1.0, 0.0, FAKE, None) == ab.ERR_INVALID
    assert f(FAKE, FAKE, ab.F32, 10, 0, 8, 0, None, None, None, 0, 1.0, 0.0, FAKE, None) == ab.ERR_INVALID
    assert f(FAKE, FAKE, ab.F32, 10, 8, 4, 0, None, None, None, 0, 1.0, 0.0, FAKE, None) == ab.ERR_INVALID
    assert "stride" in _err(L)
    assert f(None, FAKE, ab.F32, 10, 8, 8, 0, None, None, None, 0, 1.0, 0.0, FAKE, None) == ab.ERR_INVALID
    assert f(FAKE + 2, FAKE, ab.F32, 10, 8, 8, 0, None, None, None, 0, 1.0, 0.0, FAKE, None) == ab.ERR_INVALID
    # counters without a penalty table
    assert f(FAKE, FAKE, ab.F32, 10, 8, 8, 0, None, FAKE, None, 0, 1.0, 0.5, FAKE, None) == ab.ERR_INVALID
    # N == 0 is a valid no-op
    assert f(None, None, ab.F32, 0, 8, 8, 0, None, None, None, 0, 1.0, 0.0, None, None) == ab.OK


def test_select_topk_rejects_bad_arguments(L):
    f = L.astraea_select_topk
    big = 1 << 20
    assert f(FAKE, 10, 11, FAKE, None, None, None, FAKE, big, None) == ab.ERR_INVALID
    assert "k=11" in _err(L)
    assert f(FAKE, 10, -1, FAKE, None, None, None, FAKE, big, None) == ab.ERR_INVALID
    assert f(FAKE, -5, 0, FAKE, None, None, None, FAKE, big, None) == ab.ERR_INVALID
    assert f(None, 10, 3, FAKE, None, None, None, FAKE, big, None) == ab.ERR_INVALID
    assert f(FAKE, 10, 3, None, None, None, None, FAKE, big, None) == ab.ERR_INVALID
    assert f(FAKE, 10, 3, FAKE, None, None, None, None, big, None) == ab.ERR_WORKSPACE
    assert f(FAKE, 10, 3, FAKE, None, None, None, FAKE, 16, None) == ab.ERR_WORKSPACE
    assert f(FAKE, 10, 3, FAKE, None, None, None, FAKE + 8, big, None) == ab.ERR_WORKSPACE
    assert f(None, 0, 0, None, None, None, None, None, 0, None) == ab.OK


def test_kv_refresh_rejects_bad_arguments(L):
    f = L.astraea_kv_refresh
    f.restype = C.c_int
    assert f(FAKE, FAKE, FAKE, FAKE, 9, 100, 64, 64, 64, FAKE, 10, None) == ab.ERR_UNSUPPORTED
    assert f(FAKE, FAKE, FAKE, FAKE, ab.BF16, 100, 64, 32, 64, FAKE, 10, None) == ab.ERR_INVALID      # stride < row
    assert f(FAKE, None, FAKE, FAKE, ab.BF16, 100, 64, 64, 64, FAKE, 10, None) == ab.ERR_INVALID      # a NULL buffer
    assert f(FAKE, FAKE, FAKE, None, ab.BF16, 100, 64, 64, 64, FAKE, 10, None) == ab.ERR_INVALID
    assert f(FAKE, FAKE, FAKE, FAKE, ab.BF16, 100, 64, 64, 64, None, 10, None) == ab.ERR_INVALID      # no index list
    assert f(FAKE, FAKE, FAKE, FAKE, ab.BF16, 100, 64, 64, 64, FAKE, 101, None) == ab.ERR_INVALID     # k_sel > N
    assert f(None, None, None, None, ab.BF16, 100, 64, 64, 64, None, 0, None) == ab.OK                 # budget 0


def test_sparse_attn_rejects_bad_arguments(L):
    f = L.astraea_sparse_attn_fwd

    def call(dt=ab.BF16, N=100, H=2, D=128, qsn=256, qsh=128, ksn=256, ksh=128, idx=FAKE, k_sel=10, compact=0,
             scale=0.1, q=FAKE, k=FAKE, v=FAKE, o=FAKE):
        return f(q, k, v, dt, N, H, D, qsn, qsh, ksn, ksh, idx, k_sel, compact, scale, o, None, None, 0, None)

    assert call(dt=3) == ab.ERR_UNSUPPORTED
    assert call(D=64) == ab.ERR_UNSUPPORTED                     # bf16 path is head_dim 128 only
    assert call(dt=ab.F32, D=96) == ab.ERR_UNSUPPORTED
    assert call(N=0) == ab.ERR_INVALID
    assert call(H=0) == ab.ERR_INVALID
    assert call(k_sel=101) == ab.ERR_INVALID                    # more selected queries than tokens
    assert call(k_sel=-1) == ab.ERR_INVALID
    assert call(scale=0.0) == ab.ERR_INVALID and call(scale=-1.0) == ab.ERR_INVALID
    assert call(scale=float("nan")) == ab.ERR_INVALID and call(scale=float("inf")) == ab.ERR_INVALID
    assert call(q=None) == ab.ERR_INVALID
    assert call(idx=None) == ab.ERR_INVALID                     # gathering needs the index list
    assert call(q=FAKE + 8) == ab.ERR_INVALID                   # 16-byte alignment
    assert call(ksn=100) == ab.ERR_INVALID and call(ksn=260) == ab.ERR_INVALID
    assert call(k_sel=0, q=None, k=None, v=None, o=None, idx=None) == ab.OK     # budget 0: nothing to do


def test_sparse_attn_update_rejects_bad_arguments(L):
    f = L.astraea_sparse_attn_update_fwd

    def call(dt=ab.BF16, N=100, H=2, D=128, idx=FAKE, k_sel=10, compact=0, scale=0.1, q=FAKE, out=FAKE, stride=256):
        return f(q, FAKE, FAKE, dt, N, H, D, 256, 128, 256, 128, idx, k_sel, compact, scale, out, stride, None, None, 0,
                 None)

    assert call(stride=248) == ab.ERR_INVALID                   # narrower than H*D
    assert call(stride=260) == ab.ERR_INVALID                   # rows must stay 16-byte aligned
    assert call(idx=None, compact=1) == ab.ERR_INVALID          # the index list also says where rows go
    assert call(k_sel=101, compact=1) == ab.ERR_INVALID         # cannot place more rows than there are tokens
    assert call(out=None) == ab.ERR_INVALID
    assert call(out=FAKE + 8) == ab.ERR_INVALID
    assert call(dt=ab.F32, D=96) == ab.ERR_UNSUPPORTED
    assert call() == ab.ERR_WORKSPACE                           # everything else valid: the bf16 path wants its workspace
    assert call(k_sel=0, q=None, out=None, idx=None) == ab.OK   # budget 0 leaves the cache as it is


def test_sparse_linear_rejects_bad_arguments(L):
    f = L.astraea_sparse_linear

    def call(dt=ab.BF16, N=100, cin=128, cout=64, xs=128, idx=FAKE, k_sel=10, xc=0, act=0, ys=64, yc=1, x=FAKE, w=FAKE,
             b=None, y=FAKE):
        return f(x, w, b, dt, N, cin, cout, xs, idx, k_sel, xc, act, y, ys, yc, None)

    assert call(dt=ab.F32, k_sel=0, x=None, w=None, y=None, idx=None) == ab.OK      # fp32 is a supported mode
    assert call(dt=9) == ab.ERR_UNSUPPORTED
    assert call(act=2) == ab.ERR_UNSUPPORTED
    assert call(cin=96, xs=96) == ab.ERR_UNSUPPORTED            # contraction advances in steps of 64
    assert call(cout=60, ys=64) == ab.ERR_UNSUPPORTED
    assert call(xs=64) == ab.ERR_INVALID and call(ys=32) == ab.ERR_INVALID and call(xs=132) == ab.ERR_INVALID
    assert call(k_sel=101) == ab.ERR_INVALID and call(k_sel=-1) == ab.ERR_INVALID
    assert call(idx=None) == ab.ERR_INVALID                     # rows must be gathered
    assert call(idx=None, xc=1, yc=0) == ab.ERR_INVALID         # rows must be placed
    assert call(x=None) == ab.ERR_INVALID and call(y=FAKE + 8) == ab.ERR_INVALID and call(b=FAKE + 4) == ab.ERR_INVALID
    assert call(N=1 << 21, xs=1 << 11, cin=1 << 11) == ab.ERR_UNSUPPORTED    # x spans 8 GiB: beyond 32-bit offsets
    assert call(k_sel=0, x=None, w=None, y=None, idx=None) == ab.OK


def test_row_movers_reject_bad_arguments(L):
    sc, ga = L.astraea_scatter_update, L.astraea_gather_rows
    assert sc(FAKE, FAKE, 5, 10, 8, 8, 8, FAKE, 3, 0, None) == ab.ERR_UNSUPPORTED
    assert sc(FAKE, FAKE, ab.BF16, 10, 8, 8, 8, FAKE, 11, 0, None) == ab.ERR_INVALID
    assert sc(FAKE, FAKE, ab.BF16, 10, 8, 4, 8, FAKE, 3, 0, None) == ab.ERR_INVALID
    assert sc(None, FAKE, ab.BF16, 10, 8, 8, 8, FAKE, 3, 0, None) == ab.ERR_INVALID
    assert sc(FAKE, FAKE, ab.BF16, 10, 8, 8, 8, None, 3, 0, None) == ab.ERR_INVALID
    assert sc(FAKE + 1, FAKE, ab.BF16, 10, 8, 8, 8, FAKE, 3, 0, None) == ab.ERR_INVALID
    assert sc(None, None, ab.BF16, 10, 8, 8, 8, None, 0, 0, None) == ab.OK      # budget 0: cache untouched
    assert ga(FAKE, FAKE, ab.F32, 10, 8, 8, 8, FAKE, 11, None) == ab.ERR_INVALID
    assert ga(FAKE, None, ab.F32, 10, 8, 8, 8, FAKE, 3, None) == ab.ERR_INVALID
    assert ga(None, None, ab.F32, 10, 8, 8, 8, None, 0, None) == ab.OK


def test_kernel_timer_is_off_by_default_and_rejects_bad_reads(L):
    ms = C.c_double(-1.0)
    assert L.astraea_probe_kernel_count() == 0
    assert L.astraea_probe_kernel_ms(0, C.byref(ms)) == ab.ERR_INVALID
    assert L.astraea_probe_kernel_ms(-1, C.byref(ms)) == ab.ERR_INVALID
    assert L.astraea_probe_kernel_ms(0, None) == ab.ERR_INVALID
    assert ms.value == -1.0
    assert ab.kernel_times_ms() == []


def test_binding_fails_loudly_without_library(monkeypatch, tmp_path):
    monkeypatch.setattr(ab, "_lib", None)
    monkeypatch.setattr(ab, "LIB_PATH", tmp_path / "missing.so")
    with pytest.raises(ImportError):
        ab.lib()


def test_product_path_does_not_import_the_oracle():
    pkg = ROOT / "paper_2506_05096_amd"
    for f in list(pkg.glob("*.py")) + list((pkg / "csrc").glob("*")):
        text = f.read_text()
        assert "import oracle" not in text and "from oracle" not in text and "liboracle" not in text, f


def test_synthetic_workloads_have_the_configured_shapes():
    from paper_2506_05096_amd import synth
    w = synth.WORKLOADS
    assert (w["cfg0"].N, w["cfg0"].H, w["cfg0"].D, w["cfg0"].C, w["cfg0"].dtype) == (4096, 8, 64, 512, "f32")
    assert (w["cfg1"].N, w["cfg1"].H, w["cfg1"].D, w["cfg1"].budgets_pct) == (16384, 24, 128, (25, 50, 75))
    assert w["cfg2"].N == 13 * 30 * 45 and w["cfg3"].N == 33 * 45 * 80 == 118800
    for c in w.values():
        assert c.N == c.latent[0] * c.latent[1] * c.latent[2]
    sched = synth.budget_schedule(0, 50)
    assert len(sched) == 50 and set(sched) <= set(range(10, 101, 10)) and sched == synth.budget_schedule(0, 50)
    t = synth.make_layer_inputs(w["cfg2"], seed=0, N=128)
    assert t["q"].shape == (128, 24, 128) and t["x_cur"].shape == (128, 3072) and t["out_cache"].shape == (128, 3072)
    t2 = synth.make_layer_inputs(w["cfg2"], seed=0, N=128)
    assert all((t[k].view(-1) == t2[k].view(-1)).all() for k in t)


# ------------------------------------------------------ budget-aware launch plan --

def _covered(plan, H):
    """Walks every workgroup of the plan the way the header describes it and returns, per work item, the list of
    key-tile ranges its workgroups take, plus the partial-result slots used."""
    q_tiles, ipx, full, splits, tps, wgs, key_tiles, _ = (plan[n] for n in (
        "q_tiles", "items_per_xcd", "full_items", "splits", "tiles_per_split", "workgroups", "key_tiles",
        "partial_slots"))
    total = q_tiles * H
    ranges, slots = {}, []
    for wg in range(wgs):
        xcd, slot = wg % 8, wg // 8
        if slot < full:
            item, lo, hi, ps = xcd * ipx + slot, 0, key_tiles, None
        else:
            p = slot - full
            li, sp = p // splits, p % splits
            item = xcd * ipx + full + li
            lo, hi = sp * tps, min((sp + 1) * tps, key_tiles)
            ps = (xcd * (ipx - full) + li) * splits + sp
        if item >= (xcd + 1) * ipx or item >= total:
            continue
        ranges.setdefault(item, []).append((lo, hi))
        if ps is not None:
            slots.append(ps)
    return ranges, slots


def test_attention_plan_covers_every_item_and_key_tile_once():
    import random
    rnd = random.Random(0)
    cases = [(118800, 24, k) for k in (1, 255, 256, 257, 11880, 35640, 118800)]
    cases += [(17550, 24, 7020), (16384, 24, 4096), (1, 1, 1), (63, 2, 63), (77, 3, 1000), (64, 65535, 1)]
    cases += [(rnd.randint(1, 5000), rnd.randint(1, 40), rnd.randint(1, 60000)) for _ in range(300)]
    for N, H, k in cases:
        plan = ab.astraea_attn_plan(N, H, k)
        assert plan["q_tiles"] == -(-k // 256) and plan["key_tiles"] == -(-N // 64), (N, H, k)
        ranges, slots = _covered(plan, H)
        total = plan["q_tiles"] * H
        assert sorted(ranges) == list(range(total)), (N, H, k)                 # every (head, query tile) is taken
        for item, rs in ranges.items():
            rs.sort()
            assert rs[0][0] == 0 and rs[-1][1] == plan["key_tiles"], (N, H, k, item)
            assert all(a[1] == b[0] for a, b in zip(rs, rs[1:])), (N, H, k, item)   # ranges abut: each tile once
            assert all(lo < hi for lo, hi in rs), (N, H, k, item)                   # no empty share
            assert len(rs) in (1, plan["splits"])
        assert len(set(slots)) == len(slots) and all(0 <= s < plan["partial_slots"] for s in slots), (N, H, k)
        # the tail of each XCD is cut only when that shortens it, and never into more than 64 shares
        left = plan["items_per_xcd"] - plan["full_items"]
        assert 0 <= left < 32 and left * plan["splits"] <= 64 and 1 <= plan["splits"] <= 8
        assert plan["full_items"] % 32 == 0 or left == 0


def test_attention_plan_work_follows_the_budget():
    """Rounds of 32 workgroups per XCD, each weighted by the share of the keys it sweeps: the plan's cost stays
    within 10 % of proportional to k_sel from the 10 % budget up, at the headline shape."""
    N, H = 118800, 24
    cost = {}
    for pct in range(10, 101, 10):
        p = ab.astraea_attn_plan(N, H, N * pct // 100)
        left = p["items_per_xcd"] - p["full_items"]
        tail = -(-left * p["splits"] // 32) * p["tiles_per_split"] / p["key_tiles"]
        cost[pct] = p["full_items"] / 32 + tail
    unit = cost[100] / 100
    assert all(abs(cost[pct] / (unit * pct) - 1) < 0.10 for pct in cost), cost


def test_check_indices_rejects_bad_arguments(L):
    f = L.astraea_check_indices
    assert f(FAKE, 5, 0, FAKE, None) == ab.ERR_INVALID
    assert f(FAKE, -1, 10, FAKE, None) == ab.ERR_INVALID
    assert f(None, 5, 10, FAKE, None) == ab.ERR_INVALID
    assert f(FAKE, 5, 10, None, None) == ab.ERR_INVALID
    assert f(FAKE + 2, 5, 10, FAKE, None) == ab.ERR_INVALID


def test_attention_plan_rejects_bad_arguments(L):
    out = (C.c_int64 * 8)()
    assert L.astraea_attn_plan(0, 1, 1, out) == ab.ERR_INVALID
    assert L.astraea_attn_plan(10, 0, 1, out) == ab.ERR_INVALID
    assert L.astraea_attn_plan(10, 1, 0, out) == ab.ERR_INVALID
    assert L.astraea_attn_plan(10, 1, 1, None) == ab.ERR_INVALID
    assert L.astraea_attn_plan(10, 1, 1, out) == ab.OK


def test_block_flop_accounting_is_the_papers_formulas_at_k():
    """TokenSparseBlock.flops: the FLOPs appendix (self-attention 8BNH^2 + 4BN^2H in total, MLP 16BNH^2, with the
    paper's H = hidden width = E here) at k = N, and exactly the budget fraction of that at k < N."""
    import torch
    from paper_2506_05096_amd.layer import TokenSparseBlock
    N, H, D = 1000, 4, 128
    E = H * D
    blk = TokenSparseBlock.__new__(TokenSparseBlock)          # accounting only: no buffers, no GPU
    blk.N, blk.E, blk.hidden = N, E, 4 * E
    full = blk.flops(N)
    assert full["qkv_proj"] + full["attn"] + full["out_proj"] == 8.0 * N * E * E + 4.0 * N * N * E
    assert full["mlp"] == 16.0 * N * E * E
    assert full["attn"] == ab.astraea_attn_flops(N, N, H, D)
    for pct in (10, 40, 50, 70):
        part = blk.flops(N * pct // 100)
        assert all(abs(part[name] / full[name] - pct / 100) < 1e-12 for name in full)


def test_header_is_plain_c():
    """The boundary is a C ABI: the header must compile as C99 with nothing but the standard headers, and a C
    program must be able to link against the library by those declarations."""
    import subprocess
    import tempfile
    hdr = ROOT / "include" / "astraea.h"
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only", "-x", "c", str(hdr)],
                   check=True)
    prog = ('#include "astraea.h"\n#include <stdio.h>\n'
            'int main(void) { printf("%lld %s\\n", (long long)astraea_budget_to_k(118800, 30), astraea_status_string(0));'
            ' return astraea_attn_flops(2, 1, 1, 1) == 8.0 ? 0 : 1; }\n')
    with tempfile.TemporaryDirectory() as d:
        src = Path(d) / "t.c"
        src.write_text(prog)
        exe = Path(d) / "t"
        lib = ab.LIB_PATH
        subprocess.run(["gcc", "-std=c99", "-I", str(ROOT / "include"), str(src), "-o", str(exe), str(lib),
                        f"-Wl,-rpath,{lib.parent}", "-Wl,--allow-shlib-undefined"], check=True)
        out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()
    assert out == ["35640", "ok"]
