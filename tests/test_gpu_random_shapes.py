"""Random shapes within the documented limits, every entry point, against PyTorch's own fp32 operators on the
same device (softmax attention written with einsum, linear + GELU, indexing, a stable sort): a sweep for shape-
dependent mistakes (ragged tiles, tiny and odd sizes, strides, split work items) between the cases the oracle
tests fix by hand.  The oracle remains the parity reference; this one only has to be independent of the kernels.
Each case prints its parameters before it runs."""
import math
import random

import pytest
import torch

from paper_2506_05096_amd import binding as ab

pytestmark = pytest.mark.gpu
dev = "cuda"


def rel(a, b):
    return ((a.float() - b.float()).norm() / b.float().norm().clamp_min(1e-20)).item()


@pytest.mark.parametrize("seed", [0, 1, 2, 3])
def test_random_shapes_against_torch_operators(seed):
    rnd = random.Random(seed)
    bad = []
    for case in range(30):
        kind = rnd.choice(["attn_bf16", "attn_bf16", "attn_f32", "linear_bf16", "linear_f32", "rows", "topk"])
        g = torch.Generator(device=dev).manual_seed(1000 * seed + case)
        if kind.startswith("attn"):
            bf = kind == "attn_bf16"
            dt = torch.bfloat16 if bf else torch.float32
            D = 128 if bf else rnd.choice([64, 128])
            N = rnd.choice([1, 2, 63, 64, 65, 127, 200, 513, 1000, 2049, 4097, rnd.randint(1, 6000)])
            H = rnd.choice([1, 2, 3, 5, 8, 24])
            if not bf: N = min(N, 1500); H = min(H, 3)
            compact = rnd.random() < 0.3
            k_sel = rnd.randint(1, N) if not compact else rnd.randint(1, 3000 if bf else 600)
            upd = (not compact) and rnd.random() < 0.4
            layout = rnd.choice(["tok", "head", "packed"])
            print(f"case {case} {kind} N={N} H={H} D={D} k={k_sel} compact={compact} upd={upd} layout={layout}", flush=True)
            nq = k_sel if compact else N
            if layout == "tok":
                q = torch.randn(nq, H, D, device=dev, generator=g).to(dt); k = torch.randn(N, H, D, device=dev, generator=g).to(dt); v = torch.randn(N, H, D, device=dev, generator=g).to(dt)
            elif layout == "head":
                q = torch.randn(H, nq, D, device=dev, generator=g).to(dt).transpose(0, 1); k = torch.randn(H, N, D, device=dev, generator=g).to(dt).transpose(0, 1); v = torch.randn(H, N, D, device=dev, generator=g).to(dt).transpose(0, 1)
            else:
                if compact:
                    q = torch.randn(nq, H, D, device=dev, generator=g).to(dt)
                    kv = torch.randn(N, 2, H, D, device=dev, generator=g).to(dt); k, v = kv[:, 0], kv[:, 1]
                else:
                    c = torch.randn(N, 3, H, D, device=dev, generator=g).to(dt); q, k, v = c[:, 0], c[:, 1], c[:, 2]
            idx = None if compact else torch.randperm(N, device=dev, generator=g)[:k_sel].sort().values.to(torch.int32)
            scale = 1 / math.sqrt(D)
            wsb = ab.workspace_bytes(ab.OP_SPARSE_ATTN, N, k_sel, H, D)
            ws = torch.empty(max(wsb, 1), dtype=torch.uint8, device=dev) if wsb else None
            lse = torch.empty(k_sel, H, device=dev)
            qs = q if compact else q[idx.long()]
            s = torch.einsum("rhd,nhd->hrn", qs.float(), k.float()) * scale
            ref = torch.einsum("hrn,nhd->rhd", torch.softmax(s, dim=2), v.float())
            lref = torch.logsumexp(s, dim=2).transpose(0, 1)
            if upd:
                cache = torch.randn(N, H * D + 8, device=dev, generator=g).to(dt); c0 = cache.clone()
                ab.astraea_sparse_attn_update_fwd(q, k, v, idx, k_sel, cache[:, :H * D], scale, lse_sel=lse, workspace=ws)
                torch.cuda.synchronize()
                got = cache[idx.long(), :H * D].view(k_sel, H, D)
                mask = torch.ones(N, dtype=torch.bool, device=dev); mask[idx.long()] = False
                ok2 = torch.equal(cache[mask], c0[mask]) and torch.equal(cache[:, H * D:], c0[:, H * D:])
            else:
                o = torch.full((k_sel, H, D), float("nan"), device=dev).to(dt)
                ab.astraea_sparse_attn_fwd(q, k, v, idx, k_sel, o, scale, q_is_compact=compact, lse_sel=lse, workspace=ws)
                torch.cuda.synchronize()
                got, ok2 = o, True
            r = rel(got, ref); le = (lse - lref).abs().max().item()
            ok = ok2 and (r < (1e-2 if bf else 1e-5)) and le < (2e-2 if bf else 1e-4) and bool(torch.isfinite(got.float()).all())
            print(f"   rel {r:.2e} lse {le:.2e} {'ok' if ok else 'FAIL'}", flush=True)
        elif kind.startswith("linear"):
            bf = kind == "linear_bf16"
            dt = torch.bfloat16 if bf else torch.float32
            cin = 64 * rnd.randint(1, 20 if bf else 6); cout = 8 * rnd.randint(1, 150 if bf else 40)
            N = rnd.randint(1, 3000 if bf else 800); k_sel = rnd.randint(1, N)
            xc, yc = rnd.random() < 0.4, rnd.random() < 0.6
            act = rnd.choice([ab.ACT_NONE, ab.ACT_GELU_TANH]); hb = rnd.random() < 0.6
            print(f"case {case} {kind} N={N} k={k_sel} cin={cin} cout={cout} xc={xc} yc={yc} act={act} bias={hb}", flush=True)
            idx = torch.randperm(N, device=dev, generator=g)[:k_sel].sort().values.to(torch.int32)
            x = torch.randn(k_sel if xc else N, cin, device=dev, generator=g).to(dt)
            w = (torch.randn(cout, cin, device=dev, generator=g) * cin ** -0.5).to(dt)
            b = torch.randn(cout, device=dev, generator=g).to(dt) if hb else None
            xs = x if xc else x[idx.long()]
            ref = xs.float() @ w.float().T + (b.float() if hb else 0)
            if act == ab.ACT_GELU_TANH: ref = torch.nn.functional.gelu(ref, approximate="tanh")
            y = torch.randn(k_sel if yc else N, cout + 16, device=dev, generator=g).to(dt); y0 = y.clone()
            ab.astraea_sparse_linear(x, w, b, None if (xc and yc) else idx, k_sel, y[:, :cout], act=act, x_is_compact=xc, y_is_compact=yc, N=N)
            torch.cuda.synchronize()
            got = y[:, :cout] if yc else y[idx.long(), :cout]
            ok2 = torch.equal(y[:, cout:], y0[:, cout:])
            if not yc:
                mask = torch.ones(N, dtype=torch.bool, device=dev); mask[idx.long()] = False
                ok2 = ok2 and torch.equal(y[mask], y0[mask])
            r = rel(got, ref)
            ok = ok2 and r < (1e-2 if bf else 1e-5)
            print(f"   rel {r:.2e} {'ok' if ok else 'FAIL'}", flush=True)
        elif kind == "rows":
            dt = rnd.choice([torch.bfloat16, torch.float32]); E = rnd.choice([1, 3, 5, 8, 64, 100, 512, 3072, 777])
            N = rnd.randint(1, 4000); k_sel = rnd.randint(0, N); full = rnd.random() < 0.5
            print(f"case {case} rows N={N} k={k_sel} E={E} dt={dt} full={full}", flush=True)
            idx = torch.randperm(N, device=dev, generator=g)[:k_sel].sort().values.to(torch.int32)
            cache = torch.randn(N, E, device=dev, generator=g).to(dt); c0 = cache.clone()
            src = torch.randn(N if full else max(k_sel, 1), E, device=dev, generator=g).to(dt)
            ab.astraea_scatter_update(cache, src, idx, k_sel, src_is_full=full)
            dst = torch.zeros(max(k_sel, 1), E, device=dev).to(dt)
            ab.astraea_gather_rows(cache, dst, idx, k_sel)
            torch.cuda.synchronize()
            exp = c0.clone(); exp[idx.long()] = src[idx.long()] if full else src[:k_sel]
            ok = torch.equal(cache, exp) and torch.equal(dst[:k_sel], exp[idx.long()])
            print(f"   {'ok' if ok else 'FAIL'}", flush=True)
        else:
            N = rnd.choice([1, 2, 100, 2047, 2048, 2049, 5000, 70000, rnd.randint(1, 200000)]); k_sel = rnd.randint(0, N)
            mode = rnd.choice(["normal", "tied", "const"])
            print(f"case {case} topk N={N} k={k_sel} {mode}", flush=True)
            sc = torch.randn(N, device=dev, generator=g)
            if mode == "tied": sc = (sc * 4).round() / 4
            if mode == "const": sc = torch.zeros(N, device=dev)
            idx = torch.full((max(N, 1),), -1, dtype=torch.int32, device=dev)
            rem = torch.full((max(N, 1),), -1, dtype=torch.int32, device=dev)
            mask = torch.empty(N, dtype=torch.uint8, device=dev)
            ws = torch.empty(ab.workspace_bytes(ab.OP_SELECT_TOPK, N), dtype=torch.uint8, device=dev)
            ab.astraea_select_topk(sc, k_sel, idx, ws, idx_remain=rem, sel_mask=mask)
            torch.cuda.synchronize()
            order = torch.sort(-sc, stable=True).indices
            exp = order[:k_sel].sort().values.to(torch.int32)
            m = torch.zeros(N, dtype=torch.uint8, device=dev); m[exp.long()] = 1
            ok = torch.equal(idx[:k_sel], exp) and torch.equal(mask, m) and torch.equal(rem[:N - k_sel], torch.nonzero(m == 0).flatten().to(torch.int32))
            print(f"   {'ok' if ok else 'FAIL'}", flush=True)
        if not ok:
            bad.append(case)
    assert not bad, bad
