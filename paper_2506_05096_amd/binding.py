"""Thin ctypes binding of libastraea: argument marshalling only.

Every function has the name and the meaning of the C entry point declared in
include/astraea.h; tensors are torch tensors living on the GPU and only their
pointers, shapes and strides are passed on.  All arithmetic runs in the HIP
kernels.  There is no fallback: if the library cannot be loaded, importing a
symbol raises.
"""
from __future__ import annotations

import ctypes as C
from pathlib import Path
from typing import Optional

import torch

_PKG = Path(__file__).resolve().parent
LIB_PATH = _PKG / "libastraea.so"

F32, BF16 = 0, 1
DELTA_L2, DELTA_MEAN_ABS, DELTA_MEAN_SQ = 0, 1, 2
OK, ERR_INVALID, ERR_UNSUPPORTED, ERR_WORKSPACE, ERR_HIP = 0, -1, -2, -3, -4
OP_SELECT_TOPK, OP_SPARSE_ATTN = 1, 2
ACT_NONE, ACT_GELU_TANH = 0, 1
CROSSOVER_UNIFORM, CROSSOVER_BLOCK = 0, 1

EXPORTS = (
    "astraea_score", "astraea_select_topk", "astraea_select_topk_static", "astraea_sparse_attn_fwd", "astraea_sparse_attn_update_fwd",
    "astraea_scatter_update", "astraea_kv_refresh", "astraea_gather_rows", "astraea_sparse_linear", "astraea_workspace_bytes", "astraea_budget_to_k", "astraea_attn_flops",
    "astraea_probe_mfma_bf16", "astraea_probe_copy", "astraea_probe_kernel_timer", "astraea_probe_kernel_count",
    "astraea_probe_kernel_ms", "astraea_lse_weight_update", "astraea_attn_plan", "astraea_check_indices",
    "astraea_budget_search", "astraea_search_crossover", "astraea_search_mutate", "astraea_search_repair",
    "astraea_status_string", "astraea_last_error",
)


class SearchConfig(C.Structure):
    """astraea_search_config"""
    _fields_ = [("T", C.c_int32), ("population", C.c_int32), ("children", C.c_int32), ("generations", C.c_int32),
                ("budget_tenths", C.c_int64), ("p_mutation_start", C.c_double), ("p_mutation_final", C.c_double),
                ("seed", C.c_uint64)]


FITNESS_FN = C.CFUNCTYPE(C.c_double, C.POINTER(C.c_int32), C.c_int32, C.c_void_p)


class AstraeaError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"astraea status {status}: {message}")
        self.status = status


_lib = None


def lib() -> C.CDLL:
    """Load libastraea.so (built in-tree by build.py); raises if it is missing."""
    global _lib
    if _lib is None:
        if not LIB_PATH.exists():
            raise ImportError(f"{LIB_PATH} is not built; run `python -m paper_2506_05096_amd.build` "
                              "(there is no non-HIP fallback)")
        L = C.CDLL(str(LIB_PATH))
        vp, i64, i32, f32, sz = C.c_void_p, C.c_int64, C.c_int32, C.c_float, C.c_size_t
        L.astraea_score.argtypes = [vp, vp, C.c_int, i64, i64, i64, C.c_int, vp, vp, vp, i32, f32, f32, vp, vp]
        L.astraea_select_topk.argtypes = [vp, i64, i64, vp, vp, vp, vp, vp, sz, vp]
        L.astraea_select_topk_static.argtypes = [vp, i64, i64, vp, vp, vp, vp, vp]
        L.astraea_select_topk_static.restype = C.c_int
        L.astraea_sparse_attn_fwd.argtypes = [vp, vp, vp, C.c_int, i64, i32, i32, i64, i64, i64, i64, vp, i64,
                                              C.c_int, f32, vp, vp, vp, sz, vp]
        L.astraea_sparse_attn_update_fwd.argtypes = [vp, vp, vp, C.c_int, i64, i32, i32, i64, i64, i64, i64, vp, i64,
                                                     C.c_int, f32, vp, i64, vp, vp, sz, vp]
        L.astraea_scatter_update.argtypes = [vp, vp, C.c_int, i64, i64, i64, i64, vp, i64, C.c_int, vp]
        L.astraea_gather_rows.argtypes = [vp, vp, C.c_int, i64, i64, i64, i64, vp, i64, vp]
        L.astraea_kv_refresh.argtypes = [vp, vp, vp, vp, C.c_int, i64, i64, i64, i64, vp, i64, vp]
        L.astraea_kv_refresh.restype = C.c_int
        L.astraea_sparse_linear.argtypes = [vp, vp, vp, C.c_int, i64, i64, i64, i64, vp, i64, C.c_int, C.c_int, vp, i64,
                                            C.c_int, vp]
        L.astraea_sparse_linear.restype = C.c_int
        L.astraea_workspace_bytes.argtypes = [C.c_int, i64, i64, i32, i32]
        L.astraea_workspace_bytes.restype = sz
        L.astraea_budget_to_k.argtypes = [i64, i32]
        L.astraea_budget_to_k.restype = i64
        L.astraea_attn_flops.argtypes = [i64, i64, i32, i32]
        L.astraea_attn_flops.restype = C.c_double
        L.astraea_status_string.argtypes = [C.c_int]
        L.astraea_status_string.restype = C.c_char_p
        L.astraea_last_error.restype = C.c_char_p
        L.astraea_lse_weight_update.argtypes = [vp, i32, i64, vp, i64, vp, vp]
        L.astraea_lse_weight_update.restype = C.c_int
        L.astraea_probe_mfma_bf16.argtypes = [i32, i32, i32, vp, i64, C.POINTER(C.c_double), vp]
        L.astraea_probe_copy.argtypes = [vp, vp, i64, vp]
        L.astraea_check_indices.argtypes = [vp, i64, i64, vp, vp]
        L.astraea_check_indices.restype = C.c_int
        L.astraea_attn_plan.argtypes = [i64, i32, i64, C.POINTER(i64)]
        L.astraea_attn_plan.restype = C.c_int
        L.astraea_probe_kernel_timer.argtypes = [C.c_int]
        L.astraea_probe_kernel_timer.restype = C.c_int
        L.astraea_probe_kernel_count.restype = i32
        L.astraea_probe_kernel_ms.argtypes = [i32, C.POINTER(C.c_double)]
        L.astraea_probe_kernel_ms.restype = C.c_int
        L.astraea_probe_mfma_bf16.restype = C.c_int
        L.astraea_probe_copy.restype = C.c_int
        L.astraea_budget_search.argtypes = [C.POINTER(SearchConfig), FITNESS_FN, vp, vp, C.POINTER(C.c_double), vp, vp,
                                            C.POINTER(C.c_int32)]
        L.astraea_search_crossover.argtypes = [vp, vp, i32, C.c_int, C.POINTER(C.c_uint64), vp]
        L.astraea_search_mutate.argtypes = [vp, i32, C.c_double, C.POINTER(C.c_uint64)]
        L.astraea_search_repair.argtypes = [vp, i32, i64, C.POINTER(C.c_uint64)]
        for name in ("astraea_budget_search", "astraea_search_crossover", "astraea_search_mutate",
                     "astraea_search_repair"):
            getattr(L, name).restype = C.c_int
        for name in ("astraea_score", "astraea_select_topk", "astraea_sparse_attn_fwd",
                     "astraea_sparse_attn_update_fwd", "astraea_scatter_update", "astraea_gather_rows"):
            getattr(L, name).restype = C.c_int
        _lib = L
    return _lib


def _check(rc: int):
    if rc != OK:
        raise AstraeaError(rc, lib().astraea_last_error().decode() or lib().astraea_status_string(rc).decode())


def _dt(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError(f"unsupported tensor dtype {t.dtype}")


def _p(t: Optional[torch.Tensor]):
    return None if t is None else t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def workspace_bytes(op: int, N: int, k_sel: int = 0, H: int = 0, D: int = 0) -> int:
    return int(lib().astraea_workspace_bytes(op, N, k_sel, H, D))


def astraea_budget_to_k(N: int, budget_percent: int) -> int:
    return int(lib().astraea_budget_to_k(N, budget_percent))


def astraea_attn_flops(N: int, k_sel: int, H: int, D: int) -> float:
    return float(lib().astraea_attn_flops(N, k_sel, H, D))


def astraea_score(x_cur: torch.Tensor, x_prev: torch.Tensor, score_out: torch.Tensor, mode: int = DELTA_L2,
                  lse_weight: Optional[torch.Tensor] = None, skip_count: Optional[torch.Tensor] = None,
                  penalty_table: Optional[torch.Tensor] = None, w_alpha: float = 1.0, w_beta: float = 0.0) -> None:
    N, Cw = x_cur.shape
    assert x_prev.shape == x_cur.shape and x_prev.dtype == x_cur.dtype and x_cur.stride(1) == 1
    assert x_prev.stride() == x_cur.stride() and score_out.dtype == torch.float32 and score_out.is_contiguous()
    tl = 0 if penalty_table is None else int(penalty_table.numel())
    _check(lib().astraea_score(_p(x_cur), _p(x_prev), _dt(x_cur), N, Cw, x_cur.stride(0), mode, _p(lse_weight),
                               _p(skip_count), _p(penalty_table), tl, w_alpha, w_beta, _p(score_out), _stream()))


def astraea_select_topk(score: torch.Tensor, k: int, idx_sel: torch.Tensor, workspace: torch.Tensor,
                        idx_remain: Optional[torch.Tensor] = None, sel_mask: Optional[torch.Tensor] = None,
                        skip_count: Optional[torch.Tensor] = None) -> None:
    assert score.dtype == torch.float32 and score.is_contiguous() and idx_sel.dtype == torch.int32
    _check(lib().astraea_select_topk(_p(score), score.numel(), k, _p(idx_sel), _p(idx_remain), _p(sel_mask),
                                     _p(skip_count), _p(workspace), workspace.numel() * workspace.element_size(),
                                     _stream()))


def astraea_select_topk_static(score: torch.Tensor, k: int, idx_sel: torch.Tensor,
                               idx_remain: Optional[torch.Tensor] = None, sel_mask: Optional[torch.Tensor] = None,
                               skip_count: Optional[torch.Tensor] = None) -> None:
    assert score.dtype == torch.float32 and score.is_contiguous() and idx_sel.dtype == torch.int32
    _check(lib().astraea_select_topk_static(_p(score), score.numel(), k, _p(idx_sel), _p(idx_remain), _p(sel_mask),
                                            _p(skip_count), _stream()))


def astraea_sparse_attn_fwd(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, idx_sel: Optional[torch.Tensor],
                            k_sel: int, o_sel: torch.Tensor, softmax_scale: float, q_is_compact: bool = False,
                            lse_sel: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None) -> None:
    N, H, D = k.shape
    assert v.shape == k.shape and v.stride() == k.stride() and q.stride(2) == 1 and k.stride(2) == 1
    assert q.dtype == k.dtype == v.dtype == o_sel.dtype and o_sel.is_contiguous()
    wsb = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().astraea_sparse_attn_fwd(_p(q), _p(k), _p(v), _dt(k), N, H, D, q.stride(0), q.stride(1), k.stride(0),
                                         k.stride(1), _p(idx_sel), k_sel, 1 if q_is_compact else 0, softmax_scale,
                                         _p(o_sel), _p(lse_sel), _p(workspace), wsb, _stream()))


def astraea_sparse_attn_update_fwd(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, idx_sel: torch.Tensor,
                                   k_sel: int, out_cache: torch.Tensor, softmax_scale: float,
                                   q_is_compact: bool = False, lse_sel: Optional[torch.Tensor] = None,
                                   workspace: Optional[torch.Tensor] = None) -> None:
    N, H, D = k.shape
    assert v.shape == k.shape and v.stride() == k.stride() and q.stride(2) == 1 and k.stride(2) == 1
    assert q.dtype == k.dtype == v.dtype == out_cache.dtype
    assert out_cache.dim() == 2 and out_cache.shape[0] == N and out_cache.shape[1] == H * D and out_cache.stride(1) == 1
    wsb = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().astraea_sparse_attn_update_fwd(_p(q), _p(k), _p(v), _dt(k), N, H, D, q.stride(0), q.stride(1),
                                                k.stride(0), k.stride(1), _p(idx_sel), k_sel, 1 if q_is_compact else 0,
                                                softmax_scale, _p(out_cache), out_cache.stride(0), _p(lse_sel),
                                                _p(workspace), wsb, _stream()))


def astraea_scatter_update(cache: torch.Tensor, src: torch.Tensor, idx_sel: torch.Tensor, k_sel: int,
                           src_is_full: bool = False) -> None:
    assert cache.dim() == 2 and src.dim() == 2 and cache.stride(1) == 1 and src.stride(1) == 1
    assert cache.dtype == src.dtype and cache.shape[1] == src.shape[1]
    _check(lib().astraea_scatter_update(_p(cache), _p(src), _dt(cache), cache.shape[0], cache.shape[1],
                                        cache.stride(0), src.stride(0), _p(idx_sel), k_sel, 1 if src_is_full else 0,
                                        _stream()))


def astraea_kv_refresh(k_cache: torch.Tensor, v_cache: torch.Tensor, k_new: torch.Tensor, v_new: torch.Tensor,
                       idx_sel: torch.Tensor, k_sel: int) -> None:
    for c, s in ((k_cache, k_new), (v_cache, v_new)):
        assert c.dim() == 2 and s.dim() == 2 and c.stride(1) == 1 and s.stride(1) == 1 and c.shape == s.shape
        assert c.dtype == s.dtype == k_cache.dtype
    assert k_cache.shape == v_cache.shape and k_cache.stride(0) == v_cache.stride(0) and k_new.stride(0) == v_new.stride(0)
    _check(lib().astraea_kv_refresh(_p(k_cache), _p(v_cache), _p(k_new), _p(v_new), _dt(k_cache), k_cache.shape[0],
                                    k_cache.shape[1], k_cache.stride(0), k_new.stride(0), _p(idx_sel), k_sel, _stream()))


def astraea_gather_rows(src: torch.Tensor, dst: torch.Tensor, idx_sel: torch.Tensor, k_sel: int) -> None:
    assert src.dim() == 2 and dst.dim() == 2 and src.stride(1) == 1 and dst.stride(1) == 1
    assert src.dtype == dst.dtype and src.shape[1] == dst.shape[1]
    _check(lib().astraea_gather_rows(_p(src), _p(dst), _dt(src), src.shape[0], src.shape[1], src.stride(0),
                                     dst.stride(0), _p(idx_sel), k_sel, _stream()))


def astraea_sparse_linear(x: torch.Tensor, w: torch.Tensor, bias: Optional[torch.Tensor],
                          idx_sel: Optional[torch.Tensor], k_sel: int, y: torch.Tensor, act: int = ACT_NONE,
                          x_is_compact: bool = False, y_is_compact: bool = True, N: Optional[int] = None) -> None:
    """y[row_out(r)] = act(x[row_in(r)] @ w.T + bias); N is the token count the indices refer to (taken from
    whichever of x, y is not compact when omitted)."""
    assert x.dim() == 2 and y.dim() == 2 and w.dim() == 2 and w.is_contiguous()
    assert x.stride(1) == 1 and y.stride(1) == 1 and x.dtype == w.dtype == y.dtype
    assert x.shape[1] == w.shape[1] and y.shape[1] == w.shape[0]
    if N is None:
        N = x.shape[0] if not x_is_compact else (y.shape[0] if not y_is_compact else max(k_sel, 1))
    _check(lib().astraea_sparse_linear(_p(x), _p(w), _p(bias), _dt(x), N, w.shape[1], w.shape[0], x.stride(0),
                                       _p(idx_sel), k_sel, 1 if x_is_compact else 0, act, _p(y), y.stride(0),
                                       1 if y_is_compact else 0, _stream()))


def astraea_lse_weight_update(lse_sel: torch.Tensor, idx_sel: torch.Tensor, k_sel: int, lse_weight: torch.Tensor) -> None:
    assert lse_sel.dtype == torch.float32 and lse_sel.is_contiguous() and lse_weight.dtype == torch.float32
    H = lse_sel.shape[1]
    _check(lib().astraea_lse_weight_update(_p(lse_sel), H, lse_weight.numel(), _p(idx_sel), k_sel, _p(lse_weight),
                                           _stream()))


def astraea_probe_mfma_bf16(workgroups: int, iters: int, randomize: bool, sink: torch.Tensor) -> float:
    """Enqueues the MFMA loop; returns the flops it performs."""
    fl = C.c_double(0.0)
    _check(lib().astraea_probe_mfma_bf16(workgroups, iters, 1 if randomize else 0, _p(sink), sink.numel(),
                                         C.byref(fl), _stream()))
    return fl.value


def astraea_probe_copy(src: torch.Tensor, dst: torch.Tensor) -> None:
    nbytes = src.numel() * src.element_size()
    assert dst.numel() * dst.element_size() == nbytes
    _check(lib().astraea_probe_copy(_p(src), _p(dst), nbytes, _stream()))


def astraea_check_indices(idx_sel: Optional[torch.Tensor], k_sel: int, N: int, counts_out: torch.Tensor) -> None:
    assert counts_out.dtype == torch.int32 and counts_out.numel() >= 2 and counts_out.is_contiguous()
    _check(lib().astraea_check_indices(_p(idx_sel), k_sel, N, _p(counts_out), _stream()))


def astraea_attn_plan(N: int, H: int, k_sel: int) -> dict:
    out = (C.c_int64 * 8)()
    _check(lib().astraea_attn_plan(N, H, k_sel, out))
    names = ("q_tiles", "items_per_xcd", "full_items", "splits", "tiles_per_split", "workgroups", "key_tiles",
             "partial_slots")
    return dict(zip(names, (int(v) for v in out)))


def kernel_timer(enable: bool) -> None:
    _check(lib().astraea_probe_kernel_timer(1 if enable else 0))


def kernel_times_ms():
    """Durations of the attention main kernels timed since the timer was switched on."""
    out = []
    for i in range(lib().astraea_probe_kernel_count()):
        ms = C.c_double()
        _check(lib().astraea_probe_kernel_ms(i, C.byref(ms)))
        out.append(ms.value)
    return out


# ---- token-budget search (host only; numpy int32 arrays, no GPU involved) ----

def _i32(a):
    import numpy as np
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a, a.ctypes.data_as(C.c_void_p)


def astraea_search_crossover(parent0, parent1, kind: int, rng_state: int):
    """Returns (child, new rng state)."""
    import numpy as np
    p0, pp0 = _i32(parent0)
    p1, pp1 = _i32(parent1)
    child = np.empty_like(p0)
    st = C.c_uint64(rng_state)
    _check(lib().astraea_search_crossover(pp0, pp1, p0.size, kind, C.byref(st), child.ctypes.data_as(C.c_void_p)))
    return child, st.value


def astraea_search_mutate(theta, p_mutation: float, rng_state: int):
    th, p = _i32(theta)
    th = th.copy()
    st = C.c_uint64(rng_state)
    _check(lib().astraea_search_mutate(th.ctypes.data_as(C.c_void_p), th.size, p_mutation, C.byref(st)))
    return th, st.value


def astraea_search_repair(theta, budget_tenths: int, rng_state: int):
    th, p = _i32(theta)
    th = th.copy()
    st = C.c_uint64(rng_state)
    _check(lib().astraea_search_repair(th.ctypes.data_as(C.c_void_p), th.size, budget_tenths, C.byref(st)))
    return th, st.value


def astraea_budget_search(T: int, budget_tenths: int, population: int, children: int, generations: int,
                          p_mutation_start: float, p_mutation_final: float, seed: int, fitness):
    """fitness(list of T levels) -> float, lower is better.  Returns (best schedule, its fitness, final population
    best first as an int32 array [n, T], their fitness)."""
    import numpy as np
    cfg = SearchConfig(T, population, children, generations, budget_tenths, p_mutation_start, p_mutation_final, seed)
    cb = FITNESS_FN(lambda th, t, _user: float(fitness([th[i] for i in range(t)])))
    best = np.empty(T, np.int32)
    pop = np.empty((population, T), np.int32)
    fit = np.empty(population, np.float64)
    bf, n = C.c_double(), C.c_int32()
    _check(lib().astraea_budget_search(C.byref(cfg), cb, None, best.ctypes.data_as(C.c_void_p), C.byref(bf),
                                       pop.ctypes.data_as(C.c_void_p), fit.ctypes.data_as(C.c_void_p), C.byref(n)))
    return best, bf.value, pop[:n.value], fit[:n.value]
