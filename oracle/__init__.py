"""ctypes front end of the plain-C CPU oracle (test infrastructure only).

Only tests, the smoke check and the benchmark's CPU-baseline leg may import
this package.  It never imports the HIP package and shares nothing with it.
Arrays are numpy: fp32 as float32, bf16 as uint16 bit patterns.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from pathlib import Path

import numpy as np

_HERE = Path(__file__).resolve().parent
_SRC = _HERE / "astraea_oracle.c"
_LIB = _HERE / "liboracle.so"

F32, BF16 = 0, 1
DELTA_L2, DELTA_MEAN_ABS, DELTA_MEAN_SQ = 0, 1, 2
ACT_NONE, ACT_GELU_TANH = 0, 1


def build(force: bool = False) -> Path:
    """Compile the oracle with gcc (no fast-math, no contraction)."""
    if force or not _LIB.exists() or _LIB.stat().st_mtime < _SRC.stat().st_mtime:
        cmd = ["gcc", "-O2", "-std=c99", "-fopenmp", "-ffp-contract=off", "-fno-fast-math", "-fPIC", "-shared",
               "-Wall", "-Wextra", "-o", str(_LIB), str(_SRC), "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(str(_LIB))
        vp, i64, i32, f32 = C.c_void_p, C.c_int64, C.c_int32, C.c_float
        L.oracle_num_threads.restype = C.c_int
        L.oracle_score.argtypes = [vp, vp, C.c_int, i64, i64, i64, C.c_int, vp, vp, vp, i32, f32, f32, vp]
        L.oracle_score_f64.argtypes = [vp, vp, C.c_int, i64, i64, i64, C.c_int, vp, vp, C.c_double, C.c_double, vp]
        L.oracle_topk.argtypes = [vp, i64, i64, vp, vp, vp]
        L.oracle_update_skip_count.argtypes = [vp, vp, i64]
        L.oracle_sparse_attn.argtypes = [vp, vp, vp, C.c_int, i64, i32, i32, i64, i64, i64, i64, vp, i64, C.c_int,
                                         f32, C.c_int, vp, vp]
        L.oracle_lse_weight_update.argtypes = [vp, i32, i64, vp, i64, vp]
        L.oracle_round_to_dtype.argtypes = [vp, i64, C.c_int, vp]
        L.oracle_scatter.argtypes = [vp, vp, C.c_int, i64, i64, i64, i64, vp, i64, C.c_int]
        L.oracle_gather.argtypes = [vp, vp, C.c_int, i64, i64, i64, i64, vp, i64]
        L.oracle_sparse_linear.argtypes = [vp, C.c_int, i64, i64, i64, vp, i64, vp, C.c_int, vp, i64, C.c_int, vp]
        L.oracle_budget_to_k.argtypes = [i64, i32]
        L.oracle_budget_to_k.restype = i64
        _lib = L
    return _lib


def num_threads() -> int:
    return int(lib().oracle_num_threads())


def _ptr(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _dtype_code(a: np.ndarray) -> int:
    if a.dtype == np.float32:
        return F32
    if a.dtype == np.uint16:
        return BF16
    raise TypeError(f"oracle arrays must be float32 or uint16 (bf16 bits), got {a.dtype}")


def _rows(a: np.ndarray, *others: np.ndarray):
    """2-D arrays whose rows are contiguous but may lie further apart than their length (a column slice of a
    wider array): returned as they are with their common row stride in elements; anything else is copied."""
    arrs = (a,) + others
    es = a.itemsize
    ok = all(x.ndim == 2 and x.strides[1] == es and x.strides[0] % es == 0 and x.strides[0] >= x.shape[1] * es
             and x.strides[0] == a.strides[0] for x in arrs)
    if not ok:
        arrs = tuple(np.ascontiguousarray(x) for x in arrs)
    return arrs + (arrs[0].strides[0] // es,)


def _check(rc: int, what: str):
    if rc != 0:
        raise RuntimeError(f"{what} failed with status {rc}")


def score(x_cur: np.ndarray, x_prev: np.ndarray, mode: int = DELTA_L2, lse_weight=None, skip_count=None,
          penalty_table=None, w_alpha: float = 1.0, w_beta: float = 0.0) -> np.ndarray:
    assert x_cur.ndim == 2 and x_cur.shape == x_prev.shape and x_cur.dtype == x_prev.dtype
    x_cur, x_prev, stride = _rows(x_cur, x_prev)
    n, c = x_cur.shape
    out = np.empty(n, dtype=np.float32)
    if lse_weight is not None:
        lse_weight = np.ascontiguousarray(lse_weight, dtype=np.float32)
    if skip_count is not None:
        skip_count = np.ascontiguousarray(skip_count, dtype=np.int32)
        penalty_table = np.ascontiguousarray(penalty_table, dtype=np.float32)
    tl = 0 if penalty_table is None else int(penalty_table.shape[0])
    _check(lib().oracle_score(_ptr(x_cur), _ptr(x_prev), _dtype_code(x_cur), n, c, stride, mode, _ptr(lse_weight),
                              _ptr(skip_count), _ptr(penalty_table), tl, w_alpha, w_beta, _ptr(out)), "oracle_score")
    return out


def score_f64(x_cur, x_prev, mode=DELTA_L2, lse_weight=None, skip_count=None, w_alpha=1.0, w_beta=0.0) -> np.ndarray:
    x_cur, x_prev, stride = _rows(x_cur, x_prev)
    n, c = x_cur.shape
    out = np.empty(n, dtype=np.float64)
    if lse_weight is not None:
        lse_weight = np.ascontiguousarray(lse_weight, dtype=np.float32)
    if skip_count is not None:
        skip_count = np.ascontiguousarray(skip_count, dtype=np.int32)
    _check(lib().oracle_score_f64(_ptr(x_cur), _ptr(x_prev), _dtype_code(x_cur), n, c, stride, mode, _ptr(lse_weight),
                                  _ptr(skip_count), w_alpha, w_beta, _ptr(out)), "oracle_score_f64")
    return out


def penalty_table(table_len: int) -> np.ndarray:
    """e^n for n = 0..table_len-1, evaluated in fp64 and rounded to fp32 (inf past fp32 range)."""
    with np.errstate(over="ignore"):
        return np.exp(np.arange(table_len, dtype=np.float64)).astype(np.float32)


def topk(score_arr: np.ndarray, k: int, want_remain: bool = True, want_mask: bool = True):
    s = np.ascontiguousarray(score_arr, dtype=np.float32)
    n = s.shape[0]
    idx = np.empty(k, dtype=np.int32)
    rem = np.empty(n - k, dtype=np.int32) if want_remain else None
    mask = np.empty(n, dtype=np.uint8) if want_mask else None
    _check(lib().oracle_topk(_ptr(s), n, k, _ptr(idx), _ptr(rem), _ptr(mask)), "oracle_topk")
    return idx, rem, mask


def update_skip_count(skip_count: np.ndarray, sel_mask: np.ndarray) -> np.ndarray:
    out = np.ascontiguousarray(skip_count, dtype=np.int32).copy()
    m = np.ascontiguousarray(sel_mask, dtype=np.uint8)
    _check(lib().oracle_update_skip_count(_ptr(out), _ptr(m), out.shape[0]), "oracle_update_skip_count")
    return out


def sparse_attn(q: np.ndarray, k: np.ndarray, v: np.ndarray, idx_sel, scale: float, q_is_compact: bool = False,
                acc: str = "f64", want_lse: bool = True):
    """q: [N or k_sel, H, D]; k, v: [N, H, D]; returns (o [k_sel,H,D] fp64, lse [k_sel,H] fp64 or None)."""
    q, k, v = np.ascontiguousarray(q), np.ascontiguousarray(k), np.ascontiguousarray(v)
    n, h, d = k.shape
    if idx_sel is None:
        assert q_is_compact
        k_sel = q.shape[0]
        idx = None
    else:
        idx = np.ascontiguousarray(idx_sel, dtype=np.int32)
        k_sel = idx.shape[0]
    o = np.empty((k_sel, h, d), dtype=np.float64)
    lse = np.empty((k_sel, h), dtype=np.float64) if want_lse else None
    _check(lib().oracle_sparse_attn(_ptr(q), _ptr(k), _ptr(v), _dtype_code(k), n, h, d, h * d, d, h * d, d,
                                    _ptr(idx), k_sel, 1 if q_is_compact else 0, scale, 0 if acc == "f64" else 1,
                                    _ptr(o), _ptr(lse)), "oracle_sparse_attn")
    return o, lse


def lse_weight_update(lse_weight: np.ndarray, lse_sel: np.ndarray, idx_sel) -> None:
    """In place: lse_weight[idx[r]] = mean_h exp(lse_sel[r,h] - ln N)."""
    assert lse_weight.dtype == np.float32 and lse_weight.flags.c_contiguous
    lse = np.ascontiguousarray(lse_sel, dtype=np.float64)
    idx = np.ascontiguousarray(idx_sel, dtype=np.int32)
    _check(lib().oracle_lse_weight_update(_ptr(lse), lse.shape[1], lse_weight.shape[0], _ptr(idx), idx.shape[0],
                                          _ptr(lse_weight)), "oracle_lse_weight_update")


def round_to_dtype(x64: np.ndarray, dtype_code: int) -> np.ndarray:
    x64 = np.ascontiguousarray(x64, dtype=np.float64)
    out = np.empty(x64.shape, dtype=np.float32 if dtype_code == F32 else np.uint16)
    _check(lib().oracle_round_to_dtype(_ptr(x64), x64.size, dtype_code, _ptr(out)), "oracle_round_to_dtype")
    return out


def scatter(cache: np.ndarray, src: np.ndarray, idx_sel, src_is_full: bool = False) -> None:
    """In place: cache[idx[r]] = src[r] (or src[idx[r]] when src_is_full).  cache and src may be column slices
    of wider arrays."""
    assert cache.ndim == 2 and cache.dtype == src.dtype and src.ndim == 2 and src.shape[1] == cache.shape[1]
    (cache_v, cs), (src, ss) = _rows(cache), _rows(src)
    assert cache_v is cache, "the cache is updated in place: its rows must be contiguous"
    idx = np.ascontiguousarray(idx_sel, dtype=np.int32)
    n, e = cache.shape
    _check(lib().oracle_scatter(_ptr(cache), _ptr(src), _dtype_code(cache), n, e, cs, ss, _ptr(idx), idx.shape[0],
                                1 if src_is_full else 0), "oracle_scatter")


def gather(src: np.ndarray, idx_sel) -> np.ndarray:
    src, ss = _rows(src)
    idx = np.ascontiguousarray(idx_sel, dtype=np.int32)
    n, e = src.shape
    dst = np.empty((idx.shape[0], e), dtype=src.dtype)
    _check(lib().oracle_gather(_ptr(src), _ptr(dst), _dtype_code(src), n, e, ss, e, _ptr(idx), idx.shape[0]),
           "oracle_gather")
    return dst


def sparse_linear(x: np.ndarray, w: np.ndarray, idx_sel, bias=None, act: int = ACT_NONE,
                  x_is_compact: bool = False) -> np.ndarray:
    """x: [N or k_sel, c_in]; w: [c_out, c_in]; returns act(x[idx] @ w.T + bias) as [k_sel, c_out] fp64."""
    x, w = np.ascontiguousarray(x), np.ascontiguousarray(w)
    assert x.ndim == 2 and w.ndim == 2 and x.shape[1] == w.shape[1] and x.dtype == w.dtype
    if bias is not None:
        bias = np.ascontiguousarray(bias)
        assert bias.dtype == x.dtype and bias.shape == (w.shape[0],)
    if idx_sel is None:
        assert x_is_compact
        idx, k_sel = None, x.shape[0]
    else:
        idx = np.ascontiguousarray(idx_sel, dtype=np.int32)
        k_sel = idx.shape[0]
    y = np.empty((k_sel, w.shape[0]), dtype=np.float64)
    _check(lib().oracle_sparse_linear(_ptr(x), _dtype_code(x), x.shape[0], x.shape[1], x.shape[1], _ptr(w), w.shape[0],
                                      _ptr(bias), act, _ptr(idx), k_sel, 1 if x_is_compact else 0, _ptr(y)),
           "oracle_sparse_linear")
    return y


def budget_to_k(n: int, pct: int) -> int:
    return int(lib().oracle_budget_to_k(n, pct))
