"""fp64 CPU oracle for the SparseD hot path (test infrastructure, not the product).

Thin ctypes wrapper over ``oracle.c``. Only the tests, ``__graft_entry__.smoke()`` and
``bench.py``'s ``cpu_baseline`` leg may import this package; the HIP library and its
Python binding never do, and this package never imports them.

All array arguments are CPU tensors / arrays. ``q, k, v`` are given as float32
``[B, H, L, d]`` (float32 holds bf16 and fp32 inputs exactly); results are float64.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile oracle.c into liboracle.so with gcc (plain C, -O2, OpenMP)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-Wextra",
               "-o", tmp, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
    return _lib


def _f32(x) -> np.ndarray:
    """float32, C-contiguous numpy view of a tensor / array (bf16 tensors widen exactly)."""
    if hasattr(x, "detach"):
        import torch

        x = x.detach().to("cpu").to(torch.float32).contiguous().numpy()
    a = np.ascontiguousarray(x, dtype=np.float32)
    return a


def _i32(x) -> np.ndarray:
    if hasattr(x, "detach"):
        x = x.detach().to("cpu").numpy()
    return np.ascontiguousarray(x, dtype=np.int32)


def _p(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def _check(rc: int, what: str):
    if rc != 0:
        raise ValueError(f"oracle.{what} rejected its arguments (code {rc})")


def _dims(q, k):
    B, Hq, L, d = q.shape
    Bk, Hkv, Lk, dk = k.shape
    if (Bk, Lk, dk) != (B, L, d):
        raise ValueError("q and k shapes disagree")
    return B, Hq, Hkv, L, d


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def kept_blocks(rho: float, n: int) -> int:
    """How many of n key blocks "top rho%" keeps: ceil(rho*n - 1e-9) clamped to [1, n]."""
    f = _load().oracle_kept_blocks
    f.restype = ctypes.c_int
    f.argtypes = [ctypes.c_double, ctypes.c_int]
    return int(f(float(rho), int(n)))


def attn_probs_row(q, k, b: int, h: int, i: int) -> np.ndarray:
    """One row of A (Eq. 1): softmax over all L keys."""
    q, k = _f32(q), _f32(k)
    B, Hq, Hkv, L, d = _dims(q, k)
    p = np.empty(L, dtype=np.float64)
    _check(_load().oracle_attn_probs_row(_p(q), _p(k), B, Hq, Hkv, L, d, b, h, i, _p(p)), "attn_probs_row")
    return p


def attn_dense(q, k, v) -> np.ndarray:
    """Eq. 1 over the whole tensor -> float64 [B, Hq, L, d]."""
    q, k, v = _f32(q), _f32(k), _f32(v)
    B, Hq, Hkv, L, d = _dims(q, k)
    out = np.empty((B, Hq, L, d), dtype=np.float64)
    _check(_load().oracle_attn_dense(_p(q), _p(k), _p(v), B, Hq, Hkv, L, d, _p(out)), "attn_dense")
    return out


def attn_dense_rows(q, k, v, b: int, h: int, i0: int, i1: int) -> np.ndarray:
    """Eq. 1 for rows [i0, i1) of one (b, h) -> float64 [i1-i0, d]."""
    q, k, v = _f32(q), _f32(k), _f32(v)
    B, Hq, Hkv, L, d = _dims(q, k)
    out = np.empty((i1 - i0, d), dtype=np.float64)
    _check(_load().oracle_attn_dense_rows(_p(q), _p(k), _p(v), B, Hq, Hkv, L, d, b, h, i0, i1, _p(out)),
           "attn_dense_rows")
    return out


def pool_scores(q, k, bq: int, bk: int) -> np.ndarray:
    """A' = avgpool(A, bq x bk) -> float64 [B, Hq, ceil(L/bq), ceil(L/bk)] (partial last blocks: mean of what exists)."""
    q, k = _f32(q), _f32(k)
    B, Hq, Hkv, L, d = _dims(q, k)
    ap = np.empty((B, Hq, -(-L // bq), -(-L // bk)), dtype=np.float64)
    _check(_load().oracle_pool_scores(_p(q), _p(k), B, Hq, Hkv, L, d, bq, bk, _p(ap)), "pool_scores")
    return ap


def pool_scores_rows(q, k, bq: int, bk: int, b: int, h: int, I0: int, I1: int) -> np.ndarray:
    """A' rows for query blocks [I0, I1) of one (b, h) -> float64 [I1-I0, ceil(L/bk)]."""
    q, k = _f32(q), _f32(k)
    B, Hq, Hkv, L, d = _dims(q, k)
    ap = np.empty((I1 - I0, -(-L // bk)), dtype=np.float64)
    _check(_load().oracle_pool_scores_rows(_p(q), _p(k), B, Hq, Hkv, L, d, bq, bk, b, h, I0, I1, _p(ap)),
           "pool_scores_rows")
    return ap


def select_topk(apool: np.ndarray, keep: int):
    """Eq. 6 (single key range). Returns (row_ptr [B,H,nqb+1], col_idx [B,H,nqb*keep], cut [B,H,nqb,2])."""
    apool = np.ascontiguousarray(apool, dtype=np.float64)
    B, H, nqb, nkb = apool.shape
    row_ptr = np.empty((B, H, nqb + 1), dtype=np.int32)
    col_idx = np.empty((B, H, nqb * keep), dtype=np.int32)
    cut = np.empty((B, H, nqb, 2), dtype=np.float64)
    _check(_load().oracle_select_topk(_p(apool), B, H, nqb, nkb, int(keep), _p(row_ptr), _p(col_idx), _p(cut)),
           "select_topk")
    return row_ptr, col_idx, cut


def select_isolated(apool: np.ndarray, rho: float, n_pre: int):
    """Eq. 5 + Eq. 6: separate top-rho% over key blocks [0,n_pre) and [n_pre,nkb); union, ascending."""
    apool = np.ascontiguousarray(apool, dtype=np.float64)
    B, H, nqb, nkb = apool.shape
    keep = (kept_blocks(rho, n_pre) if n_pre > 0 else 0) + (kept_blocks(rho, nkb - n_pre) if nkb > n_pre else 0)
    row_ptr = np.empty((B, H, nqb + 1), dtype=np.int32)
    col_idx = np.empty((B, H, nqb * keep), dtype=np.int32)
    f = _load().oracle_select_isolated
    f.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_double,
                  ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p]
    _check(f(_p(apool), B, H, nqb, nkb, float(rho), int(n_pre), _p(row_ptr), _p(col_idx)), "select_isolated")
    return row_ptr, col_idx


def prefill_ranges(L: int, bk: int, prefill_tokens: int):
    """Key ranges for isolated selection with the boundary at a key token: one range per key block,
    except that the block holding the boundary is split in two. Returns (vstart, vend, vblock, n_pre)."""
    nkb = -(-L // bk)
    vstart, vend, vblock = [], [], []
    for J in range(nkb):
        lo, hi = J * bk, min((J + 1) * bk, L)
        if lo < prefill_tokens < hi:
            vstart += [lo, prefill_tokens]
            vend += [prefill_tokens, hi]
            vblock += [J, J]
        else:
            vstart.append(lo)
            vend.append(hi)
            vblock.append(J)
    n_pre = sum(1 for e in vend if e <= prefill_tokens)
    i32 = lambda x: np.asarray(x, dtype=np.int32)  # noqa: E731
    return i32(vstart), i32(vend), i32(vblock), n_pre


def select_isolated_tokens(q, k, bq: int, bk: int, rho: float, prefill_tokens: int):
    """Eq. 5 + Eq. 6 with the prefill / generation boundary at key token ``prefill_tokens``.

    Returns (row_ptr [B,H,nqb+1], col_idx [B,H,cap], apool_ranges [B,H,nqb,nv], n_pre, vblock);
    rows may differ in length by one (the block holding the boundary can be kept by both ranges)."""
    q, k = _f32(q), _f32(k)
    B, Hq, Hkv, L, d = _dims(q, k)
    vstart, vend, vblock, n_pre = prefill_ranges(L, bk, prefill_tokens)
    nv, nqb = len(vstart), -(-L // bq)
    ap = np.empty((B, Hq, nqb, nv), dtype=np.float64)
    lib = _load()
    _check(lib.oracle_pool_scores_ranges(_p(q), _p(k), B, Hq, Hkv, L, d, bq, nv, _p(vstart), _p(vend), _p(ap)), "pool_scores_ranges")
    keep = (kept_blocks(rho, n_pre) if n_pre > 0 else 0) + (kept_blocks(rho, nv - n_pre) if nv > n_pre else 0)
    cap = nqb * keep
    row_ptr = np.empty((B, Hq, nqb + 1), dtype=np.int32)
    col_idx = np.full((B, Hq, cap), -1, dtype=np.int32)
    f = lib.oracle_select_isolated_ranges
    f.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_double, ctypes.c_int,
                  ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p]
    _check(f(_p(ap), B, Hq, nqb, nv, float(rho), int(n_pre), _p(vblock), cap, _p(row_ptr), _p(col_idx)), "select_isolated_ranges")
    return row_ptr, col_idx, ap, n_pre, vblock


def select_pattern(q, k, bq: int, bk: int, rho: float):
    """Pooling + Eq. 6: what the selection step of Algorithm 1 produces.

    Returns (row_ptr, col_idx, apool, cut).
    """
    ap = pool_scores(q, k, bq, bk)
    keep = kept_blocks(rho, ap.shape[-1])
    row_ptr, col_idx, cut = select_topk(ap, keep)
    return row_ptr, col_idx, ap, cut


def attn_sparse(q, k, v, row_ptr, col_idx, bq: int, bk: int) -> np.ndarray:
    """Eq. 3 with the block mask of Eq. 4 -> float64 [B, Hq, L, d]."""
    q, k, v = _f32(q), _f32(k), _f32(v)
    row_ptr, col_idx = _i32(row_ptr), _i32(col_idx)
    B, Hq, Hkv, L, d = _dims(q, k)
    cap = col_idx.shape[-1]
    out = np.empty((B, Hq, L, d), dtype=np.float64)
    _check(_load().oracle_attn_sparse(_p(q), _p(k), _p(v), B, Hq, Hkv, L, d, bq, bk, _p(row_ptr), _p(col_idx),
                                      cap, _p(out)), "attn_sparse")
    return out


def attn_sparse_rows(q, k, v, row_ptr, col_idx, bq: int, bk: int, b: int, h: int, I0: int, I1: int) -> np.ndarray:
    """Eq. 3/4 for query blocks [I0, I1) of one (b, h) -> float64 [(I1-I0)*bq, d] (rows past L stay zero)."""
    q, k, v = _f32(q), _f32(k), _f32(v)
    row_ptr, col_idx = _i32(row_ptr), _i32(col_idx)
    B, Hq, Hkv, L, d = _dims(q, k)
    cap = col_idx.shape[-1]
    out = np.zeros(((I1 - I0) * bq, d), dtype=np.float64)
    _check(_load().oracle_attn_sparse_rows(_p(q), _p(k), _p(v), B, Hq, Hkv, L, d, bq, bk, _p(row_ptr),
                                           _p(col_idx), cap, b, h, I0, I1, _p(out)), "attn_sparse_rows")
    return out


def attn_masked_bruteforce(q, k, v, row_ptr, col_idx, bq: int, bk: int) -> np.ndarray:
    """Eq. 3 + Eq. 4 with an explicit L x L matrix of 0 / -inf (tiny inputs only)."""
    q, k, v = _f32(q), _f32(k), _f32(v)
    row_ptr, col_idx = _i32(row_ptr), _i32(col_idx)
    B, Hq, Hkv, L, d = _dims(q, k)
    cap = col_idx.shape[-1]
    out = np.empty((B, Hq, L, d), dtype=np.float64)
    _check(_load().oracle_attn_masked_bruteforce(_p(q), _p(k), _p(v), B, Hq, Hkv, L, d, bq, bk, _p(row_ptr),
                                                 _p(col_idx), cap, _p(out)), "attn_masked_bruteforce")
    return out
