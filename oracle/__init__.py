"""ctypes loader for the CPU oracle (oracle/vt_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg.  The product package never imports this module.

All functions take and return NumPy arrays; every real-valued result is fp64.
bf16 inputs are passed as uint16 bit patterns.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

from .selection import choose_k_min_count, choose_k_top_p, rank_order  # noqa: F401
from .tree import tree_expand, tree_rerank  # noqa: F401  (numpy-only oracle of the tree selection steps)

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "vt_oracle.c")
_LIB = os.path.join(_HERE, "libvt_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile vt_oracle.c with gcc (-O2, no fast-math, OpenMP for the row loop)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        vp, i32, i64, ci = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_int
        L.vt_oracle_set_threads.argtypes = [ci]
        L.vt_oracle_get_threads.restype = ci
        L.vt_oracle_count.argtypes = [vp, ci, i64, i32, vp, vp]
        L.vt_oracle_select.argtypes = [vp, i32, i32, vp, vp]
        L.vt_oracle_gather.argtypes = [vp, i64, i32, vp, i32, vp]
        L.vt_oracle_logits.argtypes = [vp, vp, ci, i32, i32, i32, vp]
        L.vt_oracle_log_softmax.argtypes = [vp, i32, i32, vp, vp]
        L.vt_oracle_top_m.argtypes = [vp, vp, i32, i32, vp, i32, vp, vp, vp]
        for f in ("vt_oracle_set_threads", "vt_oracle_count", "vt_oracle_select", "vt_oracle_gather",
                  "vt_oracle_logits", "vt_oracle_log_softmax", "vt_oracle_top_m"):
            getattr(L, f).restype = None
        _lib = L
    return _lib


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def set_threads(t: int) -> None:
    _load().vt_oracle_set_threads(int(t))


def get_threads() -> int:
    return int(_load().vt_oracle_get_threads())


def count(ids: np.ndarray, V: int, counts: np.ndarray | None = None):
    """Alg. 1.  Returns (counts[V] int64, n_invalid).  Accumulates into `counts` if given."""
    ids = np.ascontiguousarray(ids)
    if ids.dtype not in (np.int32, np.int64):
        raise TypeError("ids must be int32 or int64")
    if counts is None:
        counts = np.zeros(V, dtype=np.int64)
    assert counts.dtype == np.int64 and counts.shape == (V,) and counts.flags.c_contiguous
    inval = np.zeros(1, dtype=np.int64)
    _load().vt_oracle_count(_p(ids), int(ids.dtype == np.int64), ids.size, V, _p(counts), _p(inval))
    return counts, int(inval[0])


def select(counts: np.ndarray, k: int, return_rank_order: bool = False):
    """Eq. 1 line 1.  Returns map[k] int32 ascending (and optionally the frequency-rank order)."""
    counts = np.ascontiguousarray(counts, dtype=np.int64)
    V = counts.size
    assert 1 <= k <= V
    m = np.empty(k, dtype=np.int32)
    ro = np.empty(k, dtype=np.int32)
    _load().vt_oracle_select(_p(counts), V, k, _p(m), _p(ro))
    return (m, ro) if return_rank_order else m


def gather(W: np.ndarray, map_: np.ndarray) -> np.ndarray:
    """Eq. 1 line 2.  W[V,d] (float32 or uint16 bf16 bits) -> W_trim[k,d], same dtype."""
    W = np.ascontiguousarray(W)
    map_ = np.ascontiguousarray(map_, dtype=np.int32)
    out = np.empty((map_.size, W.shape[1]), dtype=W.dtype)
    _load().vt_oracle_gather(_p(W), W.dtype.itemsize, W.shape[1], _p(map_), map_.size, _p(out))
    return out


def _is_bf16(a: np.ndarray) -> int:
    if a.dtype == np.uint16:
        return 1
    if a.dtype == np.float32:
        return 0
    raise TypeError("expected float32 or uint16 (bf16 bits)")


def logits(h: np.ndarray, W_trim: np.ndarray) -> np.ndarray:
    """z[n,k] = h @ W_trim^T in fp64."""
    h = np.ascontiguousarray(h)
    W_trim = np.ascontiguousarray(W_trim)
    assert _is_bf16(h) == _is_bf16(W_trim) and h.shape[1] == W_trim.shape[1]
    n, d = h.shape
    k = W_trim.shape[0]
    z = np.empty((n, k), dtype=np.float64)
    _load().vt_oracle_logits(_p(h), _p(W_trim), _is_bf16(h), n, k, d, _p(z))
    return z


def log_softmax(z: np.ndarray):
    """Returns (lse[n], logp[n,k]) over the k trimmed logits."""
    z = np.ascontiguousarray(z, dtype=np.float64)
    n, k = z.shape
    lse = np.empty(n, dtype=np.float64)
    logp = np.empty((n, k), dtype=np.float64)
    _load().vt_oracle_log_softmax(_p(z), n, k, _p(lse), _p(logp))
    return lse, logp


def lse_only(z: np.ndarray) -> np.ndarray:
    z = np.ascontiguousarray(z, dtype=np.float64)
    n, k = z.shape
    lse = np.empty(n, dtype=np.float64)
    _load().vt_oracle_log_softmax(_p(z), n, k, _p(lse), None)
    return lse


def top_m(z: np.ndarray, lse: np.ndarray, map_: np.ndarray, m: int):
    """Returns (ids[n,m] target ids, logp[n,m] fp64, trim_idx[n,m])."""
    z = np.ascontiguousarray(z, dtype=np.float64)
    lse = np.ascontiguousarray(lse, dtype=np.float64)
    map_ = np.ascontiguousarray(map_, dtype=np.int32)
    n, k = z.shape
    assert map_.size == k and 1 <= m <= k
    ids = np.empty((n, m), dtype=np.int32)
    lp = np.empty((n, m), dtype=np.float64)
    ti = np.empty((n, m), dtype=np.int32)
    _load().vt_oracle_top_m(_p(z), _p(lse), n, k, _p(map_), m, _p(ids), _p(lp), _p(ti))
    return ids, lp, ti


def draft_head_step(h, W_trim, map_, m):
    """The whole draft step: projection, log-softmax, top-m, remap.

    Returns dict(ids, logp, lse, z, trim_idx) with fp64 reals.
    """
    z = logits(h, W_trim)
    lse = lse_only(z)
    ids, lp, ti = top_m(z, lse, map_, m)
    return {"ids": ids, "logp": lp, "lse": lse, "z": z, "trim_idx": ti}


def draft_head_step_multi(h, heads, head_of_row, m):
    """A draft step in which hidden row i uses heads[head_of_row[i]] = (W_trim, map) (Sec. 4.1, task-specific
    vocabularies next to the general one): row by row, the single-head step of that row on its head.

    Returns dict(ids [n,m], logp [n,m] fp64, lse [n] fp64).
    """
    n = h.shape[0]
    ids = np.zeros((n, m), dtype=np.int32)
    lp = np.zeros((n, m), dtype=np.float64)
    lse = np.zeros(n, dtype=np.float64)
    for i in range(n):
        W_trim, map_ = heads[int(head_of_row[i])]
        r = draft_head_step(h[i:i + 1], W_trim, map_, m)
        ids[i], lp[i], lse[i] = r["ids"][0], r["logp"][0], r["lse"][0]
    return {"ids": ids, "logp": lp, "lse": lse}
