"""ctypes front end of the CPU oracle (oracle/alaya_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
bench's cpu_baseline leg.  It never imports the HIP package, and the HIP
package never imports it.

All array arguments are numpy arrays; K and V are token-major
[n][n_kv_heads][head_dim], stored either as float32 or as bf16 bit patterns in
uint16 (dtype is inferred from the numpy dtype).  Results are fp64.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "alaya_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

BF16, F32 = 0, 1
TOPK, DIPR, FULL = 0, 1, 2


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (a second or so)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
                               "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        vp, i32, i64, f64 = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_double
        lib.oracle_scores.argtypes = [vp, vp, i32, i64, i32, i32, i32, vp]
        lib.oracle_scores.restype = None
        lib.oracle_select_topk.argtypes = [vp, i64, i64, vp]
        lib.oracle_select_topk.restype = i64
        lib.oracle_select_dipr.argtypes = [vp, i64, f64, vp]
        lib.oracle_select_dipr.restype = i64
        lib.oracle_attend.argtypes = [vp, vp, i32, i32, i32, i32, vp, i64, f64, vp]
        lib.oracle_attend.restype = None
        lib.oracle_select_window.argtypes = [vp, i64, i64, i64, i32, i64, f64, vp]
        lib.oracle_select_window.restype = i64
        lib.oracle_block_reps.argtypes = [vp, i32, i64, i32, i32, i32, i64, vp, vp]
        lib.oracle_block_reps.restype = None
        lib.oracle_block_scores.argtypes = [vp, i32, vp, vp, i64, i32, vp]
        lib.oracle_block_scores.restype = None
        lib.oracle_select_topk_in_blocks.argtypes = [vp, i64, i64, vp, i64, i64, i64, i64, vp]
        lib.oracle_select_topk_in_blocks.restype = i64
        lib.oracle_coarse_attn.argtypes = [vp, vp, vp, i32, i64, i64, i32, i32, i32, i64, i64, i64, f64, i64, i64, vp,
                                           vp, i64, vp, vp, vp, i64, vp, vp, i32]
        lib.oracle_coarse_attn.restype = i32
        lib.oracle_scores_f32.argtypes = [vp, vp, i32, i64, i32, i32, i32, vp]
        lib.oracle_scores_f32.restype = None
        lib.oracle_knn_graph.argtypes = [vp, i32, i64, i32, i32, i32, i32, vp]
        lib.oracle_knn_graph.restype = None
        lib.oracle_diprs.argtypes = [vp, i64, i32, vp, i32, i64, ctypes.c_float, i64, i64, vp, vp, vp]
        lib.oracle_diprs.restype = i64
        lib.oracle_sparse_attn.argtypes = [vp, vp, vp, i32, i64, i32, i32, i32, i32, i64, f64, f64, i64, i64,
                                           vp, vp, i64, vp, vp, i32]
        lib.oracle_sparse_attn.restype = i32
        _lib = lib
    return _lib


def _dt(a: np.ndarray) -> int:
    if a.dtype == np.float32:
        return F32
    if a.dtype == np.uint16:
        return BF16
    raise TypeError(f"oracle takes float32 or uint16 (bf16 bits), got {a.dtype}")


def _c(a: np.ndarray) -> np.ndarray:
    return np.ascontiguousarray(a)


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def scores(q_h: np.ndarray, K: np.ndarray, g: int) -> np.ndarray:
    """Raw inner products of one query head against KV head g: fp64 [n]."""
    q_h, K = _c(q_h), _c(K)
    n, hk, d = K.shape
    assert q_h.shape == (d,) and _dt(q_h) == _dt(K)
    s = np.empty(n, dtype=np.float64)
    _load().oracle_scores(_p(q_h), _p(K), _dt(K), n, hk, g, d, _p(s))
    return s


def select_topk(s: np.ndarray, k: int) -> np.ndarray:
    s = _c(s.astype(np.float64, copy=False))
    ids = np.empty(max(1, min(max(k, 0), s.size)), dtype=np.int32)
    cnt = _load().oracle_select_topk(_p(s), s.size, k, _p(ids))
    if cnt < 0:
        raise ValueError("k must be positive")
    return ids[:cnt].copy()


def select_dipr(s: np.ndarray, beta: float) -> np.ndarray:
    s = _c(s.astype(np.float64, copy=False))
    ids = np.empty(max(1, s.size), dtype=np.int32)
    cnt = _load().oracle_select_dipr(_p(s), s.size, float(beta), _p(ids))
    if cnt < 0:
        raise ValueError("beta must be >= 0")
    return ids[:cnt].copy()


def select_window(s: np.ndarray, w0: int, w1: int, mode: int, k: int = 0, beta: float = 0.0) -> np.ndarray:
    """Window tokens (first w0, last w1) plus the query's result among / beside them: ascending ids."""
    s = _c(s.astype(np.float64, copy=False))
    ids = np.empty(max(1, s.size), dtype=np.int32)
    cnt = _load().oracle_select_window(_p(s), s.size, int(w0), int(w1), int(mode), int(k), float(beta), _p(ids))
    if cnt < 0:
        raise ValueError("invalid k, beta or window")
    return ids[:cnt].copy()


def block_reps(K: np.ndarray, g: int, block: int) -> Tuple[np.ndarray, np.ndarray]:
    """Channel-wise minimum and maximum of the keys of KV head g over blocks of `block` adjacent tokens: fp64 [nb][d] each."""
    K = _c(K)
    n, hk, d = K.shape
    nb = (n + block - 1) // block
    lo, hi = np.empty((nb, d), dtype=np.float64), np.empty((nb, d), dtype=np.float64)
    _load().oracle_block_reps(_p(K), _dt(K), n, hk, g, d, int(block), _p(lo), _p(hi))
    return lo, hi


def block_scores(q_h: np.ndarray, lo: np.ndarray, hi: np.ndarray) -> np.ndarray:
    """u_b = sum_c max(q_c lo_bc, q_c hi_bc): fp64 [nb]."""
    q_h, lo, hi = _c(q_h), _c(lo.astype(np.float64, copy=False)), _c(hi.astype(np.float64, copy=False))
    nb, d = lo.shape
    assert hi.shape == lo.shape and q_h.shape == (d,)
    u = np.empty(nb, dtype=np.float64)
    _load().oracle_block_scores(_p(q_h), _dt(q_h), _p(lo), _p(hi), nb, d, _p(u))
    return u


def select_topk_in_blocks(s: np.ndarray, block: int, blocks: np.ndarray, k: int, window: Tuple[int, int] = (0, 0)) -> np.ndarray:
    """Window tokens plus the k best tokens outside the window among the tokens of the given blocks: ascending ids."""
    s = _c(s.astype(np.float64, copy=False))
    blocks = _c(np.asarray(blocks, dtype=np.int32))
    if blocks.size and (blocks.min() < 0 or blocks.max() * block >= s.size):
        raise IndexError("block out of range")
    ids = np.empty(max(1, s.size), dtype=np.int32)
    cnt = _load().oracle_select_topk_in_blocks(_p(s), s.size, int(block), _p(blocks), blocks.size, int(window[0]),
                                               int(window[1]), int(k), _p(ids))
    if cnt < 0:
        raise ValueError("invalid k, block or window")
    return ids[:cnt].copy()


def coarse_attn(q: np.ndarray, K: np.ndarray, V: np.ndarray, block: int, n_blocks: int, k: int,
                scale: Optional[float] = None, window: Tuple[int, int] = (0, 0), n_visible: Optional[int] = None,
                want_scores: bool = False, threads: int = 0) -> dict:
    """Top-k through the coarse index, one request, all heads: the n_blocks best blocks per head, then top-k
    among their tokens.  n_visible: the query sees that prefix only, through the index of the whole stored
    context (a block's representatives cover its hidden tokens too).  Returns {"out", "counts", "ids",
    "blocks": list of int32 arrays (ascending), "u": fp64 [Hq][nb] block scores, "scores": fp64 [Hq][n_visible]
    or None, "threads"}."""
    q, K, V = _c(q), _c(K), _c(V)
    n, hk, d = K.shape
    nv = n if n_visible is None else int(n_visible)
    if not 0 < nv <= n:
        raise ValueError("n_visible out of range")
    hq = q.shape[0]
    assert V.shape == K.shape and q.shape == (hq, d) and _dt(q) == _dt(K) == _dt(V)
    nb = (nv + block - 1) // block
    out = np.empty((hq, d), dtype=np.float64)
    counts, bcounts = np.zeros(hq, dtype=np.int64), np.zeros(hq, dtype=np.int64)
    ids = np.empty((hq, nv), dtype=np.int32)
    blocks = np.empty((hq, nb), dtype=np.int32)
    u = np.empty((hq, nb), dtype=np.float64)
    sc = np.empty((hq, nv), dtype=np.float64) if want_scores else None
    rc = _load().oracle_coarse_attn(_p(q), _p(K), _p(V), _dt(K), n, nv, hq, hk, d, int(block), int(n_blocks), int(k),
                                    float(scale) if scale else 0.0, int(window[0]), int(window[1]), _p(out),
                                    _p(ids), nv, _p(counts), _p(sc), _p(blocks), nb, _p(bcounts), _p(u), int(threads))
    if rc < 0:
        raise ValueError(f"oracle error {rc}")
    return {"out": out, "counts": counts, "ids": [ids[h, :counts[h]].copy() for h in range(hq)],
            "blocks": [blocks[h, :bcounts[h]].copy() for h in range(hq)], "u": u, "scores": sc, "threads": rc}


def scores_f32(q_h: np.ndarray, K: np.ndarray, g: int) -> np.ndarray:
    """Inner products in the arithmetic DIPRS decides in: fp32, one fused multiply-add per channel in order."""
    q_h, K = _c(q_h), _c(K)
    n, hk, d = K.shape
    assert q_h.shape == (d,) and _dt(q_h) == _dt(K)
    s = np.empty(n, dtype=np.float32)
    _load().oracle_scores_f32(_p(q_h), _p(K), _dt(K), n, hk, g, d, _p(s))
    return s


def knn_graph(K: np.ndarray, g: int, M: int) -> np.ndarray:
    """Exact M-nearest-neighbour graph of KV head g's keys under the inner product: int32 [n][M], best first, -1 padded."""
    K = _c(K)
    n, hk, d = K.shape
    nbr = np.empty((n, M), dtype=np.int32)
    _load().oracle_knn_graph(_p(K), _dt(K), n, hk, g, d, int(M), _p(nbr))
    return nbr


def diprs(nbr: np.ndarray, s: np.ndarray, k0: int, l0: int, beta: float, window: Tuple[int, int] = (0, 0)):
    """Algorithm 1 on the graph nbr [n][M] with fp32 scores s: returns (ids ascending, C in the order it grew)."""
    nbr = _c(np.asarray(nbr, dtype=np.int32))
    s = _c(np.asarray(s, dtype=np.float32))
    n, M = nbr.shape
    assert s.shape == (n,)
    C = np.empty(n, dtype=np.int32)
    ids = np.empty(n, dtype=np.int32)
    clen = ctypes.c_int64(0)
    cnt = _load().oracle_diprs(_p(nbr), n, M, _p(s), int(k0), int(l0), float(beta), int(window[0]), int(window[1]),
                               _p(C), ctypes.byref(clen), _p(ids))
    if cnt < 0:
        raise ValueError("invalid DIPRS arguments")
    return ids[:cnt].copy(), C[:clen.value].copy()


def attend(s: np.ndarray, V: np.ndarray, g: int, ids: np.ndarray, scale: Optional[float] = None) -> np.ndarray:
    """Softmax over the given token set and the weighted sum of its V rows: fp64 [d]."""
    s, V = _c(s.astype(np.float64, copy=False)), _c(V)
    ids = _c(np.asarray(ids, dtype=np.int32))
    n, hk, d = V.shape
    assert s.shape == (n,)
    if ids.size and (ids.min() < 0 or ids.max() >= n):
        raise IndexError("token id out of range")
    sc = float(scale) if scale is not None else 1.0 / np.sqrt(d)
    o = np.empty(d, dtype=np.float64)
    _load().oracle_attend(_p(s), _p(V), _dt(V), hk, g, d, _p(ids), ids.size, sc, _p(o))
    return o


def sparse_attn(q: np.ndarray, K: np.ndarray, V: np.ndarray, mode: int, k: int = 0, beta: float = 0.0,
                scale: Optional[float] = None, want_ids: bool = True, want_scores: bool = False,
                threads: int = 0, window: Tuple[int, int] = (0, 0), n_visible: Optional[int] = None) -> dict:
    """One request, all heads.  q [n_q_heads][d]; K, V [n][n_kv_heads][d].

    window = (first, last) tokens that are always attended; n_visible: only that prefix of K, V exists
    for the query (it is cut off here, the C code never sees the rest).

    Returns {"out": fp64 [Hq][d], "counts": int64 [Hq], "ids": list of int32 arrays (ascending),
             "scores": fp64 [Hq][n] or None, "threads": OpenMP threads used}.
    """
    if n_visible is not None:
        if not 0 < n_visible <= K.shape[0]:
            raise ValueError("n_visible out of range")
        K, V = K[:n_visible], V[:n_visible]
    q, K, V = _c(q), _c(K), _c(V)
    n, hk, d = K.shape
    hq = q.shape[0]
    assert V.shape == K.shape and q.shape == (hq, d) and _dt(q) == _dt(K) == _dt(V)
    out = np.empty((hq, d), dtype=np.float64)
    counts = np.zeros(hq, dtype=np.int64)
    stride = n if want_ids else 0
    ids = np.empty((hq, stride), dtype=np.int32) if want_ids else None
    sc = np.empty((hq, n), dtype=np.float64) if want_scores else None
    rc = _load().oracle_sparse_attn(_p(q), _p(K), _p(V), _dt(K), n, hq, hk, d, int(mode), int(k),
                                    float(beta), float(scale) if scale else 0.0, int(window[0]), int(window[1]),
                                    _p(out), _p(ids), stride, _p(counts), _p(sc), int(threads))
    if rc < 0:
        raise ValueError({-1: "bad shapes or n == 0", -2: "k must be positive",
                          -3: "beta must be >= 0", -4: "window sizes must be >= 0"}.get(rc, f"oracle error {rc}"))
    id_list = [ids[h, :counts[h]].copy() for h in range(hq)] if want_ids else None
    return {"out": out, "counts": counts, "ids": id_list, "scores": sc, "threads": rc}


def plan(context_len: int, short_context: int, reused_prefix: int, gpu_budget: int, coarse_need: int, layer_id: int):
    """The rule-based optimizer's workflow (Sec. 6.2 "Query Optimizer"): (query type, index type, visible prefix).

    Short contexts get full attention.  A long context that is only partly reused is queried under the filter
    "position < reused prefix".  With enough GPU memory for the blocks the plan is top-k on the coarse-grained
    index; otherwise DIPR, on the flat index for the first layer and on the graph for every other layer."""
    if context_len <= short_context:
        return ("full", "none", context_len)
    visible = reused_prefix if 0 < reused_prefix < context_len else context_len
    if gpu_budget >= coarse_need:
        return ("topk", "coarse", visible)
    return ("dipr", "flat" if layer_id == 0 else "fine", visible)


def full_attn(q: np.ndarray, K: np.ndarray, V: np.ndarray, scale: Optional[float] = None,
              threads: int = 0) -> np.ndarray:
    return sparse_attn(q, K, V, FULL, scale=scale, want_ids=False, threads=threads)["out"]
