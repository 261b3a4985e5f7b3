"""Seeded synthetic inputs for the sparse-attention decode path.

This module serves both the CPU oracle and the HIP path and holds none of the
method's arithmetic: it only draws random numbers, shapes them like the
paper's workload (Llama-3-8B-style heads: 32 query heads sharing 8 KV heads,
head_dim 128, bf16, Sec. 9 "Experimental Setting"; a few dominant keys among a
long tail, Sec. 2 "Sparse Attention") and rounds them once to the storage
type.  Both sides then read the very same bytes.

Recipe (per request r, KV head g, channel c, token j):
    scale[r][g][c] = exp(0.5 * N(0,1))                 lognormal(0, 0.5) per channel
    K[r][j][g][c]  = N(0,1) * scale[r][g][c]
    V[r][j][g][c]  = N(0,1)
    P[r][h]        = p distinct token ids, uniform      (h = query head, g = h // G)
    q[r][h]        = q_scale * unit_l2(sum_{j in P} K[r][j][g]) + N(0, 0.1) per channel
    bf16 workloads round K, V and q to bf16 (round to nearest even) once.

Every tensor has its own counter-based Philox stream keyed by
(seed, tensor tag, request, KV/query head), so any slice can be regenerated
on its own and generation can run in threads without changing a single byte.
"""
from __future__ import annotations

import dataclasses
import math
import os
from concurrent.futures import ThreadPoolExecutor
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

PAGE_TOKENS = 64

_TAG = {"scale": 1, "K": 2, "V": 3, "planted": 4, "qnoise": 5, "lens": 6, "pages": 7}


@dataclasses.dataclass(frozen=True)
class Workload:
    """Shape and recipe of one synthetic decode-step query."""

    name: str
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    lens: Tuple[int, ...]              # cached tokens per request
    dtype: str                         # "bf16" or "f32": storage type of K, V and q
    planted: int                       # high-affinity keys summed into each query
    mode: str                          # "topk" or "dipr"
    topk: Optional[Tuple[int, ...]] = None    # per request
    betas: Optional[Tuple[float, ...]] = None  # DIPR margins to sweep (raw inner-product units)
    permute_pages: bool = False        # physical pages handed out in a seeded random order
    seed: int = 0
    q_scale: float = 1.0               # knob on the planted direction of q (1.0 = the stated recipe)
    cluster_runs: int = 0              # per query head: runs of two adjacent pages whose keys all lean towards the query
    cluster_last: int = 0              # ... and that many last tokens of the request lean towards every query of the group
    cluster_shift: float = 0.0         # how far they lean (added along the unit query, raw inner-product units / |q|)
    page_tokens: int = PAGE_TOKENS

    @property
    def batch(self) -> int:
        return len(self.lens)

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def total_tokens(self) -> int:
        return int(sum(self.lens))

    def pages_needed(self) -> int:
        return int(sum((n + self.page_tokens - 1) // self.page_tokens for n in self.lens))


def _rng(seed: int, tag: str, a: int = 0, b: int = 0) -> np.random.Generator:
    key = (int(seed) & 0xFFFFFFFF) | (_TAG[tag] << 32) | ((a & 0xFFFF) << 40) | ((b & 0xFF) << 56)
    return np.random.Generator(np.random.Philox(key=key))


def batched_lens(seed: int, batch: int = 16, lo: int = 32768, hi: int = 262144) -> Tuple[int, ...]:
    """Context lengths of the batched-decode workload: uniform integers in [lo, hi]."""
    r = _rng(seed, "lens")
    return tuple(int(x) for x in r.integers(lo, hi + 1, size=batch))


def config(name: str, seed: int = 0) -> Workload:
    """The five workloads the build is measured and tested on, at full size."""
    if name == "tiny":
        return Workload("tiny", 1, 1, 128, (4096,), "f32", 8, "topk", topk=(64,), seed=seed)
    if name == "llama8b_128k":
        return Workload("llama8b_128k", 32, 8, 128, (131072,), "bf16", 32, "topk", topk=(2048,), seed=seed)
    if name == "range_256k":
        return Workload("range_256k", 32, 8, 128, (262144,), "bf16", 32, "dipr",
                        betas=(0.5, 1.0, 2.0, 4.0), seed=seed)
    if name == "paged_1m":
        return Workload("paged_1m", 32, 8, 128, (1048576,), "bf16", 32, "topk", topk=(4096,),
                        permute_pages=True, seed=seed)
    if name == "clustered_128k":
        # The recipe above scatters the keys that matter uniformly over the context.  In a real cache the keys of
        # adjacent tokens are alike and the recent tokens matter most (Sec. 7.1: a window of the last tokens holds
        # the best key almost always): here each head's high-affinity keys sit in four runs of two pages and in
        # the last 512 tokens.  Same shapes as llama8b_128k; a robustness measurement, not a parity bar.
        return Workload("clustered_128k", 32, 8, 128, (131072,), "bf16", 32, "topk", topk=(2048,), seed=seed,
                        cluster_runs=4, cluster_last=512, cluster_shift=6.0)
    if name == "batched_16":
        lens = batched_lens(seed)
        return Workload("batched_16", 32, 8, 128, lens, "bf16", 32, "topk",
                        topk=tuple(int(math.ceil(0.02 * n)) for n in lens), seed=seed)
    raise KeyError(name)


def resized(w: Workload, lens: Sequence[int], topk: Optional[Sequence[int]] = None, **kw) -> Workload:
    """Same recipe at other context lengths (parity cases the oracle finishes quickly)."""
    lens = tuple(int(n) for n in lens)
    if topk is None and w.topk is not None:
        if w.name.startswith("batched"):
            topk = tuple(max(1, int(math.ceil(0.02 * n))) for n in lens)
        else:
            topk = tuple(w.topk[0] for _ in lens)
    return dataclasses.replace(w, lens=lens, topk=None if topk is None else tuple(int(k) for k in topk), **kw)


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit patterns (uint16), round to nearest even. Inputs are finite."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    return (r >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def _store(x: np.ndarray, dtype: str) -> np.ndarray:
    return to_bf16_bits(x) if dtype == "bf16" else np.ascontiguousarray(x, dtype=np.float32)


def _gen_kv_head(w: Workload, r: int, g: int, K: np.ndarray, V: np.ndarray, chunk: int = 1 << 17):
    """Fill K[:, g, :] and V[:, g, :] of request r, chunk by chunk."""
    n, d = w.lens[r], w.head_dim
    scale = np.exp(0.5 * _rng(w.seed, "scale", r, g).standard_normal(d)).astype(np.float32)
    rk, rv = _rng(w.seed, "K", r, g), _rng(w.seed, "V", r, g)
    for j0 in range(0, n, chunk):
        m = min(chunk, n - j0)
        K[j0:j0 + m, g, :] = _store(rk.standard_normal((m, d), dtype=np.float32) * scale, w.dtype)
        V[j0:j0 + m, g, :] = _store(rv.standard_normal((m, d), dtype=np.float32), w.dtype)


def _as_f32(x: np.ndarray, dtype: str) -> np.ndarray:
    return bf16_bits_to_f32(x) if dtype == "bf16" else x.astype(np.float32)


def generate(w: Workload, threads: Optional[int] = None) -> Dict[str, object]:
    """Draw every tensor of the workload.

    Returns a dict with
      K, V    : list over requests of arrays [n][n_kv_heads][head_dim]  (uint16 bf16 bits, or float32)
      q       : array [batch][n_q_heads][head_dim]                      (same storage type)
      planted : int32 array [batch][n_q_heads][planted]  token ids summed into each query
      page_order : int32 array, the order in which physical pages are handed out
                   (identity unless permute_pages), length = n_phys_pages
      n_phys_pages : pages in the pool (exactly what the lengths need, plus one spare per request
                   so that a few decode steps can be appended)
    """
    st = np.uint16 if w.dtype == "bf16" else np.float32
    d, Hk, Hq, G = w.head_dim, w.n_kv_heads, w.n_q_heads, w.group
    Ks = [np.empty((n, Hk, d), dtype=st) for n in w.lens]
    Vs = [np.empty((n, Hk, d), dtype=st) for n in w.lens]
    jobs = [(r, g) for r in range(w.batch) for g in range(Hk)]
    nthr = threads or min(len(jobs), max(1, min(16, (os.cpu_count() or 1))))
    if nthr > 1:
        with ThreadPoolExecutor(nthr) as ex:
            list(ex.map(lambda rg: _gen_kv_head(w, rg[0], rg[1], Ks[rg[0]], Vs[rg[0]]), jobs))
    else:
        for r, g in jobs:
            _gen_kv_head(w, r, g, Ks[r], Vs[r])

    q = np.empty((w.batch, Hq, d), dtype=np.float32)
    planted = np.empty((w.batch, Hq, w.planted), dtype=np.int32)
    for r, n in enumerate(w.lens):
        for h in range(Hq):
            g = h // G
            ids = _rng(w.seed, "planted", r, h).choice(n, size=min(w.planted, n), replace=False)
            ids = np.sort(ids).astype(np.int32)
            planted[r, h, :len(ids)] = ids
            planted[r, h, len(ids):] = ids[-1]
            ksum = _as_f32(Ks[r][ids, g, :], w.dtype).astype(np.float64).sum(axis=0)
            unit = ksum / max(np.linalg.norm(ksum), 1e-30)
            noise = 0.1 * _rng(w.seed, "qnoise", r, h).standard_normal(d)
            q[r, h, :] = (w.q_scale * unit + noise).astype(np.float32)
    if w.cluster_runs or w.cluster_last:
        _cluster(w, Ks, q)
    qs = _store(q, w.dtype)

    n_phys = w.pages_needed() + w.batch
    order = np.arange(n_phys, dtype=np.int32)
    if w.permute_pages:
        order = _rng(w.seed, "pages").permutation(n_phys).astype(np.int32)
    return {"K": Ks, "V": Vs, "q": qs, "planted": planted, "page_order": order, "n_phys_pages": n_phys}


def _cluster(w: Workload, Ks: List[np.ndarray], q: np.ndarray) -> None:
    """Make the keys of a few page runs (per query head) and of the last tokens (per KV group) lean towards the
    queries: k += shift * q / |q| for every key of the run.  In place, after the queries are drawn."""
    G, T = w.group, w.page_tokens
    for r, n in enumerate(w.lens):
        pages = n // T
        for h in range(w.n_q_heads):
            g = h // G
            unit = (q[r, h] / max(np.linalg.norm(q[r, h]), 1e-30)).astype(np.float32)
            starts = _rng(w.seed, "pages", r + 1, h).choice(max(1, pages - 2), size=min(w.cluster_runs, max(1, pages - 2)),
                                                            replace=False)
            for p0 in starts:
                a, b = int(p0) * T, min(n, (int(p0) + 2) * T)
                Ks[r][a:b, g, :] = _store(_as_f32(Ks[r][a:b, g, :], w.dtype) + w.cluster_shift * unit, w.dtype)
        if w.cluster_last:
            a = max(0, n - w.cluster_last)
            for g in range(w.n_kv_heads):
                lean = sum(q[r, h] / max(np.linalg.norm(q[r, h]), 1e-30) for h in range(g * G, (g + 1) * G)).astype(np.float32)
                Ks[r][a:, g, :] = _store(_as_f32(Ks[r][a:, g, :], w.dtype) + 0.5 * w.cluster_shift * lean, w.dtype)


def extra_tokens(w: Workload, r: int, t: int, step: int = 0) -> Tuple[np.ndarray, np.ndarray]:
    """t further (k, v) rows [t][n_kv_heads][head_dim] for request r — what a decode step appends."""
    d, Hk = w.head_dim, w.n_kv_heads
    rk = _rng(w.seed + 7919 * (step + 1), "K", r, 0xFF)
    rv = _rng(w.seed + 7919 * (step + 1), "V", r, 0xFF)
    k = rk.standard_normal((t, Hk, d), dtype=np.float32)
    v = rv.standard_normal((t, Hk, d), dtype=np.float32)
    return _store(k, w.dtype), _store(v, w.dtype)
