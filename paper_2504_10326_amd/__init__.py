"""Python binding of libalaya.so (include/alaya.h): argument marshalling only.

Every step of the decode-step sparse-attention query runs in the HIP kernels
behind the C ABI.  PyTorch is used for device memory and for the stream handle,
nothing else.  There is no CPU fallback: if the library has not been built,
or no GPU is present when a kernel is needed, the call fails loudly.

Module-level functions carry the C names (alaya_create_cache, alaya_append_kv,
alaya_sparse_attn, alaya_full_attn, ...) and take raw pointers / torch tensors;
`Cache` bundles a handle with the torch tensors that back its pools.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence, Tuple

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libalaya.so")

ALAYA_BF16, ALAYA_F32 = 0, 1
ALAYA_TOPK, ALAYA_DIPR = 0, 1
ALAYA_OK, ALAYA_E_INVAL, ALAYA_E_NOMEM, ALAYA_E_CAPACITY, ALAYA_E_EMPTY, ALAYA_E_DEVICE = 0, -1, -2, -3, -4, -5
SCORE_PAD = 1088
N_KERNEL_SLOTS = 8
KERNEL_SLOTS = ("score", "select", "attend", "combine", "full_partial", "append", "sample", "coarse")

# include/alaya.h
EXPORTS = (
    "alaya_pool_bytes", "alaya_workspace_bytes", "alaya_scratch_bytes", "alaya_rep_bytes", "alaya_create_cache",
    "alaya_bind_scratch", "alaya_bind_reps",
    "alaya_destroy_cache", "alaya_append_kv", "alaya_append_kv_step", "alaya_seq_len", "alaya_reset_seq",
    "alaya_sparse_attn", "alaya_decode_step", "alaya_sparse_attn_static", "alaya_full_attn", "alaya_poll_status",
    "alaya_last_error",
    "alaya_graph_bytes", "alaya_graph_build_bytes", "alaya_graph_build", "alaya_graph_destroy", "alaya_graph_info",
    "alaya_diprs_attn", "alaya_plan_query",
)
# include/alaya_debug.h
DEBUG_EXPORTS = (
    "alaya_set_profiling", "alaya_kernel_times", "alaya_set_tuning", "alaya_debug_scores", "alaya_debug_pages",
    "alaya_debug_estimate", "alaya_debug_repairs", "alaya_debug_diprs_list", "alaya_debug_diprs_lds",
)


class AlayaError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"alaya status {code}: {message}")
        self.code = code


class CacheConfig(ctypes.Structure):
    _fields_ = [
        ("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
        ("page_tokens", ctypes.c_int32), ("dtype", ctypes.c_int32), ("max_seqs", ctypes.c_int32),
        ("max_batch", ctypes.c_int32), ("reserved", ctypes.c_int32),
        ("max_tokens_per_seq", ctypes.c_int64), ("max_batch_tokens", ctypes.c_int64),
        ("n_phys_pages", ctypes.c_int64),
    ]


class SparseParams(ctypes.Structure):
    _fields_ = [
        ("mode", ctypes.c_int32), ("window_init", ctypes.c_int32),
        ("topk", ctypes.POINTER(ctypes.c_int32)), ("beta", ctypes.POINTER(ctypes.c_float)),
        ("scale", ctypes.c_float), ("window_last", ctypes.c_int32),
        ("out_ids", ctypes.c_void_p), ("out_counts", ctypes.c_void_p), ("ids_stride", ctypes.c_int64),
        ("n_visible", ctypes.POINTER(ctypes.c_int32)),
        ("coarse_pages", ctypes.POINTER(ctypes.c_int32)), ("out_pages", ctypes.c_void_p),
        ("pages_stride", ctypes.c_int64),
    ]


_lib = None


class PlanInput(ctypes.Structure):
    _fields_ = [("context_len", ctypes.c_int64), ("short_context", ctypes.c_int64), ("reused_prefix", ctypes.c_int64),
                ("gpu_budget_bytes", ctypes.c_int64), ("coarse_bytes", ctypes.c_int64), ("layer_id", ctypes.c_int32),
                ("reserved", ctypes.c_int32)]


class Plan(ctypes.Structure):
    _fields_ = [("query", ctypes.c_int32), ("index", ctypes.c_int32), ("n_visible", ctypes.c_int64)]


QUERY_FULL, QUERY_TOPK, QUERY_DIPR = 0, 1, 2
INDEX_NONE, INDEX_COARSE, INDEX_FLAT, INDEX_FINE = 0, 1, 2, 3


def lib() -> ctypes.CDLL:
    """The loaded shared library.  Raises if it has not been built (python -m paper_2504_10326_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2504_10326_amd.build`; "
                               "there is no fallback path")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, i64, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_size_t
        cfgp = ctypes.POINTER(CacheConfig)
        L.alaya_pool_bytes.argtypes = [cfgp]; L.alaya_pool_bytes.restype = sz
        L.alaya_workspace_bytes.argtypes = [cfgp]; L.alaya_workspace_bytes.restype = sz
        L.alaya_scratch_bytes.argtypes = [cfgp]; L.alaya_scratch_bytes.restype = sz
        L.alaya_bind_scratch.argtypes = [vp, vp, sz]; L.alaya_bind_scratch.restype = i32
        L.alaya_rep_bytes.argtypes = [cfgp]; L.alaya_rep_bytes.restype = sz
        L.alaya_bind_reps.argtypes = [vp, vp, sz]; L.alaya_bind_reps.restype = i32
        L.alaya_create_cache.argtypes = [ctypes.POINTER(vp), cfgp, vp, vp, ctypes.POINTER(ctypes.c_int32), vp, sz]
        L.alaya_create_cache.restype = i32
        L.alaya_destroy_cache.argtypes = [vp]; L.alaya_destroy_cache.restype = i32
        L.alaya_append_kv.argtypes = [vp, i32, vp, vp, i64, vp]; L.alaya_append_kv.restype = i32
        L.alaya_append_kv_step.argtypes = [vp, ctypes.POINTER(ctypes.c_int32), i32, vp, vp, vp]
        L.alaya_append_kv_step.restype = i32
        L.alaya_seq_len.argtypes = [vp, i32]; L.alaya_seq_len.restype = i64
        L.alaya_reset_seq.argtypes = [vp, i32]; L.alaya_reset_seq.restype = i32
        L.alaya_sparse_attn.argtypes = [vp, ctypes.POINTER(ctypes.c_int32), i32, i32, vp,
                                        ctypes.POINTER(SparseParams), vp, vp]
        L.alaya_sparse_attn.restype = i32
        L.alaya_sparse_attn_static.argtypes = L.alaya_sparse_attn.argtypes
        L.alaya_sparse_attn_static.restype = i32
        L.alaya_decode_step.argtypes = [vp, ctypes.POINTER(ctypes.c_int32), i32, i32, vp, vp, vp,
                                        ctypes.POINTER(SparseParams), vp, vp]
        L.alaya_decode_step.restype = i32
        L.alaya_full_attn.argtypes = [vp, ctypes.POINTER(ctypes.c_int32), i32, i32, vp, ctypes.c_float, vp, vp]
        L.alaya_full_attn.restype = i32
        L.alaya_poll_status.argtypes = [vp, vp]; L.alaya_poll_status.restype = i32
        L.alaya_set_profiling.argtypes = [vp, i32]; L.alaya_set_profiling.restype = i32
        L.alaya_kernel_times.argtypes = [vp, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int64), i32]
        L.alaya_kernel_times.restype = i32
        L.alaya_set_tuning.argtypes = [vp, i32, i32, i32, i32]; L.alaya_set_tuning.restype = i32
        L.alaya_debug_scores.argtypes = [vp, vp, vp]; L.alaya_debug_scores.restype = i64
        L.alaya_debug_repairs.argtypes = [vp, vp]; L.alaya_debug_repairs.restype = i64
        L.alaya_debug_pages.argtypes = [vp, ctypes.POINTER(i64), ctypes.POINTER(i64)]
        L.alaya_debug_pages.restype = i32
        L.alaya_debug_estimate.argtypes = [vp, i32]; L.alaya_debug_estimate.restype = i32
        L.alaya_last_error.argtypes = []; L.alaya_last_error.restype = ctypes.c_char_p
        L.alaya_graph_bytes.argtypes = [vp, i32, i32]; L.alaya_graph_bytes.restype = sz
        L.alaya_graph_build_bytes.argtypes = [vp, i32, i32]; L.alaya_graph_build_bytes.restype = sz
        L.alaya_graph_build.argtypes = [ctypes.POINTER(vp), vp, i32, i32, vp, sz, vp, sz, vp]
        L.alaya_graph_build.restype = i32
        L.alaya_graph_destroy.argtypes = [vp]; L.alaya_graph_destroy.restype = i32
        L.alaya_graph_info.argtypes = [vp, ctypes.POINTER(i64), ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(vp),
                                       ctypes.POINTER(ctypes.c_int32)]
        L.alaya_graph_info.restype = i32
        L.alaya_diprs_attn.argtypes = [vp, vp, i32, vp, ctypes.c_float, i32, ctypes.POINTER(SparseParams), vp, vp]
        L.alaya_diprs_attn.restype = i32
        L.alaya_plan_query.argtypes = [ctypes.POINTER(PlanInput), ctypes.POINTER(Plan)]; L.alaya_plan_query.restype = i32
        L.alaya_debug_diprs_lds.argtypes = [vp, i32]; L.alaya_debug_diprs_lds.restype = i32
        L.alaya_debug_diprs_list.argtypes = [vp, i32, vp, i64, vp]; L.alaya_debug_diprs_list.restype = i64
        _lib = L
    return _lib


def alaya_last_error() -> str:
    return lib().alaya_last_error().decode()


def _check(rc: int) -> None:
    if rc != ALAYA_OK:
        raise AlayaError(rc, alaya_last_error())


def _i32_array(xs: Optional[Sequence[int]]):
    if xs is None:
        return None
    return (ctypes.c_int32 * len(xs))(*[int(x) for x in xs])


def _f32_array(xs: Optional[Sequence[float]]):
    if xs is None:
        return None
    return (ctypes.c_float * len(xs))(*[float(x) for x in xs])


def _ptr(t) -> Optional[int]:
    """Device pointer of a torch tensor (or an int passed through)."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream or None
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


# ---- functions with the C names -------------------------------------------------------------------

def alaya_pool_bytes(cfg: CacheConfig) -> int:
    return lib().alaya_pool_bytes(ctypes.byref(cfg))


def alaya_workspace_bytes(cfg: CacheConfig) -> int:
    return lib().alaya_workspace_bytes(ctypes.byref(cfg))


def alaya_scratch_bytes(cfg: CacheConfig) -> int:
    return lib().alaya_scratch_bytes(ctypes.byref(cfg))


def alaya_bind_scratch(handle: int, scratch, scratch_bytes: int) -> None:
    _check(lib().alaya_bind_scratch(handle, _ptr(scratch), scratch_bytes))


def alaya_rep_bytes(cfg: CacheConfig) -> int:
    return lib().alaya_rep_bytes(ctypes.byref(cfg))


def alaya_bind_reps(handle: int, rep_pool, rep_bytes: int) -> None:
    _check(lib().alaya_bind_reps(handle, _ptr(rep_pool), rep_bytes))


def alaya_create_cache(cfg: CacheConfig, k_pool, v_pool, phys_page_order: Optional[Sequence[int]],
                       workspace, workspace_bytes: int) -> int:
    h = ctypes.c_void_p()
    order = None
    if phys_page_order is not None:
        import numpy as np
        arr = np.ascontiguousarray(np.asarray(phys_page_order, dtype=np.int32))
        order = arr.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))
    _check(lib().alaya_create_cache(ctypes.byref(h), ctypes.byref(cfg), _ptr(k_pool), _ptr(v_pool), order,
                                    _ptr(workspace), workspace_bytes))
    return h.value


def alaya_destroy_cache(handle: int) -> None:
    _check(lib().alaya_destroy_cache(handle))


def alaya_append_kv(handle: int, seq: int, k, v, t: int, stream=0) -> None:
    _check(lib().alaya_append_kv(handle, seq, _ptr(k), _ptr(v), t, stream or None))


def alaya_append_kv_step(handle: int, seqs: Sequence[int], k, v, stream=0) -> None:
    sq = _i32_array(seqs)
    _check(lib().alaya_append_kv_step(handle, sq, len(seqs), _ptr(k), _ptr(v), stream or None))


def alaya_seq_len(handle: int, seq: int) -> int:
    return lib().alaya_seq_len(handle, seq)


def alaya_reset_seq(handle: int, seq: int) -> None:
    _check(lib().alaya_reset_seq(handle, seq))


def alaya_sparse_attn(handle: int, seqs: Sequence[int], n_q_heads: int, q, mode: int,
                      topk: Optional[Sequence[int]], beta: Optional[Sequence[float]], scale: float, out,
                      out_ids=None, out_counts=None, ids_stride: int = 0, stream=0,
                      window: Tuple[int, int] = (0, 0), n_visible: Optional[Sequence[int]] = None,
                      step_kv=None, static_scratch: bool = False, coarse_pages: Optional[Sequence[int]] = None,
                      out_pages=None, pages_stride: int = 0) -> None:
    """step_kv = (k, v): make the call an alaya_decode_step that first appends one token per sequence.
    static_scratch: call alaya_sparse_attn_static (the library's own scratch array, nothing allocated)."""
    p = SparseParams()
    p.mode = mode
    p.window_init, p.window_last = int(window[0]), int(window[1])
    nv = _i32_array(n_visible)
    p.n_visible = ctypes.cast(nv, ctypes.POINTER(ctypes.c_int32)) if nv is not None else None
    tk, bt = _i32_array(topk), _f32_array(beta)
    p.topk = ctypes.cast(tk, ctypes.POINTER(ctypes.c_int32)) if tk is not None else None
    p.beta = ctypes.cast(bt, ctypes.POINTER(ctypes.c_float)) if bt is not None else None
    p.scale = scale
    p.out_ids = _ptr(out_ids)
    p.out_counts = _ptr(out_counts)
    p.ids_stride = ids_stride
    cpg = _i32_array(coarse_pages)
    p.coarse_pages = ctypes.cast(cpg, ctypes.POINTER(ctypes.c_int32)) if cpg is not None else None
    p.out_pages = _ptr(out_pages)
    p.pages_stride = pages_stride
    sq = _i32_array(seqs)
    if step_kv is not None:
        _check(lib().alaya_decode_step(handle, sq, len(seqs), n_q_heads, _ptr(step_kv[0]), _ptr(step_kv[1]), _ptr(q),
                                       ctypes.byref(p), _ptr(out), stream or None))
        return
    fn = lib().alaya_sparse_attn_static if static_scratch else lib().alaya_sparse_attn
    _check(fn(handle, sq, len(seqs), n_q_heads, _ptr(q), ctypes.byref(p), _ptr(out), stream or None))


def alaya_sparse_attn_static(handle: int, seqs: Sequence[int], n_q_heads: int, q, mode: int,
                             topk: Optional[Sequence[int]], beta: Optional[Sequence[float]], scale: float, out,
                             out_ids=None, out_counts=None, ids_stride: int = 0, stream=0,
                             window: Tuple[int, int] = (0, 0), n_visible: Optional[Sequence[int]] = None) -> None:
    alaya_sparse_attn(handle, seqs, n_q_heads, q, mode, topk, beta, scale, out, out_ids, out_counts, ids_stride,
                      stream, window, n_visible, static_scratch=True)


def alaya_decode_step(handle: int, seqs: Sequence[int], n_q_heads: int, k, v, q, mode: int,
                      topk: Optional[Sequence[int]], beta: Optional[Sequence[float]], scale: float, out,
                      out_ids=None, out_counts=None, ids_stride: int = 0, stream=0,
                      window: Tuple[int, int] = (0, 0), n_visible: Optional[Sequence[int]] = None) -> None:
    alaya_sparse_attn(handle, seqs, n_q_heads, q, mode, topk, beta, scale, out, out_ids, out_counts, ids_stride,
                      stream, window, n_visible, step_kv=(k, v))


def alaya_full_attn(handle: int, seqs: Sequence[int], n_q_heads: int, q, scale: float, out, stream=0) -> None:
    sq = _i32_array(seqs)
    _check(lib().alaya_full_attn(handle, sq, len(seqs), n_q_heads, _ptr(q), scale, _ptr(out), stream or None))


def alaya_graph_bytes(handle: int, seq: int, degree: int) -> int:
    return lib().alaya_graph_bytes(handle, seq, degree)


def alaya_graph_build_bytes(handle: int, seq: int, degree: int) -> int:
    return lib().alaya_graph_build_bytes(handle, seq, degree)


def alaya_graph_build(handle: int, seq: int, degree: int, index_mem, index_bytes: int, build_mem, build_bytes: int,
                      stream=0) -> int:
    g = ctypes.c_void_p()
    _check(lib().alaya_graph_build(ctypes.byref(g), handle, seq, degree, _ptr(index_mem), index_bytes,
                                   _ptr(build_mem), build_bytes, stream or None))
    return g.value


def alaya_graph_destroy(graph: int) -> None:
    _check(lib().alaya_graph_destroy(graph))


def alaya_graph_info(graph: int, n_kv_heads: int) -> Tuple[int, int, int, list]:
    """(n_indexed, degree, device address of the neighbour lists, entry point of every KV head)"""
    n, m, nb = ctypes.c_int64(0), ctypes.c_int32(0), ctypes.c_void_p()
    entry = (ctypes.c_int32 * n_kv_heads)()
    _check(lib().alaya_graph_info(graph, ctypes.byref(n), ctypes.byref(m), ctypes.byref(nb), entry))
    return n.value, m.value, nb.value, list(entry)


def alaya_diprs_attn(handle: int, graph: int, n_q_heads: int, q, beta: float, l0: int, scale: float, out,
                     out_ids=None, out_counts=None, ids_stride: int = 0, stream=0,
                     window: Tuple[int, int] = (0, 0)) -> None:
    p = SparseParams()
    p.mode = ALAYA_DIPR
    p.window_init, p.window_last = int(window[0]), int(window[1])
    p.scale = scale
    p.out_ids = _ptr(out_ids)
    p.out_counts = _ptr(out_counts)
    p.ids_stride = ids_stride
    _check(lib().alaya_diprs_attn(handle, graph, n_q_heads, _ptr(q), beta, l0, ctypes.byref(p), _ptr(out),
                                  stream or None))


def alaya_plan_query(context_len: int, short_context: int, reused_prefix: int, gpu_budget_bytes: int, coarse_bytes: int,
                     layer_id: int) -> Tuple[int, int, int]:
    """(query type, index type, n_visible) by the rule-based optimizer of Sec. 6.2."""
    i, o = PlanInput(context_len, short_context, reused_prefix, gpu_budget_bytes, coarse_bytes, layer_id, 0), Plan()
    rc = lib().alaya_plan_query(ctypes.byref(i), ctypes.byref(o))
    if rc != 0:
        raise AlayaError(rc, "invalid plan input")
    return o.query, o.index, o.n_visible


def alaya_poll_status(handle: int, stream=0) -> int:
    return lib().alaya_poll_status(handle, stream or None)


# ---- a handle bundled with the torch memory behind it ---------------------------------------------

class Graph:
    """The exact nearest-neighbour graph of one sequence's keys (one per KV head), built on the GPU."""

    def __init__(self, cache: "Cache", seq: int, degree: int, stream=None):
        torch = cache.torch
        self.cache, self.seq, self.handle = cache, seq, None
        ib = alaya_graph_bytes(cache.handle, seq, degree)
        bb = alaya_graph_build_bytes(cache.handle, seq, degree)
        if ib == 0 or bb == 0:
            raise AlayaError(ALAYA_E_INVAL, alaya_last_error())
        self.index_mem = torch.empty(ib, dtype=torch.uint8, device=cache.device)
        build_mem = torch.empty(bb, dtype=torch.uint8, device=cache.device)
        self.handle = alaya_graph_build(cache.handle, seq, degree, self.index_mem, ib, build_mem, bb, _stream(stream))
        self.n_indexed, self.degree, self._nbr_addr, self.entry = alaya_graph_info(self.handle, cache.cfg.n_kv_heads)

    def neighbours(self):
        """int32 tensor [n_kv_heads][n_indexed][degree] viewing the index memory"""
        n = self.cache.cfg.n_kv_heads * self.n_indexed * self.degree
        return self.index_mem[: 4 * n].view(self.cache.torch.int32).view(self.cache.cfg.n_kv_heads, self.n_indexed, self.degree)

    def close(self) -> None:
        if self.handle:
            self.cache.torch.cuda.synchronize(self.cache.device)
            alaya_graph_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class Cache:
    """One layer's paged KV store on one GPU.  torch allocates the pools, the page-table workspace and -
    unless a tensor shared with other caches (other layers) is passed as `scratch` - the scratch memory."""

    def __init__(self, n_q_heads: int, n_kv_heads: int, head_dim: int, dtype: str, max_seqs: int,
                 max_batch: int, max_tokens_per_seq: int, max_batch_tokens: int, n_phys_pages: int,
                 phys_page_order: Optional[Sequence[int]] = None, device: str = "cuda:0", scratch=None,
                 coarse_index: bool = False):
        import torch
        if not torch.cuda.is_available():
            raise RuntimeError("no GPU visible: the sparse-attention path has no CPU fallback")
        self.torch = torch
        self.device = torch.device(device)
        self.dtype = {"bf16": ALAYA_BF16, "f32": ALAYA_F32}[dtype]
        self.torch_dtype = torch.bfloat16 if dtype == "bf16" else torch.float32
        cfg = CacheConfig(n_q_heads, n_kv_heads, head_dim, 64, self.dtype, max_seqs, max_batch, 0,
                          max_tokens_per_seq, max_batch_tokens, n_phys_pages)
        self.cfg = cfg
        pool, ws, sc = alaya_pool_bytes(cfg), alaya_workspace_bytes(cfg), alaya_scratch_bytes(cfg)
        if pool == 0 or ws == 0 or sc == 0:
            raise AlayaError(ALAYA_E_INVAL, "invalid cache configuration")
        self.k_pool = torch.empty(pool, dtype=torch.uint8, device=self.device)
        self.v_pool = torch.empty(pool, dtype=torch.uint8, device=self.device)
        self.workspace = torch.empty(ws, dtype=torch.uint8, device=self.device)
        self.workspace_bytes = ws
        self.scratch = scratch if scratch is not None else torch.empty(sc, dtype=torch.uint8, device=self.device)
        self.scratch_bytes = sc
        self.handle = alaya_create_cache(cfg, self.k_pool, self.v_pool, phys_page_order, self.workspace, ws)
        alaya_bind_scratch(self.handle, self.scratch, self.scratch.numel())
        self.rep_pool = None
        if coarse_index:      # block representatives (Sec. 6.2, coarse-grained index), kept up to date by every append
            self.rep_pool = torch.empty(alaya_rep_bytes(cfg), dtype=torch.uint8, device=self.device)
            alaya_bind_reps(self.handle, self.rep_pool, self.rep_pool.numel())

    def close(self) -> None:
        if getattr(self, "handle", None):
            self.torch.cuda.synchronize(self.device)
            alaya_destroy_cache(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- Session.update
    def append_kv(self, seq: int, k, v, stream=None) -> None:
        assert k.is_cuda and v.is_cuda and k.is_contiguous() and v.is_contiguous()
        assert k.dtype == self.torch_dtype and v.dtype == self.torch_dtype and k.shape == v.shape
        assert tuple(k.shape[1:]) == (self.cfg.n_kv_heads, self.cfg.head_dim)
        alaya_append_kv(self.handle, seq, k, v, k.shape[0], _stream(stream))

    def append_step(self, seqs: Sequence[int], k, v, stream=None) -> None:
        """One new token for each listed sequence, one launch: k, v [len(seqs)][n_kv_heads][head_dim]."""
        assert k.is_cuda and v.is_cuda and k.is_contiguous() and v.is_contiguous()
        assert k.dtype == self.torch_dtype and v.dtype == self.torch_dtype and k.shape == v.shape
        assert tuple(k.shape) == (len(seqs), self.cfg.n_kv_heads, self.cfg.head_dim)
        alaya_append_kv_step(self.handle, seqs, k, v, _stream(stream))

    def seq_len(self, seq: int) -> int:
        return alaya_seq_len(self.handle, seq)

    def reset_seq(self, seq: int) -> None:
        alaya_reset_seq(self.handle, seq)

    # -- Session.attention
    def _q_out(self, seqs, q):
        B = len(seqs)
        assert q.is_cuda and q.is_contiguous() and q.dtype == self.torch_dtype
        assert tuple(q.shape) == (B, self.cfg.n_q_heads, self.cfg.head_dim)
        return self.torch.empty((B, self.cfg.n_q_heads, self.cfg.head_dim), dtype=self.torch.float32,
                                device=self.device)

    def decode_step(self, seqs: Sequence[int], k, v, q, mode: int, **kw):
        """One token (k, v [len(seqs)][n_kv_heads][head_dim]) appended to each listed sequence, then
        sparse_attn over the grown sequences, in one call (alaya_decode_step); arguments and result as
        for sparse_attn."""
        assert k.is_cuda and v.is_cuda and k.is_contiguous() and v.is_contiguous()
        assert k.dtype == self.torch_dtype and v.dtype == self.torch_dtype and k.shape == v.shape
        assert tuple(k.shape) == (len(seqs), self.cfg.n_kv_heads, self.cfg.head_dim)
        return self.sparse_attn(seqs, q, mode, _step_kv=(k, v), **kw)

    def sparse_attn(self, seqs: Sequence[int], q, mode: int, topk=None, beta=None, scale: float = 0.0,
                    ids_stride: int = 0, out=None, stream=None, want_counts: bool = False,
                    window: Tuple[int, int] = (0, 0), n_visible: Optional[Sequence[int]] = None, _step_kv=None,
                    static_scratch: bool = False, coarse_pages: Optional[Sequence[int]] = None, pages_stride: int = 0):
        """Returns out [B][Hq][d] fp32, or (out, ids [B][Hq][ids_stride] int32, counts [B][Hq] int32) when
        ids_stride > 0, or (out, counts) when only want_counts is set.  window = (first, last) tokens
        that are always attended; n_visible[b] = the prefix of request b that the query sees.
        static_scratch: through alaya_sparse_attn_static (the library's own scratch array).
        coarse_pages[b]: answer through the coarse index, over the tokens of that many best pages per head;
        with pages_stride > 0 the chosen pages come back too: (out, ids, counts, pages [B][Hq][pages_stride])."""
        if out is None:
            out = self._q_out(seqs, q)
        ids = counts = None
        if ids_stride > 0:
            ids = self.torch.full((len(seqs), self.cfg.n_q_heads, ids_stride), -1, dtype=self.torch.int32,
                                  device=self.device)
        if ids_stride > 0 or want_counts:
            counts = self.torch.zeros((len(seqs), self.cfg.n_q_heads), dtype=self.torch.int32, device=self.device)
        pages = None
        if pages_stride > 0:
            pages = self.torch.full((len(seqs), self.cfg.n_q_heads, pages_stride), -1, dtype=self.torch.int32,
                                    device=self.device)
        alaya_sparse_attn(self.handle, seqs, self.cfg.n_q_heads, q, mode, topk, beta, scale, out, ids, counts,
                          ids_stride, _stream(stream), window, n_visible, step_kv=_step_kv,
                          static_scratch=static_scratch, coarse_pages=coarse_pages, out_pages=pages,
                          pages_stride=pages_stride)
        if pages is not None:
            return out, ids, counts, pages
        if ids is not None:
            return out, ids, counts
        return (out, counts) if want_counts else out

    # -- fine-grained index (Sec. 6.2) and DIPRS (Sec. 6.1.3, Algorithm 1)
    def build_graph(self, seq: int, degree: int, stream=None) -> "Graph":
        return Graph(self, seq, degree, stream)

    def diprs_attn(self, graph: "Graph", q, beta: float, l0: int, scale: float = 0.0, ids_stride: int = 0, out=None,
                   stream=None, window: Tuple[int, int] = (0, 0)):
        """Algorithm 1 on the graph of its sequence for the query q [1][Hq][d]; returns out [1][Hq][d] fp32, or
        (out, ids [1][Hq][ids_stride], counts [1][Hq]) when ids_stride > 0: the window's tokens, then the answer
        in the order in which the walk met it."""
        if out is None:
            out = self._q_out([graph.seq], q)
        ids = counts = None
        if ids_stride > 0:
            ids = self.torch.full((1, self.cfg.n_q_heads, ids_stride), -1, dtype=self.torch.int32, device=self.device)
            counts = self.torch.zeros((1, self.cfg.n_q_heads), dtype=self.torch.int32, device=self.device)
        alaya_diprs_attn(self.handle, graph.handle, self.cfg.n_q_heads, q, beta, l0, scale, out, ids, counts, ids_stride,
                         _stream(stream), window)
        return (out, ids, counts) if ids is not None else out

    def debug_diprs_lds(self, nbytes: int) -> None:
        _check(lib().alaya_debug_diprs_lds(self.handle, nbytes))

    def debug_diprs_list(self, head: int, stream=None):
        """The list C of the last diprs_attn call for one query head, as a numpy int32 array."""
        import numpy as np
        n = lib().alaya_debug_diprs_list(self.handle, head, None, 0, _stream(stream) or None)
        if n < 0:
            raise AlayaError(ALAYA_E_INVAL, alaya_last_error())
        ids = np.empty(max(n, 1), dtype=np.int32)
        lib().alaya_debug_diprs_list(self.handle, head, ids.ctypes.data, n, _stream(stream) or None)
        return ids[:n]

    def full_attn(self, seqs: Sequence[int], q, scale: float = 0.0, out=None, stream=None):
        if out is None:
            out = self._q_out(seqs, q)
        alaya_full_attn(self.handle, seqs, self.cfg.n_q_heads, q, scale, out, _stream(stream))
        return out

    def poll_status(self, stream=None) -> int:
        return alaya_poll_status(self.handle, _stream(stream))

    # -- measurement
    def set_profiling(self, enabled: bool) -> None:
        _check(lib().alaya_set_profiling(self.handle, int(enabled)))

    def kernel_times(self) -> dict:
        ms = (ctypes.c_double * N_KERNEL_SLOTS)()
        n = (ctypes.c_int64 * N_KERNEL_SLOTS)()
        _check(lib().alaya_kernel_times(self.handle, ms, n, N_KERNEL_SLOTS))
        return {name: {"sum_ms": ms[i], "launches": n[i]} for i, name in enumerate(KERNEL_SLOTS)}

    def debug_scores(self, lens: Sequence[int]):
        """fp32 scores that the scoring pass of the last sparse call kept (all of them if the call was made
        with write_all_scores=1), NaN elsewhere: list of tensors [Hq][n], one per request."""
        torch = self.torch
        hq = self.cfg.n_q_heads
        strides = [(n + 63) // 64 * 64 + SCORE_PAD for n in lens]
        dense = torch.full((hq * sum(strides),), float("nan"), dtype=torch.float32, device=self.device)
        if lib().alaya_debug_scores(self.handle, dense.data_ptr(), _stream(None)) < 0:
            raise AlayaError(ALAYA_E_DEVICE, alaya_last_error())
        views, off = [], 0
        for n, stride in zip(lens, strides):
            views.append(dense[off:off + hq * stride].view(hq, stride)[:, :n])
            off += hq * stride
        return views

    def debug_survivors(self, stream=None) -> int:
        """(token, score) pairs kept by the scoring pass of the last sparse call, over all heads."""
        return lib().alaya_debug_scores(self.handle, None, _stream(stream))

    def debug_repairs(self, stream=None) -> int:
        """(request, head) selections that took the repair path of the estimated bound since the last read."""
        return lib().alaya_debug_repairs(self.handle, _stream(stream))

    def debug_pages(self) -> Tuple[int, int]:
        """(pages scored by the sample pass, pages whose keys the main pass read) of the last sparse call."""
        a, b = ctypes.c_int64(0), ctypes.c_int64(0)
        _check(lib().alaya_debug_pages(self.handle, ctypes.byref(a), ctypes.byref(b)))
        return a.value, b.value

    def debug_estimate(self, mode: int) -> None:
        """0, 1: estimated bound whenever the shapes allow, 2: estimate that always needs repair, -1: never."""
        _check(lib().alaya_debug_estimate(self.handle, mode))

    def set_tuning(self, score_pages_per_wave: int = 0, attend_splits: int = 0,
                   select_batch_blocks: int = 0, write_all_scores: bool = False) -> None:
        _check(lib().alaya_set_tuning(self.handle, score_pages_per_wave, attend_splits, select_batch_blocks,
                                      int(write_all_scores)))
        self._tuning = (score_pages_per_wave, attend_splits, select_batch_blocks, bool(write_all_scores))

    def set_write_all_scores(self, flag: bool) -> None:
        """Toggle only the write-everything switch, keeping the other knobs."""
        t = getattr(self, "_tuning", (0, 0, 0, False))
        self.set_tuning(t[0], t[1], t[2], flag)
