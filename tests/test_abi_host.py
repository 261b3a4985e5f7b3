"""Host-side checks of the C ABI that need no GPU: the library loads, exports what the header
declares, and turns bad arguments into status codes before anything is launched."""
import ctypes
import os
import re

import pytest

import paper_2504_10326_amd as A

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = [0x10000000, 0x20000000, 0x30000000, 0x40000000, 0x50000000]   # aligned, never dereferenced on the host


def _cfg(**kw):
    base = dict(n_q_heads=32, n_kv_heads=8, head_dim=128, page_tokens=64, dtype=0, max_seqs=4, max_batch=4,
                reserved=0, max_tokens_per_seq=4096, max_batch_tokens=8192, n_phys_pages=70)
    base.update(kw)
    return A.CacheConfig(*[base[f[0]] for f in A.CacheConfig._fields_])


def _create(cfg=None, order=None):
    cfg = cfg or _cfg()
    return A.alaya_create_cache(cfg, FAKE[0], FAKE[1], order, FAKE[2], A.alaya_workspace_bytes(cfg))


def test_library_exports_every_declared_symbol():
    L = A.lib()
    for header, exports in (("alaya.h", A.EXPORTS), ("alaya_debug.h", A.DEBUG_EXPORTS)):
        text = open(os.path.join(ROOT, "include", header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        declared = set(re.findall(r"\b(alaya_[a-z_]+)\s*\(", text))
        for name in sorted(declared):
            assert hasattr(L, name), f"{name} declared in {header} but not exported"
        assert declared == set(exports), header
    assert {"alaya_create_cache", "alaya_append_kv", "alaya_sparse_attn", "alaya_full_attn"} <= set(A.EXPORTS)
    # the paper-defined header carries no measurement or test hooks
    assert not any("debug" in n or "tuning" in n or "profiling" in n for n in A.EXPORTS)


def test_struct_layouts_match_header():
    assert ctypes.sizeof(A.CacheConfig) == 56
    assert ctypes.sizeof(A.SparseParams) == 88


def test_sizes():
    cfg = _cfg()
    assert A.alaya_pool_bytes(cfg) == 70 * 8 * 64 * 128 * 2
    assert A.alaya_pool_bytes(_cfg(dtype=1)) == 70 * 8 * 64 * 128 * 4
    # the cache's own workspace is its page table: 4 sequences of 64 pages
    ws = A.alaya_workspace_bytes(cfg)
    assert ws == 4 * 64 * 4
    # survivor blocks and selected tokens, 8 bytes each per (q head, token), dominate the scratch memory
    sc = A.alaya_scratch_bytes(cfg)
    assert sc >= 2 * 8 * 32 * 8192 and sc % 256 == 0
    assert A.alaya_scratch_bytes(_cfg(max_batch_tokens=16384)) > sc


def test_scratch_binding_is_checked_and_may_be_shared():
    """Scratch memory is separate from the cache (one cache = one layer; layers run one after the other
    and may share it): size and alignment are checked, several caches may bind the same area, NULL unbinds."""
    cfg = _cfg()
    sc = A.alaya_scratch_bytes(cfg)
    a, b = _create(cfg), _create(cfg)
    try:
        for args, code in [((a, FAKE[3] + 8, sc), A.ALAYA_E_INVAL), ((a, FAKE[3], sc - 1), A.ALAYA_E_NOMEM),
                           ((0, FAKE[3], sc), A.ALAYA_E_INVAL)]:
            with pytest.raises(A.AlayaError) as e:
                A.alaya_bind_scratch(*args)
            assert e.value.code == code
        A.alaya_bind_scratch(a, FAKE[3], sc)
        A.alaya_bind_scratch(b, FAKE[3], sc + 4096)          # the same area, for a second layer
        A.alaya_bind_scratch(b, 0, 0)                         # unbind
        assert A.alaya_poll_status(a) == A.ALAYA_OK           # nothing launched yet: nothing to read
    finally:
        A.alaya_destroy_cache(a)
        A.alaya_destroy_cache(b)


@pytest.mark.parametrize("bad", [dict(head_dim=96), dict(page_tokens=32), dict(dtype=2), dict(n_q_heads=30),
                                 dict(n_q_heads=24, n_kv_heads=8), dict(max_seqs=0), dict(n_phys_pages=0),
                                 dict(max_tokens_per_seq=0), dict(max_tokens_per_seq=2 ** 31)])
def test_invalid_config(bad):
    cfg = _cfg(**bad)
    assert A.alaya_pool_bytes(cfg) == 0 and A.alaya_workspace_bytes(cfg) == 0
    with pytest.raises(A.AlayaError) as e:
        A.alaya_create_cache(cfg, FAKE[0], FAKE[1], None, FAKE[2], 1 << 30)
    assert e.value.code == A.ALAYA_E_INVAL


def test_create_rejects_bad_memory_arguments():
    cfg = _cfg()
    ws = A.alaya_workspace_bytes(cfg)
    for args, code in [((cfg, 0, FAKE[1], None, FAKE[2], ws), A.ALAYA_E_INVAL),
                       ((cfg, FAKE[0] + 8, FAKE[1], None, FAKE[2], ws), A.ALAYA_E_INVAL),
                       ((cfg, FAKE[0], FAKE[1], None, FAKE[2], ws - 1), A.ALAYA_E_NOMEM),
                       ((cfg, FAKE[0], FAKE[1], [0] * 70, FAKE[2], ws), A.ALAYA_E_INVAL),
                       ((cfg, FAKE[0], FAKE[1], list(range(1, 71)), FAKE[2], ws), A.ALAYA_E_INVAL)]:
        with pytest.raises(A.AlayaError) as e:
            A.alaya_create_cache(*args)
        assert e.value.code == code


def test_append_limits_are_checked_before_any_launch():
    h = _create(order=list(reversed(range(70))))
    try:
        for seq, t, code in [(-1, 1, A.ALAYA_E_INVAL), (4, 1, A.ALAYA_E_INVAL), (0, -1, A.ALAYA_E_INVAL),
                             (0, 4097, A.ALAYA_E_NOMEM)]:
            with pytest.raises(A.AlayaError) as e:
                A.alaya_append_kv(h, seq, FAKE[3], FAKE[4], t)
            assert e.value.code == code
        with pytest.raises(A.AlayaError) as e:
            A.alaya_append_kv(h, 0, 0, FAKE[4], 1)
        assert e.value.code == A.ALAYA_E_INVAL
        A.alaya_append_kv(h, 0, FAKE[3], FAKE[4], 0)           # appending nothing is fine
        assert A.alaya_seq_len(h, 0) == 0 and A.alaya_seq_len(h, 9) == -1
    finally:
        A.alaya_destroy_cache(h)


def test_pool_exhaustion_leaves_cache_unchanged():
    cfg = _cfg(n_phys_pages=3, max_tokens_per_seq=4096)
    h = A.alaya_create_cache(cfg, FAKE[0], FAKE[1], None, FAKE[2], A.alaya_workspace_bytes(cfg))
    try:
        with pytest.raises(A.AlayaError) as e:
            A.alaya_append_kv(h, 1, FAKE[3], FAKE[4], 64 * 3 + 1)   # needs 4 pages, pool has 3
        assert e.value.code == A.ALAYA_E_NOMEM and "exhausted" in str(e.value)
        assert A.alaya_seq_len(h, 1) == 0
    finally:
        A.alaya_destroy_cache(h)


def test_attention_argument_checks():
    h = _create()
    try:
        def sparse(**kw):
            a = dict(seqs=[0], n_q_heads=32, q=FAKE[3], mode=A.ALAYA_TOPK, topk=[4], beta=None, scale=0.0,
                     out=FAKE[4])
            a.update(kw)
            A.alaya_sparse_attn(h, a["seqs"], a["n_q_heads"], a["q"], a["mode"], a["topk"], a["beta"], a["scale"],
                                a["out"], a.get("out_ids"), None, a.get("ids_stride", 0))
        cases = [(dict(), A.ALAYA_E_EMPTY),                       # sequence 0 holds no tokens
                 (dict(seqs=[7]), A.ALAYA_E_INVAL),
                 (dict(seqs=[0] * 5), A.ALAYA_E_INVAL),           # batch above max_batch
                 (dict(n_q_heads=16), A.ALAYA_E_INVAL),
                 (dict(q=0), A.ALAYA_E_INVAL),
                 (dict(out=0), A.ALAYA_E_INVAL)]
        for kw, code in cases:
            with pytest.raises(A.AlayaError) as e:
                sparse(**kw)
            assert e.value.code == code, kw
        with pytest.raises(A.AlayaError) as e:
            A.alaya_full_attn(h, [0], 32, FAKE[3], 0.0, FAKE[4])
        assert e.value.code == A.ALAYA_E_EMPTY
        assert A.alaya_poll_status(h) == A.ALAYA_OK              # nothing was ever launched
    finally:
        A.alaya_destroy_cache(h)


def test_null_handle():
    L = A.lib()
    assert L.alaya_destroy_cache(None) == A.ALAYA_E_INVAL
    assert L.alaya_seq_len(None, 0) == -1
    assert L.alaya_set_tuning(None, 1, 1, 1, 0) == A.ALAYA_E_INVAL
    assert "null" in A.alaya_last_error()


def test_step_append_and_estimate_hook_argument_checks():
    h = _create()
    try:
        for seqs, code in [([0, 0], A.ALAYA_E_INVAL), ([0, 4], A.ALAYA_E_INVAL), ([-1, 0], A.ALAYA_E_INVAL),
                           ([0, 1, 2, 3, 0], A.ALAYA_E_INVAL)]:          # repeated, out of range, above max_batch
            with pytest.raises(A.AlayaError) as e:
                A.alaya_append_kv_step(h, seqs, FAKE[3], FAKE[4])
            assert e.value.code == code, seqs
        with pytest.raises(A.AlayaError) as e:
            A.alaya_append_kv_step(h, [0, 1], 0, FAKE[4])
        assert e.value.code == A.ALAYA_E_INVAL
        for seqs, kv in [([0, 0], FAKE[3]), ([0, 9], FAKE[3]), ([0, 1], 0)]:  # the decode step checks its append first
            with pytest.raises(A.AlayaError) as e:
                A.alaya_decode_step(h, seqs, 32, kv, FAKE[4], FAKE[3], A.ALAYA_TOPK, [4, 4], None, 0.0, FAKE[4])
            assert e.value.code == A.ALAYA_E_INVAL, seqs
        assert [A.alaya_seq_len(h, s) for s in range(4)] == [0, 0, 0, 0]
        L = A.lib()
        assert L.alaya_debug_estimate(h, 3) == A.ALAYA_E_INVAL and L.alaya_debug_estimate(h, -2) == A.ALAYA_E_INVAL
        assert L.alaya_debug_estimate(h, 2) == A.ALAYA_OK and L.alaya_debug_estimate(h, 0) == A.ALAYA_OK
        assert L.alaya_debug_estimate(None, 0) == A.ALAYA_E_INVAL
    finally:
        A.alaya_destroy_cache(h)


def test_bench_refuses_more_than_one_gpu_and_has_no_cpu_fallback():
    import subprocess
    import sys
    import torch
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "ONE GPU" in r.stderr and r.stdout.strip() == ""
    if not torch.cuda.is_available():
        r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py")], capture_output=True, text=True)
        assert r.returncode != 0 and "no GPU" in r.stderr and r.stdout.strip() == ""


def test_plan_query_matches_the_oracle_on_a_grid():
    """The optimizer is host code: the whole decision table is compared here, no GPU needed."""
    import itertools

    import oracle
    qn = {A.QUERY_FULL: "full", A.QUERY_TOPK: "topk", A.QUERY_DIPR: "dipr"}
    xn = {A.INDEX_NONE: "none", A.INDEX_COARSE: "coarse", A.INDEX_FLAT: "flat", A.INDEX_FINE: "fine"}
    grid = itertools.product([1, 4096, 4097, 1 << 20], [0, 4096], [0, 1, 4096, 1 << 19, 1 << 20, 1 << 21],
                             [0, 999, 1000, 1 << 40], [0, 1000], [0, 1, 31])
    for n, short, prefix, budget, need, layer in grid:
        q, x, vis = A.alaya_plan_query(n, short, prefix, budget, need, layer)
        assert (qn[q], xn[x], vis) == oracle.plan(n, short, prefix, budget, need, layer), (n, short, prefix, budget, need, layer)
    for bad in [(0, 1, 0, 0, 0, 0), (10, -1, 0, 0, 0, 0), (10, 1, -1, 0, 0, 0), (10, 1, 0, -1, 0, 0), (10, 1, 0, 0, -1, 0),
                (10, 1, 0, 0, 0, -1)]:
        with pytest.raises(A.AlayaError):
            A.alaya_plan_query(*bad)
    assert ctypes.sizeof(A.PlanInput) == 48 and ctypes.sizeof(A.Plan) == 16
