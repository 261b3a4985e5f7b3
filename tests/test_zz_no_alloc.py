"""alaya_sparse_attn_static - the entry point for callers that cannot allocate - against alaya_sparse_attn.

Runs last (file name) so that a failure here cannot hide another test; passes alone in a fresh process too.
Both entry points run the same kernels, so ids, counts and outputs must be identical bit for bit; the first
call is also checked against the oracle.  Two calls in a row, the second with a smaller input, on the one
scratch array that every call on the GPU shares.
"""
import numpy as np
import pytest
import torch

import paper_2504_10326_amd as A
import workloads as wl
from parity_util import compare_sparse, make_cache, to_device

pytestmark = pytest.mark.gpu


def _llama(lens, topk):
    return wl.resized(wl.config("llama8b_128k"), lens, topk=topk)


def test_static_scratch_entry_point_matches_the_bound_scratch_one():
    big = _llama([40000, 3000], [2048, 64])
    small = _llama([5000], [100])
    gb, gs = wl.generate(big), wl.generate(small)
    cb, cs = make_cache(big, gb), make_cache(small, gs)
    qb, qs = to_device(gb["q"], "bf16"), to_device(gs["q"], "bf16")
    for rnd in range(2):                                           # the array keeps the last call's contents
        for c, w, g, q, calls in ((cb, big, gb, qb, [(A.ALAYA_TOPK, dict(topk=[2048, 64], ids_stride=2048)),
                                                      (A.ALAYA_DIPR, dict(beta=[3.0, 1.0], ids_stride=40000,
                                                                          window=(32, 128)))]),
                                  (cs, small, gs, qs, [(A.ALAYA_TOPK, dict(topk=[100], ids_stride=100)),
                                                       (A.ALAYA_DIPR, dict(beta=[2.0], ids_stride=5000))])):
            seqs = list(range(w.batch))
            for mode, kw in calls:
                ref = c.sparse_attn(seqs, q, mode, **kw)
                got = c.sparse_attn(seqs, q, mode, static_scratch=True, **kw)
                torch.cuda.synchronize()
                for x, y in zip(ref, got):
                    assert torch.equal(x, y), (rnd, w.lens, mode)
                if rnd == 0:
                    compare_sparse(w, g, got[0], got[1], got[2], mode, kw.get("topk"), kw.get("beta"),
                                   window=kw.get("window", (0, 0)))
    # a cache with no scratch memory bound at all can still be queried through the static entry point
    A.alaya_bind_scratch(cs.handle, 0, 0)
    ref2 = cs.sparse_attn([0], qs, A.ALAYA_TOPK, topk=[100], ids_stride=100, static_scratch=True)
    with pytest.raises(A.AlayaError) as e:
        cs.sparse_attn([0], qs, A.ALAYA_TOPK, topk=[100], ids_stride=100)
    assert e.value.code == A.ALAYA_E_INVAL and "scratch" in str(e.value)
    A.alaya_bind_scratch(cs.handle, cs.scratch, cs.scratch.numel())
    ref3 = cs.sparse_attn([0], qs, A.ALAYA_TOPK, topk=[100], ids_stride=100)
    for x, y in zip(ref2, ref3):
        assert torch.equal(x, y)
    cb.close(); cs.close()


def test_static_scratch_entry_point_refuses_what_does_not_fit():
    """About 16 bytes per (query head, token): 200 thousand tokens at 32 heads exceed the 80 MiB array."""
    n = 200000
    c = A.Cache(32, 8, 128, "bf16", max_seqs=1, max_batch=1, max_tokens_per_seq=n + 64, max_batch_tokens=n + 64,
                n_phys_pages=n // 64 + 2)
    k = torch.randn((n, 8, 128), device="cuda").to(torch.bfloat16)
    c.append_kv(0, k, k)
    q = torch.randn((1, 32, 128), device="cuda").to(torch.bfloat16)
    with pytest.raises(A.AlayaError) as e:
        c.sparse_attn([0], q, A.ALAYA_TOPK, topk=[64], static_scratch=True)
    assert e.value.code == A.ALAYA_E_NOMEM and "built-in" in str(e.value)
    out = c.sparse_attn([0], q, A.ALAYA_TOPK, topk=[64])          # the bound-scratch call has no such limit
    out2 = c.sparse_attn([0], q, A.ALAYA_TOPK, topk=[64], n_visible=[100000], static_scratch=True)   # a prefix that fits
    out3 = c.sparse_attn([0], q, A.ALAYA_TOPK, topk=[64], n_visible=[100000])
    torch.cuda.synchronize()
    assert torch.isfinite(out).all() and torch.equal(out2, out3)
    c.close()
