"""Shared pieces of the GPU parity tests: load a workload into a Cache, run the HIP path, and compare
with the CPU oracle to the stated bar.

Bar:
  * selected sets: identical, except for tokens whose ORACLE score lies within BAND = 1e-4 of the
    selection boundary (the oracle's k-th largest score for top-k, its max - beta for DIPR);
  * outputs: max-abs <= OUT_TOL = 2e-3 against the oracle on its own set; if the sets differ (only
    in band tokens) the oracle's attend step is re-run on the GPU's set, which separates a
    selection difference from an accumulation error;
  * scores: max-abs <= SCORE_TOL = 2e-5 against fp64 (fp32 accumulation of 128 exact bf16 products
    of magnitude O(1): about sqrt(128) * 2^-24 * |s| ~ 1e-6 typical).
"""
from __future__ import annotations

import numpy as np
import torch

import oracle
import paper_2504_10326_amd as A
import workloads as wl

BAND = 1e-4
OUT_TOL = 2e-3
SCORE_TOL = 2e-5


def to_device(a: np.ndarray, dtype: str) -> torch.Tensor:
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype == "bf16":
        return t.cuda().view(torch.bfloat16)
    return t.cuda()


def make_cache(w: wl.Workload, g: dict, extra_tokens: int = 0, max_batch=None, chunks=None) -> A.Cache:
    """Create a cache sized for the workload and append every request's K, V (optionally in pieces)."""
    n_phys = g["n_phys_pages"] + (extra_tokens + 63) // 64 * w.batch
    order = g["page_order"]
    if n_phys != len(order):
        order = np.concatenate([order, np.arange(len(order), n_phys, dtype=np.int32)])
    c = A.Cache(w.n_q_heads, w.n_kv_heads, w.head_dim, w.dtype, max_seqs=w.batch, max_batch=max_batch or w.batch,
                max_tokens_per_seq=max(w.lens) + extra_tokens + 64,
                max_batch_tokens=w.total_tokens + w.batch * extra_tokens,
                n_phys_pages=n_phys, phys_page_order=order if w.permute_pages else None)
    # Poison everything the library did not write itself: unwritten page slots, workspace and scratch read as NaN
    # (0xFFFF is a bf16 NaN, 0xFFFFFFFF an fp32 NaN), so any use of them shows up in the outputs.
    c.k_pool.fill_(0xFF)
    c.v_pool.fill_(0xFF)
    c.workspace.fill_(0xFF)
    c.scratch.fill_(0xFF)
    for r, n in enumerate(w.lens):
        cuts = [0, n] if not chunks else sorted({0, n, *[x for x in chunks if 0 < x < n]})
        for a, b in zip(cuts[:-1], cuts[1:]):
            c.append_kv(r, to_device(g["K"][r][a:b], w.dtype), to_device(g["V"][r][a:b], w.dtype))
    torch.cuda.synchronize()
    return c


def compare_sparse(w, g, out, ids, counts, mode, topk=None, beta=None, scale=None, requests=None, heads=None,
                   scores_gpu=None, threads=0, window=(0, 0), n_visible=None):
    """Compare one sparse call with the oracle. Returns a dict of summary numbers; asserts on failure."""
    out = out.cpu().numpy()
    ids = ids.cpu().numpy()
    counts = counts.cpu().numpy()
    stats = {"band_heads": 0, "max_out_err": 0.0, "max_score_err": 0.0, "counts": []}
    for r in (requests if requests is not None else range(w.batch)):
        n = w.lens[r] if n_visible is None else int(n_visible[r])
        K, V, q = g["K"][r], g["V"][r], g["q"][r]
        k = int(topk[r]) if mode == A.ALAYA_TOPK else 0
        b = float(beta[r]) if mode == A.ALAYA_DIPR else 0.0
        orc = oracle.sparse_attn(q, K, V, oracle.TOPK if mode == A.ALAYA_TOPK else oracle.DIPR, k=k, beta=b,
                                 scale=scale, want_scores=True, threads=threads, window=window, n_visible=n)
        K, V = K[:n], V[:n]
        w0, w1 = min(window[0], n), min(window[1], n)
        outside = np.ones(n, dtype=bool)                       # tokens that the query ranks
        outside[:w0] = False
        outside[n - w1:] = False
        sg = scores_gpu[r].cpu().numpy() if scores_gpu is not None else None
        for h in (heads if heads is not None else range(w.n_q_heads)):
            s = orc["scores"][h]
            if sg is not None:
                err = float(np.abs(sg[h].astype(np.float64) - s).max())
                stats["max_score_err"] = max(stats["max_score_err"], err)
                assert err <= SCORE_TOL, f"request {r} head {h}: score error {err}"
            cnt = int(counts[r, h])
            assert cnt <= ids.shape[2], "id buffer too small for this comparison"
            gpu_ids = ids[r, h, :cnt]
            assert len(np.unique(gpu_ids)) == cnt and gpu_ids.min() >= 0 and gpu_ids.max() < n, \
                f"request {r} head {h}: ids not distinct or out of range"
            ora_ids = orc["ids"][h]
            if mode == A.ALAYA_TOPK:
                want = (n - int(outside.sum())) + min(k, int(outside.sum()))
                assert cnt == want, f"request {r} head {h}: count {cnt} != window + min(k, rest) = {want}"
                retrieved = ora_ids[outside[ora_ids]]
                boundary = s[retrieved].min() if retrieved.size else np.inf
            else:
                boundary = s.max() - b
            diff = np.setxor1d(gpu_ids, ora_ids)
            if diff.size:
                assert outside[diff].all(), f"request {r} head {h}: a window token is missing or extra"
                off = np.abs(s[diff] - boundary)
                assert off.max() <= BAND, (f"request {r} head {h}: {diff.size} ids differ, farthest "
                                           f"{off.max():.3e} from the boundary (> {BAND})")
                stats["band_heads"] += 1
                ref = oracle.attend(s, V, h // w.group, np.sort(gpu_ids), scale)
            else:
                ref = orc["out"][h]
            err = float(np.abs(out[r, h].astype(np.float64) - ref).max())
            stats["max_out_err"] = max(stats["max_out_err"], err)
            assert err <= OUT_TOL, f"request {r} head {h}: output error {err} > {OUT_TOL}"
            stats["counts"].append(cnt)
    return stats


def run_and_compare(c: A.Cache, w, g, mode, topk=None, beta=None, scale=None, ids_stride=None, check_scores=True,
                    threads=0, window=(0, 0), n_visible=None):
    q = to_device(g["q"], w.dtype)
    seqs = list(range(w.batch))
    if ids_stride is None:
        ids_stride = max(w.lens) if mode == A.ALAYA_DIPR else \
            max(min(k + window[0] + window[1], n) for k, n in zip(topk, w.lens))
    out, ids, counts = c.sparse_attn(seqs, q, mode, topk=topk, beta=beta, scale=scale or 0.0, ids_stride=ids_stride,
                                     window=window, n_visible=n_visible)
    torch.cuda.synchronize()
    assert c.poll_status() == A.ALAYA_OK
    sg = None
    if check_scores:
        # The same call with every score written: the scores themselves can then be compared, and the
        # pruned run above must have produced bit-identical ids, counts and outputs.
        c.set_write_all_scores(True)
        out2, ids2, counts2 = c.sparse_attn(seqs, q, mode, topk=topk, beta=beta, scale=scale or 0.0,
                                            ids_stride=ids_stride, window=window, n_visible=n_visible)
        torch.cuda.synchronize()
        sg = [s.clone() for s in c.debug_scores(w.lens if n_visible is None else n_visible)]
        c.set_write_all_scores(False)
        assert torch.equal(counts, counts2) and torch.equal(ids, ids2), "pruned and unpruned selections differ"
        assert torch.equal(out, out2), "pruned and unpruned outputs differ"
    return compare_sparse(w, g, out, ids, counts, mode, topk, beta, scale, scores_gpu=sg, threads=threads,
                          window=window, n_visible=n_visible)
