"""GPU parity at the full sizes of the measured workloads, in the launch configuration bench.py times
(default launch shapes, one call per step).  Every query head of every request is compared with the
oracle; the oracle runs on the host cores with OpenMP and takes a few seconds per case."""
import sys
import time

import numpy as np
import pytest
import torch

import oracle
import paper_2504_10326_amd as A
import workloads as wl
from parity_util import OUT_TOL, make_cache, run_and_compare, to_device

pytestmark = pytest.mark.gpu


def _say(msg):
    print(f"[fullsize] {msg}", file=sys.stderr, flush=True)


def _case(name, seed=0):
    t0 = time.time()
    w = wl.config(name, seed)
    _say(f"{name}: generating {w.total_tokens} tokens x {w.n_kv_heads} KV heads")
    g = wl.generate(w)
    _say(f"{name}: generated in {time.time() - t0:.1f}s, loading the cache")
    c = make_cache(w, g)
    _say(f"{name}: cache loaded")
    return w, g, c


def test_llama8b_128k_topk2048():
    w, g, c = _case("llama8b_128k")
    st = run_and_compare(c, w, g, A.ALAYA_TOPK, topk=w.topk)
    _say(f"llama8b_128k: out err {st['max_out_err']:.2e}, score err {st['max_score_err']:.2e}, "
         f"heads with band ids {st['band_heads']}")
    # the paper's own settings (Table 3): a window of [128 + 512] tokens plus 2000 / 100 retrieved ones,
    # and the window-enhanced DIPR query; then the same on a 100000-token prefix of the context
    for k in (2000, 100):
        st = run_and_compare(c, w, g, A.ALAYA_TOPK, topk=[k], window=(128, 512), check_scores=False)
        assert set(st["counts"]) == {640 + k}
        _say(f"llama8b_128k [128+512]+{k}: out err {st['max_out_err']:.2e}, band heads {st['band_heads']}")
    st = run_and_compare(c, w, g, A.ALAYA_DIPR, beta=[2.0], window=(128, 512), check_scores=False)
    _say(f"llama8b_128k [128+512] DIPR beta=2: selected {min(st['counts'])}..{max(st['counts'])}, "
         f"out err {st['max_out_err']:.2e}")
    st = run_and_compare(c, w, g, A.ALAYA_TOPK, topk=[2000], window=(128, 512), n_visible=[100000], check_scores=False)
    _say(f"llama8b_128k prefix 100000, [128+512]+2000: out err {st['max_out_err']:.2e}, band heads {st['band_heads']}")
    c.close()


def test_range_256k_dipr_betas():
    w, g, c = _case("range_256k")
    for beta in w.betas:
        st = run_and_compare(c, w, g, A.ALAYA_DIPR, beta=[beta], check_scores=(beta == w.betas[0]))
        cnt = np.array(st["counts"])
        _say(f"range_256k beta={beta}: selected per head min/median/max = {cnt.min()}/{int(np.median(cnt))}/"
             f"{cnt.max()}, out err {st['max_out_err']:.2e}, band heads {st['band_heads']}")
    c.close()


def test_paged_1m_topk4096_permuted_pages():
    w, g, c = _case("paged_1m")
    st = run_and_compare(c, w, g, A.ALAYA_TOPK, topk=w.topk)
    _say(f"paged_1m: out err {st['max_out_err']:.2e}, score err {st['max_score_err']:.2e}, "
         f"band heads {st['band_heads']}")
    # this call is large enough for the estimated threshold bound; make every head take the repair path too
    c.debug_estimate(2)
    st = run_and_compare(c, w, g, A.ALAYA_TOPK, topk=w.topk, check_scores=False)
    _say(f"paged_1m with every head repaired: out err {st['max_out_err']:.2e}, band heads {st['band_heads']}")
    c.debug_estimate(0)
    q = to_device(g["q"], w.dtype)
    full = c.full_attn([0], q).cpu().numpy()
    ref = oracle.full_attn(g["q"][0], g["K"][0], g["V"][0])
    err = float(np.abs(full[0] - ref).max())
    _say(f"paged_1m: full attention err {err:.2e}")
    assert err <= OUT_TOL
    c.close()


def test_batched_16_requests_one_launch():
    w, g, c = _case("batched_16")
    st = run_and_compare(c, w, g, A.ALAYA_TOPK, topk=w.topk)
    _say(f"batched_16: lens {w.lens}, out err {st['max_out_err']:.2e}, score err {st['max_score_err']:.2e}, "
         f"band heads {st['band_heads']}")
    c.close()
