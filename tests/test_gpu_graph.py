"""GPU parity of the fine-grained index and of DIPRS (Sec. 6.1.3 "DIPR Query Processing", Algorithm 1; Sec. 6.2
index types; Sec. 7.1 window; Sec. 7.2 late materialization) against the oracle.

Graph builder: the GPU takes k_i . k_j in fp32 on the matrix cores, the oracle in fp64.  A row's neighbour
list must hold the oracle's neighbours, except for keys whose ORACLE similarity lies within BAND_SIM of the
oracle's M-th best, and must be ordered by oracle similarity up to the same band.  BAND_SIM = 2e-3: a
similarity is a sum of 128 products with sum |terms| of a few hundred at most here, fp32 accumulation in any
order is off by at most 128 * 2^-24 * that sum, about 2e-3 (typically 1e-5).

DIPRS: which neighbours enter the list C depends on score comparisons, so both sides take scores in the same
arithmetic (fp32, one fused multiply-add per channel in channel order), and the walk runs on the same graph:
the one the GPU built, handed to the oracle.  Bar: the list C identical entry by entry, the answer identical
as a set, outputs within OUT_TOL of the oracle's attend step over that set."""
import numpy as np
import pytest
import torch

import oracle
import paper_2504_10326_amd as A
import workloads as wl
from parity_util import OUT_TOL, make_cache, to_device

pytestmark = pytest.mark.gpu
BAND_SIM = 2e-3


def _setup(n, seed=0, extra=0, **kw):
    w = wl.resized(wl.config("llama8b_128k", seed), [n], **kw)
    g = wl.generate(w)
    c = make_cache(w, g, extra_tokens=extra)
    return w, g, c


def _sims(K, g, j):
    Kf = wl.bf16_bits_to_f32(K[:, g, :]).astype(np.float64)
    return Kf @ Kf[j]


@pytest.mark.parametrize("n,M", [(1, 4), (3, 8), (64, 8), (700, 16), (4133, 32), (2500, 64)])
def test_graph_builder_matches_brute_force(n, M):
    w, g, c = _setup(n, seed=n)
    print(f"graph build n={n} M={M}", flush=True)
    gr = c.build_graph(0, M)
    nbr = gr.neighbours().cpu().numpy()
    assert nbr.shape == (w.n_kv_heads, n, M)
    K = g["K"][0]
    rows = np.unique(np.concatenate([np.arange(min(n, 40)), np.arange(max(0, n - 40), n),
                                     np.random.default_rng(n).integers(0, n, 60)]))
    band_rows = 0
    for kvh in range(w.n_kv_heads):
        want_all = oracle.knn_graph(K, kvh, M) if n <= 1000 else None
        Kf = wl.bf16_bits_to_f32(K[:, kvh, :]).astype(np.float64)
        norms = (Kf * Kf).sum(axis=1)
        # the entry point: the key of largest norm, up to fp32 rounding of the norm
        assert norms[gr.entry[kvh]] >= norms.max() * (1 - 1e-5)
        for j in (range(n) if want_all is not None else rows):
            got = nbr[kvh, j]
            m = min(M, n - 1)
            assert (got[m:] == -1).all() and (got[:m] >= 0).all() and (got[:m] < n).all()
            got = got[:m]
            assert j not in got and len(np.unique(got)) == m
            sim = Kf @ Kf[j]
            if want_all is not None:
                want = want_all[j, :m]
            else:
                sim_x = sim.copy()
                sim_x[j] = -np.inf
                want = np.lexsort((np.arange(n), -sim_x))[:m]
            if (got != want).any():
                band_rows += 1
                diff = np.setxor1d(got, want)
                if diff.size:
                    edge = sim[want[-1]]
                    assert np.abs(sim[diff] - edge).max() <= BAND_SIM, f"head {kvh} row {j}: {diff} not at the boundary"
                # order: by oracle similarity, descending, up to the band
                assert (np.diff(sim[got]) <= BAND_SIM).all(), f"head {kvh} row {j}: list out of order"
    print(f"rows with band differences: {band_rows}", flush=True)
    gr.close()
    c.close()


def _oracle_walk(w, g, nbr, entry, n_idx, l0, beta, window):
    """Per query head: (ids, C, s32) from the oracle on the GPU-built graph."""
    K, q = g["K"][0], g["q"][0]
    n = K.shape[0]
    w0, w1 = min(window[0], n), min(max(window[1], n - n_idx), n)
    res = []
    for h in range(w.n_q_heads):
        kvh = h // w.group
        s32 = oracle.scores_f32(q[h], K, kvh)
        full = np.full((n, nbr.shape[2]), -1, dtype=np.int32)
        full[:n_idx] = nbr[kvh]
        k0 = entry[kvh]
        if k0 < w0 or k0 >= n - w1:     # the entry point is a window token: start behind the initial window
            k0 = w0 if w0 < min(n - w1, n_idx) else -1
        if k0 < 0:
            ids = np.array([j for j in range(n) if j < w0 or j >= n - w1], dtype=np.int32)
            C = np.empty(0, dtype=np.int32)
        else:
            ids, C = oracle.diprs(full, s32, k0, l0, beta, window=(w0, w1))
        res.append((ids, C, s32))
    return res


def _check_walk(w, g, c, gr, l0, beta, window=(0, 0), scale=0.0):
    n = g["K"][0].shape[0]
    q = to_device(g["q"], w.dtype)
    print(f"diprs n={n} n_idx={gr.n_indexed} M={gr.degree} l0={l0} beta={beta} window={window}", flush=True)
    out, ids, counts = c.diprs_attn(gr, q, beta, l0, scale=scale, ids_stride=n, window=window)
    torch.cuda.synchronize()
    assert c.poll_status() == 0
    out, ids, counts = out.cpu().numpy(), ids.cpu().numpy(), counts.cpu().numpy()
    nbr = gr.neighbours().cpu().numpy()
    want = _oracle_walk(w, g, nbr, gr.entry, gr.n_indexed, l0, beta, window)
    lens, sizes = [], []
    for h in range(w.n_q_heads):
        want_ids, want_C, s32 = want[h]
        got_C = c.debug_diprs_list(h)
        assert len(got_C) == len(want_C), f"head {h}: list C has {len(got_C)} entries, the oracle's {len(want_C)}"
        assert (got_C == want_C).all(), f"head {h}: list C differs first at {np.argmax(got_C != want_C)}"
        cnt = int(counts[0, h])
        assert cnt == len(want_ids), f"head {h}: {cnt} selected, oracle {len(want_ids)}"
        got = ids[0, h, :cnt]
        assert (ids[0, h, cnt:] == -1).all()
        assert (np.sort(got) == want_ids).all(), f"head {h}: answers differ"
        s64 = oracle.scores(g["q"][0][h], g["K"][0], h // w.group)
        ref = oracle.attend(s64, g["V"][0], h // w.group, want_ids, scale=scale if scale > 0 else None)
        err = np.abs(out[0, h] - ref).max()
        assert err <= OUT_TOL, f"head {h}: output off by {err:.2e}"
        lens.append(len(want_C))
        sizes.append(cnt)
    return np.array(lens), np.array(sizes)


@pytest.mark.parametrize("n,M,l0,beta", [(64, 8, 0, 1.0), (700, 16, 32, 2.0), (4133, 32, 64, 2.0), (4133, 32, 0, 4.0),
                                         (2500, 64, 500, 0.0), (4133, 8, 4133, 3.0), (3000, 5, 200, 2.0), (3000, 1, 50, 8.0),
                                         (3000, 33, 100, 2.0), (9000, 4, 9000, 2.0)])
def test_diprs_list_and_answer_match_oracle(n, M, l0, beta):
    w, g, c = _setup(n, seed=100 + n)
    gr = c.build_graph(0, M)
    lens, sizes = _check_walk(w, g, c, gr, l0, beta)
    print(f"|C| {lens.min()}..{lens.max()}, answers {sizes.min()}..{sizes.max()}", flush=True)
    assert lens.max() > 1 or n == 1
    gr.close()
    c.close()


@pytest.mark.parametrize("lds_bytes", [3072, 16384, 40000])
def test_diprs_with_less_on_chip_memory(lds_bytes):
    """What a walk over a very long context does - visited bits and page table in global memory, a list far
    longer than its on-chip mirror - reached on a small one by lowering the on-chip budget: same list, same answer."""
    w, g, c = _setup(9000, seed=13)
    c.debug_diprs_lds(lds_bytes)
    for M in (4, 32):
        gr = c.build_graph(0, M)
        lens, _ = _check_walk(w, g, c, gr, 9000, 2.0, window=(4, 100))
        print(f"M={M}: |C| {lens.min()}..{lens.max()}", flush=True)
        assert lens.max() > 1500
        _check_walk(w, g, c, gr, 64, 2.0)
        gr.close()
    c.debug_diprs_lds(0)
    c.close()


def test_diprs_window_and_scale():
    w, g, c = _setup(3000, seed=7)
    gr = c.build_graph(0, 32)
    _check_walk(w, g, c, gr, 64, 2.0, window=(4, 64))
    _check_walk(w, g, c, gr, 16, 1.0, window=(130, 0), scale=0.05)
    _check_walk(w, g, c, gr, 16, 1.0, window=(0, 200))
    # a window that swallows the sequence: nothing to walk, everything attended
    lens, sizes = _check_walk(w, g, c, gr, 16, 1.0, window=(2000, 2000))
    assert (lens == 0).all() and (sizes == 3000).all()
    gr.close()
    c.close()


def test_diprs_entry_point_in_window_starts_behind_it():
    w, g, c = _setup(1500, seed=11)
    gr = c.build_graph(0, 16)
    e = max(gr.entry)
    lens, _ = _check_walk(w, g, c, gr, 32, 2.0, window=(e + 1, 0))   # every entry point lies in the initial window
    assert (lens >= 1).all()
    gr.close()
    c.close()


def test_diprs_tokens_appended_after_the_build_join_the_window():
    """Sec. 7.2 late materialization: the graph is not updated by an append; the new tokens are attended as
    window tokens until the index is rebuilt."""
    w2 = wl.resized(wl.config("llama8b_128k", 3), [2150])
    g2 = wl.generate(w2)
    first = {**g2, "K": [g2["K"][0][:2000]], "V": [g2["V"][0][:2000]]}
    c = make_cache(wl.resized(w2, [2000]), first, extra_tokens=200)
    gr = c.build_graph(0, 32)
    c.append_kv(0, to_device(g2["K"][0][2000:], w2.dtype), to_device(g2["V"][0][2000:], w2.dtype))
    assert gr.n_indexed == 2000 and c.seq_len(0) == 2150
    _check_walk(w2, g2, c, gr, 64, 2.0)
    _check_walk(w2, g2, c, gr, 64, 2.0, window=(8, 300))
    gr.close()
    c.close()


def test_diprs_recall_against_exact_range_query():
    """Not a parity bar: how much of the exact DIPR answer the walk finds on this workload (reported)."""
    w, g, c = _setup(8192, seed=5)
    gr = c.build_graph(0, 32)
    q = to_device(g["q"], w.dtype)
    beta = 2.0
    for l0 in (32, 256):
        out, ids, counts = c.diprs_attn(gr, q, beta, l0, ids_stride=8192)
        torch.cuda.synchronize()
        ids, counts = ids.cpu().numpy(), counts.cpu().numpy()
        rec = []
        for h in range(w.n_q_heads):
            s = oracle.scores(g["q"][0][h], g["K"][0], h // w.group)
            exact = oracle.select_dipr(s, beta)
            rec.append(len(np.intersect1d(ids[0, h, :counts[0, h]], exact)) / len(exact))
        print(f"l0={l0}: recall of the exact DIPR answer mean {np.mean(rec):.3f} min {np.min(rec):.3f}", flush=True)
    gr.close()
    c.close()


@pytest.mark.parametrize("seed", range(8))
def test_diprs_random_configurations_against_the_oracle(seed):
    """Random context lengths, degrees, capacities, margins, windows and on-chip budgets."""
    rng = np.random.default_rng(7000 + seed)
    n = int(rng.choice([int(rng.integers(2, 200)), int(rng.integers(1000, 6000)), int(rng.integers(10000, 30000))]))
    M = int(rng.choice([1, 3, 8, 16, 17, 32, 64]))
    w, g, c = _setup(n, seed=seed, extra=100)
    gr = c.build_graph(0, M)
    for _ in range(3):
        c.debug_diprs_lds(int(rng.choice([0, 0, 2048, 9000, 30000])))
        l0 = int(rng.choice([0, 1, 16, 64, 500, n]))
        beta = float(rng.choice([0.0, 0.5, 2.0, 5.0]))
        window = (int(rng.choice([0, 0, 3, 128])), int(rng.choice([0, 0, 64, 512])))
        _check_walk(w, g, c, gr, l0, beta, window=window)
    gr.close()
    c.close()


def test_graph_and_diprs_argument_errors():
    w, g, c = _setup(300, seed=1)
    with pytest.raises(A.AlayaError):
        c.build_graph(0, 0)
    with pytest.raises(A.AlayaError):
        c.build_graph(0, 65)
    with pytest.raises(A.AlayaError):
        c.build_graph(1, 8)
    gr = c.build_graph(0, 8)
    q = to_device(g["q"], w.dtype)
    with pytest.raises(A.AlayaError):
        c.diprs_attn(gr, q, -1.0, 8)
    with pytest.raises(A.AlayaError):
        c.diprs_attn(gr, q, 1.0, -1)
    c.reset_seq(0)
    with pytest.raises(A.AlayaError):
        c.diprs_attn(gr, q, 1.0, 8)
    gr.close()
    c.close()
