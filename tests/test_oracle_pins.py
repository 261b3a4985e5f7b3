"""Pins for the CPU oracle: facts fixed by the paper and by mathematics, none by the oracle itself.

Each test names the passage it takes its fact from.  A plausible mistake in
oracle/alaya_oracle.c (a dropped 1/sqrt(d), a softmax over all tokens instead
of the selected ones, a wrong KV-head index, '>' for '>=', a wrong tie order,
transposed K) fails at least one of them.
"""
import itertools
import math

import numpy as np
import pytest
import torch

import oracle
import workloads as wl


def _small(seed, n=96, hq=4, hk=2, d=16, dtype="f32"):
    w = wl.Workload("pin", hq, hk, d, (n,), dtype, 4, "topk", topk=(8,), seed=seed)
    g = wl.generate(w, threads=1)
    return w, g["q"][0], g["K"][0], g["V"][0]


def _f64(a, dtype):
    return (wl.bf16_bits_to_f32(a) if dtype == "bf16" else a).astype(np.float64)


def _dense(q, K, V, dtype):
    """softmax(q K^T / sqrt(d)) V with GQA, by library routines only (Eq. 1)."""
    qf, Kf, Vf = _f64(q, dtype), _f64(K, dtype), _f64(V, dtype)
    hq, d = qf.shape
    hk = Kf.shape[1]
    G = hq // hk
    s = np.einsum("hc,jhc->hj", qf, np.repeat(Kf, G, axis=1))          # [hq][n]
    z = s / math.sqrt(d)
    a = np.exp(z - z.max(axis=1, keepdims=True))
    a /= a.sum(axis=1, keepdims=True)
    o = np.einsum("hj,jhc->hc", a, np.repeat(Vf, G, axis=1))
    return s, a, o


# ---------------------------------------------------------------- closed form
def test_closed_form_weights_1_2_4():
    """Eq. (1) by hand: d = 4 so 1/sqrt(d) = 1/2; q.k_j = 2 ln w_j gives softmax weights w_j / sum w."""
    w = np.array([1.0, 2.0, 4.0])
    q = np.array([[1.0, 0.0, 0.0, 0.0]], dtype=np.float32)
    K = np.zeros((3, 1, 4), dtype=np.float32)
    K[:, 0, 0] = 2.0 * np.log(w)
    K[:, 0, 1:] = [[5.0, -3.0, 2.0], [1.0, 1.0, 1.0], [-7.0, 0.5, 0.25]]   # orthogonal to q: must not matter
    V = np.array([[[7.0, 0.0, 14.0, -7.0]], [[0.0, 7.0, 7.0, 7.0]], [[-7.0, 3.5, 0.0, 1.75]]], dtype=np.float32)
    full = oracle.full_attn(q, K, V)
    exp_full = (1 * V[0, 0] + 2 * V[1, 0] + 4 * V[2, 0]) / 7.0
    np.testing.assert_allclose(full[0], exp_full, rtol=0, atol=1e-6)
    # top-2 keeps weights 2 and 4, renormalised over the selected set: 1/3, 2/3 (Sec. 2 "Sparse Attention")
    r = oracle.sparse_attn(q, K, V, oracle.TOPK, k=2)
    assert list(r["ids"][0]) == [1, 2]
    np.testing.assert_allclose(r["out"][0], (2 * V[1, 0] + 4 * V[2, 0]) / 6.0, rtol=0, atol=1e-6)
    # scores are 0, 2 ln 2 = 1.386, 2 ln 4 = 2.773.  beta = 1.5 keeps the top two, beta = 1.3 only the top (Def. 2)
    assert list(oracle.sparse_attn(q, K, V, oracle.DIPR, beta=1.5)["ids"][0]) == [1, 2]
    assert list(oracle.sparse_attn(q, K, V, oracle.DIPR, beta=1.3)["ids"][0]) == [2]
    assert list(oracle.sparse_attn(q, K, V, oracle.DIPR, beta=2.8)["ids"][0]) == [0, 1, 2]


def test_inclusive_boundary():
    """Def. 2 uses '>=': a key exactly beta below the maximum is critical."""
    s = np.array([1.0, 3.0, 5.0, 4.0])
    assert list(oracle.select_dipr(s, 2.0)) == [1, 2, 3]
    assert list(oracle.select_dipr(s, 1.0)) == [2, 3]
    assert list(oracle.select_dipr(s, 0.999)) == [2]


# ---------------------------------------------------------------- P1: library routine
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("seed", [0, 1])
def test_scores_and_full_attention_match_dense_library(seed, dtype):
    """Eq. (1): scores, then softmax(z) V over all tokens, against numpy and torch SDPA in fp64."""
    w, q, K, V = _small(seed, n=200, hq=8, hk=2, d=32, dtype=dtype)
    s_ref, _, o_ref = _dense(q, K, V, dtype)
    G = w.group
    for h in range(w.n_q_heads):
        np.testing.assert_allclose(oracle.scores(q[h], K, h // G), s_ref[h], rtol=0, atol=1e-12)
    o = oracle.full_attn(q, K, V)
    np.testing.assert_allclose(o, o_ref, rtol=0, atol=1e-12)
    tq = torch.from_numpy(_f64(q, dtype))[None, :, None, :]                       # [1][hq][1][d]
    tk = torch.from_numpy(_f64(K, dtype)).permute(1, 0, 2).repeat_interleave(G, 0)[None]
    tv = torch.from_numpy(_f64(V, dtype)).permute(1, 0, 2).repeat_interleave(G, 0)[None]
    t = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv)[0, :, 0, :].numpy()
    np.testing.assert_allclose(o, t, rtol=0, atol=1e-10)


@pytest.mark.parametrize("seed", [0, 3])
def test_k_equal_n_and_unbounded_beta_are_full_attention(seed):
    """Selecting everything must reproduce Eq. (1) exactly."""
    w, q, K, V = _small(seed, n=150)
    full = oracle.full_attn(q, K, V)
    a = oracle.sparse_attn(q, K, V, oracle.TOPK, k=150)
    b = oracle.sparse_attn(q, K, V, oracle.TOPK, k=10 ** 6)        # k > n clamps to n
    c = oracle.sparse_attn(q, K, V, oracle.DIPR, beta=float("inf"))
    for r in (a, b, c):
        assert (r["counts"] == 150).all()
        np.testing.assert_allclose(r["out"], full, rtol=0, atol=1e-13)


def test_tiny_workload_full_attention_dense():
    """The tiny configuration (4096 tokens, fp32, d = 128) against the dense library form."""
    w = wl.config("tiny")
    g = wl.generate(w, threads=1)
    _, _, o_ref = _dense(g["q"][0], g["K"][0], g["V"][0], "f32")
    np.testing.assert_allclose(oracle.full_attn(g["q"][0], g["K"][0], g["V"][0]), o_ref, rtol=0, atol=1e-12)


# ---------------------------------------------------------------- P2: Theorem 1
@pytest.mark.parametrize("beta", [0.0, 0.3, 1.0, 2.5, 7.0])
def test_dipr_equals_alpha_form(beta):
    """Theorem 1: {q.k >= max - beta} == {a_j >= alpha max a}, alpha = exp(-beta / sqrt(d))."""
    w, q, K, V = _small(5, n=300, hq=4, hk=2, d=16)
    s, a, _ = _dense(q, K, V, "f32")
    alpha = math.exp(-beta / math.sqrt(w.head_dim))
    r = oracle.sparse_attn(q, K, V, oracle.DIPR, beta=beta)
    for h in range(w.n_q_heads):
        ratio = a[h] / a[h].max()
        far = np.abs(ratio - alpha) > 1e-9          # leave out keys on the razor's edge of fp64 rounding
        want = set(np.nonzero((ratio >= alpha) & far)[0])
        got = set(r["ids"][h])
        assert want <= got and got - want <= set(np.nonzero(~far)[0])


# ---------------------------------------------------------------- P3: beta = 0
def test_beta_zero_is_argmax_and_top1():
    w, q, K, V = _small(7, n=120)
    s, _, _ = _dense(q, K, V, "f32")
    r0 = oracle.sparse_attn(q, K, V, oracle.DIPR, beta=0.0)
    r1 = oracle.sparse_attn(q, K, V, oracle.TOPK, k=1)
    Vf = V.astype(np.float64)
    for h in range(w.n_q_heads):
        j = int(np.argmax(s[h]))
        assert list(r0["ids"][h]) == [j] == list(r1["ids"][h])
        np.testing.assert_allclose(r0["out"][h], Vf[j, h // w.group], rtol=0, atol=1e-15)
        np.testing.assert_allclose(r1["out"][h], Vf[j, h // w.group], rtol=0, atol=1e-15)


# ---------------------------------------------------------------- P4 / P5: nesting, two paths agree
def test_nesting_counts_and_cross_check():
    w, q, K, V = _small(11, n=257)
    prev_b, prev_k = None, None
    for beta in [0.0, 0.5, 1.0, 2.0, 4.0, 100.0]:
        r = oracle.sparse_attn(q, K, V, oracle.DIPR, beta=beta, want_scores=True)
        sets = [set(x) for x in r["ids"]]
        for h, S in enumerate(sets):
            assert len(S) >= 1 and int(np.argmax(r["scores"][h])) in S
            # Sec. 6.1.2 (i): a DIPR answer is the top-k' answer for k' = its own size
            kprime = len(S)
            assert S == set(oracle.select_topk(r["scores"][h], kprime))
        if prev_b is not None:
            assert all(a <= b for a, b in zip(prev_b, sets))
        prev_b = sets
    for k in [1, 2, 17, 64, 256, 257, 300]:
        r = oracle.sparse_attn(q, K, V, oracle.TOPK, k=k)
        sets = [set(x) for x in r["ids"]]
        assert all(len(S) == min(k, 257) for S in sets) and (r["counts"] == min(k, 257)).all()
        if prev_k is not None:
            assert all(a <= b for a, b in zip(prev_k, sets))
        prev_k = sets


# ---------------------------------------------------------------- P6: permutation invariance
def test_token_permutation_invariance():
    """Attention has no positional term once K, V are cached (Eq. 1): permuting tokens maps S and keeps o."""
    w, q, K, V = _small(13, n=180)
    perm = np.random.default_rng(0).permutation(180)
    inv = np.argsort(perm)
    for mode, kw in [(oracle.TOPK, dict(k=23)), (oracle.DIPR, dict(beta=1.5))]:
        a = oracle.sparse_attn(q, K, V, mode, **kw)
        b = oracle.sparse_attn(q, K[perm], V[perm], mode, **kw)
        np.testing.assert_allclose(a["out"], b["out"], rtol=0, atol=1e-13)
        for h in range(w.n_q_heads):
            assert set(a["ids"][h]) == set(perm[b["ids"][h]])
            assert set(inv[a["ids"][h]]) == set(b["ids"][h])


# ---------------------------------------------------------------- P7 / P8: brute force
@pytest.mark.parametrize("seed", range(4))
def test_bruteforce_tiny(seed):
    """n = 12: sort for top-k, enumerate every subset for the recovery ratio (Sec. 6.1.1, Observation I)."""
    n, k = 12, 4
    w, q, K, V = _small(seed, n=n, hq=2, hk=1, d=8)
    qf, Kf, Vf = q.astype(np.float64), K.astype(np.float64), V.astype(np.float64)
    r = oracle.sparse_attn(q, K, V, oracle.TOPK, k=k)
    for h in range(2):
        s = [sum(qf[h, c] * Kf[j, 0, c] for c in range(8)) for j in range(n)]
        order = sorted(range(n), key=lambda j: (-s[j], j))
        assert sorted(order[:k]) == list(r["ids"][h])
        z = [x / math.sqrt(8) for x in s]
        a = [math.exp(x - max(z)) for x in z]
        tot = sum(a)
        best = max(itertools.combinations(range(n), k), key=lambda S: sum(a[j] for j in S))
        assert set(best) == set(r["ids"][h])
        S = order[:k]
        den = sum(a[j] for j in S)
        o = [sum(a[j] / den * Vf[j, 0, c] for j in S) for c in range(8)]
        np.testing.assert_allclose(r["out"][h], o, rtol=0, atol=1e-13)
        assert sum(a[j] for j in S) / tot <= 1.0


def test_ties_prefer_smaller_index():
    """Equal scores at the k-th place: the earlier token wins (this build's reading; the paper is silent)."""
    s = np.array([1.0, 5.0, 3.0, 3.0, 3.0, 0.0, 3.0])
    assert list(oracle.select_topk(s, 1)) == [1]
    assert list(oracle.select_topk(s, 2)) == [1, 2]
    assert list(oracle.select_topk(s, 3)) == [1, 2, 3]
    assert list(oracle.select_topk(s, 4)) == [1, 2, 3, 4]
    assert list(oracle.select_topk(s, 5)) == [1, 2, 3, 4, 6]
    assert list(oracle.select_topk(s, 6)) == [0, 1, 2, 3, 4, 6]
    K = np.ones((5, 1, 4), dtype=np.float32)           # duplicate keys are legal
    V = np.arange(20, dtype=np.float32).reshape(5, 1, 4)
    q = np.ones((1, 4), dtype=np.float32)
    r = oracle.sparse_attn(q, K, V, oracle.TOPK, k=2)
    assert list(r["ids"][0]) == [0, 1]
    np.testing.assert_allclose(r["out"][0], V[:2, 0].mean(axis=0))


# ---------------------------------------------------------------- P9: partial attention merge
def test_partial_attention_merge():
    """Sec. 7.2, data-centric engine: parts computed independently and merged by (max, sum, acc) equal one pass."""
    w, q, K, V = _small(17, n=222, hq=2, hk=1, d=16)
    s, _, _ = _dense(q, K, V, "f32")
    rng = np.random.default_rng(1)
    for h in range(2):
        ids = oracle.select_topk(s[h], 50)
        whole = oracle.attend(s[h], V, 0, ids)
        cut = np.sort(rng.choice(np.arange(1, 50), size=3, replace=False))
        parts = np.split(rng.permutation(ids), cut)
        scale = 1 / math.sqrt(16)
        m = [float((s[h][p] * scale).max()) for p in parts]
        l = [float(np.exp(s[h][p] * scale - mi).sum()) for p, mi in zip(parts, m)]
        o = [oracle.attend(s[h], V, 0, np.sort(p)) for p in parts]
        M = max(m)
        wts = np.array([li * math.exp(mi - M) for li, mi in zip(l, m)])
        merged = sum(wi * oi for wi, oi in zip(wts, o)) / wts.sum()
        np.testing.assert_allclose(merged, whole, rtol=0, atol=1e-13)


# ---------------------------------------------------------------- P10: GQA
def test_gqa_equals_replicated_mha():
    """Sec. 7.2, GQA: the heads of a group query the same key/value head."""
    w, q, K, V = _small(19, n=140, hq=8, hk=2, d=16)
    G = w.group
    Kr, Vr = np.repeat(K, G, axis=1), np.repeat(V, G, axis=1)
    for mode, kw in [(oracle.TOPK, dict(k=9)), (oracle.DIPR, dict(beta=2.0)), (oracle.FULL, {})]:
        a = oracle.sparse_attn(q, K, V, mode, **kw)
        b = oracle.sparse_attn(q, Kr, Vr, mode, **kw)
        np.testing.assert_allclose(a["out"], b["out"], rtol=0, atol=1e-14)
        assert all((x == y).all() for x, y in zip(a["ids"], b["ids"]))
    # and the heads of one group do differ from each other (a wrong head index would hide behind symmetry)
    a = oracle.sparse_attn(q, K, V, oracle.TOPK, k=9)
    assert not np.allclose(a["out"][0], a["out"][1])
    assert not np.allclose(a["out"][0], a["out"][G])


# ---------------------------------------------------------------- P11: shift and scale
def test_shift_and_scale_invariance():
    """Def. 2 and softmax: adding c to every key shifts all scores by q.c; scaling q scales beta."""
    w, q, K, V = _small(23, n=160, hq=2, hk=1, d=8)
    # use exactly representable numbers so the shift itself adds no rounding
    q = np.round(q * 8) / 8
    K = np.round(K * 8) / 8
    c = (np.arange(8, dtype=np.float32) - 3.0) / 4.0
    Ks = (K + c).astype(np.float32)
    for mode, kw in [(oracle.TOPK, dict(k=11)), (oracle.DIPR, dict(beta=1.25))]:
        a = oracle.sparse_attn(q.astype(np.float32), K.astype(np.float32), V, mode, **kw)
        b = oracle.sparse_attn(q.astype(np.float32), Ks, V, mode, **kw)
        assert all((x == y).all() for x, y in zip(a["ids"], b["ids"]))
        np.testing.assert_allclose(a["out"], b["out"], rtol=0, atol=1e-12)
    a = oracle.sparse_attn(q.astype(np.float32), K.astype(np.float32), V, oracle.DIPR, beta=1.25)
    b = oracle.sparse_attn((2 * q).astype(np.float32), K.astype(np.float32), V, oracle.DIPR, beta=2.5)
    assert all((x == y).all() for x, y in zip(a["ids"], b["ids"]))
    a = oracle.sparse_attn(q.astype(np.float32), K.astype(np.float32), V, oracle.TOPK, k=11)
    b = oracle.sparse_attn((2 * q).astype(np.float32), K.astype(np.float32), V, oracle.TOPK, k=11)
    assert all((x == y).all() for x, y in zip(a["ids"], b["ids"]))


# ---------------------------------------------------------------- P12: convex hull
def test_output_in_hull_of_selected_values():
    w, q, K, V = _small(29, n=130)
    r = oracle.sparse_attn(q, K, V, oracle.TOPK, k=13)
    Vf = V.astype(np.float64)
    for h in range(w.n_q_heads):
        rows = Vf[r["ids"][h], h // w.group]
        assert (r["out"][h] >= rows.min(axis=0) - 1e-12).all() and (r["out"][h] <= rows.max(axis=0) + 1e-12).all()


# ---------------------------------------------------------------- argument handling
def test_invalid_arguments():
    w, q, K, V = _small(0, n=10)
    with pytest.raises(ValueError):
        oracle.sparse_attn(q, K, V, oracle.TOPK, k=0)
    with pytest.raises(ValueError):
        oracle.sparse_attn(q, K, V, oracle.DIPR, beta=-1.0)
    with pytest.raises(ValueError):
        oracle.sparse_attn(q, K, V, oracle.DIPR, beta=float("nan"))


def test_bf16_widening_is_exact():
    """bf16 bits are widened exactly: a score of bf16 inputs equals the fp64 sum of exact products."""
    rng = np.random.default_rng(3)
    x = rng.standard_normal((7, 1, 16)).astype(np.float32)
    kb = wl.to_bf16_bits(x)
    qb = wl.to_bf16_bits(rng.standard_normal(16).astype(np.float32))
    kf, qf = wl.bf16_bits_to_f32(kb).astype(np.float64), wl.bf16_bits_to_f32(qb).astype(np.float64)
    np.testing.assert_allclose(oracle.scores(qb, kb, 0), kf[:, 0, :] @ qf, rtol=0, atol=1e-14)
    # round-to-nearest-even of the generator: 1 + 2^-8 is a tie and goes to the even mantissa (1.0)
    assert wl.to_bf16_bits(np.array([1.0 + 2.0 ** -8], dtype=np.float32))[0] == 0x3F80
    assert wl.to_bf16_bits(np.array([1.0 + 3 * 2.0 ** -8], dtype=np.float32))[0] == 0x3F82


# ---------------------------------------------------------------- window and prefix (Sec. 7.1)
def _merge_two(parts):
    """Partial-attention merge (Sec. 7.2) of (m, l, o) triples computed from library routines."""
    M = max(m for m, _, _ in parts)
    num = sum(math.exp(m - M) * l * o for m, l, o in parts)
    den = sum(math.exp(m - M) * l for m, l, _ in parts)
    return num / den


def _dense_part(s_h, V_g, ids, d):
    """(max, sum of exponentials, normalised output) of one token set, numpy only."""
    z = s_h[ids] / math.sqrt(d)
    m = z.max()
    e = np.exp(z - m)
    return m, e.sum(), (e[:, None] * V_g[ids]).sum(axis=0) / e.sum()


def test_window_closed_form_weights():
    """Five tokens with softmax weights 1, 2, 4, 8, 16 (d = 4, q.k_j = 2 ln w_j).  Window = first 1 + last 1
    (weights 1 and 16) is always attended; top-1 retrieves the best of the OTHERS (weight 8), so the
    attended set is {0, 3, 4} with weights 1 : 8 : 16 (Table 3's "[initial + last] + retrieved")."""
    w = np.array([1.0, 2.0, 4.0, 8.0, 16.0])
    q = np.array([[1.0, 0.0, 0.0, 0.0]], dtype=np.float32)
    K = np.zeros((5, 1, 4), dtype=np.float32)
    K[:, 0, 0] = 2.0 * np.log(w)
    V = np.arange(20, dtype=np.float32).reshape(5, 1, 4) - 7.0
    r = oracle.sparse_attn(q, K, V, oracle.TOPK, k=1, window=(1, 1))
    assert list(r["ids"][0]) == [0, 3, 4]
    np.testing.assert_allclose(r["out"][0], (1 * V[0, 0] + 8 * V[3, 0] + 16 * V[4, 0]) / 25.0, rtol=0, atol=1e-5)
    # DIPR: the maximum is the window's last token (score 2 ln 16 = 5.545); beta = 1.5 reaches weight 8
    # (score 4.159) but not weight 4 (2.773): the threshold uses the maximum over window AND the rest
    r = oracle.sparse_attn(q, K, V, oracle.DIPR, beta=1.5, window=(1, 1))
    assert list(r["ids"][0]) == [0, 3, 4]
    # without the window's maximum the same beta would have kept weight 4 as well: max of the others is 4.159
    r = oracle.sparse_attn(q, K[:4], V[:4], oracle.DIPR, beta=1.5)
    assert list(r["ids"][0]) == [2, 3]
    # a window that covers everything is full attention (Eq. 1)
    r = oracle.sparse_attn(q, K, V, oracle.TOPK, k=1, window=(3, 2))
    np.testing.assert_allclose(r["out"][0], (w[:, None] * V[:, 0]).sum(axis=0) / w.sum(), rtol=0, atol=1e-5)
    r = oracle.sparse_attn(q, K, V, oracle.DIPR, beta=0.0, window=(9, 9))
    assert list(r["ids"][0]) == [0, 1, 2, 3, 4]


@pytest.mark.parametrize("seed,w0,w1,k", [(0, 5, 7, 6), (1, 0, 9, 3), (2, 11, 0, 200), (3, 1, 1, 1)])
def test_window_topk_is_window_plus_topk_of_the_rest(seed, w0, w1, k):
    """The retrieved tokens are the windowless top-k of the cache with the window rows removed, and the
    output is the merge (Sec. 7.2) of the window's attention and the retrieved tokens' attention."""
    w, q, K, V = _small(seed)
    n, d, G = K.shape[0], K.shape[2], w.n_q_heads // w.n_kv_heads
    s, _, _ = _dense(q, K, V, "f32")
    win = np.r_[np.arange(w0), np.arange(n - w1, n)]
    rest = np.arange(w0, n - w1)
    r = oracle.sparse_attn(q, K, V, oracle.TOPK, k=k, window=(w0, w1))
    sub = oracle.sparse_attn(q, K[rest], V[rest], oracle.TOPK, k=k)          # windowless, already pinned
    for h in range(w.n_q_heads):
        retrieved = rest[sub["ids"][h]]
        assert list(r["ids"][h]) == sorted(np.r_[win, retrieved])
        assert r["counts"][h] == len(win) + min(k, len(rest))
        Vg = V[:, h // G].astype(np.float64)
        parts = [_dense_part(s[h], Vg, ids, d) for ids in (win, retrieved) if len(ids)]
        np.testing.assert_allclose(r["out"][h], _merge_two(parts), rtol=0, atol=1e-12)


@pytest.mark.parametrize("seed,w0,w1,beta", [(0, 4, 4, 0.0), (1, 8, 16, 1.0), (2, 0, 3, 2.5), (3, 30, 0, 0.7)])
def test_window_dipr_is_windowless_dipr_united_with_the_window(seed, w0, w1, beta):
    """DIPR's threshold hangs on the maximum over ALL tokens (Sec. 7.1: the window's maximum is taken
    into consideration), so the result is the windowless DIPR set united with the window."""
    w, q, K, V = _small(seed)
    n, d, G = K.shape[0], K.shape[2], w.n_q_heads // w.n_kv_heads
    s, _, _ = _dense(q, K, V, "f32")
    win = np.r_[np.arange(w0), np.arange(n - w1, n)].astype(np.int64)
    r = oracle.sparse_attn(q, K, V, oracle.DIPR, beta=beta, window=(w0, w1))
    plain = oracle.sparse_attn(q, K, V, oracle.DIPR, beta=beta)               # windowless, already pinned
    for h in range(w.n_q_heads):
        want = np.union1d(win, plain["ids"][h])
        assert list(r["ids"][h]) == list(want)
        m, l, o = _dense_part(s[h], V[:, h // G].astype(np.float64), want, d)
        np.testing.assert_allclose(r["out"][h], o, rtol=0, atol=1e-12)


def test_window_select_function_alone_and_its_errors():
    s = np.array([0.5, 3.0, 1.0, 2.0, 2.0, 0.0, 9.0])
    assert list(oracle.select_window(s, 1, 1, oracle.TOPK, k=2)) == [0, 1, 3, 6]        # tie 2.0 / 2.0: smaller id
    assert list(oracle.select_window(s, 1, 1, oracle.TOPK, k=99)) == [0, 1, 2, 3, 4, 5, 6]
    assert list(oracle.select_window(s, 0, 0, oracle.TOPK, k=2)) == [1, 6]              # no window: plain top-k
    assert list(oracle.select_window(s, 2, 0, oracle.DIPR, beta=7.0)) == [0, 1, 3, 4, 6]  # 9 - 7 = 2, inclusive
    assert list(oracle.select_window(s, 0, 1, oracle.DIPR, beta=0.0)) == [6]
    with pytest.raises(ValueError):
        oracle.select_window(s, -1, 0, oracle.TOPK, k=1)
    with pytest.raises(ValueError):
        oracle.select_window(s, 0, 0, oracle.TOPK, k=0)
    with pytest.raises(ValueError):
        oracle.select_window(s, 0, 0, oracle.DIPR, beta=-1.0)


@pytest.mark.parametrize("mode,kw", [(oracle.TOPK, dict(k=7)), (oracle.DIPR, dict(beta=1.5)),
                                     (oracle.TOPK, dict(k=7, window=(3, 5)))])
def test_prefix_sees_nothing_behind_it(mode, kw):
    """Flexible context reuse (Sec. 7.1): a query on the first m tokens is the query on a cache that
    holds only those tokens, whatever lies behind them; 'last' window tokens are the prefix's last."""
    w, q, K, V = _small(5)
    m = 41
    ref = oracle.sparse_attn(q, K[:m].copy(), V[:m].copy(), mode, **kw)
    K2, V2 = K.copy(), V.copy()
    K2[m:], V2[m:] = np.nan, np.nan                                            # poison what must not be read
    r = oracle.sparse_attn(q, K2, V2, mode, n_visible=m, **kw)
    assert all(list(a) == list(b) for a, b in zip(r["ids"], ref["ids"]))
    assert np.array_equal(r["out"], ref["out"]) and np.isfinite(r["out"]).all()
    full = oracle.sparse_attn(q, K, V, mode, n_visible=K.shape[0], **kw)
    plain = oracle.sparse_attn(q, K, V, mode, **kw)
    assert np.array_equal(full["out"], plain["out"])
    with pytest.raises(ValueError):
        oracle.sparse_attn(q, K, V, mode, n_visible=0, **kw)


# ---------------------------------------------------------------- coarse-grained index (Sec. 6.2, Table 4)
def test_coarse_index_by_hand():
    """Sec. 6.2, coarse-grained index: blocks of adjacent tokens, two representative vectors (channel-wise
    min and max), block score = sum_c max(q_c lo_c, q_c hi_c), best blocks first, then top-k inside them.
    d = 2, q = (1, -2), three blocks of two tokens; every number below is worked out by hand:
      block 0: keys (1,1), (3,0)   lo (1,0)  hi (3,1)  u = max(1,3) + max(0,-2)  = 3    scores -1, 3
      block 1: keys (0,-1), (2,2)  lo (0,-1) hi (2,2)  u = max(0,2) + max(2,-4)  = 4    scores  2, -2
      block 2: keys (-1,0), (-2,1) lo (-2,0) hi (-1,1) u = max(-2,-1) + max(0,-2) = -1  scores -1, -4
    The best single block is block 1 although the best token (score 3) sits in block 0: with one block the
    query answers token 2, with two blocks token 1."""
    q = np.array([[1.0, -2.0]], dtype=np.float32)
    K = np.array([[1, 1], [3, 0], [0, -1], [2, 2], [-1, 0], [-2, 1]], dtype=np.float32).reshape(6, 1, 2)
    V = np.arange(12, dtype=np.float32).reshape(6, 1, 2)
    lo, hi = oracle.block_reps(K, 0, 2)
    assert lo.tolist() == [[1, 0], [0, -1], [-2, 0]] and hi.tolist() == [[3, 1], [2, 2], [-1, 1]]
    assert oracle.block_scores(q[0], lo, hi).tolist() == [3.0, 4.0, -1.0]
    r1 = oracle.coarse_attn(q, K, V, block=2, n_blocks=1, k=1)
    assert r1["blocks"][0].tolist() == [1] and r1["ids"][0].tolist() == [2]
    np.testing.assert_allclose(r1["out"][0], V[2, 0])
    r2 = oracle.coarse_attn(q, K, V, block=2, n_blocks=2, k=1)
    assert r2["blocks"][0].tolist() == [0, 1] and r2["ids"][0].tolist() == [1]
    # k larger than the blocks hold: every token of the chosen blocks (the paper's description read literally)
    r3 = oracle.coarse_attn(q, K, V, block=2, n_blocks=2, k=100)
    assert r3["ids"][0].tolist() == [0, 1, 2, 3]
    # weights exp(s / sqrt(2)) over scores -1, 3, 2, -2
    wgt = np.exp(np.array([-1.0, 3.0, 2.0, -2.0]) / math.sqrt(2.0))
    np.testing.assert_allclose(r3["out"][0], (wgt[:, None] * V[:4, 0]).sum(0) / wgt.sum(), rtol=1e-12)
    # window tokens are attended whatever block they are in; top-k counts the others
    r4 = oracle.coarse_attn(q, K, V, block=2, n_blocks=1, k=1, window=(1, 1))
    assert r4["ids"][0].tolist() == [0, 2, 5]
    # equal block scores: the smaller block wins (block 2 made a copy of block 1)
    K2 = K.copy(); K2[4:6] = K[2:4]
    assert oracle.coarse_attn(q, K2, V, block=2, n_blocks=1, k=1)["blocks"][0].tolist() == [1]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_coarse_representatives_and_bound_against_library_routines(dtype):
    """The representatives are plain minima and maxima (numpy's), and the block score is an upper bound of
    every inner product of the block - the property that makes min/max vectors a usable representative -
    reached exactly by blocks of one token."""
    w, q, K, V = _small(21, n=203, hq=4, hk=2, d=16, dtype=dtype)
    Kf, qf = _f64(K, dtype), _f64(q, dtype)
    for block in (1, 7, 64):
        nb = -(-203 // block)
        for g in range(2):
            lo, hi = oracle.block_reps(K, g, block)
            pad = np.full((nb * block - 203, 16), np.nan)
            kb = np.concatenate([Kf[:, g], pad]).reshape(nb, block, 16)
            np.testing.assert_array_equal(lo, np.nanmin(kb, axis=1))
            np.testing.assert_array_equal(hi, np.nanmax(kb, axis=1))
            for h in (2 * g, 2 * g + 1):
                u = oracle.block_scores(q[h], lo, hi)
                s = Kf[:, g] @ qf[h]
                smax = np.array([s[b * block:(b + 1) * block].max() for b in range(nb)])
                assert (u >= smax - 1e-12).all()
                if block == 1:
                    np.testing.assert_allclose(u, s, rtol=0, atol=1e-12)


def test_coarse_query_reduces_to_the_exact_one():
    """All blocks chosen = the exact top-k query; blocks of one token with P = k too; and so does any P that
    takes every block whose bound reaches the exact k-th score (no token that belongs to the answer can lie
    in a block whose upper bound is below it).  Chosen blocks are nested in P."""
    w, q, K, V = _small(22, n=500, hq=4, hk=2, d=16, dtype="bf16")
    exact = oracle.sparse_attn(q, K, V, oracle.TOPK, k=20, want_scores=True, window=(3, 5))
    nb = -(-500 // 16)
    allb = oracle.coarse_attn(q, K, V, block=16, n_blocks=nb, k=20, window=(3, 5))
    for h in range(4):
        assert allb["ids"][h].tolist() == exact["ids"][h].tolist()
        np.testing.assert_allclose(allb["out"][h], exact["out"][h], rtol=0, atol=1e-12)
    one = oracle.coarse_attn(q, K, V, block=1, n_blocks=20, k=20)
    ex0 = oracle.sparse_attn(q, K, V, oracle.TOPK, k=20)
    prev = [set() for _ in range(4)]
    for P in (1, 2, 5, 11, nb):
        r = oracle.coarse_attn(q, K, V, block=16, n_blocks=P, k=20)
        for h in range(4):
            assert one["ids"][h].tolist() == ex0["ids"][h].tolist()
            assert len(r["blocks"][h]) == min(P, nb) and prev[h] <= set(r["blocks"][h].tolist())
            prev[h] = set(r["blocks"][h].tolist())
    for h in range(4):
        s = exact["scores"][h]
        kth = np.sort(s)[-20]
        u = allb["u"][h]
        P = int((u >= kth).sum())
        r = oracle.coarse_attn(q, K, V, block=16, n_blocks=P, k=20)
        assert r["ids"][h].tolist() == ex0["ids"][h].tolist()


def test_coarse_prefix_uses_the_stored_index():
    """Sec. 7.1 flexible context reuse on the coarse index: the query sees a prefix through the index of the
    stored context, so the half-visible block keeps the representatives of all its stored tokens; whole
    blocks behind the prefix take no part, and hidden tokens are never returned."""
    w, q, K, V = _small(23, n=160, hq=2, hk=1, d=16, dtype="f32")
    Kp = K.copy()
    Kp[100:112] *= 50.0            # hidden tokens of the half-visible block 6 (tokens 96..111; 100 are visible)
    r = oracle.coarse_attn(q, Kp, V, block=16, n_blocks=3, k=8, n_visible=100)
    lo, hi = oracle.block_reps(Kp, 0, 16)
    for h in range(2):
        assert r["u"][h].shape == (7,)                                        # blocks 0..6 only
        np.testing.assert_array_equal(r["u"][h], oracle.block_scores(q[h], lo, hi)[:7])
        assert 6 in r["blocks"][h]                                            # its (hidden) outliers raise the bound
        assert r["ids"][h].max() < 100
        np.testing.assert_array_equal(r["ids"][h], oracle.select_topk_in_blocks(
            oracle.scores(q[h], Kp[:100], 0), 16, r["blocks"][h], 8))
    with pytest.raises(ValueError):
        oracle.coarse_attn(q, K, V, block=16, n_blocks=0, k=8)


# ---------------------------------------------------------------- DIPRS (Sec. 6.1.3, Algorithm 1)
_G7 = np.array([[1, 2], [3, 4], [5, 4], [6, 0], [6, 5], [3, 6], [0, 1]], dtype=np.int32)   # neighbours of nodes 0..6


def test_diprs_by_hand_three_cases_of_try_append():
    """Algorithm 1 walked by hand on a 7-node graph (neighbour lists above), start key 0, beta = 1.
    Scores 5, 1, 9, 8.5, 3, 8.9, 0.
    l0 = 1: node 1 is appended although it is not critical (|C| <= l0, case a of the paper's figure); node 2
    (9 >= 5 - 1) is appended by the threshold (case c) and raises the best to 9; node 3 (8.5 >= 8) and
    node 5 (8.9 >= 8) follow; nodes 4 (3) and 6 (0) are pruned (case b).  C = 0, 1, 2, 3, 5; answer 2, 3, 5.
    l0 = 0: node 1 is pruned at once; C grows 0, 2, 5, 3; the same answer."""
    s = np.array([5.0, 1.0, 9.0, 8.5, 3.0, 8.9, 0.0], dtype=np.float32)
    ids, C = oracle.diprs(_G7, s, 0, 1, 1.0)
    assert C.tolist() == [0, 1, 2, 3, 5] and ids.tolist() == [2, 3, 5]
    ids, C = oracle.diprs(_G7, s, 0, 0, 1.0)
    assert C.tolist() == [0, 2, 5, 3] and ids.tolist() == [2, 3, 5]
    # the threshold moves with the best so far: node 2 at 5.2 enters under the early threshold (4.5) and is
    # dropped from the answer once 8.9 has been found; beta = 0.5
    s2 = s.copy(); s2[2] = 5.2
    ids, C = oracle.diprs(_G7, s2, 0, 0, 0.5)
    assert C.tolist() == [0, 2, 5, 3] and ids.tolist() == [3, 5]
    # inclusive comparison: a neighbour exactly beta below the best is appended and answered
    s3 = np.array([5.0, 4.0, 4.0, 0.0, 0.0, 0.0, 0.0], dtype=np.float32)
    ids, C = oracle.diprs(_G7, s3, 0, 0, 1.0)
    assert C.tolist() == [0, 1, 2] and ids.tolist() == [0, 1, 2]


def test_diprs_is_approximate_and_l0_buys_exploration():
    """The best key (node 3, score 9) hangs behind node 1 (score 1).  With l0 = 0 node 1 is pruned and the
    walk ends at once: the answer is the start key, not the true range.  With l0 = 1 node 1 is kept, node 3 is
    reached, and the answer is the exact DIPR set {3}: principle (i) of Sec. 6.1.3."""
    s = np.array([5.0, 1.0, 2.0, 9.0, 3.0, 0.5, 0.0], dtype=np.float32)
    ids, C = oracle.diprs(_G7, s, 0, 0, 1.0)
    assert C.tolist() == [0] and ids.tolist() == [0]
    ids, C = oracle.diprs(_G7, s, 0, 1, 1.0)
    assert C.tolist() == [0, 1, 3] and ids.tolist() == [3]
    assert oracle.select_dipr(s, 1.0).tolist() == [3]


def test_diprs_window_seeds_the_best_and_is_always_answered():
    """Sec. 7.1: the best so far also counts the cached window.  Token 6 (last one) scores 9.5: from the start
    the threshold is 8.5, so node 2 (9) is appended, node 1 (1) is not - even with l0 = 0 the walk goes straight
    for the critical tokens - and the answer holds the window whatever it scores."""
    s = np.array([5.0, 1.0, 9.0, 8.5, 3.0, 8.9, 9.5], dtype=np.float32)
    ids, C = oracle.diprs(_G7, s, 0, 0, 1.0, window=(0, 1))
    assert C.tolist() == [0, 2, 5, 3] and ids.tolist() == [2, 3, 5, 6]
    s[6] = -4.0
    ids, C = oracle.diprs(_G7, s, 0, 0, 1.0, window=(0, 1))
    assert ids.tolist() == [2, 3, 5, 6]
    # with node 2 at 6.0 the seeded threshold (9.5 - 1) prunes it and the walk never leaves the start key, whose
    # own 5.0 is not within beta of the window's 9.5; unseeded, 6.0 >= 5 - 1 would have been appended
    s2 = np.array([5.0, 1.0, 6.0, 8.5, 3.0, 8.9, 9.5], dtype=np.float32)
    ids, C = oracle.diprs(_G7, s2, 0, 0, 1.0, window=(0, 1))
    assert C.tolist() == [0] and ids.tolist() == [6]
    with pytest.raises(ValueError):
        oracle.diprs(_G7, s, 6, 0, 1.0, window=(0, 1))      # the start key may not be a window token


def test_diprs_on_a_complete_graph_is_the_exact_range_query():
    """If every key neighbours every other and l0 >= n nothing is ever pruned before it is scored: C holds
    every key and the answer is Def. 2's set; and the nearest-neighbour graph itself against a library sort."""
    w, q, K, V = _small(31, n=60, hq=2, hk=1, d=16, dtype="bf16")
    full = oracle.knn_graph(K, 0, 59)
    Kf = _f64(K, "bf16")[:, 0]
    sim = Kf @ Kf.T
    for j in range(60):
        order = sorted((i for i in range(60) if i != j), key=lambda i: (-sim[i, j], i))
        assert full[j].tolist() == order
    assert (oracle.knn_graph(K, 0, 5) == full[:, :5]).all()
    assert (oracle.knn_graph(K[:4], 0, 5)[:, 3:] == -1).all()
    for h in range(2):
        s32 = oracle.scores_f32(q[h], K, 0)
        np.testing.assert_allclose(s32, oracle.scores(q[h], K, 0), rtol=0, atol=2e-5)
        for beta in (0.0, 0.7, 3.0):
            ids, C = oracle.diprs(full, s32, 7, 60, beta)
            assert sorted(C.tolist()) == list(range(60))
            assert ids.tolist() == oracle.select_dipr(s32.astype(np.float64), beta).tolist()
    # the fp32 score is a chain of fused multiply-adds in channel order: on small integers it is exact
    qi = np.arange(1, 17, dtype=np.float32)
    Ki = (np.arange(32, dtype=np.float32).reshape(2, 1, 16) % 7) - 3
    assert oracle.scores_f32(qi, Ki, 0).tolist() == (Ki[:, 0] @ qi).tolist()


def test_diprs_invariants_on_a_sparse_graph():
    """On a 6-nearest-neighbour graph: C starts with the start key, holds no key twice, every entry but the
    first is a neighbour of an earlier entry, the answer is exactly the part of C within beta of C's best,
    and a larger l0 never returns fewer keys of the exact range set when it finds the same best."""
    w, q, K, V = _small(32, n=400, hq=2, hk=1, d=16, dtype="bf16")
    nbr = oracle.knn_graph(K, 0, 6)
    norms = (_f64(K, "bf16")[:, 0] ** 2).sum(1)
    k0 = int(norms.argmax())
    for h in range(2):
        s = oracle.scores_f32(q[h], K, 0)
        exact = set(oracle.select_dipr(s.astype(np.float64), 2.0).tolist())
        for l0 in (0, 8, 64, 400):
            ids, C = oracle.diprs(nbr, s, k0, l0, 2.0)
            assert C[0] == k0 and len(set(C.tolist())) == len(C)
            pos = {int(c): i for i, c in enumerate(C)}
            for i, c in enumerate(C[1:], 1):
                assert any(int(c) in nbr[int(p)] for p in C[:i])
            best = s[C].max()
            assert ids.tolist() == sorted(int(c) for c in C if s[c] >= best - np.float32(2.0))
            if best == s.max():
                assert set(ids.tolist()) <= exact


def test_plan_follows_the_optimizer_workflow():
    """Sec. 6.2 "Query Optimizer": the outcomes the text states, one per branch of the workflow."""
    GB = 1 << 30
    assert oracle.plan(2000, 4096, 0, 80 * GB, 10 * GB, 3) == ("full", "none", 2000)          # short: full attention
    assert oracle.plan(2000, 4096, 500, 0, 10 * GB, 0) == ("full", "none", 2000)              # ... whatever else holds
    assert oracle.plan(200000, 4096, 0, 80 * GB, 10 * GB, 3) == ("topk", "coarse", 200000)    # budget is enough
    assert oracle.plan(200000, 4096, 0, 10 * GB, 10 * GB, 0) == ("topk", "coarse", 200000)
    assert oracle.plan(200000, 4096, 0, 4 * GB, 10 * GB, 0) == ("dipr", "flat", 200000)       # limited: first layer scans
    assert oracle.plan(200000, 4096, 0, 4 * GB, 10 * GB, 1) == ("dipr", "fine", 200000)       # ... the others walk the graph
    assert oracle.plan(200000, 4096, 0, 4 * GB, 10 * GB, 31) == ("dipr", "fine", 200000)
    assert oracle.plan(200000, 4096, 150000, 4 * GB, 10 * GB, 7) == ("dipr", "fine", 150000)  # partial reuse: filter
    assert oracle.plan(200000, 4096, 150000, 40 * GB, 10 * GB, 7) == ("topk", "coarse", 150000)
    assert oracle.plan(200000, 4096, 200000, 4 * GB, 10 * GB, 7)[2] == 200000                 # whole context reused: no filter
