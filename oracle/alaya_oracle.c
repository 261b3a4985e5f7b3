/*
 * CPU oracle for the decode-step sparse-attention query.
 *
 * TEST INFRASTRUCTURE ONLY.  Plain, slow, and written from the paper's
 * definitions; it shares no code with the HIP library and must never be
 * called from the product path.  Only the tests, the smoke check and the
 * bench's cpu_baseline leg may load it.
 *
 * What it computes, per query head h (KV head g = h / G), over n cached tokens:
 *   scores   s_j = q_h . k_{g,j}                      raw inner product (Eq. 1 numerator; Def. 2)
 *   top-k    the min(k, n) tokens with the largest s_j (Sec. 6.1.1); equal scores: smaller j first
 *   DIPR     every j with s_j >= max_s s_s - beta, beta >= 0, inclusive (Def. 2, Def. 3)
 *   attend   z_j = s_j * scale (scale = 1/sqrt(d)); a = softmax over the SELECTED set only;
 *            o = sum_j a_j v_{g,j}                    (Eq. 1 restricted to the critical tokens,
 *                                                      Sec. 2 "Sparse Attention")
 *   full     the same with every token selected       (Eq. 1)
 *   window   (Sec. 7.1 "Window Caching Enhanced DIPR"; Table 3 counts "[initial + last] + retrieved"
 *            tokens) the first w0 and the last w1 tokens are always attended; top-k retrieves its k
 *            tokens among the others; DIPR keeps the others that are within beta of the maximum over
 *            ALL tokens, the window's included
 *   prefix   (Sec. 7.1 "Flexible Context Reuse") only the first n_visible tokens exist for the query:
 *            the caller hands over that prefix of K and V, nothing else changes
 *   coarse   (Sec. 6.2 "Query Optimizer", coarse-grained index; Table 4: top-k and filter queries) adjacent
 *            tokens form blocks, each block is represented by two vectors - the channel-wise minimum lo and
 *            maximum hi of its keys - and scored by u_b = sum_c max(q_c lo_bc, q_c hi_bc), which no q.k of
 *            the block exceeds; the P blocks with the largest u_b (equal u: smaller block first) are the
 *            critical blocks, and the top-k query runs over their tokens only (window tokens are still
 *            always attended).  The paper fixes neither the block size, nor the representatives, nor P:
 *            they are parameters here.
 *
 *   DIPRS    (Sec. 6.1.3 "DIPR Query Processing", Algorithm 1) the approximate DIPR query on a graph index: a
 *            list C starts with the start key; its entries are visited in order, and every unvisited
 *            neighbour k of the visited entry is appended if C holds at most l0 entries or q.k is within beta
 *            of the best inner product in C so far; the answer is every c in C within beta of the best of C.
 *            With a window (Sec. 7.1 "Window Caching Enhanced DIPR") the best so far also counts the window's
 *            tokens, which are always attended and take no part in the walk.  The graph here is the exact
 *            M-nearest-neighbour graph of the keys under the inner product (the paper builds RoarGraph; any
 *            graph index serves Algorithm 1).  Which neighbours are appended depends on comparisons of
 *            scores, so DIPRS - alone in this file - takes its scores in the GPU kernel's arithmetic: fp32,
 *            one fused multiply-add per channel in channel order (oracle_scores_f32).
 *
 * All other arithmetic is fp64.  Inputs are the stored bytes (bf16 or fp32), widened
 * exactly.  K and V are token-major: element (j, g, c) sits at (j*n_kv_heads + g)*d + c.
 *
 * Every function here is pinned by tests/test_oracle_pins.py against facts that
 * do not depend on this file (a dense library softmax, Theorem 1's alpha form,
 * brute force, invariances, a hand-derived closed form).
 */
#define _GNU_SOURCE /* qsort_r */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_BF16 = 0, ORACLE_F32 = 1 };
enum { ORACLE_TOPK = 0, ORACLE_DIPR = 1, ORACLE_FULL = 2 };

static double widen(const void *base, int dtype, int64_t idx)
{
    if (dtype == ORACLE_F32)
        return (double)((const float *)base)[idx];
    uint32_t bits = (uint32_t)((const uint16_t *)base)[idx] << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

/* s_j = sum_c q[c] * K[j][g][c]  for j < n.  q points at this head's d elements. */
void oracle_scores(const void *q, const void *K, int dtype, int64_t n,
                   int n_kv_heads, int g, int d, double *s)
{
    for (int64_t j = 0; j < n; ++j) {
        double acc = 0.0;
        int64_t row = (j * n_kv_heads + g) * (int64_t)d;
        for (int c = 0; c < d; ++c)
            acc += widen(q, dtype, c) * widen(K, dtype, row + c);
        s[j] = acc;
    }
}

static int by_score_desc_then_id(const void *a, const void *b, void *ctx)
{
    const double *s = (const double *)ctx;
    int32_t ia = *(const int32_t *)a, ib = *(const int32_t *)b;
    if (s[ia] > s[ib]) return -1;
    if (s[ia] < s[ib]) return 1;
    return (ia > ib) - (ia < ib);
}

static int by_id(const void *a, const void *b)
{
    int32_t ia = *(const int32_t *)a, ib = *(const int32_t *)b;
    return (ia > ib) - (ia < ib);
}

/* Top-k query: rank every token by score, keep the first min(k, n); ids come
 * back ascending.  Returns the count, or -1 if k <= 0. */
int64_t oracle_select_topk(const double *s, int64_t n, int64_t k, int32_t *ids)
{
    if (k <= 0) return -1;
    if (n <= 0) return 0;
    int64_t kk = k < n ? k : n;
    int32_t *order = (int32_t *)malloc((size_t)n * sizeof *order);
    for (int64_t j = 0; j < n; ++j) order[j] = (int32_t)j;
    qsort_r(order, (size_t)n, sizeof *order, by_score_desc_then_id, (void *)s);
    memcpy(ids, order, (size_t)kk * sizeof *ids);
    free(order);
    qsort(ids, (size_t)kk, sizeof *ids, by_id);
    return kk;
}

/* DIPR(q, beta): all tokens whose inner product is within beta of the maximum.
 * ids ascending.  Returns the count (>= 1 for n >= 1), or -1 if beta < 0 or NaN. */
int64_t oracle_select_dipr(const double *s, int64_t n, double beta, int32_t *ids)
{
    if (!(beta >= 0.0)) return -1;
    if (n <= 0) return 0;
    double m = s[0];
    for (int64_t j = 1; j < n; ++j)
        if (s[j] > m) m = s[j];
    int64_t cnt = 0;
    for (int64_t j = 0; j < n; ++j)
        if (s[j] >= m - beta) ids[cnt++] = (int32_t)j;
    return cnt;
}

/* Query with a window of always-attended tokens W = {j < w0} U {j >= n - w1}.
 *   top-k: W plus the min(k, n - |W|) best tokens outside W (equal scores: smaller j first);
 *   DIPR : W plus every token outside W with s_j >= max over all n tokens - beta.
 * ids ascending.  Returns the count, or -1 on an invalid k / beta / window. */
int64_t oracle_select_window(const double *s, int64_t n, int64_t w0, int64_t w1, int mode, int64_t k,
                             double beta, int32_t *ids)
{
    if (w0 < 0 || w1 < 0) return -1;
    if (mode == ORACLE_TOPK && k <= 0) return -1;
    if (mode == ORACLE_DIPR && !(beta >= 0.0)) return -1;
    if (n <= 0) return 0;
    char *inwin = (char *)malloc((size_t)n);
    int64_t n_out = 0;
    for (int64_t j = 0; j < n; ++j) {
        inwin[j] = (j < w0 || j >= n - w1) ? 1 : 0;
        n_out += !inwin[j];
    }
    char *take = (char *)calloc((size_t)n, 1);
    if (mode == ORACLE_TOPK) {
        int32_t *order = (int32_t *)malloc((size_t)(n_out > 0 ? n_out : 1) * sizeof *order);
        int64_t m = 0;
        for (int64_t j = 0; j < n; ++j)
            if (!inwin[j]) order[m++] = (int32_t)j;
        qsort_r(order, (size_t)n_out, sizeof *order, by_score_desc_then_id, (void *)s);
        int64_t kk = k < n_out ? k : n_out;
        for (int64_t i = 0; i < kk; ++i) take[order[i]] = 1;
        free(order);
    } else {
        double m = s[0];
        for (int64_t j = 1; j < n; ++j)
            if (s[j] > m) m = s[j];
        for (int64_t j = 0; j < n; ++j)
            if (!inwin[j] && s[j] >= m - beta) take[j] = 1;
    }
    int64_t cnt = 0;
    for (int64_t j = 0; j < n; ++j)
        if (inwin[j] || take[j]) ids[cnt++] = (int32_t)j;
    free(take);
    free(inwin);
    return cnt;
}

/* Coarse index, step 1: representatives of block b = tokens [b*block, min(n, (b+1)*block)) of KV head g:
 * lo[b][c] = min_j K[j][g][c], hi[b][c] = max_j K[j][g][c].  lo, hi: [ceil(n/block)][d]. */
void oracle_block_reps(const void *K, int dtype, int64_t n, int n_kv_heads, int g, int d, int64_t block,
                       double *lo, double *hi)
{
    for (int64_t b = 0; b * block < n; ++b) {
        for (int c = 0; c < d; ++c) {
            double mn = 0.0, mx = 0.0;
            for (int64_t j = b * block; j < n && j < (b + 1) * block; ++j) {
                double x = widen(K, dtype, (j * n_kv_heads + g) * (int64_t)d + c);
                if (j == b * block || x < mn) mn = x;
                if (j == b * block || x > mx) mx = x;
            }
            lo[b * d + c] = mn;
            hi[b * d + c] = mx;
        }
    }
}

/* Coarse index, step 2: u_b = sum_c max(q_c * lo[b][c], q_c * hi[b][c]) for nb blocks. */
void oracle_block_scores(const void *q, int dtype, const double *lo, const double *hi, int64_t nb, int d, double *u)
{
    for (int64_t b = 0; b < nb; ++b) {
        double acc = 0.0;
        for (int c = 0; c < d; ++c) {
            double qc = widen(q, dtype, c);
            double a = qc * lo[b * d + c], z = qc * hi[b * d + c];
            acc += a > z ? a : z;
        }
        u[b] = acc;
    }
}

/* Coarse index, step 3 is oracle_select_topk(u, nb, P, blocks): the P best blocks, smaller block first among
 * equal scores.  Step 4: the top-k query over the tokens of the given blocks (ascending block numbers):
 * the window W = {j < w0} U {j >= n - w1} plus the min(k, candidates) best tokens outside W that lie in one
 * of the blocks (equal scores: smaller j first).  ids ascending.  Returns the count, -1 on invalid arguments. */
int64_t oracle_select_topk_in_blocks(const double *s, int64_t n, int64_t block, const int32_t *blocks, int64_t nblk,
                                     int64_t w0, int64_t w1, int64_t k, int32_t *ids)
{
    if (w0 < 0 || w1 < 0 || k <= 0 || block <= 0) return -1;
    if (n <= 0) return 0;
    char *cand = (char *)calloc((size_t)n, 1);
    for (int64_t i = 0; i < nblk; ++i)
        for (int64_t j = (int64_t)blocks[i] * block; j < n && j < ((int64_t)blocks[i] + 1) * block; ++j) cand[j] = 1;
    int32_t *order = (int32_t *)malloc((size_t)n * sizeof *order);
    int64_t m = 0;
    for (int64_t j = 0; j < n; ++j) {
        int inwin = j < w0 || j >= n - w1;
        if (cand[j] && !inwin) order[m++] = (int32_t)j;
    }
    qsort_r(order, (size_t)m, sizeof *order, by_score_desc_then_id, (void *)s);
    int64_t kk = k < m ? k : m;
    char *take = (char *)calloc((size_t)n, 1);
    for (int64_t i = 0; i < kk; ++i) take[order[i]] = 1;
    int64_t cnt = 0;
    for (int64_t j = 0; j < n; ++j)
        if (j < w0 || j >= n - w1 || take[j]) ids[cnt++] = (int32_t)j;
    free(take);
    free(order);
    free(cand);
    return cnt;
}

/*
 * One request, all query heads, top-k through the coarse index: scores -> block representatives -> block
 * scores -> the P best blocks -> top-k among their tokens -> attend.
 *   blocks_out  optional [n_q_heads][blocks_stride] ascending block numbers (first min(count, stride))
 *   bcounts     optional [n_q_heads] blocks chosen = min(P, number of blocks)
 *   u_out       optional [n_q_heads][number of blocks] block scores
 *   n_vis       the query sees only the first n_vis <= n tokens (prefix reuse, Sec. 7.1), through the index of
 *               the STORED context: the representatives of a block cover all of its stored tokens, also those
 *               behind the prefix; only blocks that hold a visible token take part
 * Other arguments as oracle_sparse_attn.  Returns the threads used, negative on invalid arguments.
 */
void oracle_attend(const double *s, const void *V, int dtype, int n_kv_heads, int g, int d,
                   const int32_t *ids, int64_t cnt, double scale, double *o);
int oracle_coarse_attn(const void *q, const void *K, const void *V, int dtype, int64_t n, int64_t n_vis, int n_q_heads,
                       int n_kv_heads, int d, int64_t block, int64_t P, int64_t k, double scale, int64_t w0, int64_t w1, double *out,
                       int32_t *ids, int64_t ids_stride, int64_t *counts, double *scores, int32_t *blocks_out,
                       int64_t blocks_stride, int64_t *bcounts, double *u_out, int n_threads)
{
    if (n <= 0 || n_q_heads <= 0 || n_kv_heads <= 0 || d <= 0 || n_q_heads % n_kv_heads) return -1;
    if (w0 < 0 || w1 < 0) return -4;
    if (k <= 0) return -2;
    if (block <= 0 || P <= 0) return -5;
    if (n_vis <= 0 || n_vis > n) return -6;
    if (!(scale > 0.0)) scale = 1.0 / sqrt((double)d);
    const int G = n_q_heads / n_kv_heads;
    const size_t esz = dtype == ORACLE_F32 ? 4 : 2;
    const int64_t nb = (n_vis + block - 1) / block;            /* blocks that hold a visible token */
    const int64_t n_rep = nb * block < n ? nb * block : n;     /* stored tokens that their representatives cover */
    int used = 1;
#ifdef _OPENMP
    if (n_threads <= 0) n_threads = omp_get_max_threads();
    if (n_threads > n_q_heads) n_threads = n_q_heads;
    used = n_threads;
#pragma omp parallel for schedule(dynamic, 1) num_threads(n_threads)
#endif
    for (int h = 0; h < n_q_heads; ++h) {
        const int g = h / G;
        const void *qh = (const char *)q + (size_t)h * (size_t)d * esz;
        double *s = scores ? scores + (size_t)h * (size_t)n_vis : (double *)malloc((size_t)n_vis * sizeof(double));
        double *lo = (double *)malloc((size_t)nb * d * sizeof(double)), *hi = (double *)malloc((size_t)nb * d * sizeof(double));
        double *u = u_out ? u_out + (size_t)h * (size_t)nb : (double *)malloc((size_t)nb * sizeof(double));
        int32_t *blk = (int32_t *)malloc((size_t)nb * sizeof(int32_t));
        int32_t *sel = (int32_t *)malloc((size_t)n_vis * sizeof(int32_t));
        oracle_scores(qh, K, dtype, n_vis, n_kv_heads, g, d, s);
        oracle_block_reps(K, dtype, n_rep, n_kv_heads, g, d, block, lo, hi);
        oracle_block_scores(qh, dtype, lo, hi, nb, d, u);
        int64_t nblk = oracle_select_topk(u, nb, P, blk);
        int64_t cnt = oracle_select_topk_in_blocks(s, n_vis, block, blk, nblk, w0, w1, k, sel);
        oracle_attend(s, V, dtype, n_kv_heads, g, d, sel, cnt, scale, out + (size_t)h * (size_t)d);
        if (counts) counts[h] = cnt;
        if (bcounts) bcounts[h] = nblk;
        if (ids) memcpy(ids + (size_t)h * (size_t)ids_stride, sel, (size_t)(cnt < ids_stride ? cnt : ids_stride) * sizeof(int32_t));
        if (blocks_out)
            memcpy(blocks_out + (size_t)h * (size_t)blocks_stride, blk,
                   (size_t)(nblk < blocks_stride ? nblk : blocks_stride) * sizeof(int32_t));
        free(sel); free(blk); free(lo); free(hi);
        if (!u_out) free(u);
        if (!scores) free(s);
    }
    return used;
}

/* Scores in the arithmetic DIPRS decides in: fp32, acc = fma(q_c, k_c, acc) for c = 0 .. d-1 in order. */
void oracle_scores_f32(const void *q, const void *K, int dtype, int64_t n, int n_kv_heads, int g, int d, float *s)
{
    for (int64_t j = 0; j < n; ++j) {
        float acc = 0.0f;
        int64_t row = (j * n_kv_heads + g) * (int64_t)d;
        for (int c = 0; c < d; ++c)
            acc = fmaf((float)widen(q, dtype, c), (float)widen(K, dtype, row + c), acc);
        s[j] = acc;
    }
}

static int by_sim_desc_then_id(const void *a, const void *b, void *ctx)
{
    const double *sim = (const double *)ctx;
    int32_t ia = *(const int32_t *)a, ib = *(const int32_t *)b;
    if (sim[ia] > sim[ib]) return -1;
    if (sim[ia] < sim[ib]) return 1;
    return (ia > ib) - (ia < ib);
}

/* The exact M-nearest-neighbour graph of the first n keys of KV head g under the inner product: nbr[j][0..M)
 * = the M keys i != j with the largest k_i . k_j, best first (equal products: smaller i first); -1 where
 * fewer than M other keys exist.  Brute force, fp64. */
void oracle_knn_graph(const void *K, int dtype, int64_t n, int n_kv_heads, int g, int d, int M, int32_t *nbr)
{
#ifdef _OPENMP
#pragma omp parallel
#endif
    {
        double *sim = (double *)malloc((size_t)n * sizeof(double));
        int32_t *order = (int32_t *)malloc((size_t)n * sizeof(int32_t));
#ifdef _OPENMP
#pragma omp for schedule(dynamic, 16)
#endif
        for (int64_t j = 0; j < n; ++j) {
            int64_t m = 0;
            for (int64_t i = 0; i < n; ++i) {
                double acc = 0.0;
                for (int c = 0; c < d; ++c)
                    acc += widen(K, dtype, (i * n_kv_heads + g) * (int64_t)d + c) *
                           widen(K, dtype, (j * n_kv_heads + g) * (int64_t)d + c);
                sim[i] = acc;
                if (i != j) order[m++] = (int32_t)i;
            }
            qsort_r(order, (size_t)m, sizeof *order, by_sim_desc_then_id, sim);
            for (int t = 0; t < M; ++t) nbr[j * M + t] = t < m ? order[t] : -1;
        }
        free(order);
        free(sim);
    }
}

/* Algorithm 1, DIPRS(G, q, k0, l0, beta), on the graph nbr[n][M] (-1 = no neighbour) with the scores s[n].
 * Window tokens W = {j < w0} U {j >= n - w1} are always attended, count as visited from the start and seed
 * the best-so-far; k0 must lie outside W.
 *   C, c_len   the list C in the order in which it grew (C[0] = k0)
 *   ids        the answer, ascending: W plus every c in C with s_c >= best - beta, best = max over C and W
 * Returns the size of the answer, -1 on invalid arguments. */
int64_t oracle_diprs(const int32_t *nbr, int64_t n, int M, const float *s, int32_t k0, int64_t l0, float beta,
                     int64_t w0, int64_t w1, int32_t *C, int64_t *c_len, int32_t *ids)
{
    if (n <= 0 || M <= 0 || !(beta >= 0.0f) || l0 < 0 || w0 < 0 || w1 < 0) return -1;
    if (k0 < 0 || k0 >= n || k0 < w0 || k0 >= n - w1) return -1;
    char *visited = (char *)calloc((size_t)n, 1);
    int have_best = 0;
    float best = 0.0f;
    for (int64_t j = 0; j < n; ++j)
        if (j < w0 || j >= n - w1) {
            visited[j] = 1;
            if (!have_best || s[j] > best) { best = s[j]; have_best = 1; }
        }
    int64_t len = 0;
    C[len++] = k0;
    visited[k0] = 1;
    if (!have_best || s[k0] > best) { best = s[k0]; have_best = 1; }
    for (int64_t i = 0; i < len; ++i) {
        const int32_t c = C[i];
        for (int t = 0; t < M; ++t) {
            const int32_t k = nbr[(int64_t)c * M + t];
            if (k < 0 || k >= n || visited[k]) continue;
            visited[k] = 1;                                   /* tryAppend(q, k, beta, C, l0) */
            if (len <= l0 || s[k] >= best - beta) {
                C[len++] = k;
                if (s[k] > best) best = s[k];
            }
        }
    }
    *c_len = len;
    char *take = (char *)calloc((size_t)n, 1);
    for (int64_t i = 0; i < len; ++i)
        if (s[C[i]] >= best - beta) take[C[i]] = 1;
    int64_t cnt = 0;
    for (int64_t j = 0; j < n; ++j)
        if (j < w0 || j >= n - w1 || take[j]) ids[cnt++] = (int32_t)j;
    free(take);
    free(visited);
    return cnt;
}

/* Softmax over the selected set and the weighted sum of its value rows. */
void oracle_attend(const double *s, const void *V, int dtype, int n_kv_heads, int g, int d,
                   const int32_t *ids, int64_t cnt, double scale, double *o)
{
    for (int c = 0; c < d; ++c) o[c] = 0.0;
    if (cnt <= 0) return;
    double zmax = s[ids[0]] * scale;
    for (int64_t i = 1; i < cnt; ++i) {
        double z = s[ids[i]] * scale;
        if (z > zmax) zmax = z;
    }
    double denom = 0.0;
    for (int64_t i = 0; i < cnt; ++i)
        denom += exp(s[ids[i]] * scale - zmax);
    for (int64_t i = 0; i < cnt; ++i) {
        double a = exp(s[ids[i]] * scale - zmax) / denom;
        int64_t row = ((int64_t)ids[i] * n_kv_heads + g) * (int64_t)d;
        for (int c = 0; c < d; ++c)
            o[c] += a * widen(V, dtype, row + c);
    }
}

/*
 * One request, all query heads: scores -> select -> attend.
 *   q        [n_q_heads][d]          storage dtype
 *   K, V     [n][n_kv_heads][d]      storage dtype
 *   mode     ORACLE_TOPK (uses k), ORACLE_DIPR (uses beta), ORACLE_FULL
 *   w0, w1   window of always-attended first / last tokens (0, 0 = none)
 *   scale    softmax scale; <= 0 means 1/sqrt(d)
 *   out      [n_q_heads][d] fp64
 *   ids      optional [n_q_heads][ids_stride] ascending token ids (first min(count, stride))
 *   counts   optional [n_q_heads] true selected count
 *   scores   optional [n_q_heads][n] fp64 raw inner products
 * Heads run in an OpenMP loop with at most n_threads threads (0 = library default).
 * Returns the number of threads used, or a negative value on invalid arguments.
 */
int oracle_sparse_attn(const void *q, const void *K, const void *V, int dtype, int64_t n,
                       int n_q_heads, int n_kv_heads, int d, int mode, int64_t k, double beta,
                       double scale, int64_t w0, int64_t w1, double *out, int32_t *ids, int64_t ids_stride,
                       int64_t *counts, double *scores, int n_threads)
{
    if (n <= 0 || n_q_heads <= 0 || n_kv_heads <= 0 || d <= 0 || n_q_heads % n_kv_heads) return -1;
    if (w0 < 0 || w1 < 0) return -4;
    if (mode == ORACLE_TOPK && k <= 0) return -2;
    if (mode == ORACLE_DIPR && !(beta >= 0.0)) return -3;
    if (!(scale > 0.0)) scale = 1.0 / sqrt((double)d);
    const int G = n_q_heads / n_kv_heads;
    const size_t esz = dtype == ORACLE_F32 ? 4 : 2;
    int used = 1;
#ifdef _OPENMP
    if (n_threads <= 0) n_threads = omp_get_max_threads();
    if (n_threads > n_q_heads) n_threads = n_q_heads;
    used = n_threads;
#pragma omp parallel for schedule(dynamic, 1) num_threads(n_threads)
#endif
    for (int h = 0; h < n_q_heads; ++h) {
        const int g = h / G;
        double *s = scores ? scores + (size_t)h * (size_t)n : (double *)malloc((size_t)n * sizeof(double));
        int32_t *sel = (int32_t *)malloc((size_t)n * sizeof(int32_t));
        oracle_scores((const char *)q + (size_t)h * (size_t)d * esz, K, dtype, n, n_kv_heads, g, d, s);
        int64_t cnt;
        if (mode != ORACLE_FULL && (w0 > 0 || w1 > 0)) {
            cnt = oracle_select_window(s, n, w0, w1, mode, k, beta, sel);
        } else if (mode == ORACLE_TOPK) {
            cnt = oracle_select_topk(s, n, k, sel);
        } else if (mode == ORACLE_DIPR) {
            cnt = oracle_select_dipr(s, n, beta, sel);
        } else {
            for (int64_t j = 0; j < n; ++j) sel[j] = (int32_t)j;
            cnt = n;
        }
        oracle_attend(s, V, dtype, n_kv_heads, g, d, sel, cnt, scale, out + (size_t)h * (size_t)d);
        if (counts) counts[h] = cnt;
        if (ids) {
            int64_t m = cnt < ids_stride ? cnt : ids_stride;
            memcpy(ids + (size_t)h * (size_t)ids_stride, sel, (size_t)m * sizeof(int32_t));
        }
        free(sel);
        if (!scores) free(s);
    }
    return used;
}
