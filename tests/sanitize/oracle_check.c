/* Calls every function of the oracle on small, ragged inputs whose buffers have exactly the documented sizes,
 * in a build with AddressSanitizer and UBSan: an index that runs past a buffer, or an overflow in an index
 * computation, ends the program.  Results are only checked for plausibility here; what they must be is the
 * business of the pins. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

void oracle_scores(const void *q, const void *K, int dtype, int64_t n, int n_kv_heads, int g, int d, double *s);
int64_t oracle_select_topk(const double *s, int64_t n, int64_t k, int32_t *ids);
int64_t oracle_select_dipr(const double *s, int64_t n, double beta, int32_t *ids);
int64_t oracle_select_window(const double *s, int64_t n, int64_t w0, int64_t w1, int mode, int64_t k, double beta, int32_t *ids);
void oracle_block_reps(const void *K, int dtype, int64_t n, int n_kv_heads, int g, int d, int64_t block, double *lo, double *hi);
void oracle_block_scores(const void *q, int dtype, const double *lo, const double *hi, int64_t nb, int d, double *u);
int64_t oracle_select_topk_in_blocks(const double *s, int64_t n, int64_t block, const int32_t *blocks, int64_t nblk, int64_t w0,
                                     int64_t w1, int64_t k, int32_t *ids);
int oracle_coarse_attn(const void *q, const void *K, const void *V, int dtype, int64_t n, int64_t n_vis, int n_q_heads,
                       int n_kv_heads, int d, int64_t block, int64_t P, int64_t k, double scale, int64_t w0, int64_t w1,
                       double *out, int32_t *ids, int64_t ids_stride, int64_t *counts, double *scores, int32_t *blocks_out,
                       int64_t blocks_stride, int64_t *bcounts, double *u_out, int n_threads);
void oracle_scores_f32(const void *q, const void *K, int dtype, int64_t n, int n_kv_heads, int g, int d, float *s);
void oracle_knn_graph(const void *K, int dtype, int64_t n, int n_kv_heads, int g, int d, int M, int32_t *nbr);
int64_t oracle_diprs(const int32_t *nbr, int64_t n, int M, const float *s, int32_t k0, int64_t l0, float beta, int64_t w0,
                     int64_t w1, int32_t *C, int64_t *c_len, int32_t *ids);
void oracle_attend(const double *s, const void *V, int dtype, int n_kv_heads, int g, int d, const int32_t *ids, int64_t cnt,
                   double scale, double *o);
int oracle_sparse_attn(const void *q, const void *K, const void *V, int dtype, int64_t n, int n_q_heads, int n_kv_heads, int d,
                       int mode, int64_t k, double beta, double scale, int64_t w0, int64_t w1, double *out, int32_t *ids,
                       int64_t ids_stride, int64_t *counts, double *scores, int n_threads);

static uint32_t rng = 12345u;
static float frand(void)
{
    rng = rng * 1664525u + 1013904223u;
    return (float)((rng >> 8) & 0xFFFF) / 32768.0f - 1.0f;
}
static uint16_t bf16(float f)
{
    union { float f; uint32_t u; } x = {f};
    return (uint16_t)((x.u + 0x7FFFu + ((x.u >> 16) & 1u)) >> 16);
}

static int bad = 0;
#define CHECK(c) do { if (!(c)) { fprintf(stderr, "CHECK failed: %s (line %d)\n", #c, __LINE__); ++bad; } } while (0)

static void run(int dtype, int64_t n, int hq, int hk, int d, int64_t block, int M)
{
    const size_t kv = (size_t)n * hk * d, es = dtype == 0 ? 2 : 4;
    void *K = malloc(kv * es), *V = malloc(kv * es), *q = malloc((size_t)hq * d * es);
    for (size_t i = 0; i < kv; ++i) {
        if (dtype == 0) { ((uint16_t *)K)[i] = bf16(frand()); ((uint16_t *)V)[i] = bf16(frand()); }
        else { ((float *)K)[i] = frand(); ((float *)V)[i] = frand(); }
    }
    for (size_t i = 0; i < (size_t)hq * d; ++i) {
        if (dtype == 0) ((uint16_t *)q)[i] = bf16(frand()); else ((float *)q)[i] = frand();
    }
    const int G = hq / hk;
    double *s = malloc((size_t)n * sizeof *s), *o = malloc((size_t)d * sizeof *o);
    int32_t *ids = malloc((size_t)n * sizeof *ids);
    const void *q0 = q;
    oracle_scores(q0, K, dtype, n, hk, hk - 1, d, s);
    CHECK(oracle_select_topk(s, n, 1, ids) == 1);
    CHECK(oracle_select_topk(s, n, n + 5, ids) == n);
    CHECK(oracle_select_topk(s, n, 0, ids) == -1);
    int64_t c = oracle_select_dipr(s, n, 0.5, ids);
    CHECK(c >= 1 && c <= n);
    CHECK(oracle_select_dipr(s, n, INFINITY, ids) == n);
    c = oracle_select_window(s, n, 3, 5, 0, 4, 0.0, ids);
    CHECK(c >= 1 && c <= n);
    c = oracle_select_window(s, n, n + 2, n + 2, 1, 0, 1.0, ids);
    CHECK(c == n);
    oracle_attend(s, V, dtype, hk, hk - 1, d, ids, c, 0.1, o);
    CHECK(isfinite(o[0]) && isfinite(o[d - 1]));

    const int64_t nb = (n + block - 1) / block;
    double *lo = malloc((size_t)nb * d * sizeof *lo), *hi = malloc((size_t)nb * d * sizeof *hi), *u = malloc((size_t)nb * sizeof *u);
    oracle_block_reps(K, dtype, n, hk, hk - 1, d, block, lo, hi);
    oracle_block_scores(q0, dtype, lo, hi, nb, d, u);
    int32_t *blk = malloc((size_t)nb * sizeof *blk);
    for (int64_t b = 0; b < nb; ++b) blk[b] = (int32_t)b;
    c = oracle_select_topk_in_blocks(s, n, block, blk + nb / 2, nb - nb / 2, 2, 2, 7, ids);
    CHECK(c >= 1 && c <= n);

    double *out = malloc((size_t)hq * d * sizeof *out), *sc = malloc((size_t)hq * n * sizeof *sc), *uo = malloc((size_t)hq * nb * sizeof *uo);
    int32_t *idm = malloc((size_t)hq * n * sizeof *idm), *bo = malloc((size_t)hq * nb * sizeof *bo);
    int64_t *cnt = malloc((size_t)hq * sizeof *cnt), *bc = malloc((size_t)hq * sizeof *bc);
    for (int mode = 0; mode < 3; ++mode)
        CHECK(oracle_sparse_attn(q, K, V, dtype, n, hq, hk, d, mode, 9, 0.7, 0.0, mode, 2 * mode, out, idm, n, cnt, sc, 3) >= 1);
    CHECK(oracle_sparse_attn(q, K, V, dtype, n, hq, hk, d, 0, 9, 0.7, 0.0, 0, 0, out, idm, 4, cnt, NULL, 0) >= 1); /* short id rows */
    CHECK(oracle_sparse_attn(q, K, V, dtype, n, hq, hk, d, 2, 0, 0.0, 0.25, 0, 0, out, NULL, 0, NULL, NULL, 2) >= 1); /* full attention */
    CHECK(oracle_coarse_attn(q, K, V, dtype, n, n, hq, hk, d, block, 2, 5, 0.0, 1, 3, out, idm, n, cnt, sc, bo, nb, bc, uo, 2) >= 1);
    CHECK(oracle_coarse_attn(q, K, V, dtype, n, n - n / 3, hq, hk, d, block, nb + 3, n + 1, 0.0, 0, 0, out, idm, 3, cnt, NULL, bo, 1,
                             bc, NULL, 1) >= 1);

    float *s32 = malloc((size_t)n * sizeof *s32);
    int32_t *nbr = malloc((size_t)n * M * sizeof *nbr), *C = malloc((size_t)n * sizeof *C);
    oracle_scores_f32(q0, K, dtype, n, hk, 0, d, s32);
    oracle_knn_graph(K, dtype, n, hk, 0, d, M, nbr);
    int64_t cl = 0;
    c = oracle_diprs(nbr, n, M, s32, (int32_t)(n / 2), 3, 0.5f, 0, 0, C, &cl, ids);
    CHECK(c >= 1 && cl >= 1 && cl <= n);
    c = oracle_diprs(nbr, n, M, s32, (int32_t)(n / 2), n, 0.0f, 2, 2, C, &cl, ids);
    CHECK(c >= 4 || n < 6);
    CHECK(oracle_diprs(nbr, n, M, s32, 0, 3, 0.5f, 1, 0, C, &cl, ids) == -1); /* start key inside the window */
    (void)G;
    free(K); free(V); free(q); free(s); free(o); free(ids); free(lo); free(hi); free(u); free(blk); free(out); free(sc); free(uo);
    free(idm); free(bo); free(cnt); free(bc); free(s32); free(nbr); free(C);
}

int main(void)
{
    run(0, 131, 4, 2, 16, 64, 5);   /* bf16, ragged last block */
    run(1, 64, 2, 1, 8, 16, 70);    /* fp32, more neighbours asked for than keys exist */
    run(0, 7, 8, 8, 4, 3, 2);       /* tiny, one query head per KV head */
    run(1, 300, 6, 2, 32, 64, 9);
    printf("oracle_check: %d failures\n", bad);
    return bad ? 1 : 0;
}
