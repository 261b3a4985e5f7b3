// Drives the host half of the library - page bookkeeping, descriptor building, scratch layout, argument checks,
// the optimizer - through the C ABI on a machine without a GPU, linked against hip_stub.hip and built with
// AddressSanitizer and UBSan.  "Device" memory that the host code itself copies to or from (page table, scratch,
// representatives, graph) is real host memory of exactly the size the library asks for, so that a copy or a
// layout that overruns it is caught; the K and V pools, which only kernels touch, are fake addresses.
#include "../../include/alaya.h"
#include "../../include/alaya_debug.h"

#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

extern int g_launches, g_check_failures;
static int failures = 0;

#define CHECK(cond)                                                                  \
    do {                                                                             \
        if (!(cond)) {                                                               \
            std::fprintf(stderr, "CHECK failed: %s (line %d): %s\n", #cond, __LINE__, alaya_last_error()); \
            ++failures;                                                              \
        }                                                                            \
    } while (0)

static void *dev_alloc(size_t n, int fill)
{
    void *p = nullptr;
    if (posix_memalign(&p, 256, n ? n : 256) != 0) std::abort();
    std::memset(p, fill, n);
    return p;
}

int main()
{
    void *const FAKE_K = (void *)0x10000000, *const FAKE_V = (void *)0x20000000, *const FAKE_Q = (void *)0x30000000,
                *const FAKE_OUT = (void *)0x40000000, *const FAKE_KV = (void *)0x50000000;
    alaya_cache_config cfg{};
    cfg.n_q_heads = 32; cfg.n_kv_heads = 8; cfg.head_dim = 128; cfg.page_tokens = 64; cfg.dtype = ALAYA_BF16;
    cfg.max_seqs = 4; cfg.max_batch = 4; cfg.max_tokens_per_seq = 9000; cfg.max_batch_tokens = 20000; cfg.n_phys_pages = 200;
    const size_t ws_b = alaya_workspace_bytes(&cfg), sc_b = alaya_scratch_bytes(&cfg), rep_b = alaya_rep_bytes(&cfg);
    CHECK(alaya_pool_bytes(&cfg) == (size_t)200 * 8 * 64 * 128 * 2 && ws_b > 0 && sc_b > 0 && rep_b > 0);
    void *ws = dev_alloc(ws_b, 0xFF), *sc = dev_alloc(sc_b, 0xFF), *rep = dev_alloc(rep_b, 0xFF);
    std::vector<int32_t> order(200);
    for (int i = 0; i < 200; ++i) order[i] = (i * 77) % 200; // a permutation: 77 and 200 are coprime
    alaya_cache *c = nullptr;
    CHECK(alaya_create_cache(&c, &cfg, FAKE_K, FAKE_V, order.data(), ws, ws_b) == ALAYA_OK && c);
    CHECK(alaya_bind_scratch(c, sc, sc_b) == ALAYA_OK);
    CHECK(alaya_bind_reps(c, rep, rep_b) == ALAYA_OK);

    // Session.update in ragged pieces, across page boundaries
    const int64_t pieces[] = {1, 62, 1, 64, 65, 1000, 3807, 0};
    int64_t n0 = 0;
    for (int64_t t : pieces) { CHECK(alaya_append_kv(c, 0, FAKE_KV, FAKE_KV, t, nullptr) == ALAYA_OK); n0 += t; }
    CHECK(alaya_seq_len(c, 0) == n0 && n0 == 5000);
    CHECK(alaya_append_kv(c, 1, FAKE_KV, FAKE_KV, 300, nullptr) == ALAYA_OK);
    CHECK(alaya_append_kv(c, 2, FAKE_KV, FAKE_KV, 64, nullptr) == ALAYA_OK);
    const int32_t s012[] = {0, 1, 2};
    for (int i = 0; i < 3; ++i) CHECK(alaya_append_kv_step(c, s012, 3, FAKE_KV, FAKE_KV, nullptr) == ALAYA_OK);
    CHECK(alaya_seq_len(c, 0) == 5003 && alaya_seq_len(c, 1) == 303 && alaya_seq_len(c, 2) == 67 && alaya_seq_len(c, 3) == 0);
    // the pool has 200 pages; sequence 3 cannot take what is left plus one
    const int64_t used = (5003 + 63) / 64 + (303 + 63) / 64 + (67 + 63) / 64;
    CHECK(alaya_append_kv(c, 3, FAKE_KV, FAKE_KV, (200 - used) * 64 + 1, nullptr) == ALAYA_E_NOMEM && alaya_seq_len(c, 3) == 0);
    CHECK(alaya_append_kv(c, 3, FAKE_KV, FAKE_KV, 9001, nullptr) == ALAYA_E_NOMEM);

    // Session.attention: every plan, with and without windows, prefixes, returned ids
    std::vector<int32_t> ids((size_t)3 * 32 * 2600), counts(3 * 32), pages((size_t)3 * 32 * 8);
    const int32_t topk[] = {2048, 100, 1000}, nvis[] = {4097, 303, 1}, cpages[] = {8, 2, 100};
    const float beta[] = {2.f, 0.f, 1e30f};
    for (int variant = 0; variant < 7; ++variant) {
        alaya_sparse_params p{};
        p.mode = variant == 1 || variant == 4 ? ALAYA_DIPR : ALAYA_TOPK;
        p.topk = topk; p.beta = beta;
        if (variant >= 2) { p.window_init = 128; p.window_last = 512; }
        if (variant == 3 || variant == 4) p.n_visible = nvis;
        if (variant >= 5) { p.coarse_pages = cpages; p.out_pages = pages.data(); p.pages_stride = 8; }
        if (variant == 6) p.n_visible = nvis;
        p.out_ids = ids.data(); p.out_counts = counts.data(); p.ids_stride = 2600;
        g_launches = 0;
        CHECK(alaya_sparse_attn(c, s012, 3, 32, FAKE_Q, &p, (float *)FAKE_OUT, nullptr) == ALAYA_OK);
        CHECK(g_launches >= 6);
        // one request: its descriptor travels in the kernel arguments
        alaya_sparse_params p1 = p;
        p1.topk = topk + 1; p1.beta = beta + 1;
        if (p1.n_visible) p1.n_visible = nvis + 1;
        if (p1.coarse_pages) p1.coarse_pages = cpages + 1;
        CHECK(alaya_sparse_attn(c, s012 + 1, 1, 32, FAKE_Q, &p1, (float *)FAKE_OUT, nullptr) == ALAYA_OK);
    }
    {
        alaya_sparse_params p{};
        p.mode = ALAYA_TOPK; p.topk = topk;
        CHECK(alaya_decode_step(c, s012, 3, 32, FAKE_KV, FAKE_KV, FAKE_Q, &p, (float *)FAKE_OUT, nullptr) == ALAYA_OK);
        CHECK(alaya_seq_len(c, 0) == 5004);
        CHECK(alaya_sparse_attn_static(c, s012, 3, 32, FAKE_Q, &p, (float *)FAKE_OUT, nullptr) == ALAYA_OK);
        CHECK(alaya_set_profiling(c, 1) == ALAYA_OK);
        for (int i = 0; i < 40; ++i) CHECK(alaya_sparse_attn(c, s012, 3, 32, FAKE_Q, &p, (float *)FAKE_OUT, nullptr) == ALAYA_OK);
        double ms[7]; int64_t n[7];
        CHECK(alaya_kernel_times(c, ms, n, 7) == ALAYA_OK && n[0] == 40);
        CHECK(alaya_set_profiling(c, 0) == ALAYA_OK);
        CHECK(alaya_set_tuning(c, 4, 64, 1, 1) == ALAYA_OK);
        CHECK(alaya_sparse_attn(c, s012, 3, 32, FAKE_Q, &p, (float *)FAKE_OUT, nullptr) == ALAYA_OK);
        CHECK(alaya_set_tuning(c, 0, 0, 0, 0) == ALAYA_OK);
        int64_t a = 0, b = 0;
        CHECK(alaya_debug_pages(c, &a, &b) == ALAYA_OK && b == (5004 + 63) / 64 + (304 + 63) / 64 + (68 + 63) / 64);
        (void)alaya_debug_repairs(c, nullptr);
        CHECK(alaya_full_attn(c, s012, 3, 32, FAKE_Q, 0.f, (float *)FAKE_OUT, nullptr) == ALAYA_OK);
        (void)alaya_poll_status(c, nullptr);
        // bad arguments never reach a launcher
        g_launches = 0;
        const int32_t far[] = {9};
        CHECK(alaya_sparse_attn(c, far, 1, 32, FAKE_Q, &p, (float *)FAKE_OUT, nullptr) == ALAYA_E_INVAL);
        CHECK(alaya_sparse_attn(c, s012, 3, 16, FAKE_Q, &p, (float *)FAKE_OUT, nullptr) == ALAYA_E_INVAL);
        const int32_t s3[] = {3};
        CHECK(alaya_sparse_attn(c, s3, 1, 32, FAKE_Q, &p, (float *)FAKE_OUT, nullptr) == ALAYA_E_EMPTY);
        CHECK(g_launches == 0);
    }

    // the fine-grained index: the build's chunks stay inside the build memory, the walk's areas inside the scratch
    {
        const size_t ib = alaya_graph_bytes(c, 0, 32), bb = alaya_graph_build_bytes(c, 0, 32);
        CHECK(ib > 0 && bb > 0);
        void *im = dev_alloc(ib, 0xFF), *bm = dev_alloc(bb, 0xFF);
        alaya_graph *g = nullptr;
        CHECK(alaya_graph_build(&g, c, 3, 32, im, ib, bm, bb, nullptr) == ALAYA_E_EMPTY && !g);
        CHECK(alaya_graph_build(&g, c, 0, 32, im, ib - 1, bm, bb, nullptr) == ALAYA_E_NOMEM && !g);
        CHECK(alaya_graph_build(&g, c, 0, 32, im, ib, bm, bb, nullptr) == ALAYA_OK && g);
        int64_t ni = 0; int32_t deg = 0, entry[8]; const int32_t *nb = nullptr;
        CHECK(alaya_graph_info(g, &ni, &deg, &nb, entry) == ALAYA_OK && ni == 5004 && deg == 32 && nb == im && entry[7] == 2502);
        CHECK(alaya_append_kv_step(c, s012, 1, FAKE_KV, FAKE_KV, nullptr) == ALAYA_OK); // a token the graph does not know
        alaya_sparse_params p{};
        p.window_init = 4; p.window_last = 64; p.out_ids = ids.data(); p.out_counts = counts.data(); p.ids_stride = 2600;
        CHECK(alaya_diprs_attn(c, g, 32, FAKE_Q, 2.f, 64, &p, (float *)FAKE_OUT, nullptr) == ALAYA_OK);
        CHECK(alaya_diprs_attn(c, g, 32, FAKE_Q, 2.f, 64, nullptr, (float *)FAKE_OUT, nullptr) == ALAYA_OK);
        CHECK(alaya_diprs_attn(c, g, 32, FAKE_Q, -1.f, 64, nullptr, (float *)FAKE_OUT, nullptr) == ALAYA_E_INVAL);
        int32_t lst[4];
        CHECK(alaya_debug_diprs_list(c, 31, lst, 4, nullptr) == 0);
        CHECK(alaya_graph_destroy(g) == ALAYA_OK);
        std::free(im); std::free(bm);
    }

    // a sequence is reset and its pages are handed out again
    CHECK(alaya_reset_seq(c, 0) == ALAYA_OK && alaya_seq_len(c, 0) == 0);
    CHECK(alaya_append_kv(c, 3, FAKE_KV, FAKE_KV, 5000, nullptr) == ALAYA_OK);
    CHECK(alaya_append_kv(c, 0, FAKE_KV, FAKE_KV, 4000, nullptr) == ALAYA_OK);
    const int32_t s30[] = {3, 0, 1, 2};
    {
        alaya_sparse_params p{};
        p.mode = ALAYA_DIPR; p.beta = beta; // (beta has three entries: a fourth is needed)
        const float b4[] = {1.f, 2.f, 3.f, 4.f};
        p.beta = b4;
        CHECK(alaya_sparse_attn(c, s30, 4, 32, FAKE_Q, &p, (float *)FAKE_OUT, nullptr) == ALAYA_OK);
    }

    // scratch shared by a second cache (another layer), then unbound
    {
        void *ws2 = dev_alloc(ws_b, 0xFF);
        alaya_cache *c2 = nullptr;
        CHECK(alaya_create_cache(&c2, &cfg, FAKE_K, FAKE_V, nullptr, ws2, ws_b) == ALAYA_OK);
        CHECK(alaya_bind_scratch(c2, sc, sc_b) == ALAYA_OK);
        CHECK(alaya_append_kv(c2, 0, FAKE_KV, FAKE_KV, 700, nullptr) == ALAYA_OK);
        alaya_sparse_params p{};
        p.mode = ALAYA_TOPK; p.topk = topk;
        const int32_t s0[] = {0};
        CHECK(alaya_sparse_attn(c2, s0, 1, 32, FAKE_Q, &p, (float *)FAKE_OUT, nullptr) == ALAYA_OK);
        CHECK(alaya_bind_scratch(c2, nullptr, 0) == ALAYA_OK);
        CHECK(alaya_sparse_attn(c2, s0, 1, 32, FAKE_Q, &p, (float *)FAKE_OUT, nullptr) == ALAYA_E_INVAL);
        CHECK(alaya_destroy_cache(c2) == ALAYA_OK);
        std::free(ws2);
    }

    // the optimizer
    {
        alaya_plan_input in{200000, 4096, 150000, 1 << 20, 1 << 30, 3, 0};
        alaya_plan out{};
        CHECK(alaya_plan_query(&in, &out) == ALAYA_OK && out.query == ALAYA_QUERY_DIPR && out.index == ALAYA_INDEX_FINE &&
              out.n_visible == 150000);
        CHECK(alaya_plan_query(nullptr, &out) == ALAYA_E_INVAL);
    }

    CHECK(alaya_destroy_cache(c) == ALAYA_OK);
    std::free(ws); std::free(sc); std::free(rep);
    if (g_check_failures) std::fprintf(stderr, "%d launch checks failed\n", g_check_failures);
    std::printf("host_check: %d failures, %d launch-check failures\n", failures, g_check_failures);
    return failures || g_check_failures ? 1 : 0;
}
