// Host-only stand-in for the HIP runtime and for the kernel launchers, so that the host half of the library
// (api.hip, plan.hip) can run on a machine without a GPU under AddressSanitizer and UBSan.  "Device" memory is
// ordinary host memory that the test allocates; copies are memcpy; a launcher launches nothing and instead
// checks on the host what its kernel would assume of the descriptors and sizes it is handed.
#include "../../paper_2504_10326_amd/csrc/alaya_internal.h"

#include <cstdio>
#include <cstdlib>
#include <cstring>

int g_launches = 0;      // launcher calls since the last reset (read by the driver)
int g_check_failures = 0;

#define EXPECT(cond)                                                                        \
    do {                                                                                    \
        if (!(cond)) {                                                                      \
            std::fprintf(stderr, "launch check failed: %s (%s:%d)\n", #cond, __FILE__, __LINE__); \
            ++g_check_failures;                                                             \
        }                                                                                   \
    } while (0)

extern "C" {
void **__hipRegisterFatBinary(const void *) { static void *h; return &h; }
void __hipUnregisterFatBinary(void **) {}
void __hipRegisterVar(void **, void *, char *, const char *, int, size_t, int, int) {}
void __hipRegisterFunction(void **, const void *, char *, const char *, unsigned, void *, void *, void *, void *, int *) {}
}

hipError_t hipGetDevice(int *d) { *d = 0; return hipSuccess; }
hipError_t hipGetLastError() { return hipSuccess; }
const char *hipGetErrorString(hipError_t) { return "stub"; }
hipError_t hipStreamSynchronize(hipStream_t) { return hipSuccess; }
hipError_t hipMemcpyAsync(void *dst, const void *src, size_t n, hipMemcpyKind, hipStream_t)
{
    std::memcpy(dst, src, n); // both sides are host memory here: the sanitizer sees every byte of the copy
    return hipSuccess;
}
hipError_t hipHostMalloc(void **p, size_t n, unsigned) { *p = std::malloc(n); return *p ? hipSuccess : hipErrorOutOfMemory; }
hipError_t hipHostFree(void *p) { std::free(p); return hipSuccess; }
hipError_t hipEventCreate(hipEvent_t *e) { *e = (hipEvent_t)std::malloc(1); return hipSuccess; }
hipError_t hipEventCreateWithFlags(hipEvent_t *e, unsigned) { return hipEventCreate(e); }
hipError_t hipEventDestroy(hipEvent_t e) { std::free((void *)e); return hipSuccess; }
hipError_t hipEventRecord(hipEvent_t, hipStream_t) { return hipSuccess; }
hipError_t hipEventSynchronize(hipEvent_t) { return hipSuccess; }
hipError_t hipEventElapsedTime(float *ms, hipEvent_t, hipEvent_t) { *ms = 0.01f; return hipSuccess; }
hipError_t hipGetSymbolAddress(void **p, const void *symbol)
{
    *p = const_cast<void *>(symbol); // the host-side array itself stands for the device's copy
    return hipSuccess;
}

namespace alaya {

static ReqDesc desc_of(const DescArgs &d, int r) { return d.n == 1 ? d.in : d.mem[r]; }

// What every kernel assumes of a call's descriptors.
static void check_descs(const Shape &sh, const DescArgs &d, int B)
{
    EXPECT(d.n == B && B >= 1);
    int64_t off = 0;
    for (int r = 0; r < B; ++r) {
        const ReqDesc q = desc_of(d, r);
        EXPECT(q.n >= 1 && q.n_pages == (q.n + kPageTokens - 1) / kPageTokens);
        EXPECT(q.head_stride >= q.n_pages * kPageTokens);
        EXPECT(q.score_off >= off);
        off = q.score_off + (int64_t)sh.n_q_heads * q.head_stride;
        EXPECT(q.w0 >= 0 && q.w1 >= 0 && q.w0 <= q.n && q.w1 <= q.n && q.nwin <= q.n);
        EXPECT(q.k >= 0 && q.k <= q.n);
        EXPECT(q.sample_stride >= 1 && (q.sample_stride & (q.sample_stride - 1)) == 0 && q.sample_stride <= 32);
        EXPECT(q.xf >= 0 && q.xf <= q.xb && q.xb <= q.n_pages);
    }
}

hipError_t launch_append(const Shape &, const int32_t *pt_row, void *k_pool, void *v_pool, const void *k, const void *v,
                         int64_t n_old, int64_t t, hipStream_t)
{
    ++g_launches;
    EXPECT(pt_row && k_pool && v_pool && k && v && n_old >= 0 && t > 0);
    for (int64_t p = n_old / kPageTokens; p <= (n_old + t - 1) / kPageTokens; ++p) EXPECT(pt_row[p] >= 0); // pages are mapped
    return hipSuccess;
}
hipError_t launch_append_step(const Shape &sh, const DeviceViews &dv, void *, void *, const void *k, const void *v, int B,
                              hipStream_t)
{
    ++g_launches;
    EXPECT(k && v && dv.desc.n == B);
    for (int r = 0; r < B; ++r) {
        const ReqDesc q = desc_of(dv.desc, r);
        EXPECT(q.n >= 1 && dv.page_table[q.pt_off + (q.n - 1) / kPageTokens] >= 0);
    }
    (void)sh;
    return hipSuccess;
}
hipError_t launch_sample(const Shape &sh, const DeviceViews &dv, int B, const void *q, int total_tiles, int mode, bool coarse,
                         hipStream_t)
{
    ++g_launches;
    if (total_tiles <= 0) return hipSuccess;
    check_descs(sh, dv.desc, B);
    EXPECT(q && (mode == 0 || mode == 1) && (!coarse || (mode == 0 && dv.pmask)));
    int prev = 0;
    for (int r = 0; r < B; ++r) {
        const ReqDesc d = desc_of(dv.desc, r);
        EXPECT(d.tile_start >= prev && d.tile_start <= total_tiles);
        prev = d.tile_start;
        // every mapped page of the request is readable through the page table
        for (int p = 0; p < d.n_pages; ++p) EXPECT(dv.page_table[d.pt_off + p] >= 0);
    }
    return hipSuccess;
}
hipError_t launch_tau(const Shape &sh, const DeviceViews &dv, int B, int, hipStream_t)
{
    ++g_launches;
    check_descs(sh, dv.desc, B);
    return hipSuccess;
}
hipError_t launch_score(const Shape &sh, const DeviceViews &dv, int B, const void *q, int total_tiles, int cp, bool, int,
                        bool coarse, hipStream_t, hipEvent_t, hipEvent_t)
{
    ++g_launches;
    check_descs(sh, dv.desc, B);
    EXPECT(q && (cp == 1 || cp == 2 || cp == 4));
    const int G = sh.n_q_heads / sh.n_kv_heads;
    // a full block fits: its dense part, and the rest of it in the second area
    EXPECT(dv.area.hdrs && dv.area.head && dv.area.rest_stride >= (int64_t)kScoreWaves * cp * kPageTokens * G - kHeadStride);
    EXPECT(dv.area.n_tiles == total_tiles);
    int next = 0;
    for (int r = 0; r < B; ++r) {
        const ReqDesc d = desc_of(dv.desc, r);
        EXPECT(d.tileb_start == next);
        EXPECT(d.ntiles_b == (d.n_pages + kScoreWaves * cp - 1) / (kScoreWaves * cp));
        next += d.ntiles_b;
        if (coarse) EXPECT(d.pm_stride >= d.n_pages && d.pm_off >= 0);
    }
    EXPECT(next == total_tiles);
    return hipSuccess;
}
hipError_t launch_select(const Shape &sh, const DeviceViews &, const SelectIO &io, int B, int mode, bool, int batch_blocks,
                         int32_t *out_ids, int32_t *, int64_t ids_stride, hipStream_t)
{
    ++g_launches;
    EXPECT(io.desc.n == B && io.area.head && io.ids && io.scores && io.counts && io.head_M);
    EXPECT(mode == 0 || mode == 1);
    EXPECT(batch_blocks >= 0);
    EXPECT(!out_ids || ids_stride > 0);
    for (int r = 0; r < B; ++r) {
        const ReqDesc d = desc_of(io.desc, r);
        EXPECT(d.head_stride >= d.n && d.k <= d.n);
        if (io.pmask) EXPECT(d.pm_off >= 0 && d.pm_stride >= d.n); // (pages: one mask byte per (KV head, page))
    }
    (void)sh;
    return hipSuccess;
}
hipError_t launch_attend(const Shape &, const DeviceViews &dv, int B, float scale, int splits, int min_splits, hipStream_t)
{
    ++g_launches;
    EXPECT(B >= 1 && (min_splits & 0xFFFF) >= 1 && (min_splits & 0xFFFF) <= splits && splits <= kMaxSplits && scale > 0.f && dv.partials);
    EXPECT((min_splits >> 16) == 7 || (min_splits >> 16) == 8);
    return hipSuccess;
}
hipError_t launch_combine(const Shape &, const DeviceViews &, int B, int splits, int min_splits, int per_request_tiles, int ppt,
                          float *out, hipStream_t)
{
    ++g_launches;
    EXPECT(B >= 1 && out && (per_request_tiles ? ppt >= 1 : (min_splits & 0xFFFF) >= 1 && (min_splits & 0xFFFF) <= splits && splits <= kMaxSplits));
    return hipSuccess;
}
hipError_t launch_full_partial(const Shape &sh, const DeviceViews &dv, int B, const void *q, float scale, int total_tiles,
                               int ppt, hipStream_t)
{
    ++g_launches;
    EXPECT(q && scale > 0.f && ppt >= 1);
    int next = 0;
    for (int r = 0; r < B; ++r) {
        const ReqDesc d = desc_of(dv.desc, r);
        EXPECT(d.tile_start == next);
        next += ((d.n + kPageTokens - 1) / kPageTokens + ppt - 1) / ppt;
    }
    EXPECT(next == total_tiles);
    (void)sh;
    return hipSuccess;
}
hipError_t launch_fill_u32(uint32_t *p, size_t n, uint32_t v, hipStream_t)
{
    ++g_launches;
    for (size_t i = 0; i < n; ++i) p[i] = v; // (host memory here: an overrun is the sanitizer's to find)
    return hipSuccess;
}
hipError_t launch_debug_scatter(const Shape &, const DeviceViews &, int, int, float *, unsigned long long *, hipStream_t)
{
    ++g_launches;
    return hipSuccess;
}
hipError_t launch_reps_range(const Shape &, const int32_t *pt_row, const void *k_pool, void *rep_pool, int first, int count,
                             int64_t n_new, hipStream_t)
{
    ++g_launches;
    EXPECT(k_pool && rep_pool && first >= 0 && count >= 1 && n_new > (int64_t)first * kPageTokens);
    for (int p = first; p < first + count; ++p) EXPECT(pt_row[p] >= 0);
    return hipSuccess;
}
hipError_t launch_reps_step(const Shape &, const DeviceViews &dv, void *rep_pool, int B, hipStream_t)
{
    ++g_launches;
    EXPECT(rep_pool && dv.desc.n == B);
    return hipSuccess;
}
hipError_t launch_coarse_score(const Shape &sh, const DeviceViews &, const DescArgs &pd, int B, const void *q, const void *rep_pool,
                               int total_tiles, const BlockArea &area, uint8_t *pmask, hipStream_t)
{
    ++g_launches;
    EXPECT(q && rep_pool && pmask && pd.n == B && area.hdrs && area.head && area.n_tiles == total_tiles &&
           area.rest_stride >= 256 * (sh.n_q_heads / sh.n_kv_heads) - kHeadStride);
    int next = 0;
    for (int r = 0; r < B; ++r) {
        const ReqDesc d = desc_of(pd, r);
        EXPECT(d.tileb_start == next && d.k >= 1 && d.k <= d.n);
        EXPECT(d.pm_off >= 0 && d.pm_stride >= d.n); // the kernel clears one mask byte per (KV head, page)
        next += d.ntiles_b;
    }
    EXPECT(next == total_tiles);
    return hipSuccess;
}
hipError_t launch_graph_knn(const Shape &sh, const void *k_pool, const int32_t *pt_row, int n, int M, int32_t *nbr, hipStream_t)
{
    ++g_launches;
    EXPECT(k_pool && pt_row && nbr && n >= 1 && M >= 1 && M <= 64);
    for (int p = 0; p < (n + kPageTokens - 1) / kPageTokens; ++p) EXPECT(pt_row[p] >= 0);
    // the lists that the kernel writes lie inside the index memory: touch their first and last element
    nbr[0] = -1;
    nbr[(size_t)sh.n_kv_heads * n * M - 1] = -1;
    return hipSuccess;
}
hipError_t launch_graph_norm(const Shape &sh, const void *, const int32_t *, int n, unsigned long long *best, hipStream_t)
{
    ++g_launches;
    for (int g = 0; g < sh.n_kv_heads; ++g) best[g] = (1ull << 32) | (0xFFFFFFFFu - (uint32_t)(n / 2)); // token n / 2
    return hipSuccess;
}
hipError_t launch_diprs(const Shape &sh, const DeviceViews &dv, const void *q, const int32_t *nbr, int n_idx, int M,
                        const int32_t *k0s, int l0, float beta, uint2 *clist, int64_t cap, uint32_t *visited, int64_t vis_words,
                        int32_t *c_lens, int32_t *, int32_t *, int64_t, int, hipStream_t)
{
    ++g_launches;
    const ReqDesc d = dv.desc.in;
    EXPECT(dv.desc.n == 1 && q && nbr && k0s && clist && visited && c_lens && l0 >= 0 && beta >= 0.f && M >= 1);
    EXPECT(n_idx <= d.n && cap >= n_idx && vis_words * 32 >= d.n && d.head_stride >= d.n);
    for (int g = 0; g < sh.n_kv_heads; ++g) EXPECT(k0s[g] >= 0 && k0s[g] < n_idx);
    // the areas one head's walk may write lie inside the scratch memory: touch their ends
    clist[(size_t)sh.n_q_heads * cap - 1] = make_uint2(0u, 0u);
    visited[(size_t)sh.n_q_heads * vis_words - 1] = 0u;
    c_lens[sh.n_q_heads - 1] = 0;
    return hipSuccess;
}

} // namespace alaya
