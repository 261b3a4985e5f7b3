// Host side of the C ABI declared in include/alaya.h: argument checks, the page allocator and page
// table, per-call descriptors, launch shapes, event timing.  No device memory is allocated here.
#include "../../include/alaya.h"
#include "../../include/alaya_debug.h"
#include "alaya_internal.h"

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <string>
#include <vector>

using namespace alaya;

static_assert(sizeof(alaya_cache_config) == 56 && sizeof(alaya_sparse_params) == 88, "C ABI struct layout");

namespace {

thread_local std::string g_err;

// Scratch memory for alaya_sparse_attn_static, the entry point for callers that cannot allocate: one
// array per GPU, in the library's own device image, held until the process ends.  In host code the
// array's name is only a stand-in for the symbol: every use of the memory goes through the address that
// hipGetSymbolAddress returns for the current device.
constexpr size_t kStaticScratchBytes = ALAYA_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
char *g_static_scratch[kMaxDevices]; // per device: address of that device's copy of `scratch`, once looked up

int fail(int code, const char *fmt, ...)
{
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    g_err = buf;
    return code;
}

int fail_hip(hipError_t e, const char *what)
{
    return fail(ALAYA_E_DEVICE, "%s: %s", what, hipGetErrorString(e));
}

constexpr int kRing = 16;          // descriptor slots in pinned host memory
constexpr int kProfPairs = 1024;   // event pairs before a forced harvest
constexpr int kTargetGroups = 2048;

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

bool cfg_ok(const alaya_cache_config *c)
{
    if (!c) return false;
    if (c->head_dim != 64 && c->head_dim != 128) return false;
    if (c->page_tokens != kPageTokens) return false;
    if (c->dtype != ALAYA_BF16 && c->dtype != ALAYA_F32) return false;
    if (c->n_kv_heads <= 0 || c->n_q_heads <= 0 || c->n_q_heads % c->n_kv_heads) return false;
    const int G = c->n_q_heads / c->n_kv_heads;
    if (G != 1 && G != 2 && G != 4 && G != 8) return false;
    if (c->max_seqs <= 0 || c->max_batch <= 0 || c->max_tokens_per_seq <= 0 || c->max_batch_tokens <= 0) return false;
    if (c->n_phys_pages <= 0 || c->n_phys_pages > INT32_MAX / kPageTokens) return false; // V-pool row numbers are int32
    if (c->max_tokens_per_seq > (int64_t)INT32_MAX - 64) return false; // token ids are int32
    const int64_t mpps = (c->max_tokens_per_seq + kPageTokens - 1) / kPageTokens;
    if (mpps * c->max_seqs > INT32_MAX) return false;                 // page-table offsets are int32
    return true;
}

// The cache's own device memory: the page table.
struct Layout {
    size_t page_table, total;
    int64_t mpps; // max pages per sequence
};

Layout make_layout(const alaya_cache_config &c)
{
    Layout L{};
    L.mpps = (c.max_tokens_per_seq + kPageTokens - 1) / kPageTokens;
    L.page_table = 0;
    L.total = align_up((size_t)L.mpps * c.max_seqs * sizeof(int32_t), 256);
    return L;
}

// Scratch memory of one attention call (nothing in it outlives the call, except that the words between
// zero_begin and zero_end are zero from one call to the next): survivor blocks, selected tokens,
// statistics, partial results.  Sized by the largest call it must serve.
struct Scratch {
    size_t desc, blocks, sel_scores, sel_ids, sel_rows, zero_begin, hist, head_maxkey, sample_max, fail, zero_end, tau,
        tau_safe, head_M, counts, partials, status, dbg_total, pg_ids, pg_scores, pg_counts, pg_M, pmask, visited, samp, total;
    int64_t samp_pages;  // capacity of the sample pass's score area, in pages
    int64_t visited_words; // capacity of the DIPRS visited bits, 32-bit words
    int64_t pg_elems;    // capacity of the chosen-page arrays of the coarse index
    int64_t pmask_bytes; // capacity of its page mask
    int64_t block_words; // capacity of the survivor blocks, 8-byte words
    int64_t sel_elems;   // capacity of each selected-token array
    int64_t max_tiles;   // full-attention tiles
};

// Survivor-block words that a call of `pages` pages in `batch` requests can need with cp pages per wavefront.
int64_t block_words_for(int64_t pages, int64_t batch, int n_kv_heads, int G, int cp)
{
    const int64_t tiles = (pages + (int64_t)kScoreWaves * cp - 1) / ((int64_t)kScoreWaves * cp) + batch;
    return block_area_words(tiles, n_kv_heads, G, (int64_t)kScoreWaves * cp * kPageTokens * G);
}

Scratch make_scratch(int n_q_heads, int n_kv_heads, int head_dim, int64_t max_batch, int64_t max_batch_tokens)
{
    Scratch S{};
    const int G = n_q_heads / n_kv_heads;
    const int64_t pages = max_batch_tokens / kPageTokens + max_batch;
    S.block_words = 0;
    for (int cp = 1; cp <= kMaxPagesPerWave && cp * G <= 16; cp *= 2)
        S.block_words = std::max(S.block_words, block_words_for(pages, max_batch, n_kv_heads, G, cp));
    S.sel_elems = (int64_t)n_q_heads * (max_batch_tokens + (int64_t)(kPageTokens + kScorePad) * max_batch);
    S.max_tiles = kTargetGroups / n_kv_heads + 1 + max_batch;
    const size_t heads = (size_t)max_batch * n_q_heads;
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o = align_up(o + bytes, 256); return at; };
    S.desc = take((size_t)max_batch * 2 * sizeof(ReqDesc)); // token-level and page-level descriptors
    S.blocks = take((size_t)S.block_words * sizeof(uint2));
    S.sel_scores = take((size_t)S.sel_elems * sizeof(float));
    S.sel_ids = take((size_t)S.sel_elems * sizeof(int32_t));
    S.sel_rows = take((size_t)S.sel_elems * sizeof(int32_t));
    S.zero_begin = o;
    S.hist = take(heads * kHistBins * sizeof(uint32_t));
    S.head_maxkey = take(heads * sizeof(uint32_t));
    S.sample_max = take(heads * kMaxSlots * sizeof(uint32_t));
    S.fail = take((heads + 1) * sizeof(uint32_t)); // + the any-head word
    S.zero_end = o;
    S.tau = take(heads * sizeof(uint32_t));
    S.tau_safe = take(heads * sizeof(uint32_t));
    S.head_M = take(heads * sizeof(float));
    S.counts = take(heads * sizeof(int32_t));
    const size_t sparse_slots = heads * kMaxSplits;
    const size_t full_slots = (size_t)S.max_tiles * n_q_heads;
    S.partials = take((sparse_slots > full_slots ? sparse_slots : full_slots) * (head_dim + 2) * sizeof(float));
    S.status = take(256);
    S.dbg_total = take(256);
    // coarse index: the chosen pages of every head, and one byte per (KV head, page)
    S.pg_elems = (int64_t)n_q_heads * (pages + (int64_t)kPageTokens * max_batch);
    S.pg_ids = take((size_t)S.pg_elems * sizeof(int32_t));
    S.pg_scores = take((size_t)S.pg_elems * sizeof(float));
    S.pg_counts = take(heads * sizeof(int32_t));
    S.pg_M = take(heads * sizeof(float));
    S.pmask_bytes = (int64_t)n_kv_heads * (pages + 4 * max_batch);
    S.pmask = take((size_t)S.pmask_bytes);
    // DIPRS: one visited bit per (query head, token)
    S.visited_words = (int64_t)n_q_heads * ((max_batch_tokens + 31) / 32 + 8 * max_batch);
    S.visited = take((size_t)S.visited_words * sizeof(uint32_t));
    // scores of the sample pass's pages: every S-th page, S >= kSampScoresMinStride, of every request
    S.samp_pages = pages / kSampScoresMinStride + max_batch;
    S.samp = take((size_t)S.samp_pages * n_q_heads * kPageTokens * sizeof(float));
    S.total = o;
    return S;
}

} // namespace

struct alaya_cache {
    alaya_cache_config cfg;
    Layout L;
    Scratch S;                       // layout of the bound scratch memory
    char *ws;                        // the cache's own device memory (page table)
    char *scratch_mem;               // bound scratch memory, or null
    void *k_pool, *v_pool;
    void *rep_pool;                  // block representatives of the coarse index, or null
    DeviceViews dv;
    // host bookkeeping
    std::vector<int32_t> free_pages; // stack: back() is handed out next
    std::vector<int64_t> seq_len;
    int32_t *h_page_table;           // pinned when a device is present
    bool h_page_table_pinned;
    ReqDesc *h_desc;                 // pinned ring [kRing][max_batch]
    hipEvent_t ring_ev[kRing];
    bool ring_used[kRing];
    int ring_pos;
    bool scratch_ready;              // the must-be-zero words of the bound scratch were cleared by this cache
    int tune_ppw, tune_splits, tune_batch, tune_noprune;
    int estimate_mode; // alaya_debug_estimate
    int diprs_lds_limit; // alaya_debug_diprs_lds
    int last_B, last_tiles_b;        // of the last sparse call, for the inspection hooks
    int64_t last_pages_a, last_pages_b; // pages of the last sparse call scored by the sample / the main pass
    // profiling
    bool prof;
    std::vector<hipEvent_t> ev;      // 2 * kProfPairs, created on demand
    int ev_slot[kProfPairs];
    int ev_n;
    double sum_ms[ALAYA_N_KERNEL_SLOTS];
    int64_t launches[ALAYA_N_KERNEL_SLOTS];
};

namespace {

int harvest(alaya_cache *c)
{
    for (int i = 0; i < c->ev_n; ++i) {
        hipError_t e = hipEventSynchronize(c->ev[2 * i + 1]);
        if (e != hipSuccess) return fail_hip(e, "hipEventSynchronize");
        float ms = 0.f;
        e = hipEventElapsedTime(&ms, c->ev[2 * i], c->ev[2 * i + 1]);
        if (e != hipSuccess) return fail_hip(e, "hipEventElapsedTime");
        c->sum_ms[c->ev_slot[i]] += ms;
        c->launches[c->ev_slot[i]] += 1;
    }
    c->ev_n = 0;
    return ALAYA_OK;
}

// Brackets one or more launches with events when profiling is on; with `attach` the events are not
// recorded here but handed to ONE launch (begin() / end()), which attaches them to its dispatch.
struct Timed {
    alaya_cache *c;
    hipStream_t st;
    int idx;
    bool attach;
    hipEvent_t begin() const { return idx >= 0 ? c->ev[2 * idx] : nullptr; }
    hipEvent_t end() const { return idx >= 0 ? c->ev[2 * idx + 1] : nullptr; }
    Timed(alaya_cache *c_, int slot, hipStream_t st_, bool attach_ = false) : c(c_), st(st_), idx(-1), attach(attach_)
    {
        if (!c->prof) return;
        if (c->ev_n == kProfPairs && harvest(c) != ALAYA_OK) return;
        if (c->ev.empty()) {
            c->ev.resize(2 * kProfPairs);
            for (auto &e : c->ev)
                if (hipEventCreate(&e) != hipSuccess) { c->ev.clear(); return; }
        }
        idx = c->ev_n++;
        c->ev_slot[idx] = slot;
        if (!attach) (void)hipEventRecord(c->ev[2 * idx], st);
    }
    ~Timed()
    {
        if (idx >= 0 && !attach) (void)hipEventRecord(c->ev[2 * idx + 1], st);
    }
};

// Points the device views at a scratch area laid out as S.
void bind_views(DeviceViews &dv, const Scratch &S, char *base)
{
    dv.desc.mem = (const ReqDesc *)(base + S.desc);
    dv.blocks = (uint2 *)(base + S.blocks);
    dv.sel_scores = (float *)(base + S.sel_scores);
    dv.sel_ids = (int32_t *)(base + S.sel_ids);
    dv.sel_rows = (int32_t *)(base + S.sel_rows);
    dv.hist = (uint32_t *)(base + S.hist);
    dv.head_maxkey = (uint32_t *)(base + S.head_maxkey);
    dv.sample_max = (uint32_t *)(base + S.sample_max);
    dv.fail = (uint32_t *)(base + S.fail);
    dv.any_fail = dv.fail + (S.zero_end - S.fail) / sizeof(uint32_t) - 1; // the last word of the cleared range
    dv.tau = (uint32_t *)(base + S.tau);
    dv.tau_safe = (uint32_t *)(base + S.tau_safe);
    dv.head_M = (float *)(base + S.head_M);
    dv.counts = (int32_t *)(base + S.counts);
    dv.partials = (float *)(base + S.partials);
    dv.status = (int32_t *)(base + S.status);
    dv.pmask = (const uint8_t *)(base + S.pmask);
    dv.repairs = (uint32_t *)(base + S.dbg_total + 8);
    dv.samp = (float *)(base + S.samp);
}

// Clears what must be zero before a scratch area's first use: statistics, repair marks, status.
hipError_t clear_scratch(const Scratch &S, char *base, hipStream_t st)
{
    hipError_t e = launch_fill_u32((uint32_t *)(base + S.zero_begin), (S.zero_end - S.zero_begin) / sizeof(uint32_t), 0u, st);
    if (e == hipSuccess) e = launch_fill_u32((uint32_t *)(base + S.status), 1, 0u, st);
    if (e == hipSuccess) e = launch_fill_u32((uint32_t *)(base + S.dbg_total), 4, 0u, st);
    return e;
}

int need_scratch(alaya_cache *c, hipStream_t st)
{
    if (!c->scratch_mem) return fail(ALAYA_E_INVAL, "no scratch memory bound to this cache (alaya_bind_scratch)");
    if (c->scratch_ready) return ALAYA_OK;
    const hipError_t e = clear_scratch(c->S, c->scratch_mem, st);
    if (e != hipSuccess) return fail_hip(e, "scratch initialisation");
    c->scratch_ready = true;
    return ALAYA_OK;
}

// Reserve the next descriptor slot; waits only if the copy issued kRing calls ago is still pending.
int ring_acquire(alaya_cache *c, int B, ReqDesc **slot, int *idx)
{
    const int i = c->ring_pos;
    if (c->ring_used[i]) {
        hipError_t e = hipEventSynchronize(c->ring_ev[i]);
        if (e != hipSuccess) return fail_hip(e, "hipEventSynchronize(descriptor ring)");
    }
    if (B > kInlineDescs && !c->ring_ev[i]) { // (normally created with the cache)
        hipError_t e = hipEventCreateWithFlags(&c->ring_ev[i], hipEventDisableTiming);
        if (e != hipSuccess) { c->ring_ev[i] = nullptr; return fail_hip(e, "hipEventCreate"); }
    }
    *slot = c->h_desc + (size_t)i * 2 * c->cfg.max_batch; // room for two sets of descriptors
    *idx = i;
    return ALAYA_OK;
}

// Hands the descriptors in ring slot idx to the kernels launched after this: in their arguments for a
// call of one request, through an asynchronous copy into `dev` (device memory) otherwise.
int ring_publish(alaya_cache *c, DeviceViews &dv, int idx, int B, hipStream_t st, bool two_sets = false)
{
    const ReqDesc *src = c->h_desc + (size_t)idx * 2 * c->cfg.max_batch;
    dv.desc.n = B;
    if (B <= kInlineDescs) {
        dv.desc.in = src[0];
        return ALAYA_OK; // the slot is free again at once
    }
    hipError_t e = hipMemcpyAsync((void *)dv.desc.mem, src, (size_t)B * (two_sets ? 2 : 1) * sizeof(ReqDesc),
                                  hipMemcpyHostToDevice, st);
    if (e != hipSuccess) return fail_hip(e, "descriptor copy");
    e = hipEventRecord(c->ring_ev[idx], st);
    if (e != hipSuccess) return fail_hip(e, "hipEventRecord");
    c->ring_used[idx] = true;
    c->ring_pos = (idx + 1) % kRing;
    return ALAYA_OK;
}

// Checks shared by both attention calls.
int check_call(alaya_cache *c, const int32_t *seqs, int B, int n_q_heads, const void *q, const float *out,
               int64_t *total_pages, int64_t *total_tokens)
{
    if (!c) return fail(ALAYA_E_INVAL, "null cache handle");
    if (!seqs || !q || !out) return fail(ALAYA_E_INVAL, "null seqs, q or out");
    if (B <= 0 || B > c->cfg.max_batch) return fail(ALAYA_E_INVAL, "batch %d outside 1..%d", B, c->cfg.max_batch);
    if (n_q_heads != c->cfg.n_q_heads)
        return fail(ALAYA_E_INVAL, "n_q_heads %d differs from the cache's %d", n_q_heads, c->cfg.n_q_heads);
    int64_t pages = 0, toks = 0;
    for (int b = 0; b < B; ++b) {
        if (seqs[b] < 0 || seqs[b] >= c->cfg.max_seqs)
            return fail(ALAYA_E_INVAL, "request %d: sequence id %d outside 0..%d", b, seqs[b], c->cfg.max_seqs - 1);
        const int64_t n = c->seq_len[seqs[b]];
        if (n <= 0) return fail(ALAYA_E_EMPTY, "request %d: sequence %d holds no tokens", b, seqs[b]);
        pages += (n + kPageTokens - 1) / kPageTokens;
        toks += n;
    }
    if (toks > c->cfg.max_batch_tokens)
        return fail(ALAYA_E_NOMEM, "call covers %lld tokens, the cache was configured for %lld", (long long)toks,
                    (long long)c->cfg.max_batch_tokens);
    *total_pages = pages;
    *total_tokens = toks;
    return ALAYA_OK;
}

} // namespace

extern "C" {

const char *alaya_last_error(void) { return g_err.c_str(); }

size_t alaya_pool_bytes(const alaya_cache_config *cfg)
{
    if (!cfg_ok(cfg)) return 0;
    return (size_t)cfg->n_phys_pages * cfg->n_kv_heads * kPageTokens * cfg->head_dim *
           (cfg->dtype == ALAYA_BF16 ? 2 : 4);
}

size_t alaya_workspace_bytes(const alaya_cache_config *cfg)
{
    if (!cfg_ok(cfg)) return 0;
    return make_layout(*cfg).total;
}

size_t alaya_scratch_bytes(const alaya_cache_config *cfg)
{
    if (!cfg_ok(cfg)) return 0;
    return make_scratch(cfg->n_q_heads, cfg->n_kv_heads, cfg->head_dim, cfg->max_batch, cfg->max_batch_tokens).total;
}

int alaya_create_cache(alaya_cache **out, const alaya_cache_config *cfg, void *k_pool, void *v_pool,
                       const int32_t *phys_page_order, void *workspace, size_t workspace_bytes)
{
    if (!out) return fail(ALAYA_E_INVAL, "null out pointer");
    *out = nullptr;
    if (!cfg_ok(cfg)) return fail(ALAYA_E_INVAL, "invalid cache configuration");
    if (!k_pool || !v_pool || !workspace) return fail(ALAYA_E_INVAL, "null pool or workspace");
    if (((uintptr_t)k_pool | (uintptr_t)v_pool | (uintptr_t)workspace) & 255)
        return fail(ALAYA_E_INVAL, "pools and workspace must be 256-byte aligned");
    const Layout L = make_layout(*cfg);
    if (workspace_bytes < L.total)
        return fail(ALAYA_E_NOMEM, "workspace has %zu bytes, %zu needed", workspace_bytes, L.total);
    const int64_t np = cfg->n_phys_pages;
    std::vector<int32_t> order((size_t)np);
    if (phys_page_order) {
        std::vector<char> seen((size_t)np, 0);
        for (int64_t i = 0; i < np; ++i) {
            const int32_t p = phys_page_order[i];
            if (p < 0 || p >= np || seen[(size_t)p]) return fail(ALAYA_E_INVAL, "phys_page_order is not a permutation");
            seen[(size_t)p] = 1;
            order[(size_t)i] = p;
        }
    } else {
        for (int64_t i = 0; i < np; ++i) order[(size_t)i] = (int32_t)i;
    }
    alaya_cache *c = new (std::nothrow) alaya_cache();
    if (!c) return fail(ALAYA_E_NOMEM, "host allocation failed");
    c->cfg = *cfg;
    c->L = L;
    c->S = Scratch{};
    c->ws = (char *)workspace;
    c->scratch_mem = nullptr;
    c->k_pool = k_pool;
    c->v_pool = v_pool;
    c->rep_pool = nullptr;
    c->dv = DeviceViews{};
    c->dv.fused = FusedAppend{nullptr, nullptr, nullptr, nullptr};
    c->dv.page_table = (const int32_t *)(c->ws + L.page_table);
    c->dv.k_pool = k_pool;
    c->dv.v_pool = v_pool;
    c->free_pages.assign(order.rbegin(), order.rend()); // back() == first page of the order
    c->seq_len.assign((size_t)cfg->max_seqs, 0);
    const size_t pt_bytes = (size_t)L.mpps * cfg->max_seqs * sizeof(int32_t);
    const size_t ring_bytes = (size_t)kRing * 2 * cfg->max_batch * sizeof(ReqDesc);
    // Pinned host memory lets the table and descriptor copies run asynchronously.  Without a device
    // (host-only use: argument and allocator checks) plain memory serves.
    void *p = nullptr;
    if (hipHostMalloc(&p, pt_bytes + ring_bytes, hipHostMallocDefault) == hipSuccess) {
        c->h_page_table_pinned = true;
    } else {
        (void)hipGetLastError();
        p = malloc(pt_bytes + ring_bytes);
        c->h_page_table_pinned = false;
        if (!p) { delete c; return fail(ALAYA_E_NOMEM, "host allocation failed"); }
    }
    c->h_page_table = (int32_t *)p;
    c->h_desc = (ReqDesc *)((char *)p + pt_bytes);
    for (int i = 0; i < kRing; ++i) {
        c->ring_ev[i] = nullptr;
        c->ring_used[i] = false;
        // (with a device: now, so that no later call has to create one; without: on first use)
        if (c->h_page_table_pinned && hipEventCreateWithFlags(&c->ring_ev[i], hipEventDisableTiming) != hipSuccess) {
            (void)hipGetLastError();
            c->ring_ev[i] = nullptr;
        }
    }
    c->ring_pos = 0;
    c->scratch_ready = false;
    c->tune_ppw = 0;
    c->tune_splits = 0;
    c->tune_batch = 0;
    c->tune_noprune = 0;
    c->estimate_mode = 0;
    c->diprs_lds_limit = 0;
    c->last_B = c->last_tiles_b = 0;
    c->last_pages_a = c->last_pages_b = 0;
    c->prof = false;
    c->ev_n = 0;
    for (int i = 0; i < ALAYA_N_KERNEL_SLOTS; ++i) { c->sum_ms[i] = 0.0; c->launches[i] = 0; }
    *out = c;
    return ALAYA_OK;
}

int alaya_bind_scratch(alaya_cache *c, void *scratch, size_t scratch_bytes)
{
    if (!c) return fail(ALAYA_E_INVAL, "null cache handle");
    if (!scratch) { // unbind
        c->scratch_mem = nullptr;
        c->scratch_ready = false;
        return ALAYA_OK;
    }
    if ((uintptr_t)scratch & 255) return fail(ALAYA_E_INVAL, "scratch memory must be 256-byte aligned");
    const Scratch S = make_scratch(c->cfg.n_q_heads, c->cfg.n_kv_heads, c->cfg.head_dim, c->cfg.max_batch,
                                   c->cfg.max_batch_tokens);
    if (scratch_bytes < S.total)
        return fail(ALAYA_E_NOMEM, "scratch has %zu bytes, %zu needed", scratch_bytes, S.total);
    c->S = S;
    c->scratch_mem = (char *)scratch;
    c->scratch_ready = false;
    bind_views(c->dv, S, c->scratch_mem);
    return ALAYA_OK;
}

size_t alaya_rep_bytes(const alaya_cache_config *cfg)
{
    if (!cfg_ok(cfg)) return 0;
    return (size_t)cfg->n_phys_pages * cfg->n_kv_heads * 2 * cfg->head_dim * (cfg->dtype == ALAYA_BF16 ? 2 : 4);
}

int alaya_bind_reps(alaya_cache *c, void *rep_pool, size_t rep_bytes)
{
    if (!c) return fail(ALAYA_E_INVAL, "null cache handle");
    if (!rep_pool) return fail(ALAYA_E_INVAL, "null representative pool");
    if ((uintptr_t)rep_pool & 255) return fail(ALAYA_E_INVAL, "representative pool must be 256-byte aligned");
    if (rep_bytes < alaya_rep_bytes(&c->cfg))
        return fail(ALAYA_E_NOMEM, "representative pool has %zu bytes, %zu needed", rep_bytes, alaya_rep_bytes(&c->cfg));
    for (int64_t n : c->seq_len)
        if (n > 0) return fail(ALAYA_E_INVAL, "bind the representative pool while every sequence is empty");
    c->rep_pool = rep_pool;
    return ALAYA_OK;
}

int alaya_destroy_cache(alaya_cache *c)
{
    if (!c) return fail(ALAYA_E_INVAL, "null cache handle");
    for (int i = 0; i < kRing; ++i)
        if (c->ring_ev[i]) { (void)hipEventSynchronize(c->ring_ev[i]); (void)hipEventDestroy(c->ring_ev[i]); }
    for (auto &e : c->ev) (void)hipEventDestroy(e);
    if (c->h_page_table_pinned) (void)hipHostFree(c->h_page_table);
    else free(c->h_page_table);
    delete c;
    return ALAYA_OK;
}

int64_t alaya_seq_len(const alaya_cache *c, int seq)
{
    if (!c || seq < 0 || seq >= c->cfg.max_seqs) { fail(ALAYA_E_INVAL, "bad handle or sequence id"); return -1; }
    return c->seq_len[(size_t)seq];
}

int alaya_reset_seq(alaya_cache *c, int seq)
{
    if (!c || seq < 0 || seq >= c->cfg.max_seqs) return fail(ALAYA_E_INVAL, "bad handle or sequence id");
    const int64_t pages = (c->seq_len[(size_t)seq] + kPageTokens - 1) / kPageTokens;
    const int32_t *row = c->h_page_table + (size_t)seq * c->L.mpps;
    for (int64_t i = pages - 1; i >= 0; --i) c->free_pages.push_back(row[i]);
    c->seq_len[(size_t)seq] = 0;
    return ALAYA_OK;
}

int alaya_append_kv(alaya_cache *c, int seq, const void *k, const void *v, int64_t t, void *stream)
{
    if (!c) return fail(ALAYA_E_INVAL, "null cache handle");
    if (seq < 0 || seq >= c->cfg.max_seqs) return fail(ALAYA_E_INVAL, "sequence id %d outside 0..%d", seq, c->cfg.max_seqs - 1);
    if (t < 0) return fail(ALAYA_E_INVAL, "negative token count");
    if (t == 0) return ALAYA_OK;
    if (!k || !v) return fail(ALAYA_E_INVAL, "null k or v");
    const int64_t n_old = c->seq_len[(size_t)seq], n_new = n_old + t;
    if (n_new > c->cfg.max_tokens_per_seq)
        return fail(ALAYA_E_NOMEM, "sequence %d would hold %lld tokens, limit %lld", seq, (long long)n_new,
                    (long long)c->cfg.max_tokens_per_seq);
    const int64_t have = (n_old + kPageTokens - 1) / kPageTokens, want = (n_new + kPageTokens - 1) / kPageTokens;
    const int64_t take = want - have;
    if (take > (int64_t)c->free_pages.size())
        return fail(ALAYA_E_NOMEM, "page pool exhausted: %lld pages needed, %zu free", (long long)take, c->free_pages.size());
    hipStream_t st = (hipStream_t)stream;
    int32_t *row = c->h_page_table + (size_t)seq * c->L.mpps;
    for (int64_t i = 0; i < take; ++i) {
        row[have + i] = c->free_pages.back();
        c->free_pages.pop_back();
    }
    auto rollback = [&]() {
        for (int64_t i = take - 1; i >= 0; --i) c->free_pages.push_back(row[have + i]);
    };
    int32_t *d_row = (int32_t *)c->dv.page_table + (size_t)seq * c->L.mpps;
    if (take > 0) {
        hipError_t e = hipMemcpyAsync(d_row + have, row + have, (size_t)take * sizeof(int32_t), hipMemcpyHostToDevice, st);
        if (e != hipSuccess) { rollback(); return fail_hip(e, "page table copy"); }
    }
    const Shape sh{c->cfg.dtype, c->cfg.head_dim, c->cfg.n_q_heads, c->cfg.n_kv_heads};
    hipError_t e;
    {
        Timed tm(c, 5, st);
        e = launch_append(sh, d_row, c->k_pool, c->v_pool, k, v, n_old, t, st);
    }
    if (e != hipSuccess) { rollback(); return fail_hip(e, "append launch"); }
    if (c->rep_pool) { // coarse index: the representatives of the pages this append touched
        const int first = (int)(n_old / kPageTokens);
        e = launch_reps_range(sh, d_row, c->k_pool, c->rep_pool, first, (int)(want - first), n_new, st);
        if (e != hipSuccess) { rollback(); return fail_hip(e, "representative update launch"); }
    }
    c->seq_len[(size_t)seq] = n_new;
    return ALAYA_OK;
}

namespace {

// Host side of a decode step's append: checks, then takes a page for every listed sequence that starts
// a new one and sends the new page-table entries.  Lengths are left as they are; `taken` lists the
// sequences that got a page, for step_rollback.
int step_reserve(alaya_cache *c, const int32_t *seqs, int B, hipStream_t st, std::vector<int32_t> &taken)
{
    size_t need = 0;
    for (int b = 0; b < B; ++b) {
        if (seqs[b] < 0 || seqs[b] >= c->cfg.max_seqs)
            return fail(ALAYA_E_INVAL, "entry %d: sequence id %d outside 0..%d", b, seqs[b], c->cfg.max_seqs - 1);
        for (int a = 0; a < b; ++a)
            if (seqs[a] == seqs[b]) return fail(ALAYA_E_INVAL, "sequence %d is listed twice", seqs[b]);
        const int64_t n_old = c->seq_len[(size_t)seqs[b]];
        if (n_old + 1 > c->cfg.max_tokens_per_seq)
            return fail(ALAYA_E_NOMEM, "sequence %d would hold %lld tokens, limit %lld", seqs[b],
                        (long long)(n_old + 1), (long long)c->cfg.max_tokens_per_seq);
        if (n_old % kPageTokens == 0) ++need;
    }
    if (need > c->free_pages.size())
        return fail(ALAYA_E_NOMEM, "page pool exhausted: %zu pages needed, %zu free", need, c->free_pages.size());
    for (int b = 0; b < B; ++b) {
        const int s = seqs[b];
        const int64_t n_old = c->seq_len[(size_t)s];
        if (n_old % kPageTokens != 0) continue;
        int32_t *row = c->h_page_table + (size_t)s * c->L.mpps;
        row[n_old / kPageTokens] = c->free_pages.back();
        c->free_pages.pop_back();
        taken.push_back(s);
        hipError_t e = hipMemcpyAsync((int32_t *)c->dv.page_table + (size_t)s * c->L.mpps + n_old / kPageTokens,
                                      row + n_old / kPageTokens, sizeof(int32_t), hipMemcpyHostToDevice, st);
        if (e != hipSuccess) return fail_hip(e, "page table copy");
    }
    return ALAYA_OK;
}

// Gives the pages of a failed step back; `back` = 1 if the lengths already count the new token.
void step_rollback(alaya_cache *c, const std::vector<int32_t> &taken, int back)
{
    for (size_t i = taken.size(); i-- > 0;) {
        const int s = taken[i];
        c->free_pages.push_back(c->h_page_table[(size_t)s * c->L.mpps + (c->seq_len[(size_t)s] - back) / kPageTokens]);
    }
}

// The append kernel for one new token per listed sequence; `back` as above.  A batch needs the bound
// scratch memory for its descriptors.
int step_launch_append(alaya_cache *c, const int32_t *seqs, int B, const void *k, const void *v, int back,
                       hipStream_t st)
{
    if (B > kInlineDescs && !c->scratch_mem)
        return fail(ALAYA_E_INVAL, "no scratch memory bound to this cache (alaya_bind_scratch)");
    ReqDesc *hd;
    int slot;
    int rc = ring_acquire(c, B, &hd, &slot);
    if (rc != ALAYA_OK) return rc;
    for (int b = 0; b < B; ++b) {
        std::memset(&hd[b], 0, sizeof(ReqDesc));
        hd[b].pt_off = (int32_t)((int64_t)seqs[b] * c->L.mpps);
        hd[b].n = (int32_t)(c->seq_len[(size_t)seqs[b]] - back);
    }
    rc = ring_publish(c, c->dv, slot, B, st);
    if (rc != ALAYA_OK) return rc;
    const Shape sh{c->cfg.dtype, c->cfg.head_dim, c->cfg.n_q_heads, c->cfg.n_kv_heads};
    hipError_t e;
    {
        Timed tm(c, 5, st);
        e = launch_append_step(sh, c->dv, c->k_pool, c->v_pool, k, v, B, st);
        if (e == hipSuccess && c->rep_pool) e = launch_reps_step(sh, c->dv, c->rep_pool, B, st);
    }
    if (e != hipSuccess) return fail_hip(e, "append launch");
    return ALAYA_OK;
}

// Scratch memory other than the one bound to the cache: views into it and its layout.
struct ScratchUse {
    DeviceViews *dv;
    const Scratch *S;
};

int sparse_attn_impl(alaya_cache *c, const ScratchUse *use, const int32_t *seqs, int B, int n_q_heads,
                     const void *q, const alaya_sparse_params *p, float *out, void *stream, const void *fused_k,
                     const void *fused_v, bool *appended);

} // namespace

int alaya_append_kv_step(alaya_cache *c, const int32_t *seqs, int B, const void *k, const void *v, void *stream)
{
    if (!c) return fail(ALAYA_E_INVAL, "null cache handle");
    if (!seqs || !k || !v) return fail(ALAYA_E_INVAL, "null seqs, k or v");
    if (B <= 0 || B > c->cfg.max_batch) return fail(ALAYA_E_INVAL, "batch %d outside 1..%d", B, c->cfg.max_batch);
    if (B == 1) return alaya_append_kv(c, seqs[0], k, v, 1, stream);
    hipStream_t st = (hipStream_t)stream;
    // From step_reserve on pages are taken; on a failure they go back and no length changes.
    std::vector<int32_t> taken;
    int rc = step_reserve(c, seqs, B, st, taken);
    if (rc == ALAYA_OK) rc = step_launch_append(c, seqs, B, k, v, 0, st);
    if (rc != ALAYA_OK) { step_rollback(c, taken, 0); return rc; }
    for (int b = 0; b < B; ++b) c->seq_len[(size_t)seqs[b]] += 1;
    return ALAYA_OK;
}

int alaya_decode_step(alaya_cache *c, const int32_t *seqs, int B, int n_q_heads, const void *k, const void *v,
                      const void *q, const alaya_sparse_params *p, float *out, void *stream)
{
    if (!c) return fail(ALAYA_E_INVAL, "null cache handle");
    if (!seqs || !k || !v) return fail(ALAYA_E_INVAL, "null seqs, k or v");
    if (B <= 0 || B > c->cfg.max_batch) return fail(ALAYA_E_INVAL, "batch %d outside 1..%d", B, c->cfg.max_batch);
    // (with a visible prefix the new token may lie outside what the query sees; with a coarse index the
    // append also updates the page's representatives: nothing to fuse, the two calls are made in turn)
    if ((p && p->n_visible) || c->rep_pool) {
        const int rc = alaya_append_kv_step(c, seqs, B, k, v, stream);
        return rc != ALAYA_OK ? rc : alaya_sparse_attn(c, seqs, B, n_q_heads, q, p, out, stream);
    }
    hipStream_t st = (hipStream_t)stream;
    std::vector<int32_t> taken;
    int rc = step_reserve(c, seqs, B, st, taken);
    if (rc != ALAYA_OK) { step_rollback(c, taken, 0); return rc; }
    for (int b = 0; b < B; ++b) c->seq_len[(size_t)seqs[b]] += 1;
    // The attention call's sample pass writes the new rows.  If the call is turned down before that
    // launch, the plain append kernel writes them: the token is appended either way.
    bool appended = false;
    rc = sparse_attn_impl(c, nullptr, seqs, B, n_q_heads, q, p, out, stream, k, v, &appended);
    if (!appended) {
        const int rc2 = step_launch_append(c, seqs, B, k, v, 1, st);
        if (rc2 != ALAYA_OK) { // nothing was written: undo the step
            step_rollback(c, taken, 1);
            for (int b = 0; b < B; ++b) c->seq_len[(size_t)seqs[b]] -= 1;
            return rc2;
        }
    }
    return rc;
}

int alaya_sparse_attn(alaya_cache *c, const int32_t *seqs, int B, int n_q_heads, const void *q,
                      const alaya_sparse_params *p, float *out, void *stream)
{
    bool appended = false;
    return sparse_attn_impl(c, nullptr, seqs, B, n_q_heads, q, p, out, stream, nullptr, nullptr, &appended);
}

namespace {

// alaya_sparse_attn; with fused_k / fused_v (a decode step whose lengths already count the new token)
// the sample pass also writes each request's newest key and value rows.  *appended is set once that
// launch is out.  use: null = the scratch memory bound to the cache; otherwise a scratch area that the
// caller of this function has made ready (cleared), with room for this call.
int sparse_attn_impl(alaya_cache *c, const ScratchUse *use, const int32_t *seqs, int B, int n_q_heads,
                     const void *q, const alaya_sparse_params *p, float *out, void *stream, const void *fused_k,
                     const void *fused_v, bool *appended)
{
    int64_t total_pages = 0, total_tokens = 0;
    int rc = check_call(c, seqs, B, n_q_heads, q, out, &total_pages, &total_tokens);
    if (rc != ALAYA_OK) return rc;
    if (!p) return fail(ALAYA_E_INVAL, "null params");
    if (p->mode != ALAYA_TOPK && p->mode != ALAYA_DIPR) return fail(ALAYA_E_INVAL, "unknown mode %d", p->mode);
    if (!(p->scale >= 0.f) || std::isinf(p->scale)) return fail(ALAYA_E_INVAL, "scale must be finite and >= 0");
    if (p->mode == ALAYA_TOPK) {
        if (!p->topk) return fail(ALAYA_E_INVAL, "top-k mode needs topk[]");
        for (int b = 0; b < B; ++b)
            if (p->topk[b] <= 0) return fail(ALAYA_E_INVAL, "request %d: k = %d must be positive", b, p->topk[b]);
    } else {
        if (!p->beta) return fail(ALAYA_E_INVAL, "DIPR mode needs beta[]");
        for (int b = 0; b < B; ++b)
            if (!(p->beta[b] >= 0.f)) return fail(ALAYA_E_INVAL, "request %d: beta must be >= 0", b);
    }
    if (p->out_ids && p->ids_stride <= 0) return fail(ALAYA_E_INVAL, "out_ids given with ids_stride <= 0");
    if (p->window_init < 0 || p->window_last < 0)
        return fail(ALAYA_E_INVAL, "window sizes %d + %d must be >= 0", p->window_init, p->window_last);
    if (p->n_visible)
        for (int b = 0; b < B; ++b)
            if (p->n_visible[b] <= 0 || p->n_visible[b] > c->seq_len[(size_t)seqs[b]])
                return fail(ALAYA_E_INVAL, "request %d: n_visible = %d outside 1..%lld", b, p->n_visible[b],
                            (long long)c->seq_len[(size_t)seqs[b]]);
    const bool coarse = p->coarse_pages != nullptr;
    if (coarse) {
        if (p->mode != ALAYA_TOPK) return fail(ALAYA_E_INVAL, "the coarse index answers top-k queries only");
        if (!c->rep_pool) return fail(ALAYA_E_INVAL, "no representative pool bound to this cache (alaya_bind_reps)");
        for (int b = 0; b < B; ++b)
            if (p->coarse_pages[b] <= 0)
                return fail(ALAYA_E_INVAL, "request %d: coarse_pages = %d must be positive", b, p->coarse_pages[b]);
        if (p->out_pages && p->pages_stride <= 0) return fail(ALAYA_E_INVAL, "out_pages given with pages_stride <= 0");
        if (fused_k) return fail(ALAYA_E_INVAL, "internal: a fused append cannot go with the coarse index");
    }
    if (!use && !c->scratch_mem) return fail(ALAYA_E_INVAL, "no scratch memory bound to this cache (alaya_bind_scratch)");
    DeviceViews &dv = use ? *use->dv : c->dv;
    const Scratch &S = use ? *use->S : c->S;

    hipStream_t st = (hipStream_t)stream;
    const int G = n_q_heads / c->cfg.n_kv_heads;
    // Pages per wavefront of the main pass (= pages per survivor block / 4): one, or four where that still leaves
    // about 3072 workgroups or more (from 384K tokens of 8 KV heads on): the selection likes few, large blocks (at 1M
    // one page per wavefront makes 4096 blocks per KV head and costs it 47 us more), and the pass itself runs as fast
    // either way for one long request (us with 1 / 2 / 4: 512K tokens 164 / 164 / 163, 768K 241 / 243 / 242; a 256K
    // threshold query is faster with one: 78 against 88).  A call of many requests runs faster with one (the batched
    // workload: 758 against 776 us, selection 53 against 46 us), as long as none of them is so long that the
    // selection pays more than that.  The staging area of a workgroup (4 * cp * 64 * G pairs) stays within 32 KiB.
    int cp = 1;
    {
        int64_t max_pages = 0;
        for (int b = 0; b < B; ++b) {
            const int64_t n = p->n_visible ? (int64_t)p->n_visible[b] : c->seq_len[(size_t)seqs[b]];
            max_pages = std::max(max_pages, (n + kPageTokens - 1) / kPageTokens);
        }
        int want = c->tune_ppw;
        if (want <= 0) {
            want = total_pages * c->cfg.n_kv_heads / (kScoreWaves * kMaxPagesPerWave) >= 3072 ? kMaxPagesPerWave : 1;
            if (B > 1 && max_pages <= 4096) want = 1;
        }
        if (want > kMaxPagesPerWave) want = kMaxPagesPerWave;
        if (c->tune_ppw > 0) { // (the tests ask for every value)
            while (2 * cp <= want && 2 * cp * G <= 16) cp *= 2;
        } else if (want * G <= 16) {
            cp = want;
        }
    }
    // The attend pass: `splits` workgroups per head in the grid, of which a head with `count` selected tokens
    // uses clamp(count / rows, min_splits, splits); rows = 128 tokens per workgroup (what the gather of 256-byte
    // rows runs fastest with), 256 in calls of thousands of workgroups (they gather as fast, and the merge has
    // half as many partial results to read); more workgroups when the call is small.  The grid is sized for the
    // longest list the call can have (a threshold set's size is not known here: 4096 is assumed, and a longer
    // list gets more tokens per workgroup).  The launchers get min_splits | log2(rows) << 16.
    int splits = c->tune_splits, min_splits = c->tune_splits | (7 << 16);
    if (splits <= 0) {
        int kmax = 4096;
        if (p->mode == ALAYA_TOPK) {
            kmax = 1;
            for (int b = 0; b < B; ++b) kmax = p->topk[b] > kmax ? p->topk[b] : kmax;
        }
        const int64_t kw = (int64_t)kmax + p->window_init + p->window_last;
        const int rows_log2 = (int64_t)B * n_q_heads * ((kw + 127) / 128) >= 8192 ? 8 : 7;
        const int per = (int)std::min<int64_t>((kw + (1 << rows_log2) - 1) >> rows_log2, kMaxSplits);
        const int fill = (int)std::min<int64_t>((kw + 31) / 32, (512 + B * n_q_heads - 1) / (B * n_q_heads));
        splits = std::min(std::max(std::max(per, fill), 1), kMaxSplits);
        min_splits = std::min(std::max(fill, 1), splits) | (rows_log2 << 16);
    }

    ReqDesc *hd;
    int slot;
    rc = ring_acquire(c, B, &hd, &slot);
    if (rc != ALAYA_OK) return rc;
    int tiles = 0, tiles_b = 0, tiles_p = 0;
    int64_t pg_off = 0, pm_off = 0;
    ReqDesc *hp = hd + B; // page-level descriptors of the coarse index (the ring slot holds max_batch >= B more)
    const bool estimate = c->estimate_mode >= 0;
    bool any_est = false;
    int64_t pages_a = 0, pages_all = 0, samp_off = 0, pages_handed = 0;
    int64_t off = 0;
    for (int b = 0; b < B; ++b) {
        // the tokens this query sees: the whole sequence, or the prefix asked for
        const int64_t n = p->n_visible ? (int64_t)p->n_visible[b] : c->seq_len[(size_t)seqs[b]];
        const int64_t pages = (n + kPageTokens - 1) / kPageTokens;
        ReqDesc &d = hd[b];
        std::memset(&d, 0, sizeof d);
        d.pt_off = (int32_t)((int64_t)seqs[b] * c->L.mpps);
        d.n = (int32_t)n;
        d.head_stride = (int32_t)(pages * kPageTokens + kScorePad);
        d.w0 = (int32_t)((int64_t)p->window_init < n ? p->window_init : n);
        d.w1 = (int32_t)((int64_t)p->window_last < n ? p->window_last : n);
        d.nwin = (int32_t)((int64_t)d.w0 + d.w1 < n ? d.w0 + d.w1 : n);
        const int64_t n_out = n - d.nwin; // tokens outside the window: what top-k ranks
        d.k = p->mode == ALAYA_TOPK ? (int32_t)((int64_t)p->topk[b] < n_out ? p->topk[b] : n_out) : 0;
        d.beta = p->mode == ALAYA_DIPR ? p->beta[b] : 0.f;
        d.score_off = off;
        if (pages > 131072)
            return fail(ALAYA_E_INVAL, "request %d: %lld tokens exceed the selection layout (%lld)", b, (long long)n,
                        (long long)131072 * kPageTokens);
        d.n_pages = (int32_t)pages;
        // Sample stride S: the sample pass reads n / S keys, the main pass writes about k * S survivors
        // (guaranteed bound).  Powers of two, at most 32.
        int S = 1;
        d.k_est = 0;
        // Through the coarse index top-k ranks the tokens of the P pages a head chose: at least cand of them,
        // whichever pages those are.  With fewer than k such tokens possible, everything found is taken and
        // nothing is pruned; otherwise the estimated bound works as it does on the whole sequence, with the
        // chosen pages in the place of all pages.
        int64_t rank_pages = pages, rank_tokens = n_out;
        if (coarse) {
            rank_pages = std::min<int64_t>(p->coarse_pages[b], pages);
            rank_tokens = kPageTokens * (rank_pages - 1) + 1 - d.nwin;
            d.flags = 1;
        }
        if (!c->tune_noprune && pages >= 4) {
            // (never when top-k takes every token outside the window: nothing checks the bound then)
            // (through the coarse index only when the chosen pages hold more tokens than the selection keeps in
            // registers: below that a bound saves the selection nothing and costs a sample pass)
            if (p->mode == ALAYA_TOPK && estimate && d.k >= 512 && d.k < rank_tokens && rank_pages >= 64 &&
                (!coarse || rank_pages * kPageTokens > 16384)) {
                d.flags = 0; // at least k tokens can be ranked: fewer survivors means that the bound was too high
                if (coarse) d.est_cand = (int32_t)(rank_pages * kPageTokens);
                // Estimated bound: a 1-in-S sample holds about mu = k / S of the k best
                // scores, so its (mu + 6 sqrt(mu) + 8)-th largest score lies below the true threshold
                // unless the sample is far from representative - which the selection detects and
                // repairs.  The main pass then writes about k (1 + 6 / sqrt(mu)) survivors whatever S
                // is, so S only has to keep mu at 64 or more.
                while (S < 32 && d.k / (2 * S) >= 64) S *= 2;
                while (S > 1 && rank_pages / S < 2) S /= 2;
                const double mu = (double)d.k / S;
                d.k_est = c->estimate_mode == 2 ? 1 : (int32_t)(mu + 6.0 * std::sqrt(mu) + 8.0);
                if (d.k_est > d.k) d.k_est = d.k;
                if (S > 1) any_est = true; else d.k_est = 0;
                // a sample-pass workgroup (four sampled pages) adds at most this much to one bucket: four
                // times what all buckets down to the estimate's rank get from four pages on average, 8 at least
                const int64_t sampled_pages = (rank_pages + S - 1) / S;
                d.hist_cap = (int32_t)std::max<int64_t>(8, (16 * (int64_t)d.k_est + sampled_pages - 1) / sampled_pages);
            } else if (coarse) {
                // (no bound: every token of a chosen page survives)
            } else if (p->mode == ALAYA_TOPK) {
                while (S < 32 && (int64_t)(2 * S) * (2 * S) * d.k <= n && (int64_t)2 * S * d.k * 2 <= n) S *= 2;
                while (S > 1 && pages / S < 2) S /= 2;
            } else {
                // (the sample only has to come close to the maximum; its pages are handed to the main pass scored, so a
                // denser sample costs little: 256K tokens, beta = 4: 135 -> 126 us with 8 instead of 16, beta = 2 the same)
                S = pages >= 8192 ? 32 : 8;
                while (S > 1 && pages / S < 2) S /= 2;
            }
        }
        if (d.k_est == 0) d.hist_cap = 1 << 16; // guaranteed bound only: the counts must be exact
        d.sample_stride = S;
        // DIPR with a window (Sec. 7.1): the maximum mostly sits among the window's tokens, so the pages
        // that hold them join the sample and seed the bound.
        d.xf = 0;
        d.xb = d.n_pages;
        if (p->mode == ALAYA_DIPR && S > 1 && d.nwin > 0) {
            d.xf = std::min(d.n_pages, (d.w0 + kPageTokens - 1) / kPageTokens);
            d.xb = std::max(d.xf, d.w1 > 0 ? (d.n - d.w1) / kPageTokens : d.n_pages);
        }
        // a decode step: the page of the newest token belongs to the sample pass, which writes that token
        if (fused_k) d.xb = std::max(d.xf, std::min(d.xb, (d.n - 1) / kPageTokens));
        const int every = S > 1 ? (d.n_pages + S - 1) / S : 0;
        if (!coarse) {
            d.pm_off = samp_off; // the main pass takes the scores of these pages from the sample pass
            if (S >= kSampScoresMinStride) { samp_off += every; pages_handed += every; }
        }
        auto not_every = [S](int a, int b) { return S > 1 ? (b - a) - ((b + S - 1) / S - (a + S - 1) / S) : b - a; }; // in [a, b)
        pages_a += every + not_every(0, d.xf) + not_every(d.xb, d.n_pages);
        const int n_a = every + d.xf + (d.n_pages - d.xb); // wavefronts of the sample pass
        d.tile_start = tiles;
        d.tileb_start = tiles_b;
        d.ntiles_b = (int32_t)((d.n_pages + (int64_t)kScoreWaves * cp - 1) / ((int64_t)kScoreWaves * cp));
        tiles += (n_a + kScoreWaves - 1) / kScoreWaves; // one page per wavefront
        tiles_b += d.ntiles_b;
        if (coarse) {
            d.pm_off = pm_off;
            d.pm_stride = (int32_t)((pages + 3) / 4 * 4);
            pm_off += (int64_t)c->cfg.n_kv_heads * d.pm_stride;
            ReqDesc &e = hp[b]; // the same request seen as a sequence of pages: n, k count pages
            std::memset(&e, 0, sizeof e);
            e.pt_off = d.pt_off;
            e.n = (int32_t)pages;
            e.n_pages = (int32_t)((pages + kPageTokens - 1) / kPageTokens);
            e.k = (int32_t)((int64_t)p->coarse_pages[b] < pages ? p->coarse_pages[b] : pages);
            e.head_stride = (int32_t)(pages + kPageTokens);
            e.score_off = pg_off;
            e.sample_stride = 1;
            e.pm_off = d.pm_off; // (the block-score kernel clears the mask)
            e.pm_stride = d.pm_stride;
            e.tileb_start = tiles_p;
            e.ntiles_b = (int32_t)((pages + 255) / 256);
            tiles_p += e.ntiles_b;
            pg_off += (int64_t)n_q_heads * e.head_stride;
        }
        pages_all += pages;
        off += (int64_t)n_q_heads * d.head_stride;
    }
    {
        // selection workgroups take the requests in descending order of what they have to go through
        std::vector<int> order((size_t)B);
        for (int b = 0; b < B; ++b) order[(size_t)b] = b;
        std::stable_sort(order.begin(), order.end(), [&](int x, int y) { return hd[x].n_pages > hd[y].n_pages; });
        for (int b = 0; b < B; ++b) {
            hd[b].flags = (hd[b].flags & 1) | (order[(size_t)b] << 8);
            if (coarse) hp[b].flags = (hp[b].flags & 1) | (order[(size_t)b] << 8);
        }
    }
    const int64_t block_full = (int64_t)kScoreWaves * cp * kPageTokens * G;
    if (off > S.sel_elems) return fail(ALAYA_E_NOMEM, "scratch too small for the selected-token arrays");
    if (samp_off > S.samp_pages) return fail(ALAYA_E_NOMEM, "scratch too small for the sample pass's scores");
    if (block_area_words(tiles_b, c->cfg.n_kv_heads, G, block_full) > S.block_words)
        return fail(ALAYA_E_NOMEM, "scratch too small for the survivor blocks");
    // page level: a block holds the scores of 256 pages
    const int64_t block_full_p = (int64_t)256 * G;
    if (coarse && (block_area_words(tiles_p, c->cfg.n_kv_heads, G, block_full_p) > S.block_words || pg_off > S.pg_elems ||
                   pm_off > S.pmask_bytes))
        return fail(ALAYA_E_NOMEM, "scratch too small for the coarse index");
    if (!use) {
        rc = need_scratch(c, st);
        if (rc != ALAYA_OK) return rc;
    }
    rc = ring_publish(c, dv, slot, B, st, coarse);
    if (rc != ALAYA_OK) return rc;
    dv.area = make_block_area(dv.blocks, tiles_b, c->cfg.n_kv_heads, G, block_full);
    if (!use) {
        c->last_B = B;
        c->last_tiles_b = tiles_b;
        c->last_pages_a = pages_a;
        c->last_pages_b = pages_all - pages_handed; // (pages whose keys the main pass reads)
    }

    const Shape sh{c->cfg.dtype, c->cfg.head_dim, n_q_heads, c->cfg.n_kv_heads};
    const float scale = p->scale > 0.f ? p->scale : 1.0f / std::sqrt((float)c->cfg.head_dim);
    // (a launch that fails below may leave the statistics half-filled: scratch_ready is dropped so that
    // the next call clears them again)
    hipError_t e;
    char *sbase = (char *)dv.sel_scores - S.sel_scores; // the scratch area the views point into
    if (coarse) {
        // Coarse index: block scores of every page (and a cleared page mask) -> the best pages of every head
        // (the selection kernel, over pages), marked in one byte per (KV head, page) for the main pass.
        Timed tm(c, 7, st);
        DescArgs pd = dv.desc;
        pd.mem = dv.desc.mem + B;
        pd.in = hp[0];
        int32_t *pg_ids = (int32_t *)(sbase + S.pg_ids), *pg_counts = (int32_t *)(sbase + S.pg_counts);
        e = launch_coarse_score(sh, dv, pd, B, q, c->rep_pool, tiles_p,
                                make_block_area(dv.blocks, tiles_p, c->cfg.n_kv_heads, G, block_full_p),
                                (uint8_t *)(sbase + S.pmask), st);
        const SelectIO pio{pd, make_block_area(dv.blocks, tiles_p, c->cfg.n_kv_heads, G, block_full_p), pg_ids, (float *)(sbase + S.pg_scores), nullptr, pg_counts,
                           (float *)(sbase + S.pg_M), (uint32_t *)(sbase + S.pmask)};
        if (e == hipSuccess)
            e = launch_select(sh, dv, pio, B, ALAYA_TOPK, false, c->tune_batch, p->out_pages, nullptr, p->pages_stride, st);
        if (e != hipSuccess) { c->scratch_ready = false; return fail_hip(e, "coarse index launch"); }
    }
    {
        Timed tm(c, 6, st);
        if (fused_k) dv.fused = FusedAppend{(uint4 *)c->k_pool, (uint4 *)c->v_pool, (const uint4 *)fused_k, (const uint4 *)fused_v};
        e = launch_sample(sh, dv, B, q, tiles, p->mode, coarse, st);
        dv.fused = FusedAppend{nullptr, nullptr, nullptr, nullptr};
        if (e == hipSuccess) *appended = fused_k != nullptr && tiles > 0;
        if (e == hipSuccess) e = launch_tau(sh, dv, B, p->mode, st);
    }
    if (e != hipSuccess) { c->scratch_ready = false; return fail_hip(e, "sample scoring launch"); }
    {
        Timed tm(c, 0, st, true); // the roofline kernel: timed by its own dispatch
        e = launch_score(sh, dv, B, q, tiles_b, cp, false, p->mode, coarse, st, tm.begin(), tm.end());
    }
    if (e != hipSuccess) { c->scratch_ready = false; return fail_hip(e, "score launch"); }
    {
        Timed tm(c, 1, st);
        const SelectIO io{dv.desc, dv.area, dv.sel_ids, dv.sel_scores, dv.sel_rows, dv.counts, dv.head_M, nullptr};
        e = launch_select(sh, dv, io, B, p->mode, false, c->tune_batch, p->out_ids, p->out_counts, p->ids_stride, st);
        // repair of the heads whose estimated bound lost tokens (normally none: both launches are idle)
        if (e == hipSuccess && any_est) e = launch_score(sh, dv, B, q, tiles_b, cp, true, p->mode, coarse, st);
        if (e == hipSuccess && any_est)
            e = launch_select(sh, dv, io, B, p->mode, true, c->tune_batch, p->out_ids, p->out_counts, p->ids_stride, st);
    }
    if (e != hipSuccess) { c->scratch_ready = false; return fail_hip(e, "select launch"); }
    {
        Timed tm(c, 2, st);
        e = launch_attend(sh, dv, B, scale, splits, min_splits, st);
    }
    if (e != hipSuccess) return fail_hip(e, "attend launch");
    { Timed tm(c, 3, st); e = launch_combine(sh, dv, B, splits, min_splits, 0, 0, out, st); }
    if (e != hipSuccess) return fail_hip(e, "combine launch");
    return ALAYA_OK;
}

} // namespace

int alaya_sparse_attn_static(alaya_cache *c, const int32_t *seqs, int B, int n_q_heads, const void *q,
                             const alaya_sparse_params *p, float *out, void *stream)
{
    int64_t total_pages = 0, total_tokens = 0;
    int rc = check_call(c, seqs, B, n_q_heads, q, out, &total_pages, &total_tokens);
    if (rc != ALAYA_OK) return rc;
    // The layout for exactly this call; it must fit the array.
    int64_t tokens = total_tokens;
    if (p && p->n_visible) {
        tokens = 0;
        for (int b = 0; b < B; ++b) tokens += p->n_visible[b] > 0 ? p->n_visible[b] : 0;
    }
    const Scratch S = make_scratch(n_q_heads, c->cfg.n_kv_heads, c->cfg.head_dim, B, tokens);
    if (S.total > kStaticScratchBytes)
        return fail(ALAYA_E_NOMEM, "call needs %zu bytes of scratch memory, the built-in area holds %zu "
                    "(alaya_sparse_attn with bound scratch memory has no such limit)", S.total, kStaticScratchBytes);
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail_hip(e, "hipGetDevice");
    if (dev < 0 || dev >= kMaxDevices) return fail(ALAYA_E_DEVICE, "device %d outside 0..%d", dev, kMaxDevices - 1);
    if (!g_static_scratch[dev]) {
        char *ptr = nullptr;
        e = hipGetSymbolAddress((void **)&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr) return fail_hip(e, "hipGetSymbolAddress(scratch)");
        g_static_scratch[dev] = ptr;
    }
    char *base = g_static_scratch[dev];
    hipStream_t st = (hipStream_t)stream;
    // The array keeps what the call before this one left (of any cache, with any layout): clear what must start at zero.
    e = clear_scratch(S, base, st);
    if (e != hipSuccess) return fail_hip(e, "scratch clear");
    if (B > kInlineDescs && !c->ring_ev[c->ring_pos])
        return fail(ALAYA_E_DEVICE, "descriptor ring not initialised (no device when the cache was created)");
    DeviceViews dv = c->dv; // page table and pools; the rest is pointed at the array
    bind_views(dv, S, base);
    const ScratchUse use{&dv, &S};
    const bool prof = c->prof; // (the profiling mode creates events on first use: not here)
    c->prof = false;
    bool appended = false;
    rc = sparse_attn_impl(c, &use, seqs, B, n_q_heads, q, p, out, stream, nullptr, nullptr, &appended);
    c->prof = prof;
    return rc;
}

// ---- fine-grained index and DIPRS ------------------------------------------------------------------

struct alaya_graph {
    alaya_cache *cache;
    int seq;
    int64_t n_idx;           // tokens of the sequence that the graph covers
    int degree;              // neighbours per key
    int32_t *nbr;            // DEVICE [n_kv_heads][n_idx][degree]
    unsigned long long *best; // DEVICE [n_kv_heads] (ordered norm << 32 | ~token) of the entry points
    int32_t *entry_dev;      // DEVICE [n_kv_heads]
    std::vector<int32_t> entry; // HOST copy
};

namespace {

int graph_args_ok(const alaya_cache *c, int seq, int degree)
{
    if (!c) return fail(ALAYA_E_INVAL, "null cache handle");
    if (seq < 0 || seq >= c->cfg.max_seqs) return fail(ALAYA_E_INVAL, "sequence id %d outside 0..%d", seq, c->cfg.max_seqs - 1);
    if (degree < 1 || degree > 64) return fail(ALAYA_E_INVAL, "degree %d outside 1..64", degree);
    if (c->cfg.dtype != ALAYA_BF16 || c->cfg.head_dim != 128)
        return fail(ALAYA_E_INVAL, "the graph index is built for bf16 caches of head_dim 128 only");
    if (c->seq_len[(size_t)seq] <= 0) return fail(ALAYA_E_EMPTY, "sequence %d holds no tokens", seq);
    return ALAYA_OK;
}

} // namespace

size_t alaya_graph_bytes(const alaya_cache *c, int seq, int degree)
{
    if (graph_args_ok(c, seq, degree) != ALAYA_OK) return 0;
    const int64_t n = c->seq_len[(size_t)seq];
    return align_up((size_t)c->cfg.n_kv_heads * (size_t)n * degree * sizeof(int32_t), 256) + 512;
}

size_t alaya_graph_build_bytes(const alaya_cache *c, int seq, int degree)
{
    if (graph_args_ok(c, seq, degree) != ALAYA_OK) return 0;
    return 256; // (the build keeps its working lists on chip; the argument is kept for builders that do not)
}

int alaya_graph_build(alaya_graph **out, alaya_cache *c, int seq, int degree, void *index_mem, size_t index_bytes,
                      void *build_mem, size_t build_bytes, void *stream)
{
    if (!out) return fail(ALAYA_E_INVAL, "null out pointer");
    *out = nullptr;
    int rc = graph_args_ok(c, seq, degree);
    if (rc != ALAYA_OK) return rc;
    if (!index_mem || !build_mem || (((uintptr_t)index_mem | (uintptr_t)build_mem) & 255))
        return fail(ALAYA_E_INVAL, "index and build memory must be given and 256-byte aligned");
    if (index_bytes < alaya_graph_bytes(c, seq, degree) || build_bytes < alaya_graph_build_bytes(c, seq, degree))
        return fail(ALAYA_E_NOMEM, "index or build memory too small");
    const int64_t n = c->seq_len[(size_t)seq];
    hipStream_t st = (hipStream_t)stream;
    alaya_graph *g = new (std::nothrow) alaya_graph();
    if (!g) return fail(ALAYA_E_NOMEM, "host allocation failed");
    g->cache = c;
    g->seq = seq;
    g->n_idx = n;
    g->degree = degree;
    g->nbr = (int32_t *)index_mem;
    char *tail = (char *)index_mem + align_up((size_t)c->cfg.n_kv_heads * (size_t)n * degree * sizeof(int32_t), 256);
    g->best = (unsigned long long *)tail;
    g->entry_dev = (int32_t *)(tail + 256);
    const Shape sh{c->cfg.dtype, c->cfg.head_dim, c->cfg.n_q_heads, c->cfg.n_kv_heads};
    const int32_t *pt_row = c->dv.page_table + (size_t)seq * c->L.mpps;
    hipError_t e = launch_graph_knn(sh, c->k_pool, pt_row, (int)n, degree, g->nbr, st);
    if (e == hipSuccess) e = launch_graph_norm(sh, c->k_pool, pt_row, (int)n, g->best, st);
    std::vector<unsigned long long> best((size_t)c->cfg.n_kv_heads);
    if (e == hipSuccess) e = hipMemcpyAsync(best.data(), g->best, best.size() * sizeof(unsigned long long), hipMemcpyDeviceToHost, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    if (e != hipSuccess) { delete g; return fail_hip(e, "graph build"); }
    g->entry.resize(best.size());
    for (size_t i = 0; i < best.size(); ++i) g->entry[i] = (int32_t)(0xFFFFFFFFu - (uint32_t)(best[i] & 0xFFFFFFFFull));
    e = hipMemcpyAsync(g->entry_dev, g->entry.data(), g->entry.size() * sizeof(int32_t), hipMemcpyHostToDevice, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    if (e != hipSuccess) { delete g; return fail_hip(e, "graph build"); }
    *out = g;
    return ALAYA_OK;
}

int alaya_graph_destroy(alaya_graph *g)
{
    if (!g) return fail(ALAYA_E_INVAL, "null graph handle");
    delete g;
    return ALAYA_OK;
}

int alaya_graph_info(const alaya_graph *g, int64_t *n_indexed, int32_t *degree, const int32_t **neighbours, int32_t *entry)
{
    if (!g) return fail(ALAYA_E_INVAL, "null graph handle");
    if (n_indexed) *n_indexed = g->n_idx;
    if (degree) *degree = g->degree;
    if (neighbours) *neighbours = g->nbr;
    if (entry) std::memcpy(entry, g->entry.data(), g->entry.size() * sizeof(int32_t));
    return ALAYA_OK;
}

int alaya_diprs_attn(alaya_cache *c, const alaya_graph *g, int n_q_heads, const void *q, float beta, int32_t l0,
                     const alaya_sparse_params *p, float *out, void *stream)
{
    if (!c || !g) return fail(ALAYA_E_INVAL, "null cache or graph handle");
    if (g->cache != c) return fail(ALAYA_E_INVAL, "the graph belongs to another cache");
    const int32_t seq = g->seq;
    int64_t total_pages = 0, total_tokens = 0;
    int rc = check_call(c, &seq, 1, n_q_heads, q, out, &total_pages, &total_tokens);
    if (rc != ALAYA_OK) return rc;
    if (!(beta >= 0.f)) return fail(ALAYA_E_INVAL, "beta must be >= 0");
    if (l0 < 0) return fail(ALAYA_E_INVAL, "capacity threshold l0 = %d must be >= 0", l0);
    if (p && (p->window_init < 0 || p->window_last < 0))
        return fail(ALAYA_E_INVAL, "window sizes %d + %d must be >= 0", p->window_init, p->window_last);
    if (p && (!(p->scale >= 0.f) || std::isinf(p->scale))) return fail(ALAYA_E_INVAL, "scale must be finite and >= 0");
    if (p && p->out_ids && p->ids_stride <= 0) return fail(ALAYA_E_INVAL, "out_ids given with ids_stride <= 0");
    if (!c->scratch_mem) return fail(ALAYA_E_INVAL, "no scratch memory bound to this cache (alaya_bind_scratch)");
    const int64_t n = c->seq_len[(size_t)seq];
    if (n < g->n_idx) return fail(ALAYA_E_INVAL, "the sequence is shorter (%lld) than its graph (%lld): it was reset", (long long)n, (long long)g->n_idx);
    hipStream_t st = (hipStream_t)stream;
    const int64_t pages = (n + kPageTokens - 1) / kPageTokens;
    ReqDesc d;
    std::memset(&d, 0, sizeof d);
    d.pt_off = (int32_t)((int64_t)seq * c->L.mpps);
    d.n = (int32_t)n;
    d.n_pages = (int32_t)pages;
    d.head_stride = (int32_t)(pages * kPageTokens + kScorePad);
    d.beta = beta;
    d.sample_stride = 1;
    // Tokens appended after the graph was built are not in it (Sec. 7.2 "Late Materialization for Index
    // Updating"): they belong to the window of last tokens, which is attended as it is.
    const int64_t w0 = p ? p->window_init : 0, w1 = std::max<int64_t>(p ? p->window_last : 0, n - g->n_idx);
    d.w0 = (int32_t)std::min(w0, n);
    d.w1 = (int32_t)std::min(w1, n);
    d.nwin = (int32_t)std::min<int64_t>((int64_t)d.w0 + d.w1, n);
    const int64_t cap = pages * kPageTokens, vis_words = (n + 31) / 32 + 8;
    if ((int64_t)n_q_heads * cap > c->S.block_words || (int64_t)n_q_heads * vis_words > c->S.visited_words ||
        (int64_t)n_q_heads * d.head_stride > c->S.sel_elems)
        return fail(ALAYA_E_NOMEM, "scratch too small for the DIPRS walk");
    rc = need_scratch(c, st);
    if (rc != ALAYA_OK) return rc;
    c->dv.desc.n = 1;
    c->dv.desc.in = d;
    const Shape sh{c->cfg.dtype, c->cfg.head_dim, n_q_heads, c->cfg.n_kv_heads};
    const float scale = p && p->scale > 0.f ? p->scale : 1.0f / std::sqrt((float)c->cfg.head_dim);
    uint32_t *visited = (uint32_t *)(c->scratch_mem + c->S.visited);
    int32_t *c_lens = (int32_t *)(c->scratch_mem + c->S.pg_counts);
    hipError_t e;
    {
        Timed tm(c, 1, st);
        e = launch_diprs(sh, c->dv, q, g->nbr, (int)g->n_idx, g->degree, g->entry_dev, l0, beta, c->dv.blocks, cap, visited,
                             vis_words, c_lens, p ? p->out_ids : nullptr, p ? p->out_counts : nullptr, p ? p->ids_stride : 0,
                             c->diprs_lds_limit, st);
    }
    if (e != hipSuccess) return fail_hip(e, "DIPRS launch");
    int splits = c->tune_splits > 0 ? c->tune_splits : 16;
    { Timed tm(c, 2, st); e = launch_attend(sh, c->dv, 1, scale, splits, splits | (7 << 16), st); }
    if (e != hipSuccess) return fail_hip(e, "attend launch");
    { Timed tm(c, 3, st); e = launch_combine(sh, c->dv, 1, splits, splits | (7 << 16), 0, 0, out, st); }
    if (e != hipSuccess) return fail_hip(e, "combine launch");
    c->last_B = 0; // (no survivor blocks to inspect after this call)
    c->last_tiles_b = 0;
    return ALAYA_OK;
}

int alaya_debug_diprs_lds(alaya_cache *c, int bytes)
{
    if (!c || bytes < 0) return fail(ALAYA_E_INVAL, "bad arguments");
    c->diprs_lds_limit = bytes;
    return ALAYA_OK;
}

int64_t alaya_debug_diprs_list(alaya_cache *c, int head, int32_t *ids, int64_t cap, void *stream)
{
    if (!c || !c->scratch_mem || head < 0 || head >= c->cfg.n_q_heads) { fail(ALAYA_E_INVAL, "bad arguments"); return -1; }
    hipStream_t st = (hipStream_t)stream;
    const ReqDesc &d = c->dv.desc.in;
    int32_t len = 0;
    hipError_t e = hipMemcpyAsync(&len, (int32_t *)(c->scratch_mem + c->S.pg_counts) + head, sizeof len, hipMemcpyDeviceToHost, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    if (e != hipSuccess) { fail_hip(e, "list length read"); return -1; }
    const int64_t m = len < cap ? len : cap;
    if (ids && m > 0) {
        std::vector<uint2> tmp((size_t)m);
        const int64_t stride = (int64_t)d.n_pages * kPageTokens;
        e = hipMemcpyAsync(tmp.data(), c->dv.blocks + (size_t)head * stride, (size_t)m * sizeof(uint2), hipMemcpyDeviceToHost, st);
        if (e == hipSuccess) e = hipStreamSynchronize(st);
        if (e != hipSuccess) { fail_hip(e, "list read"); return -1; }
        for (int64_t i = 0; i < m; ++i) ids[i] = (int32_t)tmp[(size_t)i].y;
    }
    return len;
}

int alaya_full_attn(alaya_cache *c, const int32_t *seqs, int B, int n_q_heads, const void *q, float scale_in,
                    float *out, void *stream)
{
    int64_t total_pages = 0, total_tokens = 0;
    int rc = check_call(c, seqs, B, n_q_heads, q, out, &total_pages, &total_tokens);
    if (rc != ALAYA_OK) return rc;
    if (!(scale_in >= 0.f) || std::isinf(scale_in)) return fail(ALAYA_E_INVAL, "scale must be finite and >= 0");
    if (!c->scratch_mem) return fail(ALAYA_E_INVAL, "no scratch memory bound to this cache (alaya_bind_scratch)");
    hipStream_t st = (hipStream_t)stream;
    int64_t ppt = (total_pages * c->cfg.n_kv_heads + kTargetGroups - 1) / kTargetGroups;
    ppt = (ppt + 3) / 4 * 4;
    if (ppt < 4) ppt = 4;

    ReqDesc *hd;
    int slot;
    rc = ring_acquire(c, B, &hd, &slot);
    if (rc != ALAYA_OK) return rc;
    int tiles = 0;
    for (int b = 0; b < B; ++b) {
        const int64_t n = c->seq_len[(size_t)seqs[b]];
        const int64_t pages = (n + kPageTokens - 1) / kPageTokens;
        ReqDesc &d = hd[b];
        std::memset(&d, 0, sizeof d);
        d.pt_off = (int32_t)((int64_t)seqs[b] * c->L.mpps);
        d.n = (int32_t)n;
        d.tile_start = tiles;
        d.sample_stride = 1;
        tiles += (int)((pages + ppt - 1) / ppt);
    }
    if (tiles > c->S.max_tiles) return fail(ALAYA_E_NOMEM, "scratch too small for the partial results");
    rc = need_scratch(c, st);
    if (rc != ALAYA_OK) return rc;
    rc = ring_publish(c, c->dv, slot, B, st);
    if (rc != ALAYA_OK) return rc;

    const Shape sh{c->cfg.dtype, c->cfg.head_dim, n_q_heads, c->cfg.n_kv_heads};
    const float scale = scale_in > 0.f ? scale_in : 1.0f / std::sqrt((float)c->cfg.head_dim);
    hipError_t e;
    { Timed tm(c, 4, st); e = launch_full_partial(sh, c->dv, B, q, scale, tiles, (int)ppt, st); }
    if (e != hipSuccess) return fail_hip(e, "full-attention launch");
    { Timed tm(c, 3, st); e = launch_combine(sh, c->dv, B, 0, 0, 1, (int)ppt, out, st); }
    if (e != hipSuccess) return fail_hip(e, "combine launch");
    return ALAYA_OK;
}

int alaya_poll_status(alaya_cache *c, void *stream)
{
    if (!c) return fail(ALAYA_E_INVAL, "null cache handle");
    if (!c->scratch_mem || !c->scratch_ready) return ALAYA_OK;
    hipStream_t st = (hipStream_t)stream;
    int32_t word = 0;
    hipError_t e = hipMemcpyAsync(&word, c->dv.status, sizeof word, hipMemcpyDeviceToHost, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    if (e != hipSuccess) return fail_hip(e, "status read");
    if (word) {
        e = launch_fill_u32((uint32_t *)c->dv.status, 1, 0u, st);
        if (e != hipSuccess) return fail_hip(e, "status clear");
        return fail(ALAYA_E_CAPACITY, "a selected set was larger than ids_stride; out_counts holds the true sizes");
    }
    return ALAYA_OK;
}

// ---- include/alaya_debug.h ---------------------------------------------------------------------

int alaya_set_profiling(alaya_cache *c, int enabled)
{
    if (!c) return fail(ALAYA_E_INVAL, "null cache handle");
    if (c->prof) {
        int rc = harvest(c);
        if (rc != ALAYA_OK) return rc;
    }
    c->prof = enabled != 0;
    if (c->prof)
        for (int i = 0; i < ALAYA_N_KERNEL_SLOTS; ++i) { c->sum_ms[i] = 0.0; c->launches[i] = 0; }
    return ALAYA_OK;
}

int alaya_kernel_times(alaya_cache *c, double *sum_ms, int64_t *launches, int n_slots)
{
    if (!c || !sum_ms || !launches || n_slots < 0 || n_slots > ALAYA_N_KERNEL_SLOTS)
        return fail(ALAYA_E_INVAL, "bad arguments");
    int rc = harvest(c);
    if (rc != ALAYA_OK) return rc;
    for (int i = 0; i < n_slots; ++i) { sum_ms[i] = c->sum_ms[i]; launches[i] = c->launches[i]; }
    return ALAYA_OK;
}

int alaya_debug_estimate(alaya_cache *c, int mode)
{
    if (!c) return fail(ALAYA_E_INVAL, "null cache handle");
    if (mode < -1 || mode > 2) return fail(ALAYA_E_INVAL, "estimate mode %d outside -1..2", mode);
    c->estimate_mode = mode;
    return ALAYA_OK;
}

int alaya_debug_pages(const alaya_cache *c, int64_t *sampled, int64_t *main_pass)
{
    if (!c || !sampled || !main_pass) return fail(ALAYA_E_INVAL, "bad arguments");
    *sampled = c->last_pages_a;
    *main_pass = c->last_pages_b;
    return ALAYA_OK;
}

int64_t alaya_debug_scores(alaya_cache *c, float *out, void *stream)
{
    if (!c) { fail(ALAYA_E_INVAL, "null cache handle"); return -1; }
    if (!c->scratch_mem || c->last_tiles_b <= 0) return 0;
    hipStream_t st = (hipStream_t)stream;
    unsigned long long *total = (unsigned long long *)(c->scratch_mem + c->S.dbg_total);
    hipError_t e = launch_fill_u32((uint32_t *)total, 2, 0u, st);
    const Shape sh{c->cfg.dtype, c->cfg.head_dim, c->cfg.n_q_heads, c->cfg.n_kv_heads};
    if (e == hipSuccess) e = launch_debug_scatter(sh, c->dv, c->last_B, c->last_tiles_b, out, total, st);
    unsigned long long h = 0;
    if (e == hipSuccess) e = hipMemcpyAsync(&h, total, sizeof h, hipMemcpyDeviceToHost, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    if (e != hipSuccess) { fail_hip(e, "survivor read"); return -1; }
    return (int64_t)h;
}

int64_t alaya_debug_repairs(alaya_cache *c, void *stream)
{
    if (!c) { fail(ALAYA_E_INVAL, "null cache handle"); return -1; }
    if (!c->scratch_mem || !c->scratch_ready) return 0;
    hipStream_t st = (hipStream_t)stream;
    uint32_t h = 0;
    hipError_t e = hipMemcpyAsync(&h, c->dv.repairs, sizeof h, hipMemcpyDeviceToHost, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    if (e == hipSuccess) e = launch_fill_u32(c->dv.repairs, 1, 0u, st);
    if (e != hipSuccess) { fail_hip(e, "repair counter read"); return -1; }
    return (int64_t)h;
}

int alaya_set_tuning(alaya_cache *c, int score_pages_per_wave, int attend_splits, int select_batch_blocks,
                     int write_all_scores)
{
    if (!c) return fail(ALAYA_E_INVAL, "null cache handle");
    if (score_pages_per_wave > 16 || attend_splits > kMaxSplits || select_batch_blocks > kSelBatch)
        return fail(ALAYA_E_INVAL, "knob out of range");
    c->tune_ppw = score_pages_per_wave > 0 ? score_pages_per_wave : 0;
    c->tune_splits = attend_splits > 0 ? attend_splits : 0;
    c->tune_batch = select_batch_blocks > 0 ? select_batch_blocks : 0;
    c->tune_noprune = write_all_scores > 0 ? 1 : 0;
    return ALAYA_OK;
}

} // extern "C"
