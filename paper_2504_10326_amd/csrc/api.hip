// Host side of the C ABI declared in include/alaya.h: argument checks, the page allocator and page
// table, per-call descriptors, launch shapes, event timing.  No device memory is allocated here.
#include "../../include/alaya.h"
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

static_assert(sizeof(alaya_cache_config) == 56 && sizeof(alaya_sparse_params) == 64, "C ABI struct layout");

namespace {

thread_local std::string g_err;

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
    if (c->n_phys_pages <= 0 || c->n_phys_pages > INT32_MAX) return false;
    if (c->max_tokens_per_seq > (int64_t)INT32_MAX - 64) return false; // token ids are int32
    const int64_t mpps = (c->max_tokens_per_seq + kPageTokens - 1) / kPageTokens;
    if (mpps * c->max_seqs > INT32_MAX) return false;                 // page-table offsets are int32
    return true;
}

struct Layout {
    size_t page_table, desc, cand, loc_scores, loc_ids, sel_scores, sel_ids, page_cnt, hist,
        head_maxkey, sample_max, fail, tau, tau_safe, seg_counts, head_M, head_info, counts, partials, status, total;
    int64_t mpps;        // max pages per sequence
    int64_t score_elems; // capacity of each per-token array
    int64_t max_tiles;   // full-attention tiles
    int64_t max_pages;   // pages over one call
};

Layout make_layout(const alaya_cache_config &c)
{
    Layout L{};
    L.mpps = (c.max_tokens_per_seq + kPageTokens - 1) / kPageTokens;
    L.score_elems = (int64_t)c.n_q_heads * (c.max_batch_tokens + (int64_t)(kPageTokens + kScorePad) * c.max_batch);
    L.max_tiles = kTargetGroups / c.n_kv_heads + 1 + c.max_batch;
    L.max_pages = c.max_batch_tokens / kPageTokens + c.max_batch;
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o = align_up(o + bytes, 256); return at; };
    L.page_table = take((size_t)L.mpps * c.max_seqs * sizeof(int32_t));
    L.desc = take((size_t)c.max_batch * sizeof(ReqDesc));
    L.cand = take((size_t)L.score_elems * sizeof(uint2));
    L.loc_scores = take((size_t)L.score_elems * sizeof(float));
    L.loc_ids = take((size_t)L.score_elems * sizeof(int32_t));
    L.sel_scores = take((size_t)L.score_elems * sizeof(float));
    L.sel_ids = take((size_t)L.score_elems * sizeof(int32_t));
    L.page_cnt = take((size_t)L.max_pages * c.n_q_heads * sizeof(int32_t));
    L.hist = take((size_t)c.max_batch * c.n_q_heads * kHistBins * sizeof(uint32_t));
    L.head_maxkey = take((size_t)c.max_batch * c.n_q_heads * sizeof(uint32_t));
    L.sample_max = take((size_t)c.max_batch * c.n_q_heads * kMaxSlots * sizeof(uint32_t));
    L.fail = take(((size_t)c.max_batch * c.n_q_heads + 1) * sizeof(uint32_t)); // + the any-head word
    L.tau = take((size_t)c.max_batch * c.n_q_heads * sizeof(uint32_t));
    L.tau_safe = take((size_t)c.max_batch * c.n_q_heads * sizeof(uint32_t));
    L.seg_counts = take((size_t)c.max_batch * c.n_q_heads * kMaxSegs * 2 * sizeof(int32_t));
    L.head_M = take((size_t)c.max_batch * c.n_q_heads * sizeof(float));
    L.head_info = take((size_t)c.max_batch * c.n_q_heads * 2 * sizeof(int32_t));
    L.counts = take((size_t)c.max_batch * c.n_q_heads * sizeof(int32_t));
    const size_t sparse_slots = (size_t)c.max_batch * c.n_q_heads * kMaxSplits;
    const size_t full_slots = (size_t)L.max_tiles * c.n_q_heads;
    L.partials = take((sparse_slots > full_slots ? sparse_slots : full_slots) * (c.head_dim + 2) * sizeof(float));
    L.status = take(256);
    L.total = o;
    return L;
}

} // namespace

struct alaya_cache {
    alaya_cache_config cfg;
    Layout L;
    char *ws;
    void *k_pool, *v_pool;
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
    bool dev_ready;
    int tune_ppw, tune_splits, tune_seg, tune_noprune;
    int estimate_mode; // alaya_debug_estimate
    int last_pages, last_heads;
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

int ensure_device(alaya_cache *c, hipStream_t st)
{
    if (c->dev_ready) return ALAYA_OK;
    // the histograms and the running maxima sit next to each other in the workspace: one fill
    const size_t nh = (size_t)(c->L.tau - c->L.hist) / sizeof(uint32_t);
    hipError_t e = launch_fill_u32(c->dv.hist, nh, 0u, st);
    if (e == hipSuccess) e = launch_fill_u32((uint32_t *)c->dv.status, 1, 0u, st);
    if (e != hipSuccess) return fail_hip(e, "workspace initialisation");
    c->dev_ready = true;
    return ALAYA_OK;
}

// Reserve the next descriptor slot; waits only if the copy issued kRing calls ago is still pending.
int ring_acquire(alaya_cache *c, ReqDesc **slot, int *idx)
{
    const int i = c->ring_pos;
    if (c->ring_used[i]) {
        hipError_t e = hipEventSynchronize(c->ring_ev[i]);
        if (e != hipSuccess) return fail_hip(e, "hipEventSynchronize(descriptor ring)");
    }
    *slot = c->h_desc + (size_t)i * c->cfg.max_batch;
    *idx = i;
    return ALAYA_OK;
}

// Hands the descriptors in ring slot idx to the kernels launched after this: in their arguments for a
// small call, through an asynchronous copy into the workspace otherwise.
int ring_publish(alaya_cache *c, int idx, int B, hipStream_t st)
{
    const ReqDesc *src = c->h_desc + (size_t)idx * c->cfg.max_batch;
    c->dv.desc.n = B;
    if (B <= kInlineDescs) {
        c->dv.desc.in = src[0];
        return ALAYA_OK; // the slot is free again at once
    }
    hipError_t e = hipMemcpyAsync((void *)c->dv.desc.mem, src,
                                  (size_t)B * sizeof(ReqDesc), hipMemcpyHostToDevice, st);
    if (e != hipSuccess) return fail_hip(e, "descriptor copy");
    e = hipEventRecord(c->ring_ev[idx], st);
    if (e != hipSuccess) return fail_hip(e, "hipEventRecord");
    c->ring_used[idx] = true;
    c->ring_pos = (idx + 1) % kRing;
    return ALAYA_OK;
}

// Checks shared by both attention calls; fills n[] with the sequence lengths.
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
        return fail(ALAYA_E_NOMEM, "call covers %lld tokens, workspace was sized for %lld", (long long)toks,
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
    c->ws = (char *)workspace;
    c->k_pool = k_pool;
    c->v_pool = v_pool;
    c->dv.desc.mem = (const ReqDesc *)(c->ws + L.desc);
    c->dv.desc.n = 0;
    c->dv.fused = FusedAppend{nullptr, nullptr, nullptr, nullptr};
    c->dv.page_table = (const int32_t *)(c->ws + L.page_table);
    c->dv.k_pool = k_pool;
    c->dv.v_pool = v_pool;
    c->dv.cand = (uint2 *)(c->ws + L.cand);
    c->dv.loc_scores = (float *)(c->ws + L.loc_scores);
    c->dv.loc_ids = (int32_t *)(c->ws + L.loc_ids);
    c->dv.sel_scores = (float *)(c->ws + L.sel_scores);
    c->dv.sel_ids = (int32_t *)(c->ws + L.sel_ids);
    c->dv.page_cnt = (int32_t *)(c->ws + L.page_cnt);
    c->dv.hist = (uint32_t *)(c->ws + L.hist);
    c->dv.head_maxkey = (uint32_t *)(c->ws + L.head_maxkey);
    c->dv.sample_max = (uint32_t *)(c->ws + L.sample_max);
    c->dv.fail = (uint32_t *)(c->ws + L.fail);
    c->dv.any_fail = c->dv.fail + (size_t)cfg->max_batch * cfg->n_q_heads;
    c->dv.tau = (uint32_t *)(c->ws + L.tau);
    c->dv.tau_safe = (uint32_t *)(c->ws + L.tau_safe);
    c->dv.seg_counts = (int32_t *)(c->ws + L.seg_counts);
    c->dv.head_info = (int32_t *)(c->ws + L.head_info);
    c->dv.head_M = (float *)(c->ws + L.head_M);
    c->dv.counts = (int32_t *)(c->ws + L.counts);
    c->dv.partials = (float *)(c->ws + L.partials);
    c->dv.status = (int32_t *)(c->ws + L.status);
    c->free_pages.assign(order.rbegin(), order.rend()); // back() == first page of the order
    c->seq_len.assign((size_t)cfg->max_seqs, 0);
    const size_t pt_bytes = (size_t)L.mpps * cfg->max_seqs * sizeof(int32_t);
    const size_t ring_bytes = (size_t)kRing * cfg->max_batch * sizeof(ReqDesc);
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
    for (int i = 0; i < kRing; ++i) { c->ring_ev[i] = nullptr; c->ring_used[i] = false; }
    c->ring_pos = 0;
    c->dev_ready = false;
    c->tune_ppw = 0;
    c->tune_splits = 0;
    c->tune_seg = 0;
    c->tune_noprune = 0;
    c->estimate_mode = 0;
    c->last_pages = c->last_heads = 0;
    c->last_pages_a = c->last_pages_b = 0;
    c->prof = false;
    c->ev_n = 0;
    for (int i = 0; i < ALAYA_N_KERNEL_SLOTS; ++i) { c->sum_ms[i] = 0.0; c->launches[i] = 0; }
    *out = c;
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
    int rc = ensure_device(c, st);
    if (rc != ALAYA_OK) { rollback(); return rc; }
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
    int rc = ensure_device(c, st);
    if (rc != ALAYA_OK) return rc;
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

// The append kernel for one new token per listed sequence; `back` as above.
int step_launch_append(alaya_cache *c, const int32_t *seqs, int B, const void *k, const void *v, int back,
                       hipStream_t st)
{
    ReqDesc *hd;
    int slot;
    int rc = ring_acquire(c, &hd, &slot);
    if (rc != ALAYA_OK) return rc;
    if (!c->ring_ev[slot]) {
        hipError_t e = hipEventCreateWithFlags(&c->ring_ev[slot], hipEventDisableTiming);
        if (e != hipSuccess) { c->ring_ev[slot] = nullptr; return fail_hip(e, "hipEventCreate"); }
    }
    for (int b = 0; b < B; ++b) {
        std::memset(&hd[b], 0, sizeof(ReqDesc));
        hd[b].pt_off = (int32_t)((int64_t)seqs[b] * c->L.mpps);
        hd[b].n = (int32_t)(c->seq_len[(size_t)seqs[b]] - back);
    }
    rc = ring_publish(c, slot, B, st);
    if (rc != ALAYA_OK) return rc;
    const Shape sh{c->cfg.dtype, c->cfg.head_dim, c->cfg.n_q_heads, c->cfg.n_kv_heads};
    hipError_t e;
    {
        Timed tm(c, 5, st);
        e = launch_append_step(sh, c->dv, c->k_pool, c->v_pool, k, v, B, st);
    }
    if (e != hipSuccess) return fail_hip(e, "append launch");
    return ALAYA_OK;
}

int sparse_attn_impl(alaya_cache *c, const int32_t *seqs, int B, int n_q_heads, const void *q,
                     const alaya_sparse_params *p, float *out, void *stream, const void *fused_k,
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
    if (p && p->n_visible) { // the new token may lie outside what the query sees: nothing to fuse
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
    rc = sparse_attn_impl(c, seqs, B, n_q_heads, q, p, out, stream, k, v, &appended);
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
    return sparse_attn_impl(c, seqs, B, n_q_heads, q, p, out, stream, nullptr, nullptr, &appended);
}

namespace {

// alaya_sparse_attn; with fused_k / fused_v (a decode step whose lengths already count the new token)
// the sample pass also writes each request's newest key and value rows.  *appended is set once that
// launch is out.
int sparse_attn_impl(alaya_cache *c, const int32_t *seqs, int B, int n_q_heads, const void *q,
                     const alaya_sparse_params *p, float *out, void *stream, const void *fused_k,
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

    hipStream_t st = (hipStream_t)stream;
    int ppw = c->tune_ppw; // pages per wavefront in the main scoring pass; chosen below if not given
    // pages per selection segment: about 512 segment workgroups in all, 128 to 2048 pages each
    int64_t seg_pages_want = c->tune_seg;
    if (seg_pages_want <= 0) {
        seg_pages_want = 128;
        while (seg_pages_want < kMaxSegPages && seg_pages_want * 512 < total_pages * n_q_heads) seg_pages_want *= 2;
    }
    int splits = c->tune_splits;
    if (splits <= 0) {
        // enough workgroups to fill the chip, and at most about 512 selected tokens per workgroup
        // (a threshold set's size is not known here: assume 4096)
        int kmax = 4096;
        if (p->mode == ALAYA_TOPK) {
            kmax = 1;
            for (int b = 0; b < B; ++b) kmax = p->topk[b] > kmax ? p->topk[b] : kmax;
        }
        const int fill = (2048 + B * n_q_heads - 1) / (B * n_q_heads);
        const int per = (int)(((int64_t)kmax + 511) / 512);
        splits = fill > per ? fill : per;
        if (splits < 1) splits = 1;
        if (splits > 32) splits = 32;
    }

    ReqDesc *hd;
    int slot;
    rc = ring_acquire(c, &hd, &slot);
    if (rc != ALAYA_OK) return rc;
    int tiles = 0, tiles_b = 0, segs = 0, all_pages = 0;
    // Large top-k calls filter with an estimated bound and pay two (normally idle) repair launches for
    // it; below about a quarter of a million tokens in the call the guaranteed bound is as fast.
    const bool estimate = c->estimate_mode > 0 || (c->estimate_mode == 0 && total_pages >= 4096);
    bool any_est = false;
    double survive = 0.0;
    int64_t pages_a = 0;
    int64_t off = 0;
    for (int b = 0; b < B; ++b) {
        // the tokens this query sees: the whole sequence, or the prefix asked for
        const int64_t n = p->n_visible ? (int64_t)p->n_visible[b] : c->seq_len[(size_t)seqs[b]];
        const int64_t pages = (n + kPageTokens - 1) / kPageTokens;
        ReqDesc &d = hd[b];
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
        if (pages > (int64_t)kMaxSegs * kMaxSegPages)
            return fail(ALAYA_E_INVAL, "request %d: %lld tokens exceed the selection layout (%lld)", b, (long long)n,
                        (long long)kMaxSegs * kMaxSegPages * kPageTokens);
        d.n_pages = (int32_t)pages;
        d.page_start = all_pages;
        // selection segments: seg_pages pages each, at most kMaxSegs per head
        int64_t per = seg_pages_want;
        if ((pages + per - 1) / per > kMaxSegs) per = (pages + kMaxSegs - 1) / kMaxSegs;
        per = (per + kMaxPagesPerWave - 1) / kMaxPagesPerWave * kMaxPagesPerWave; // whole scoring chunks
        d.seg_pages = (int32_t)per;
        d.nseg = (int32_t)((pages + per - 1) / per);
        d.seg_start = segs;
        // Sample stride S: phase A writes n / S scores, phase B about k * S survivors; their sum is
        // smallest at S = sqrt(n / k).  Powers of two, at most 32, and the sample must hold 2k tokens.
        int S = 1;
        d.k_est = 0;
        if (!c->tune_noprune && pages >= 4) {
            // (never when top-k takes every token outside the window: nothing checks the bound then)
            if (p->mode == ALAYA_TOPK && estimate && d.k >= 512 && d.k < n_out && pages >= 64) {
                // Estimated bound (large calls): a 1-in-S sample holds about mu = k / S of the k best
                // scores, so its (mu + 6 sqrt(mu) + 8)-th largest score lies below the true threshold
                // unless the sample is far from representative - which the selection detects and
                // repairs.  The main pass then writes about k (1 + 6 / sqrt(mu)) survivors whatever S
                // is, so S only has to keep mu at 64 or more.
                while (S < 32 && d.k / (2 * S) >= 64) S *= 2;
                while (S > 1 && pages / S < 2) S /= 2;
                const double mu = (double)d.k / S;
                d.k_est = c->estimate_mode == 2 ? 1 : (int32_t)(mu + 6.0 * std::sqrt(mu) + 8.0);
                if (d.k_est > d.k) d.k_est = d.k;
                if (S > 1) any_est = true; else d.k_est = 0;
            } else if (p->mode == ALAYA_TOPK) {
                while (S < 32 && (int64_t)(2 * S) * (2 * S) * d.k <= n && (int64_t)2 * S * d.k * 2 <= n) S *= 2;
                while (S > 1 && pages / S < 2) S /= 2;
            } else {
                S = pages >= 8192 ? 32 : 16; // the sample only has to come close to the maximum
                while (S > 1 && pages / S < 2) S /= 2;
            }
        }
        d.sample_stride = S;
        // share of the main pass's scores that is expected to survive
        const double f = p->mode == ALAYA_TOPK && S > 1 ? (double)(d.k_est > 0 ? d.k_est : d.k) * S / (double)n : 0.0;
        if (f > survive) survive = f;
        all_pages += (int)pages;
        segs += d.nseg;
        off += (int64_t)n_q_heads * d.head_stride;
    }
    // Several pages per wavefront (about 8192 workgroups, survivors staged in registers and written as
    // one list) pay when many scores survive; with few survivors one page per wavefront is faster.
    if (ppw <= 0) {
        ppw = 1;
        if (survive > 0.03)
            ppw = (int)((total_pages * c->cfg.n_kv_heads + (int64_t)kScoreWaves * 8192 - 1) /
                        ((int64_t)kScoreWaves * 8192));
        if (ppw < 1) ppw = 1;
        if (ppw > 8) ppw = 8;
    }
    for (int b = 0; b < B; ++b) {
        ReqDesc &d = hd[b];
        const int S = d.sample_stride;
        int cp = 1; // pages per wavefront in the main pass: a power of two, at most min(ppw, S)
        while (2 * cp <= ppw && 2 * cp <= S) cp *= 2;
        d.chunk_pages = cp;
        // DIPR with a window (Sec. 7.1): the maximum mostly sits among the window's tokens, which are
        // attended anyway, so the pages that hold them join the sample and seed the bound.  Whole
        // main-pass chunks, so that a chunk never mixes the two kinds of page.
        d.xf = 0;
        d.xb = d.n_pages;
        if (p->mode == ALAYA_DIPR && S > 1 && d.nwin > 0) {
            const int wp0 = (d.w0 + kPageTokens - 1) / kPageTokens;
            const int pb = d.w1 > 0 ? (d.n - d.w1) / kPageTokens : d.n_pages;
            d.xf = std::min(d.n_pages, (wp0 + cp - 1) / cp * cp);
            d.xb = std::max(d.xf, pb / cp * cp);
        }
        // a decode step: the page of the newest token belongs to the sample pass, which writes that token
        if (fused_k && S > 1) d.xb = std::max(d.xf, std::min(d.xb, (d.n - 1) / kPageTokens / cp * cp));
        const int every = (d.n_pages + S - 1) / S;
        auto not_every = [S](int a, int b) { return (b - a) - ((b + S - 1) / S - (a + S - 1) / S); }; // in [a, b)
        pages_a += every + not_every(0, d.xf) + not_every(d.xb, d.n_pages);
        const int n_a = every + d.xf + (d.n_pages - d.xb); // wavefronts of the sample pass
        d.tile_start = tiles;
        d.tileb_start = tiles_b;
        tiles += (n_a + kScoreWaves - 1) / kScoreWaves;                                  // one page per wavefront
        if (S > 1) tiles_b += (int)((d.n_pages + (int64_t)kScoreWaves * cp - 1) / ((int64_t)kScoreWaves * cp));
    }
    c->last_pages = all_pages;
    c->last_pages_a = pages_a;
    c->last_pages_b = all_pages - pages_a;
    c->last_heads = n_q_heads;
    if (off > c->L.score_elems) return fail(ALAYA_E_NOMEM, "score workspace too small");
    if (all_pages > c->L.max_pages) return fail(ALAYA_E_NOMEM, "page-count workspace too small");
    if (!c->ring_ev[slot]) {
        hipError_t e = hipEventCreateWithFlags(&c->ring_ev[slot], hipEventDisableTiming);
        if (e != hipSuccess) { c->ring_ev[slot] = nullptr; return fail_hip(e, "hipEventCreate"); }
    }
    rc = ensure_device(c, st);
    if (rc != ALAYA_OK) return rc;
    rc = ring_publish(c, slot, B, st);
    if (rc != ALAYA_OK) return rc;

    const Shape sh{c->cfg.dtype, c->cfg.head_dim, n_q_heads, c->cfg.n_kv_heads};
    const float scale = p->scale > 0.f ? p->scale : 1.0f / std::sqrt((float)c->cfg.head_dim);
    // (a launch that fails below may leave the running histogram and maximum half-filled: dev_ready is
    // dropped so that the next call zeroes them again)
    hipError_t e;
    {
        Timed tm(c, 6, st);
        if (fused_k) c->dv.fused = FusedAppend{(uint4 *)c->k_pool, (uint4 *)c->v_pool, (const uint4 *)fused_k, (const uint4 *)fused_v};
        e = launch_score(sh, c->dv, B, q, tiles, 1, 0, p->mode, st);
        c->dv.fused = FusedAppend{nullptr, nullptr, nullptr, nullptr};
        if (e == hipSuccess) *appended = fused_k != nullptr;
        // (DIPR: the bound kernel also gathers the sample pass's maxima, so it runs even with no main pass)
        if (e == hipSuccess && (tiles_b > 0 || p->mode == ALAYA_DIPR)) e = launch_tau(sh, c->dv, B, p->mode, st);
    }
    if (e != hipSuccess) { c->dev_ready = false; return fail_hip(e, "sample scoring launch"); }
    if (tiles_b > 0) {
        Timed tm(c, 0, st, true); // the roofline kernel: timed by its own dispatch
        e = launch_score(sh, c->dv, B, q, tiles_b, ppw, 1, p->mode, st, tm.begin(), tm.end());
    }
    if (e != hipSuccess) { c->dev_ready = false; return fail_hip(e, "score launch"); }
    {
        Timed tm(c, 1, st);
        e = launch_select_front(sh, c->dv, B, p->mode, segs, st);
        // repair of the heads whose estimated bound lost tokens (normally none: both launches are idle)
        if (e == hipSuccess && any_est) e = launch_score(sh, c->dv, B, q, tiles_b, ppw, 2, p->mode, st);
        if (e == hipSuccess && p->mode == ALAYA_TOPK)
            e = launch_select_back(sh, c->dv, B, p->mode, segs, any_est, p->out_ids, p->out_counts, p->ids_stride, st);
    }
    if (e != hipSuccess) { c->dev_ready = false; return fail_hip(e, "select launch"); }
    {
        // (a DIPR call has no finishing pass: the gather reads select_local's lists and reports the ids)
        Timed tm(c, 2, st);
        e = launch_attend(sh, c->dv, B, scale, splits, p->mode == ALAYA_DIPR, p->out_ids, p->out_counts, p->ids_stride, st);
    }
    if (e != hipSuccess) return fail_hip(e, "attend launch");
    { Timed tm(c, 3, st); e = launch_combine(sh, c->dv, B, splits, 0, 0, out, st); }
    if (e != hipSuccess) return fail_hip(e, "combine launch");
    return ALAYA_OK;
}

} // namespace

int alaya_full_attn(alaya_cache *c, const int32_t *seqs, int B, int n_q_heads, const void *q, float scale_in,
                    float *out, void *stream)
{
    int64_t total_pages = 0, total_tokens = 0;
    int rc = check_call(c, seqs, B, n_q_heads, q, out, &total_pages, &total_tokens);
    if (rc != ALAYA_OK) return rc;
    if (!(scale_in >= 0.f) || std::isinf(scale_in)) return fail(ALAYA_E_INVAL, "scale must be finite and >= 0");
    hipStream_t st = (hipStream_t)stream;
    int64_t ppt = (total_pages * c->cfg.n_kv_heads + kTargetGroups - 1) / kTargetGroups;
    ppt = (ppt + 3) / 4 * 4;
    if (ppt < 4) ppt = 4;

    ReqDesc *hd;
    int slot;
    rc = ring_acquire(c, &hd, &slot);
    if (rc != ALAYA_OK) return rc;
    int tiles = 0;
    for (int b = 0; b < B; ++b) {
        const int64_t n = c->seq_len[(size_t)seqs[b]];
        const int64_t pages = (n + kPageTokens - 1) / kPageTokens;
        ReqDesc &d = hd[b];
        d.pt_off = (int32_t)((int64_t)seqs[b] * c->L.mpps);
        d.n = (int32_t)n;
        d.head_stride = 0;
        d.k = 0;
        d.beta = 0.f;
        d.tile_start = tiles;
        d.score_off = 0;
        d.page_start = d.n_pages = d.seg_start = d.nseg = d.seg_pages = 0;
        d.tileb_start = 0;
        d.sample_stride = 1;
        d.chunk_pages = 1;
        d.w0 = d.w1 = d.nwin = d.k_est = 0;
        d.xf = d.xb = 0;
        tiles += (int)((pages + ppt - 1) / ppt);
    }
    if (tiles > c->L.max_tiles) return fail(ALAYA_E_NOMEM, "partial-result workspace too small");
    if (!c->ring_ev[slot]) {
        hipError_t e = hipEventCreateWithFlags(&c->ring_ev[slot], hipEventDisableTiming);
        if (e != hipSuccess) { c->ring_ev[slot] = nullptr; return fail_hip(e, "hipEventCreate"); }
    }
    rc = ensure_device(c, st);
    if (rc != ALAYA_OK) return rc;
    rc = ring_publish(c, slot, B, st);
    if (rc != ALAYA_OK) return rc;

    const Shape sh{c->cfg.dtype, c->cfg.head_dim, n_q_heads, c->cfg.n_kv_heads};
    const float scale = scale_in > 0.f ? scale_in : 1.0f / std::sqrt((float)c->cfg.head_dim);
    hipError_t e;
    { Timed tm(c, 4, st); e = launch_full_partial(sh, c->dv, B, q, scale, tiles, (int)ppt, st); }
    if (e != hipSuccess) return fail_hip(e, "full-attention launch");
    { Timed tm(c, 3, st); e = launch_combine(sh, c->dv, B, 0, 1, (int)ppt, out, st); }
    if (e != hipSuccess) return fail_hip(e, "combine launch");
    return ALAYA_OK;
}

int alaya_poll_status(alaya_cache *c, void *stream)
{
    if (!c) return fail(ALAYA_E_INVAL, "null cache handle");
    if (!c->dev_ready) return ALAYA_OK;
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

const float *alaya_debug_scores(const alaya_cache *c)
{
    if (!c) { fail(ALAYA_E_INVAL, "null cache handle"); return nullptr; }
    return (const float *)c->dv.cand;
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

int64_t alaya_debug_survivors(alaya_cache *c, void *stream)
{
    if (!c) { fail(ALAYA_E_INVAL, "null cache handle"); return -1; }
    const size_t n = (size_t)c->last_pages * c->last_heads;
    if (n == 0) return 0;
    std::vector<int32_t> h(n);
    hipStream_t st = (hipStream_t)stream;
    hipError_t e = hipMemcpyAsync(h.data(), c->dv.page_cnt, n * sizeof(int32_t), hipMemcpyDeviceToHost, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    if (e != hipSuccess) { fail_hip(e, "survivor count read"); return -1; }
    int64_t tot = 0;
    for (size_t i = 0; i < n; ++i) tot += h[i];
    return tot;
}

int alaya_set_tuning(alaya_cache *c, int score_pages_per_wave, int attend_splits, int select_segment_pages,
                     int write_all_scores)
{
    if (!c) return fail(ALAYA_E_INVAL, "null cache handle");
    if (score_pages_per_wave > kMaxPagesPerWave || attend_splits > kMaxSplits ||
        select_segment_pages > kMaxSegPages)
        return fail(ALAYA_E_INVAL, "knob out of range");
    c->tune_ppw = score_pages_per_wave > 0 ? score_pages_per_wave : 0;
    c->tune_splits = attend_splits > 0 ? attend_splits : 0;
    c->tune_seg = select_segment_pages > 0 ? select_segment_pages : 0;
    c->tune_noprune = write_all_scores > 0 ? 1 : 0;
    return ALAYA_OK;
}

} // extern "C"
