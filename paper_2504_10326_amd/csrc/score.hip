// Append (Session.update) and the scoring passes: s[h][j] = q_h . k_{h/G, j} for every cached token
// (numerator of Eq. 1; the inner product of Def. 2).  This is the paper's "flat index" plan
// (Sec. 6.2 "Query Optimizer": scan all keys) executed from HBM.
//
// Layout that makes the scan coalesce: inside a page the K tile of one KV head is stored
// [head_dim / E][64 tokens][E] with E = 16 bytes of elements.  A wavefront takes one page,
// lane = token: each 16-byte load instruction of the wave covers one contiguous 1 KiB run, every
// lane ends up with its own token's whole key, and the G query heads of the group are reduced in
// registers with no cross-lane traffic.  One K read serves all G heads of the group (GQA, Sec. 7.2).
#include "alaya_internal.h"
#include "score_page.h"
#include <hip/hip_ext.h>

#include <algorithm>

namespace alaya {

// ------------------------------------------------------------------------------------------------
// Append: one thread moves one 16-byte slice of one token's key and of its value.
//   k, v   [t][H_kv][D] token-major (what the model emits)
//   K pool [page][kvh][D/E][64][E]      V pool [page][kvh][64][D]
__global__ __launch_bounds__(256) void append_kernel(const int32_t *__restrict__ pt_row,
                                                      uint4 *__restrict__ k_pool, uint4 *__restrict__ v_pool,
                                                      const uint4 *__restrict__ k, const uint4 *__restrict__ v,
                                                      int64_t n_old, int64_t t, int H_kv, int NC)
{
    const int64_t total = t * H_kv * NC;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total;
         i += (int64_t)gridDim.x * blockDim.x) {
        const int c = (int)(i % NC);
        const int kvh = (int)((i / NC) % H_kv);
        const int64_t tok = n_old + i / ((int64_t)NC * H_kv);
        const int phys = pt_row[tok >> 6];
        const int slot = (int)(tok & 63);
        const size_t tile = ((size_t)phys * H_kv + kvh) * (size_t)(NC * 64);
        k_pool[tile + (size_t)c * 64 + slot] = k[i];
        v_pool[tile + (size_t)slot * NC + c] = v[i];
    }
}

// The same for many tokens at once (a context being loaded).  Grid: (page that the new tokens touch, KV head).
// The model's rows are 256-byte runs (one token's key for one KV head); the K tile wants the tokens of a
// 16-byte slice column next to each other.  The workgroup reads the page's key rows as they lie, turns the
// tile over in LDS and writes it column by column, 1 KiB in a row per wavefront; the value rows are copied as
// they are.  (One thread per slice with the slice as the fastest index, as above, writes every 16 bytes of a
// key to a line of its own, 1 KiB from the next: 3.3 ms for a million tokens; with the token as the fastest
// index and scattered reads instead, 2.3 ms.)
constexpr int kAppendMaxNC = 32; // 16-byte slices per row: fp32, head_dim 128

__global__ __launch_bounds__(256) void append_bulk_kernel(const int32_t *__restrict__ pt_row,
                                                           uint4 *__restrict__ k_pool, uint4 *__restrict__ v_pool,
                                                           const uint4 *__restrict__ k, const uint4 *__restrict__ v,
                                                           int64_t n_old, int64_t t, int H_kv, int NC, int64_t first_page)
{
    __shared__ uint4 turn[64][kAppendMaxNC + 1]; // (+ 1: the column reads of the second phase spread over the banks)
    const int kvh = blockIdx.x % H_kv;
    const int64_t page = first_page + blockIdx.x / H_kv;
    const size_t tile = ((size_t)pt_row[page] * H_kv + kvh) * (size_t)(NC * 64);
    // the page's slots that this append writes
    const int s0 = (int)(n_old > page * 64 ? n_old - page * 64 : 0);
    const int s1 = (int)(n_old + t < (page + 1) * 64 ? n_old + t - page * 64 : 64);
    const int rows_per_turn = 256 / NC; // NC is 8, 16 or 32
    const int c1 = threadIdx.x % NC;
    for (int slot = s0 + threadIdx.x / NC; slot < s1; slot += rows_per_turn) {
        const size_t src = ((size_t)(page * 64 + slot - n_old) * H_kv + kvh) * NC + c1;
        turn[slot][c1] = k[src];
        v_pool[tile + (size_t)slot * NC + c1] = v[src];
    }
    __syncthreads();
    const int slot = threadIdx.x & 63;
    if (slot >= s0 && slot < s1)
        for (int c = threadIdx.x >> 6; c < NC; c += 4) k_pool[tile + (size_t)c * 64 + slot] = turn[slot][c];
}

hipError_t launch_append(const Shape &sh, const int32_t *pt_row, void *k_pool, void *v_pool, const void *k,
                         const void *v, int64_t n_old, int64_t t, hipStream_t st)
{
    const int NC = sh.head_dim * (sh.dtype == 0 ? 2 : 4) / 16;
    if (t >= 4 * kPageTokens) {
        if (NC > kAppendMaxNC || 256 % NC != 0) return hipErrorInvalidValue;
        const int64_t first_page = n_old / kPageTokens, n_pages = (n_old + t + kPageTokens - 1) / kPageTokens - first_page;
        append_bulk_kernel<<<dim3((unsigned)(n_pages * sh.n_kv_heads)), dim3(256), 0, st>>>(
            pt_row, (uint4 *)k_pool, (uint4 *)v_pool, (const uint4 *)k, (const uint4 *)v, n_old, t, sh.n_kv_heads, NC, first_page);
        return hipGetLastError();
    }
    const int64_t total = t * sh.n_kv_heads * NC;
    int64_t blocks = (total + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    if (blocks < 1) blocks = 1;
    append_kernel<<<dim3((unsigned)blocks), dim3(256), 0, st>>>(pt_row, (uint4 *)k_pool, (uint4 *)v_pool,
                                                                (const uint4 *)k, (const uint4 *)v, n_old, t,
                                                                sh.n_kv_heads, NC);
    return hipGetLastError();
}

// One new token for each of B sequences (a decode step of a batch) in one launch.
//   k, v   [B][H_kv][D]; desc[b].pt_off / desc[b].n = the sequence's page-table row / its length before
__global__ __launch_bounds__(256) void append_step_kernel(const ReqDesc *__restrict__ desc_mem, const ReqDesc desc0, int desc_n,
                                                           const int32_t *__restrict__ page_table,
                                                           uint4 *__restrict__ k_pool, uint4 *__restrict__ v_pool,
                                                           const uint4 *__restrict__ k, const uint4 *__restrict__ v,
                                                           int B, int H_kv, int NC)
{
    const Descs desc{desc_mem, desc0, desc_n};
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= B * H_kv * NC) return;
    const int c = i % NC;
    const int kvh = (i / NC) % H_kv;
    const int b = i / (NC * H_kv);
    const int tok = desc[b].n;
    const int phys = page_table[desc[b].pt_off + (tok >> 6)];
    const int slot = tok & 63;
    const size_t tile = ((size_t)phys * H_kv + kvh) * (size_t)(NC * 64);
    k_pool[tile + (size_t)c * 64 + slot] = k[i];
    v_pool[tile + (size_t)slot * NC + c] = v[i];
}

hipError_t launch_append_step(const Shape &sh, const DeviceViews &dv, void *k_pool, void *v_pool, const void *k,
                              const void *v, int B, hipStream_t st)
{
    const int NC = sh.head_dim * (sh.dtype == 0 ? 2 : 4) / 16;
    const int total = B * sh.n_kv_heads * NC;
    append_step_kernel<<<dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st>>>(
        dv.desc.mem, dv.desc.in, dv.desc.n, dv.page_table, (uint4 *)k_pool, (uint4 *)v_pool, (const uint4 *)k, (const uint4 *)v, B,
        sh.n_kv_heads, NC);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// Scoring.  Grid: one workgroup per (tile, KV head); KV head is the fastest index so that with
// 8 KV heads each head's stream stays on one XCD (workgroups are dealt to XCDs round-robin).
// A tile is four wavefronts' worth of pages; a wavefront scores one or a few pages of one request,
// lane = token.
//
// bf16 uses the packed dot-product instruction (two bf16 products and the fp32 accumulate in one op,
// both operands used as stored); fp32 uses fused multiply-add.  The group's queries come from scalar registers in
// dense attention, and from LDS (a broadcast read per 16 bytes) in the sample and main passes, where G * 64
// words of them do not fit the scalar registers next to everything else that is wave-uniform there.  (The same contraction on the matrix cores - v_mfma_f32_16x16x32_bf16 with the four
// heads of a group on four rows of the 16-row operand - was measured on a 2 GiB pool and runs at the
// same speed, 6.09 against 6.03 TB/s: the pass is bound by the memory system, not by the arithmetic.)
//
// What is written.  Writing every fp32 score back costs far more than its 6 % share of the bytes, and
// nearly all of those scores can never be selected.  So a workgroup writes only the SURVIVORS of its
// pages - (score, token id) pairs at or above `tau`, a lower bound of the head's final selection
// threshold (window tokens always survive) - and it writes them as ONE contiguous block: the four
// wavefronts stage their survivors in LDS, and the block leaves as {count, start} per head followed
// by the pairs, head after head, ascending by token.  Small scattered writes mixed into the read
// stream cost far more than their bytes (5.2 TB/s with a list per page against 5.7 with a block per
// workgroup at 1.6 % survivors; with the keys loaded non-temporally 5.7 against 6.3).
// The bound comes from a sample; the workgroups of one launch never wait for or feed back to each other:
//   sample pass  scores every S-th page of each request and enters those scores into the head's
//                histogram (top-k) or maximum (DIPR); it writes no scores;
//   bound        (tau_kernel) top-k: the k-th largest score of a SUBSET is never above the k-th largest
//                of the whole, so the lower edge of the histogram bucket holding the sample's k-th
//                largest score is a valid tau; DIPR: tau = (sample max) - beta <= (true max) - beta.
//                Large top-k calls filter with a tighter ESTIMATE instead, which the selection
//                verifies afterwards;
//   main pass    scores every page against tau.
// A guaranteed tau never exceeds the final threshold, so nothing that can be selected is dropped;
// an estimated one that does is detected (fewer than k survivors) and repaired.  Either way the
// selection that follows is exact, and deterministic - the blocks depend on the data only, not on timing.
// ------------------------------------------------------------------------------------------------
// Sample pass: one page per wavefront.  Wavefront w of a request takes the sampled page w * S; the
// wavefronts after those take the pages [0, xf) and [xb, n_pages) that are scored on top (a DIPR
// window, the page of a token that this pass appends), leaving out the S-th pages among them.
// DIPR: the workgroup raises one of the head's kMaxSlots sample maxima (many atomics on ONE address are
// slow: they are carried out one after the other at the memory side).  top-k: it counts the scores of
// the every-S-th pages per bucket in LDS and adds the non-empty buckets to the head's histogram (the
// pages scored on top are no uniform sample of the request, so the estimate must not see them).
template <int DT, int D, int G>
__global__ __launch_bounds__(256) void sample_kernel(const ReqDesc *__restrict__ desc_mem, const ReqDesc desc0, int desc_n,
                                                      int B, const int32_t *__restrict__ page_table,
                                                      const uint32_t *__restrict__ qw, const uint4 *__restrict__ k_pool,
                                                      uint32_t *__restrict__ hist, uint32_t *__restrict__ sample_max,
                                                      int H_kv, int mode, const FusedAppend fa,
                                                      const uint8_t *__restrict__ pmask, float *__restrict__ samp)
{
    const Descs desc{desc_mem, desc0, desc_n};
    constexpr int NC = D * (DT == 0 ? 2 : 4) / 16;
    constexpr int QW = D * (DT == 0 ? 2 : 4) / 4;
    // two 16-bit counters per word: a workgroup scores 4 pages = 256 tokens per head
    __shared__ uint32_t lhist[G][kHistBins / 2];
    __shared__ float wmax[kScoreWaves][G];
    __shared__ uint4 q_lds[G * NC]; // the group's queries
    const int kvh = blockIdx.x % H_kv;
    const int tile = blockIdx.x / H_kv;
    int r = 0;
    while (r + 1 < B && desc[r + 1].tile_start <= tile) ++r;
    const ReqDesc dsc = desc[r];
    const int H_q = H_kv * G;
    const int rh0 = r * H_q + kvh * G; // first head of this group
    const bool hist_on = mode == 0;
    if (threadIdx.x < G * NC) q_lds[threadIdx.x] = ((const uint4 *)(qw + (size_t)rh0 * QW))[threadIdx.x];
    if (hist_on)
        for (int i = threadIdx.x; i < G * (kHistBins / 2); i += 256) (&lhist[0][0])[i] = 0u;
    if (threadIdx.x < kScoreWaves * G) (&wmax[0][0])[threadIdx.x] = -INFINITY;
    __syncthreads();

    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    const int S = dsc.sample_stride;
    const int w_req = (tile - dsc.tile_start) * kScoreWaves + wave;
    const int ns = S > 1 ? (dsc.n_pages + S - 1) >> (__ffs(S) - 1) : 0; // every S-th page
    const int x = w_req - ns;
    const bool every_sth = x < 0;
    int p = x < 0 ? w_req * S : x < dsc.xf ? x : dsc.xb + (x - dsc.xf);
    if (x >= 0 && S > 1 && (p & (S - 1)) == 0) p = dsc.n_pages; // an S-th page: another wavefront's
    float lmax[G];
#pragma unroll
    for (int g = 0; g < G; ++g) lmax[g] = -INFINITY;

    // Coarse index: a page that no head of the group chose is not read, and a head counts only the tokens of
    // pages it chose itself (the sample then is 1-in-S of every head's own candidates).
    uint32_t chosen = 0xFFu;
    if (pmask && p < dsc.n_pages) {
        chosen = pmask[(size_t)dsc.pm_off + (size_t)kvh * dsc.pm_stride + p];
        if (chosen == 0u) p = dsc.n_pages;
    }
    if (p < dsc.n_pages) {
        const int phys = page_table[dsc.pt_off + p];
        const uint4 *kp = k_pool;
        if (fa.k) {
            // A decode step: the newest token's rows are not in the pools yet.  The wavefront that scores
            // its page writes them (this KV head's), waits for the writes, and reads the page through
            // the same pointer; the value row is read by later kernels only.
            kp = fa.k_pool;
            if (p == (dsc.n - 1) >> 6) {
                const int slot = (dsc.n - 1) & 63;
                const size_t t = ((size_t)phys * H_kv + kvh) * (size_t)(NC * 64);
                const size_t src = ((size_t)r * H_kv + kvh) * NC;
                for (int c = lane; c < NC; c += 64) {
                    fa.k_pool[t + (size_t)c * 64 + slot] = fa.k[src + c];
                    fa.v_pool[t + (size_t)slot * NC + c] = fa.v[src + c];
                }
                asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            }
        }
        const uint4 *base = kp + ((size_t)phys * H_kv + kvh) * (size_t)(NC * 64) + lane;
        float acc[G];
        score_page_lds<DT, D, G>(base, q_lds, acc);
        // The main pass takes the scores of the every-S-th pages from here instead of reading their keys again.
        if (every_sth && S >= kSampScoresMinStride && !pmask) {
            float *dst = samp + ((size_t)(dsc.pm_off + w_req) * H_kv + kvh) * (size_t)(G * 64) + lane;
#pragma unroll
            for (int g = 0; g < G; ++g) dst[g * 64] = acc[g];
        }
        const int j = p * kPageTokens + lane;
        const bool valid = j < dsc.n;
        const bool win = in_window(dsc, j);
#pragma unroll
        for (int g = 0; g < G; ++g) {
            if (!valid) continue;
            lmax[g] = acc[g];
            if (hist_on && every_sth && !win && ((chosen >> g) & 1u)) {
                const uint32_t bin = ord_key(acc[g]) >> 21;
                atomicAdd(&lhist[g][bin >> 1], 1u << ((bin & 1u) * 16u));
            }
        }
    }
    if (mode == 1) {
#pragma unroll
        for (int g = 0; g < G; ++g) {
            float m = lmax[g];
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o));
            if (lane == 0) wmax[wave][g] = m;
        }
    }
    __syncthreads();
    if (mode == 1) {
        if (threadIdx.x < G) {
            float m = wmax[0][threadIdx.x];
#pragma unroll
            for (int w = 1; w < kScoreWaves; ++w) m = fmaxf(m, wmax[w][threadIdx.x]);
            if (m > -INFINITY)
                atomicMax(sample_max + (size_t)(rh0 + threadIdx.x) * kMaxSlots + (tile & (kMaxSlots - 1)), ord_key(m));
        }
    } else {
        // What the four pages add to one bucket is capped (hist_cap, several times what a bucket of the
        // threshold region gets from four pages of unclustered keys).  Keys of neighbouring tokens are
        // alike, so a sampled page may hold dozens of scores of one bucket where the pages between the
        // sampled ones hold none; uncapped, the estimate would take them for 1-in-S of the cache and come
        // out too high.  The cap can only lower the bound (more survivors), never lose a token.
        uint32_t *gh = hist + (size_t)rh0 * kHistBins;
        const uint32_t cap = (uint32_t)dsc.hist_cap;
        for (int i = threadIdx.x; i < G * (kHistBins / 2); i += 256) {
            const uint32_t v = (&lhist[0][0])[i];
            if (v & 0xFFFFu) atomicAdd(&gh[2 * i], min(v & 0xFFFFu, cap));
            if (v >> 16) atomicAdd(&gh[2 * i + 1], min(v >> 16, cap));
        }
    }
}

template <int DT, int D>
static hipError_t launch_sample_g(const Shape &sh, const DeviceViews &dv, int B, const void *q, int total_tiles,
                                  int mode, bool coarse, hipStream_t st)
{
    const int G = sh.n_q_heads / sh.n_kv_heads;
    const dim3 grid((unsigned)(total_tiles * sh.n_kv_heads)), block(256);
#define ALAYA_SAMPLE(GG)                                                                                      \
    sample_kernel<DT, D, GG><<<grid, block, 0, st>>>(dv.desc.mem, dv.desc.in, dv.desc.n, B, dv.page_table,     \
                                                     (const uint32_t *)q, (const uint4 *)dv.k_pool, dv.hist,  \
                                                     dv.sample_max, sh.n_kv_heads, mode, dv.fused,           \
                                                     coarse ? dv.pmask : nullptr, dv.samp)
    switch (G) {
    case 1: ALAYA_SAMPLE(1); break;
    case 2: ALAYA_SAMPLE(2); break;
    case 4: ALAYA_SAMPLE(4); break;
    case 8: ALAYA_SAMPLE(8); break;
    default: return hipErrorInvalidValue;
    }
#undef ALAYA_SAMPLE
    return hipGetLastError();
}

hipError_t launch_sample(const Shape &sh, const DeviceViews &dv, int B, const void *q, int total_tiles, int mode,
                         bool coarse, hipStream_t st)
{
    if (total_tiles <= 0) return hipSuccess;
    if (sh.dtype == 0) {
        if (sh.head_dim == 128) return launch_sample_g<0, 128>(sh, dv, B, q, total_tiles, mode, coarse, st);
        if (sh.head_dim == 64) return launch_sample_g<0, 64>(sh, dv, B, q, total_tiles, mode, coarse, st);
    } else {
        if (sh.head_dim == 128) return launch_sample_g<1, 128>(sh, dv, B, q, total_tiles, mode, coarse, st);
        if (sh.head_dim == 64) return launch_sample_g<1, 64>(sh, dv, B, q, total_tiles, mode, coarse, st);
    }
    return hipErrorInvalidValue;
}

// ------------------------------------------------------------------------------------------------
// tau: the lower bound of each head's selection threshold, from what the sample pass accumulated.
// One 1024-thread workgroup per (request, head); runs between the sample pass and the main pass, and
// leaves the sample's histogram and maxima zero for the next call.
__global__ __launch_bounds__(kSelectThreads) void tau_kernel(const ReqDesc *__restrict__ desc_mem, const ReqDesc desc0, int desc_n, int H_q, int mode,
                                                              uint32_t *__restrict__ hist,
                                                              uint32_t *__restrict__ sample_max,
                                                              uint32_t *__restrict__ head_maxkey,
                                                              uint32_t *__restrict__ tau,
                                                              uint32_t *__restrict__ tau_safe,
                                                              uint32_t *__restrict__ any_fail)
{
    const Descs desc{desc_mem, desc0, desc_n};
    __shared__ int32_t wtot[kSelectThreads / 64];
    __shared__ int32_t found, found_est;

    const int rh = blockIdx.x;
    const ReqDesc dsc = desc[rh / H_q];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (rh == 0 && tid == 0) *any_fail = 0u; // (the selection of the call before this one is over)

    if (mode == 1) { // DIPR: (maximum over the sample) - beta
        if (tid < 64) {
            static_assert(kMaxSlots == 64, "one slot per lane");
            uint32_t mk = sample_max[(size_t)rh * kMaxSlots + tid];
            sample_max[(size_t)rh * kMaxSlots + tid] = 0u; // consumed: zero for the next call
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) mk = max(mk, (uint32_t)__shfl_xor((int)mk, o));
            if (tid == 0) {
                const bool prune = dsc.sample_stride > 1 && mk != 0u;
                head_maxkey[rh] = mk; // the main pass raises it further
                tau[rh] = tau_safe[rh] = prune ? ord_key(ord_float(mk) - dsc.beta) : 0u;
            }
        }
        return;
    }
    // top-k: lower edge of the bucket that holds the k-th largest score of the sample.
    // Walk down from the top bucket: two buckets per thread, thread 0 holding the top ones.
    __shared__ int32_t cnts[kHistBins];
    __shared__ int32_t above_est;
    uint32_t *gh = hist + (size_t)rh * kHistBins;
    const int b0 = kHistBins - 1 - 2 * tid;
    const int c0 = (int)gh[b0], c1 = (int)gh[b0 - 1];
    gh[b0] = 0u; // consumed: zero for the next call
    gh[b0 - 1] = 0u;
    cnts[b0] = c0;
    cnts[b0 - 1] = c1;
    if (tid == 0) found = found_est = -1;
    const int inc = wave_scan(c0 + c1);
    if (lane == 63) wtot[wave] = inc;
    __syncthreads();
    int above = inc - (c0 + c1);
    for (int w = 0; w < wave; ++w) above += wtot[w];
    if (above < dsc.k && above + c0 + c1 >= dsc.k) found = above + c0 >= dsc.k ? b0 : b0 - 1;
    // The estimated bound: the sample's k_est-th largest score, k_est being the share of k that a
    // 1-in-S sample is expected to hold plus a wide margin.  Nothing guarantees it; the selection
    // checks the survivor count against k and has the head repaired if it fell short.
    int ke = dsc.k_est;
    if (dsc.est_cand > 0 && ke > 1) {
        // Through the coarse index the sample is every S-th page among the pages the head chose - about P / S of
        // them, but the number varies from head to head, and with it the share of the k best that the sample
        // holds.  The histogram's total says how large the sample is.
        int total = 0;
        for (int w = 0; w < kSelectThreads / 64; ++w) total += wtot[w];
        const float mu = (float)dsc.k * (float)total / (float)dsc.est_cand;
        ke = min(dsc.k, (int)(mu + 6.f * sqrtf(mu) + 8.f));
    }
    if (ke > 0 && above < ke && above + c0 + c1 >= ke) {
        const bool first = above + c0 >= ke;
        found_est = first ? b0 : b0 - 1;
        above_est = first ? above : above + c0;
    }
    __syncthreads();
    if (tid == 0) {
        // fewer than k scores in the sample (or no sample at all): no bound
        const uint32_t safe = dsc.sample_stride > 1 && found >= 0 ? (uint32_t)found << 21 : 0u;
        tau_safe[rh] = safe;
        uint32_t est = safe;
        if (dsc.sample_stride > 1 && ke > 0 && found_est >= 0) {
            // A bucket spans a factor 2^(1/4) of score, and far more scores sit near its lower edge than
            // the estimate needs.  Place the bound inside the bucket: with cb scores in [lo, hi), r of which
            // are wanted, and a density that falls off exponentially at the rate the next bucket's count
            // suggests, the r-th largest lies at x with  N(x) = cb (e^-L(x-lo) - e^-Lw) / (1 - e^-Lw) = r.
            const uint32_t kb = (uint32_t)found_est << 21;
            est = kb;
            const int cb = cnts[found_est], r = ke - above_est; // 1 <= r <= cb
            const float lo = ord_float(kb), hi = found_est + 1 < kHistBins ? ord_float(kb + (1u << 21)) : lo;
            const float w = hi - lo;
            if (w > 0.f && w < 1e30f && cb > r) {
                const int cn = found_est + 1 < kHistBins ? cnts[found_est + 1] : 0;
                float x;
                if (cn > 0 && cn < cb) {
                    const float hi2 = found_est + 2 < kHistBins ? ord_float(kb + (2u << 21)) : hi + w;
                    const float w2 = hi2 - hi;
                    // decay rate from the two buckets' mean densities, taken at their mid-points
                    const float L = __logf(((float)cb / w) / ((float)cn / w2)) / (0.5f * (w + w2));
                    const float eLw = __expf(-L * w);
                    const float frac = (float)r / (float)cb;
                    x = L > 1e-6f ? lo - __logf(eLw + frac * (1.f - eLw)) / L : hi - w * frac;
                } else {
                    x = hi - w * (float)r / (float)cb; // flat density
                }
                if (x > lo && x < hi) est = ord_key(x);
            }
        }
        tau[rh] = est;
    }
}

hipError_t launch_tau(const Shape &sh, const DeviceViews &dv, int B, int mode, hipStream_t st)
{
    tau_kernel<<<dim3((unsigned)(B * sh.n_q_heads)), dim3(kSelectThreads), 0, st>>>(
        dv.desc.mem, dv.desc.in, dv.desc.n, sh.n_q_heads, mode, dv.hist, dv.sample_max, dv.head_maxkey, dv.tau,
        dv.tau_safe, dv.any_fail);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// Main pass.  `block` = tile * H_kv + KV head: what one 256-thread workgroup scores and the survivor
// block it writes.  Wavefront w of the tile takes the CP consecutive pages from (4 * tile_in_request + w) * CP.
// REPAIR: only for the groups with a head marked in `fail` - those whose estimated bound turned out to
// lie above the true threshold - and for those heads against the guaranteed bound; the whole block is
// written again (the other heads' parts come out as before).
// COARSE (coarse-grained index): only the pages that some head of the group chose (dv.pmask), and the pages
// that hold window tokens, are read; a head keeps a token only if it chose the token's page itself.
template <int DT, int D, int G, int CP, bool REPAIR, bool COARSE>
__device__ __forceinline__ void main_block(const int block, const Descs &desc, int B,
                                           const int32_t *__restrict__ page_table,
                                           const uint32_t *__restrict__ qw, const uint4 *__restrict__ k_pool,
                                           const BlockArea &area,
                                           const uint32_t *__restrict__ tau_in,
                                           const uint32_t *__restrict__ tau_safe,
                                           const uint32_t *__restrict__ fail, int H_kv, int mode,
                                           uint32_t *head_maxkey, const void *__restrict__ aux)
{
    // aux: COARSE - the page mask; otherwise the scores that the sample pass left of its every-S-th pages
    const uint8_t *pmask = (const uint8_t *)aux;
    const float *samp = (const float *)aux;
    constexpr int NC = D * (DT == 0 ? 2 : 4) / 16;
    constexpr int QW = D * (DT == 0 ? 2 : 4) / 4;
    constexpr int CAP = kPageTokens * CP; // survivors of one wavefront and head, at most
    __shared__ uint2 stage[kScoreWaves][G][CAP];
    __shared__ int32_t wcnt[G][kScoreWaves];
    __shared__ uint4 q_lds[G * NC]; // the group's queries

    const int kvh = block % H_kv;
    const int tile = block / H_kv;
    int r = 0;
    while (r + 1 < B && desc[r + 1].tileb_start <= tile) ++r;
    const ReqDesc dsc = desc[r];
    const int H_q = H_kv * G;
    const int rh0 = r * H_q + kvh * G; // first head of this group
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;

    uint32_t tau[G];
    uint32_t smax[G]; // DIPR: the head's maximum as this wavefront knows it
    bool any_act = !REPAIR;
#pragma unroll
    for (int g = 0; g < G; ++g) {
        const bool failed = REPAIR && fail[rh0 + g] != 0u;
        any_act |= failed;
        tau[g] = failed ? tau_safe[rh0 + g] : tau_in[rh0 + g];
        smax[g] = !REPAIR && mode == 1 ? head_maxkey[rh0 + g] : 0xFFFFFFFFu;
    }
    if (REPAIR && !any_act) return; // whole workgroup
    const unsigned long long lt_mask = (1ull << lane) - 1ull;
    if (threadIdx.x < G * NC) q_lds[threadIdx.x] = ((const uint4 *)(qw + (size_t)rh0 * QW))[threadIdx.x];
    __syncthreads();
    int cnt[G];
#pragma unroll
    for (int g = 0; g < G; ++g) cnt[g] = 0;

    const int p0 = ((tile - dsc.tileb_start) * kScoreWaves + wave) * CP;
#pragma unroll 1
    for (int i = 0; i < CP; ++i) {
        const int p = p0 + i;
        if (p >= dsc.n_pages) break;
        uint32_t chosen = 0xFFu; // bit g: head g takes tokens of this page
        if (COARSE) {
            chosen = pmask[(size_t)dsc.pm_off + (size_t)kvh * dsc.pm_stride + p];
            const bool holds_window = p * kPageTokens < dsc.w0 || (dsc.w1 > 0 && (p + 1) * kPageTokens > dsc.n - dsc.w1);
            if (chosen == 0u && !holds_window) continue; // (wave-uniform) the page's keys are not read
        }
        float acc[G];
        const int S = dsc.sample_stride;
        if (!COARSE && S >= kSampScoresMinStride && (p & (S - 1)) == 0) {
            // (wave-uniform) a page of the sample: scored there, 1 KiB of scores instead of 16 KiB of keys
            const float *src = samp + ((size_t)(dsc.pm_off + (p >> (__ffs(S) - 1))) * H_kv + kvh) * (size_t)(G * 64) + lane;
#pragma unroll
            for (int g = 0; g < G; ++g) acc[g] = src[g * 64];
        } else {
            const int phys = page_table[dsc.pt_off + p];
            const uint4 *base = k_pool + ((size_t)phys * H_kv + kvh) * (size_t)(NC * 64) + lane;
            score_page_lds<DT, D, G>(base, q_lds, acc);
        }
        const int j = p * kPageTokens + lane;
        const bool valid = j < dsc.n;
        const bool win = in_window(dsc, j); // always a survivor; top-k neither counts nor ranks it
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const uint32_t key = ord_key(acc[g]);
            const bool keep = valid && (win || (((chosen >> g) & 1u) != 0u && key >= tau[g]));
            // DIPR: a score above the sample's maximum raises the head's maximum.  About S - 1 scores
            // per head do (the expected number of tokens ahead of the best of a 1-in-S sample), so
            // these atomics on one address are few; one per wavefront and page at most.
            if (!REPAIR && __ballot(valid && key > smax[g])) {
                uint32_t m = valid ? key : 0u;
#pragma unroll
                for (int o = 32; o > 0; o >>= 1) m = max(m, (uint32_t)__shfl_xor((int)m, o));
                if (lane == 0) atomicMax(&head_maxkey[rh0 + g], m);
                smax[g] = m;
            }
            const unsigned long long m = __ballot(keep);
            if (keep) stage[wave][g][cnt[g] + __popcll(m & lt_mask)] = make_uint2(__float_as_uint(acc[g]), (uint32_t)j);
            cnt[g] += __popcll(m);
        }
    }
    if (lane < G) {
        int c = cnt[0];
#pragma unroll
        for (int g = 1; g < G; ++g) c = lane == g ? cnt[g] : c;
        wcnt[lane][wave] = c;
    }
    __syncthreads();
    // order inside the block: head after head, wavefront after wavefront = ascending by token
    int off[G * kScoreWaves + 1];
    off[0] = 0;
#pragma unroll
    for (int s = 0; s < G * kScoreWaves; ++s) off[s + 1] = off[s] + (&wcnt[0][0])[s];
    const int total = off[G * kScoreWaves];
    if (threadIdx.x < G)
        *area.hdr(tile, kvh * G + (int)threadIdx.x) =
            make_uint2((uint32_t)(off[kScoreWaves * threadIdx.x + kScoreWaves] - off[kScoreWaves * threadIdx.x]),
                       (uint32_t)off[kScoreWaves * threadIdx.x]);
    for (int i = threadIdx.x; i < total; i += 256) {
        int s = 0;
#pragma unroll
        for (int t = 1; t < G * kScoreWaves; ++t) s += (off[t] <= i) ? 1 : 0;
        *area.at(block, i) = stage[s % kScoreWaves][s / kScoreWaves][i - off[s]];
    }
}

template <int DT, int D, int G, int CP, bool REPAIR, bool COARSE>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu((D * (DT == 0 ? 2 : 4) / 4 + 8 * G <= 96 && G <= 4) ? 4 : 2)))
void main_kernel(const ReqDesc *__restrict__ desc_mem, const ReqDesc desc0, int desc_n, int B,
                                                    const int32_t *__restrict__ page_table,
                                                    const uint32_t *__restrict__ qw, const uint4 *__restrict__ k_pool,
                                                    const BlockArea area,
                                                    const uint32_t *__restrict__ tau_in,
                                                    const uint32_t *__restrict__ tau_safe,
                                                    const uint32_t *__restrict__ fail,
                                                    const uint32_t *__restrict__ any_fail, int H_kv, int mode,
                                                    int total_blocks, uint32_t *head_maxkey,
                                                    const void *__restrict__ aux)
{
    const Descs desc{desc_mem, desc0, desc_n};
    if (REPAIR) {
        // launched with a small grid whose workgroups leave at once unless some head was marked
        if (*any_fail == 0u) return;
        for (int b = blockIdx.x; b < total_blocks; b += gridDim.x) {
            main_block<DT, D, G, CP, REPAIR, COARSE>(b, desc, B, page_table, qw, k_pool, area, tau_in,
                                                     tau_safe, fail, H_kv, mode, head_maxkey, aux);
            __syncthreads(); // the staging area is reused
        }
    } else {
        main_block<DT, D, G, CP, REPAIR, COARSE>(blockIdx.x, desc, B, page_table, qw, k_pool, area,
                                                 tau_in, tau_safe, fail, H_kv, mode, head_maxkey, aux);
    }
}

// With events given, they are attached to the dispatch itself (hipExtLaunchKernelGGL): their
// timestamps are then the kernel's own begin and end, without the gaps an event pair recorded
// around a launch also sees.
template <typename Kern, typename... Args>
static void launch_maybe_timed(Kern kern, dim3 grid, dim3 block, hipStream_t st, hipEvent_t ev0, hipEvent_t ev1,
                               Args... args)
{
    if (ev0 && ev1) hipExtLaunchKernelGGL(kern, grid, block, 0, st, ev0, ev1, 0, args...);
    else kern<<<grid, block, 0, st>>>(args...);
}

template <int DT, int D, int G>
static hipError_t launch_score_cp(const Shape &sh, const DeviceViews &dv, int B, const void *q, int total_tiles,
                                  int cp, bool repair, int mode, bool coarse, hipStream_t st, hipEvent_t ev0,
                                  hipEvent_t ev1)
{
    const int total_blocks = total_tiles * sh.n_kv_heads;
    const dim3 grid((unsigned)(repair && total_blocks > kRepairGrid ? kRepairGrid : total_blocks)), block(256);
#define ALAYA_MAIN_K(CPP, RP, CO)                                                                             \
    launch_maybe_timed(main_kernel<DT, D, G, CPP, RP, CO>, grid, block, st, ev0, ev1, dv.desc.mem, dv.desc.in, \
                       dv.desc.n, B, dv.page_table, (const uint32_t *)q, (const uint4 *)dv.k_pool, dv.area,   \
                       (const uint32_t *)dv.tau, (const uint32_t *)dv.tau_safe,                               \
                       (const uint32_t *)dv.fail, (const uint32_t *)dv.any_fail, sh.n_kv_heads, mode,         \
                       total_blocks, dv.head_maxkey, CO ? (const void *)dv.pmask : (const void *)dv.samp)
#define ALAYA_MAIN(CPP)                                                                                       \
    do {                                                                                                      \
        if (coarse && repair) ALAYA_MAIN_K(CPP, true, true);                                                  \
        else if (coarse) ALAYA_MAIN_K(CPP, false, true);                                                      \
        else if (repair) ALAYA_MAIN_K(CPP, true, false);                                                      \
        else ALAYA_MAIN_K(CPP, false, false);                                                                 \
    } while (0)
    // (the staging area holds 4 * G * 64 * CP pairs: at most 32 KiB)
    if (cp == 1) ALAYA_MAIN(1);
    else if (cp == 2 && G <= 8) ALAYA_MAIN(2);
    else if (cp == 4 && G <= 4) {
        if constexpr (G <= 4) ALAYA_MAIN(4);
    } else return hipErrorInvalidValue;
#undef ALAYA_MAIN
#undef ALAYA_MAIN_K
    return hipGetLastError();
}

template <int DT, int D>
static hipError_t launch_score_g(const Shape &sh, const DeviceViews &dv, int B, const void *q, int total_tiles,
                                 int cp, bool repair, int mode, bool coarse, hipStream_t st, hipEvent_t ev0,
                                 hipEvent_t ev1)
{
    switch (sh.n_q_heads / sh.n_kv_heads) {
    case 1: return launch_score_cp<DT, D, 1>(sh, dv, B, q, total_tiles, cp, repair, mode, coarse, st, ev0, ev1);
    case 2: return launch_score_cp<DT, D, 2>(sh, dv, B, q, total_tiles, cp, repair, mode, coarse, st, ev0, ev1);
    case 4: return launch_score_cp<DT, D, 4>(sh, dv, B, q, total_tiles, cp, repair, mode, coarse, st, ev0, ev1);
    case 8: return launch_score_cp<DT, D, 8>(sh, dv, B, q, total_tiles, cp, repair, mode, coarse, st, ev0, ev1);
    default: return hipErrorInvalidValue;
    }
}

hipError_t launch_score(const Shape &sh, const DeviceViews &dv, int B, const void *q, int total_tiles, int cp,
                        bool repair, int mode, bool coarse, hipStream_t st, hipEvent_t ev0, hipEvent_t ev1)
{
    if (total_tiles <= 0) return hipSuccess;
    if (sh.dtype == 0) {
        if (sh.head_dim == 128) return launch_score_g<0, 128>(sh, dv, B, q, total_tiles, cp, repair, mode, coarse, st, ev0, ev1);
        if (sh.head_dim == 64) return launch_score_g<0, 64>(sh, dv, B, q, total_tiles, cp, repair, mode, coarse, st, ev0, ev1);
    } else {
        if (sh.head_dim == 128) return launch_score_g<1, 128>(sh, dv, B, q, total_tiles, cp, repair, mode, coarse, st, ev0, ev1);
        if (sh.head_dim == 64) return launch_score_g<1, 64>(sh, dv, B, q, total_tiles, cp, repair, mode, coarse, st, ev0, ev1);
    }
    return hipErrorInvalidValue;
}

__global__ void fill_u32_kernel(uint32_t *p, size_t n, uint32_t v)
{
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
        p[i] = v;
}

hipError_t launch_fill_u32(uint32_t *p, size_t n, uint32_t v, hipStream_t st)
{
    if (n == 0) return hipSuccess;
    size_t blocks = (n + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    fill_u32_kernel<<<dim3((unsigned)blocks), dim3(256), 0, st>>>(p, n, v);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// Inspection: scatter the survivors' scores of the last call into dense rows, and count them.
__global__ __launch_bounds__(256) void debug_scatter_kernel(const ReqDesc *__restrict__ desc_mem, const ReqDesc desc0, int desc_n, int B,
                                                             const BlockArea area,
                                                             int H_kv, int G, float *__restrict__ out,
                                                             unsigned long long *__restrict__ total)
{
    const Descs desc{desc_mem, desc0, desc_n};
    const int kvh = blockIdx.x % H_kv;
    const int tile = blockIdx.x / H_kv;
    int r = 0;
    while (r + 1 < B && desc[r + 1].tileb_start <= tile) ++r;
    const ReqDesc dsc = desc[r];
    unsigned long long sum = 0;
    for (int g = 0; g < G; ++g) {
        const uint2 hd = *area.hdr(tile, kvh * G + g);
        sum += hd.x;
        if (out)
            for (uint32_t i = threadIdx.x; i < hd.x; i += 256) {
                const uint2 pr = *area.at(blockIdx.x, (int)(hd.y + i));
                out[(size_t)dsc.score_off + (size_t)(kvh * G + g) * dsc.head_stride + pr.y] = __uint_as_float(pr.x);
            }
    }
    if (threadIdx.x == 0 && total) atomicAdd(total, sum);
}

hipError_t launch_debug_scatter(const Shape &sh, const DeviceViews &dv, int B, int total_tiles, float *out,
                                unsigned long long *total, hipStream_t st)
{
    if (total_tiles <= 0) return hipSuccess;
    debug_scatter_kernel<<<dim3((unsigned)(total_tiles * sh.n_kv_heads)), dim3(256), 0, st>>>(
        dv.desc.mem, dv.desc.in, dv.desc.n, B, dv.area, sh.n_kv_heads, sh.n_q_heads / sh.n_kv_heads,
        out, total);
    return hipGetLastError();
}

} // namespace alaya
