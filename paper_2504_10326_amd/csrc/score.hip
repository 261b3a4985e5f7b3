// Append (Session.update) and the scoring pass: s[h][j] = q_h . k_{h/G, j} for every cached token
// (numerator of Eq. 1; the inner product of Def. 2).  This is the paper's "flat index" plan
// (Sec. 5.2: scan all keys) executed from HBM.
//
// Layout that makes the scan coalesce: inside a page the K tile of one KV head is stored
// [head_dim / E][64 tokens][E] with E = 16 bytes of elements.  A wavefront takes one page,
// lane = token: each 16-byte load instruction of the wave covers one contiguous 1 KiB run, every
// lane ends up with its own token's whole key, and the G query heads of the group are reduced in
// registers with no cross-lane traffic.  One K read serves all G heads of the group (GQA, Sec. 6.2).
#include "alaya_internal.h"
#include <hip/hip_ext.h>

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

hipError_t launch_append(const Shape &sh, const int32_t *pt_row, void *k_pool, void *v_pool, const void *k,
                         const void *v, int64_t n_old, int64_t t, hipStream_t st)
{
    const int NC = sh.head_dim * (sh.dtype == 0 ? 2 : 4) / 16;
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
// A tile is four wavefronts' worth of pages; a wavefront scores one or a few pages of one request.
//
// bf16 uses the packed dot-product instruction (two bf16 products and the fp32 accumulate in one op,
// both operands used as stored), the query streamed through scalar registers; fp32 uses fused
// multiply-add.
//
// What is written.  Writing every fp32 score back costs far more than its 6 % share of the bytes (a
// read-only scan of the same keys runs at 6.3 TB/s, the same scan writing all scores at 5.3), and
// nearly all of those scores can never be selected.  So a wavefront writes only the SURVIVORS of its
// pages - (score, token id) pairs, compacted, ascending, plus their count - where a survivor is a
// score at or above `tau`, a lower bound of the head's final selection threshold (window tokens
// always survive).  The bound comes from a sample; the workgroups of one launch never wait for or
// feed back to each other:
//   sample pass  (phase 0) scores every S-th page of each request, writes all of those scores and
//                enters them into the head's histogram (top-k) or maximum (DIPR);
//   bound        (tau_kernel) top-k: the k-th largest score of a SUBSET is never above the k-th largest
//                of the whole, so the lower edge of the histogram bucket holding the sample's k-th
//                largest score is a valid tau; DIPR: tau = (sample max) - beta <= (true max) - beta.
//                Large top-k calls filter with a tighter ESTIMATE instead, which the selection
//                verifies afterwards (tau_kernel, phase 2);
//   main pass    (phase 1) scores the remaining pages against tau.
// A guaranteed tau never exceeds the final threshold, so nothing that can be selected is dropped;
// an estimated one that does is detected and repaired.  Either way the selection that follows is
// exact, and deterministic - the survivor lists depend on the data only, not on timing.
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;

__device__ __forceinline__ float dot2_bf16(uint32_t a, uint32_t b, float c)
{
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a), __builtin_bit_cast(bf16x2_t, b), c,
                                           false);
}

// PHASE 0 (sample pass): the workgroup also enters its scores into the head's statistics: for DIPR it
// raises one of the head's kMaxSlots sample maxima (many atomics on ONE address are slow: they are
// carried out one after the other at the memory side), for top-k it counts them per bucket in LDS
// and adds the non-empty buckets to the histogram.  The bound kernel reads both right after this
// pass; the selection later adds only the survivors of the OTHER pages to them.  Few workgroups run
// in phase 0 (a 1/S share of the pages), so these atomics are cheap; the main pass (PHASE 1) has none.
// PHASE 2 (repair pass): as the main pass, but only for the heads marked in `fail` - those whose
// estimated bound turned out to lie above the true threshold - and against the guaranteed bound; it
// rewrites those heads' lists and adds the scores between the two bounds to their histograms.  It
// runs after every call that used an estimated bound and normally finds nothing to do.
// RING: a wavefront may cover several pages; their survivors are staged and leave as one list.
// `block` = tile * H_kv + KV head: what one 256-thread workgroup scores.
template <int DT, int D, int G, int PHASE, bool RING>
__device__ __forceinline__ void score_block(const int block, const Descs &desc, int B,
                                            const int32_t *__restrict__ page_table,
                                            const uint32_t *__restrict__ qw, const uint4 *__restrict__ k_pool,
                                            uint2 *__restrict__ cand, int32_t *__restrict__ page_cnt,
                                            const uint32_t *__restrict__ tau_in,
                                            const uint32_t *__restrict__ tau_safe,
                                            const uint32_t *__restrict__ fail, uint32_t *__restrict__ hist,
                                            uint32_t *__restrict__ sample_max, int H_kv, int ppw, int mode,
                                            const FusedAppend &fa, uint32_t *head_maxkey)
{
    constexpr int phase = PHASE == 0 ? 0 : 1; // page mapping: the repair pass walks the main pass's pages
    constexpr int NC = D * (DT == 0 ? 2 : 4) / 16; // 16-byte chunks per key
    constexpr int QW = D * (DT == 0 ? 2 : 4) / 4;  // 32-bit words per query head
    // two 16-bit counters per word: a phase-0 workgroup scores 4 pages = 256 tokens per head
    __shared__ uint32_t lhist[PHASE == 0 ? G : 1][PHASE == 0 ? kHistBins / 2 : 1];
    __shared__ float wmax[kScoreWaves][G];
    const bool sample_hist_on = PHASE == 0 && mode == 0 && ppw == 1;
    if (PHASE == 0) {
        if (sample_hist_on)
            for (int i = threadIdx.x; i < G * (kHistBins / 2); i += 256) (&lhist[0][0])[i] = 0u;
        if (threadIdx.x < kScoreWaves * G) (&wmax[0][0])[threadIdx.x] = -INFINITY;
        __syncthreads();
    }

    const int kvh = block % H_kv;
    const int tile = block / H_kv;
    int r = 0;
    if (phase == 0) while (r + 1 < B && desc[r + 1].tile_start <= tile) ++r;
    else while (r + 1 < B && desc[r + 1].tileb_start <= tile) ++r;
    const ReqDesc dsc = desc[r];
    const int H_q = H_kv * G;
    const int rh0 = r * H_q + kvh * G; // first head of this group

    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    const int S = dsc.sample_stride;
    // Phase 0: wavefront w of the request takes the sampled page w * S; the wavefronts after those take
    // the pages [0, xf) and [xb, n_pages) that are sampled on top (a DIPR window, the page of a token
    // that this pass appends), leaving out the S-th pages among them.  Phase 1: wavefront w takes the aligned
    // chunk of `cp` consecutive pages [w * cp, (w + 1) * cp) without the sampled ones; cp is a power of
    // two <= S and divides xf and xb, so a chunk is either all window pages or holds at most one
    // sampled page, its first.
    const int w_req = (tile - (phase == 0 ? dsc.tile_start : dsc.tileb_start)) * kScoreWaves + wave;
    const int cp = phase == 0 ? 1 : dsc.chunk_pages;
    int p_first = w_req * cp;
    bool every_sth = true; // phase 0: this wavefront's page is one of the every-S-th sample
    if (phase == 0) {
        const int ns = (dsc.n_pages + S - 1) >> (__ffs(S) - 1); // every S-th page
        const int x = w_req - ns;
        every_sth = x < 0;
        p_first = x < 0 ? w_req * S : x < dsc.xf ? x : dsc.xb + (x - dsc.xf);
        if (x >= 0 && (p_first & (S - 1)) == 0) p_first = dsc.n_pages; // an S-th page: not this wavefront's
    }
    const int p_end = min(p_first + cp, dsc.n_pages);
    const int p_begin = (phase == 1 && (p_first & (S - 1)) == 0) ? p_first + 1 : p_first;
    if (PHASE == 1 && p_begin >= p_end) return;                  // whole wavefront; the main pass has no barriers
    if (phase == 1 && (p_first < dsc.xf || p_first >= dsc.xb)) return; // window pages: the sample pass had them
    const uint4 *qh = (const uint4 *)(qw + (size_t)rh0 * QW);    // wave-uniform address: scalar loads

    uint32_t tau[G], tau_hi[G]; // keep key >= tau; repair pass: count tau <= key < tau_hi
    uint32_t smax[G];           // main pass of a DIPR call: the head's maximum as the sample knows it
    bool act[G];                // repair pass: this head is being repaired
    bool any_act = PHASE != 2;
#pragma unroll
    for (int g = 0; g < G; ++g) {
        act[g] = PHASE != 2 || fail[rh0 + g] != 0u;
        any_act |= act[g];
        tau[g] = PHASE == 0 ? 0u : PHASE == 1 ? tau_in[rh0 + g] : tau_safe[rh0 + g];
        tau_hi[g] = PHASE == 2 ? tau_in[rh0 + g] : 0u;
        smax[g] = PHASE == 1 && mode == 1 ? head_maxkey[rh0 + g] : 0xFFFFFFFFu;
    }
    if (PHASE == 2 && !any_act) return; // whole workgroup: the usual case
    const unsigned long long lt_mask = (1ull << lane) - 1ull;

    float lmax[G];
#pragma unroll
    for (int g = 0; g < G; ++g) lmax[g] = -INFINITY;

    // The survivors of the wavefront's pages form ONE list per head.  It starts in the slot of the
    // wavefront's first page and runs on through the slots of its other pages.  Small writes mixed
    // into the read stream cost far more than their bytes, so with several pages per wavefront the
    // survivors are staged in a ring of 64 entries per head held in registers (entry i in lane i) and
    // leave as whole 512-byte blocks, plus one partial block when the wavefront is done.
    uint32_t ring_s[G], ring_j[G]; // staged entries: score bits, token id
    int pend[G], flushed[G];       // wave-uniform: entries staged / entries already written
#pragma unroll
    for (int g = 0; g < G; ++g) { ring_s[g] = 0u; ring_j[g] = 0u; pend[g] = 0; flushed[g] = 0; }
    const size_t list0 = (size_t)dsc.score_off + (size_t)p_begin * kPageTokens; // + head * head_stride

    for (int p = p_begin; p < p_end; ++p) {
        const int phys = page_table[dsc.pt_off + p];
        const uint4 *kp = k_pool;
        if (PHASE == 0 && fa.k) {
            // A decode step: the newest token's rows are not in the pools yet.  The wavefront that scores
            // its page writes them (this KV head's), waits for the writes, and reads the page through
            // the same pointer; the value row is read by later kernels only.
            kp = fa.k_pool;
            if (p == (dsc.n - 1) >> 6) {
                const int slot = (dsc.n - 1) & 63;
                const size_t tile = ((size_t)phys * H_kv + kvh) * (size_t)(NC * 64);
                const size_t src = ((size_t)r * H_kv + kvh) * NC;
                for (int c = lane; c < NC; c += 64) {
                    fa.k_pool[tile + (size_t)c * 64 + slot] = fa.k[src + c];
                    fa.v_pool[tile + (size_t)slot * NC + c] = fa.v[src + c];
                }
                asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            }
        }
        const uint4 *base = kp + ((size_t)phys * H_kv + kvh) * (size_t)(NC * 64) + lane;
        uint4 kc[NC];
#pragma unroll
        for (int c = 0; c < NC; ++c) kc[c] = base[c * 64];
        // The query (64 * G words) is streamed through scalar registers for every page.  The offset
        // is opaque to the compiler so that it does not hoist all of it out of the page loop.
        int opaque_zero = 0;
        asm volatile("" : "+s"(opaque_zero));
        const uint4 *qp = qh + opaque_zero;
        float acc[G];
#pragma unroll
        for (int g = 0; g < G; ++g) acc[g] = 0.f;
#pragma unroll
        for (int c = 0; c < NC; ++c) {
#pragma unroll
            for (int g = 0; g < G; ++g) {
                const uint4 qc = qp[g * (QW / 4) + c];
                if constexpr (DT == 0) {
                    acc[g] = dot2_bf16(kc[c].x, qc.x, acc[g]);
                    acc[g] = dot2_bf16(kc[c].y, qc.y, acc[g]);
                    acc[g] = dot2_bf16(kc[c].z, qc.z, acc[g]);
                    acc[g] = dot2_bf16(kc[c].w, qc.w, acc[g]);
                } else {
                    acc[g] = fmaf(__uint_as_float(kc[c].x), __uint_as_float(qc.x), acc[g]);
                    acc[g] = fmaf(__uint_as_float(kc[c].y), __uint_as_float(qc.y), acc[g]);
                    acc[g] = fmaf(__uint_as_float(kc[c].z), __uint_as_float(qc.z), acc[g]);
                    acc[g] = fmaf(__uint_as_float(kc[c].w), __uint_as_float(qc.w), acc[g]);
                }
            }
        }
        const int j = p * kPageTokens + lane;
        const bool valid = j < dsc.n;
        const bool win = in_window(dsc, j); // always a survivor; top-k's statistics leave it out
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const uint32_t key = ord_key(acc[g]);
            const bool keep = act[g] && valid && (win || key >= tau[g]);
            // DIPR: a score above the sample's maximum raises the head's maximum.  About S - 1 scores
            // per head do (the expected number of tokens ahead of the best of a 1-in-S sample), so
            // these atomics on one address are few; they replace a statistics kernel.
            if (PHASE == 1 && valid && key > smax[g]) atomicMax(&head_maxkey[rh0 + g], key);
            if (PHASE == 2 && keep && !win && key < tau_hi[g]) // a score the estimated bound had dropped
                atomicAdd(&hist[(size_t)(rh0 + g) * kHistBins + (key >> 21)], 1u);
            const unsigned long long m = __ballot(keep);
            const int c = __popcll(m);
            if constexpr (!RING) { // one page per wavefront: its list goes straight out
                if (keep)
                    cand[list0 + (size_t)(kvh * G + g) * dsc.head_stride + __popcll(m & lt_mask)] =
                        make_uint2(__float_as_uint(acc[g]), (uint32_t)j);
                if (lane == g && act[g])
                    page_cnt[(size_t)dsc.page_start * H_q + (size_t)(kvh * G + g) * dsc.n_pages + p] = c;
            } else if (c) {
                // Send the survivors, in lane order, to the ring positions pend .. pend + c - 1 (mod 64);
                // the other lanes take the positions left over, so that the move is a permutation.
                const int dst = keep ? pend[g] + __popcll(m & lt_mask) : pend[g] + c + __popcll(~m & lt_mask);
                const uint32_t ts = (uint32_t)__builtin_amdgcn_ds_permute((dst & 63) << 2, (int)__float_as_uint(acc[g]));
                const uint32_t tj = (uint32_t)__builtin_amdgcn_ds_permute((dst & 63) << 2, j);
                const bool fresh = ((lane - pend[g]) & 63) < c; // this lane received a survivor
                if (fresh && lane >= pend[g]) { ring_s[g] = ts; ring_j[g] = tj; }
                if (pend[g] + c >= 64) { // the ring is full: one 512-byte block leaves
                    cand[list0 + (size_t)(kvh * G + g) * dsc.head_stride + flushed[g] + lane] =
                        make_uint2(ring_s[g], ring_j[g]);
                    flushed[g] += 64;
                    if (fresh && lane < pend[g]) { ring_s[g] = ts; ring_j[g] = tj; } // those that wrapped around
                    pend[g] += c - 64;
                } else {
                    pend[g] += c;
                }
            }
            if (PHASE == 0 && valid) {
                lmax[g] = fmaxf(lmax[g], acc[g]);
                // (the pages sampled on top are no uniform sample of the request: top-k's estimate must
                // not see them; the statistics kernel counts them with the other pages' survivors)
                if (sample_hist_on && !win && every_sth) {
                    const uint32_t bin = key >> 21;
                    atomicAdd(&lhist[g][bin >> 1], 1u << ((bin & 1u) * 16u));
                }
            }
        }
    }
    // the rest of each list; its length goes to the first page's count, zero to the other pages'
#pragma unroll
    for (int g = 0; RING && g < G; ++g) {
        if (!act[g]) continue;
        if (lane < pend[g])
            cand[list0 + (size_t)(kvh * G + g) * dsc.head_stride + flushed[g] + lane] = make_uint2(ring_s[g], ring_j[g]);
        if (lane < p_end - p_begin)
            page_cnt[(size_t)dsc.page_start * H_q + (size_t)(kvh * G + g) * dsc.n_pages + p_begin + lane] =
                lane == 0 ? flushed[g] + pend[g] : 0;
    }
    if (PHASE == 0) {
        // what the sample says about this head: bucket counts (top-k) or the maximum (DIPR)
#pragma unroll
        for (int g = 0; g < G; ++g) {
            float m = lmax[g];
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o));
            if (lane == 0) wmax[wave][g] = m;
        }
        __syncthreads();
        if (mode == 1) {
            if (threadIdx.x < G) {
                float m = wmax[0][threadIdx.x];
#pragma unroll
                for (int w = 1; w < kScoreWaves; ++w) m = fmaxf(m, wmax[w][threadIdx.x]);
                if (m > -INFINITY) {
                    const uint32_t key = ord_key(m);
                    atomicMax(sample_max + (size_t)(rh0 + threadIdx.x) * kMaxSlots + (tile & (kMaxSlots - 1)), key);
                }
            }
        }
        if (sample_hist_on) {
            uint32_t *gh = hist + (size_t)rh0 * kHistBins;
            for (int i = threadIdx.x; i < G * (kHistBins / 2); i += 256) {
                const uint32_t v = (&lhist[0][0])[i];
                if (v & 0xFFFFu) atomicAdd(&gh[2 * i], v & 0xFFFFu);
                if (v >> 16) atomicAdd(&gh[2 * i + 1], v >> 16);
            }
        }
    }
}

// Phases 0 and 1: one workgroup per block.  Phase 2 is launched with a small grid whose workgroups
// leave at once unless some head was marked for repair, and otherwise share all blocks out.
template <int DT, int D, int G, int PHASE, bool RING>
__global__ __launch_bounds__(256) void score_kernel(const ReqDesc *__restrict__ desc_mem, const ReqDesc desc0, int desc_n, int B,
                                                     const int32_t *__restrict__ page_table,
                                                     const uint32_t *__restrict__ qw, const uint4 *__restrict__ k_pool,
                                                     uint2 *__restrict__ cand, int32_t *__restrict__ page_cnt,
                                                     const uint32_t *__restrict__ tau_in,
                                                     const uint32_t *__restrict__ tau_safe,
                                                     const uint32_t *__restrict__ fail,
                                                     const uint32_t *__restrict__ any_fail,
                                                     uint32_t *__restrict__ hist,
                                                     uint32_t *__restrict__ sample_max, int H_kv, int ppw, int mode,
                                                     int total_blocks, const FusedAppend fa,
                                                     uint32_t *head_maxkey)
{
    const Descs desc{desc_mem, desc0, desc_n};
    if (PHASE == 2) {
        if (*any_fail == 0u) return;
        for (int b = blockIdx.x; b < total_blocks; b += gridDim.x)
            score_block<DT, D, G, PHASE, RING>(b, desc, B, page_table, qw, k_pool, cand, page_cnt, tau_in, tau_safe,
                                               fail, hist, sample_max, H_kv, ppw, mode, fa, head_maxkey);
    } else {
        score_block<DT, D, G, PHASE, RING>(blockIdx.x, desc, B, page_table, qw, k_pool, cand, page_cnt, tau_in,
                                           tau_safe, fail, hist, sample_max, H_kv, ppw, mode, fa, head_maxkey);
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

template <int DT, int D>
static hipError_t launch_score_g(const Shape &sh, const DeviceViews &dv, int B, const void *q, int total_tiles,
                                 int ppw, int phase, int mode, hipStream_t st, hipEvent_t ev0, hipEvent_t ev1)
{
    const int G = sh.n_q_heads / sh.n_kv_heads;
    const int total_blocks = total_tiles * sh.n_kv_heads;
    const dim3 grid((unsigned)(phase == 2 && total_blocks > kRepairGrid ? kRepairGrid : total_blocks)), block(256);
#define ALAYA_SCORE_K(GG, PH, RG)                                                                             \
    launch_maybe_timed(score_kernel<DT, D, GG, PH, RG>, grid, block, st, ev0, ev1, dv.desc.mem, dv.desc.in, dv.desc.n, B, dv.page_table, \
                       (const uint32_t *)q, (const uint4 *)dv.k_pool, dv.cand, dv.page_cnt,                   \
                       (const uint32_t *)dv.tau, (const uint32_t *)dv.tau_safe, (const uint32_t *)dv.fail,    \
                       (const uint32_t *)dv.any_fail, dv.hist, dv.sample_max, sh.n_kv_heads, ppw, mode,       \
                       total_blocks, PH == 0 ? dv.fused : FusedAppend{nullptr, nullptr, nullptr, nullptr},       \
                       dv.head_maxkey)
#define ALAYA_SCORE(GG)                                                                                       \
    do {                                                                                                      \
        if (phase == 0) ALAYA_SCORE_K(GG, 0, false);                                                          \
        else if (phase == 1 && ppw == 1) ALAYA_SCORE_K(GG, 1, false);                                         \
        else if (phase == 1) ALAYA_SCORE_K(GG, 1, true);                                                      \
        else if (ppw == 1) ALAYA_SCORE_K(GG, 2, false);                                                       \
        else ALAYA_SCORE_K(GG, 2, true);                                                                      \
    } while (0)
    switch (G) {
    case 1: ALAYA_SCORE(1); break;
    case 2: ALAYA_SCORE(2); break;
    case 4: ALAYA_SCORE(4); break;
    case 8: ALAYA_SCORE(8); break;
    default: return hipErrorInvalidValue;
    }
#undef ALAYA_SCORE
#undef ALAYA_SCORE_K
    return hipGetLastError();
}

hipError_t launch_score(const Shape &sh, const DeviceViews &dv, int B, const void *q, int total_tiles, int ppw,
                        int phase, int mode, hipStream_t st, hipEvent_t ev0, hipEvent_t ev1)
{
    if (total_tiles <= 0) return hipSuccess;
    if (sh.dtype == 0) {
        if (sh.head_dim == 128) return launch_score_g<0, 128>(sh, dv, B, q, total_tiles, ppw, phase, mode, st, ev0, ev1);
        if (sh.head_dim == 64) return launch_score_g<0, 64>(sh, dv, B, q, total_tiles, ppw, phase, mode, st, ev0, ev1);
    } else {
        if (sh.head_dim == 128) return launch_score_g<1, 128>(sh, dv, B, q, total_tiles, ppw, phase, mode, st, ev0, ev1);
        if (sh.head_dim == 64) return launch_score_g<1, 64>(sh, dv, B, q, total_tiles, ppw, phase, mode, st, ev0, ev1);
    }
    return hipErrorInvalidValue;
}

// ------------------------------------------------------------------------------------------------
// tau: the lower bound of each head's selection threshold, from what the sample pass accumulated.
// One 1024-thread workgroup per (request, head); runs between the sample pass and the main pass, when
// the histogram and the maximum hold the sampled pages only.
__global__ __launch_bounds__(kSelectThreads) void tau_kernel(const ReqDesc *__restrict__ desc_mem, const ReqDesc desc0, int desc_n, int H_q, int mode,
                                                              const uint32_t *__restrict__ hist,
                                                              uint32_t *__restrict__ sample_max,
                                                              uint32_t *__restrict__ head_maxkey,
                                                              uint32_t *__restrict__ tau,
                                                              uint32_t *__restrict__ tau_safe)
{
    const Descs desc{desc_mem, desc0, desc_n};
    __shared__ int32_t wtot[kSelectThreads / 64];
    __shared__ int32_t found, found_est;

    const int rh = blockIdx.x;
    const ReqDesc dsc = desc[rh / H_q];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

    if (mode == 1) { // DIPR: (maximum over the sample) - beta
        if (tid < 64) {
            static_assert(kMaxSlots == 64, "one slot per lane");
            uint32_t mk = sample_max[(size_t)rh * kMaxSlots + tid];
            sample_max[(size_t)rh * kMaxSlots + tid] = 0u; // consumed: zero for the next call
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) mk = max(mk, (uint32_t)__shfl_xor((int)mk, o));
            if (tid == 0) {
                head_maxkey[rh] = mk; // the selection raises it further with the other pages' survivors
                tau[rh] = tau_safe[rh] = mk ? ord_key(ord_float(mk) - dsc.beta) : 0u;
            }
        }
        return;
    }
    // top-k: lower edge of the bucket that holds the k-th largest score of the sample.
    // Walk down from the top bucket: two buckets per thread, thread 0 holding the top ones.
    const uint32_t *gh = hist + (size_t)rh * kHistBins;
    const int b0 = kHistBins - 1 - 2 * tid;
    const int c0 = (int)gh[b0], c1 = (int)gh[b0 - 1];
    if (tid == 0) found = found_est = -1;
    int inc = c0 + c1;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int t = __shfl_up(inc, o);
        if (lane >= o) inc += t;
    }
    if (lane == 63) wtot[wave] = inc;
    __syncthreads();
    int above = inc - (c0 + c1);
    for (int w = 0; w < wave; ++w) above += wtot[w];
    if (above < dsc.k && above + c0 + c1 >= dsc.k) found = above + c0 >= dsc.k ? b0 : b0 - 1;
    // The estimated bound: the bucket of the sample's k_est-th largest score, k_est being the share
    // of k that a 1-in-S sample is expected to hold plus a wide margin.  Nothing guarantees it; the
    // selection checks the survivor count against k and has the head repaired if it fell short.
    const int ke = dsc.k_est;
    if (ke > 0 && above < ke && above + c0 + c1 >= ke) found_est = above + c0 >= ke ? b0 : b0 - 1;
    __syncthreads();
    if (tid == 0) {
        const uint32_t safe = found >= 0 ? (uint32_t)found << 21 : 0u; // fewer than k scores in the sample: no bound
        tau_safe[rh] = safe;
        tau[rh] = (ke > 0 && found_est >= 0) ? (uint32_t)found_est << 21 : safe;
    }
}

hipError_t launch_tau(const Shape &sh, const DeviceViews &dv, int B, int mode, hipStream_t st)
{
    tau_kernel<<<dim3((unsigned)(B * sh.n_q_heads)), dim3(kSelectThreads), 0, st>>>(
        dv.desc.mem, dv.desc.in, dv.desc.n, sh.n_q_heads, mode, dv.hist, dv.sample_max, dv.head_maxkey, dv.tau, dv.tau_safe);
    return hipGetLastError();
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

} // namespace alaya
