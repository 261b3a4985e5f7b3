// Selection of the critical tokens of every (request, query head) from the survivors the scoring
// passes wrote (every token that can possibly be selected is among them; each list is ascending).
//   top-k (Sec. 5.1.1): the k largest scores; equal scores at the k-th place go to the smaller id.
//   DIPR  (Def. 2, 3) : every token with score >= max - beta.
//   window (Sec. 7.1) : window tokens are always selected; top-k neither counts nor ranks them.
// Everything is exact and order-deterministic: counting is integer (radix select on the
// order-preserving image of the score) and placement is an ordered compaction, so the selected list
// is the same on every run.
//
// A head's pages are cut into segments; one 1024-thread workgroup owns one (head, segment).  The
// survivors of a segment are addressed through a FLAT index: the pages' survivor counts are scanned
// in LDS, and element t of the concatenation is found by a binary search over the prefix sums.  All
// loads of a pass are therefore independent, and the flat order is ascending token order.
//   stats   (top-k only) adds the survivors of the main pass's pages to what the sample pass already
//           entered for its own pages: the bucket counts (top 11 bits of the ordered key).  LDS first,
//           then at most kMaxSegs workgroups per head add to the global counters.  A DIPR call needs
//           no such pass: its main pass raises the head's maximum itself, with the few scores that
//           lie above the sample's maximum.
//   local   top-k: reads the bucket b of the k-th largest score off the histogram and checks that it
//           lies in the part of the histogram that is complete (at or above the bucket of the bound
//           the main pass filtered with); if not - possible only with an estimated bound - the head
//           is marked for the repair pass and left alone until `local` runs a second time.
//           Then classifies each survivor: "definite" (window token; top-k: bucket above b; DIPR:
//           score >= max - beta), "candidate" (top-k only: bucket == b) or neither, and compacts the
//           segment into its own region: definite tokens from the front, candidates from the back,
//           both in ascending token order.
//   finish  (top-k only; the gather kernel of a DIPR call reads the segments' lists as they are)
//           per head: gather the segments' definite lists into the head's final list (a binary search
//           over the segment prefix sums finds each element's source), gather the candidates behind
//           them, radix-refine the remaining 21 key bits over the candidates and keep key > T and the
//           first `ties` tokens with key == T (from registers when they are at most 16384, in place
//           otherwise); take the head maximum from the finished list; publish the count, copy ids
//           out if asked, and reset the head's histogram, maximum and repair mark for the next call.
#include "alaya_internal.h"

namespace alaya {

constexpr int kSelE = 4;                       // elements per thread per chunk
constexpr int kSelWaves = kSelectThreads / 64; // 16
constexpr int kSelChunk = kSelE * kSelectThreads;
constexpr int kFinSets = 4;                    // chunks of tie-bucket tokens the finishing pass keeps in registers
static_assert(kSelE * kSelWaves == 64, "the cross-wave scan maps one (e, wave) pair to one lane of wave 0");
static_assert(kMaxSegPages == 2 * kSelectThreads, "the page-count scan takes two pages per thread");

struct ScanShared {
    int32_t cnt[2][2][64]; // [parity][list][e * 16 + wave]
    int32_t tot[2][2];     // [parity][list]
};

// Ordered ranks of two flag lists over one chunk.  Element (e, tid) is chunk position e*1024 + tid.
// On return exA[e] / exB[e] are the number of flagged elements before it inside the chunk (for every
// element, flagged or not) and totA / totB the chunk totals.  Two barriers; `parity` alternates per call.
__device__ __forceinline__ void chunk_ranks(ScanShared &sh, int parity, const bool *fa, const bool *fb,
                                            int *exA, int *exB, int &totA, int &totB)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int ra[kSelE], rb[kSelE];
#pragma unroll
    for (int e = 0; e < kSelE; ++e) {
        const unsigned long long ba = __ballot(fa[e]), bb = __ballot(fb[e]);
        const unsigned long long lt = (1ull << lane) - 1ull;
        ra[e] = __popcll(ba & lt);
        rb[e] = __popcll(bb & lt);
        if (lane == 0) {
            sh.cnt[parity][0][e * kSelWaves + wave] = __popcll(ba);
            sh.cnt[parity][1][e * kSelWaves + wave] = __popcll(bb);
        }
    }
    __syncthreads();
    if (wave == 0) {
        const int a = sh.cnt[parity][0][lane], b = sh.cnt[parity][1][lane];
        int ia = a, ib = b;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int ta = __shfl_up(ia, o), tb = __shfl_up(ib, o);
            if (lane >= o) { ia += ta; ib += tb; }
        }
        sh.cnt[parity][0][lane] = ia - a;
        sh.cnt[parity][1][lane] = ib - b;
        if (lane == 63) { sh.tot[parity][0] = ia; sh.tot[parity][1] = ib; }
    }
    __syncthreads();
#pragma unroll
    for (int e = 0; e < kSelE; ++e) {
        exA[e] = sh.cnt[parity][0][e * kSelWaves + wave] + ra[e];
        exB[e] = sh.cnt[parity][1][e * kSelWaves + wave] + rb[e];
    }
    totA = sh.tot[parity][0];
    totB = sh.tot[parity][1];
}

// Find the bin that holds the `need`-th largest element of a histogram, walking from the top bin
// down: res[0] = bin, res[1] = elements in bins above it.  All 1024 threads take part (nbins is 1024
// or 2048: one or two bins per thread, thread 0 holding the top ones).  Two barriers.  If the
// histogram holds fewer than `need` elements nothing is written.
__device__ __forceinline__ void block_find_bin(const uint32_t *hist, int nbins, int need, int32_t *wtot,
                                               int32_t *res)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int per = nbins / kSelectThreads;
    const int b0 = nbins - 1 - per * tid;
    const int c0 = (int)hist[b0];
    const int c1 = per == 2 ? (int)hist[b0 - 1] : 0;
    const int local = c0 + c1;
    int inc = local;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int t = __shfl_up(inc, o);
        if (lane >= o) inc += t;
    }
    if (lane == 63) wtot[wave] = inc;
    __syncthreads();
    int above = inc - local;
    for (int w = 0; w < wave; ++w) above += wtot[w];
    if (above < need && above + local >= need) {
        if (above + c0 >= need) { res[0] = b0; res[1] = above; }
        else { res[0] = b0 - 1; res[1] = above + c0; }
    }
    __syncthreads();
}

// blockIdx -> (request, head, segment).  Heads are the fastest index.
struct SegId { int r, h, seg; };
__device__ __forceinline__ SegId seg_of_block(const Descs &desc, int B, int H_q)
{
    const int h = blockIdx.x % H_q;
    const int gs = blockIdx.x / H_q;
    int r = 0;
    while (r + 1 < B && desc[r + 1].seg_start <= gs) ++r;
    return {r, h, gs - desc[r].seg_start};
}

// The survivors of the pages [p_begin, p_end) of one head, addressed by a flat index.  A list may be
// longer than its page's 64 slots (it then covers the slots of the pages behind it, whose own counts
// are 0); no list crosses a segment boundary.
struct SegView {
    int p_begin, np, total; // first page, pages, survivors
    size_t base;            // element offset of (page 0, this head) in the survivor arrays
    size_t page_stride;     // elements between the slots of consecutive pages
};

// Loads the pages' survivor counts (two pages per thread) ...
__device__ __forceinline__ SegView begin_segment(const ReqDesc &dsc, int H_q, int h, int seg,
                                                 const int32_t *__restrict__ page_cnt, int &a0, int &a1)
{
    const int tid = threadIdx.x;
    SegView v;
    v.p_begin = seg * dsc.seg_pages;
    v.np = min(dsc.n_pages, v.p_begin + dsc.seg_pages) - v.p_begin;
    v.base = (size_t)dsc.score_off + (size_t)h * dsc.head_stride;
    v.page_stride = kPageTokens;
    v.total = 0;
    const int32_t *cnt = page_cnt + (size_t)dsc.page_start * H_q + (size_t)h * dsc.n_pages + v.p_begin;
    const int i0 = 2 * tid, i1 = 2 * tid + 1;
    a0 = i0 < v.np ? cnt[i0] : 0;
    a1 = i1 < v.np ? cnt[i1] : 0;
    return v;
}

// ... and leaves their exclusive prefix sums in off[0 .. np] (off[np] = total).  Two barriers.
__device__ __forceinline__ void scan_segment(SegView &v, int a0, int a1, int32_t *off, int32_t *wtot)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int i0 = 2 * tid, i1 = 2 * tid + 1;
    int inc = a0 + a1;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int t = __shfl_up(inc, o);
        if (lane >= o) inc += t;
    }
    if (lane == 63) wtot[wave] = inc;
    __syncthreads();
    int pre = inc - (a0 + a1);
    for (int w = 0; w < wave; ++w) pre += wtot[w];
    if (i0 <= v.np) off[i0] = pre;
    if (i1 <= v.np) off[i1] = pre + a0;
    if (tid == kSelectThreads - 1 && v.np == kMaxSegPages) off[v.np] = pre + a0 + a1;
    __syncthreads();
    v.total = off[v.np];
}

// Flat index t -> element offset in the survivor arrays.
__device__ __forceinline__ size_t flat_to_offset(const SegView &v, const int32_t *off, int t)
{
    int lo = 0, hi = v.np; // page index in [lo, hi): the last page whose prefix is <= t
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (off[mid] <= t) lo = mid; else hi = mid;
    }
    return v.base + (size_t)(v.p_begin + lo) * v.page_stride + (size_t)(t - off[lo]);
}

// What a survivor's score means for the selection, given the head's threshold data.
struct Rule {
    int topk;     // 1: bucket rule, 0: threshold rule
    uint32_t b1;  // bucket of the k-th score
    float thr;    // threshold rule: definite iff score >= thr
    // win: the token is in the window (always selected; top-k neither counts nor ranks it)
    __device__ __forceinline__ void classify(float v, bool in, bool win, bool &definite, bool &candidate) const
    {
        if (topk) {
            const uint32_t bin = ord_key(v) >> 21;
            definite = in && (win || bin > b1);
            candidate = in && !win && bin == b1;
        } else {
            definite = in && (win || v >= thr);
            candidate = false;
        }
    }
};

// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kSelectThreads) void select_stats_kernel(
    const ReqDesc *__restrict__ desc_mem, const ReqDesc desc0, int desc_n, int B, int H_q, const uint2 *__restrict__ cand,
    const int32_t *__restrict__ page_cnt, uint32_t *__restrict__ hist)
{
    const Descs desc{desc_mem, desc0, desc_n};
    __shared__ uint32_t lh[kHistBins];
    __shared__ int32_t off[kMaxSegPages + 1];
    __shared__ int32_t wtot[kSelWaves];

    const SegId id = seg_of_block(desc, B, H_q);
    const ReqDesc dsc = desc[id.r];
    const int rh = id.r * H_q + id.h;
    const int tid = threadIdx.x;
    // The every-S-th pages entered the histogram when they were scored.
    const int S = dsc.sample_stride;
    if (S == 1) return;                        // whole workgroup: every page was a sampled page
    if (dsc.k >= dsc.n - dsc.nwin) return;     // every token is taken: nothing to rank
    for (int i = tid; i < kHistBins; i += kSelectThreads) lh[i] = 0u;
    int a0, a1;
    SegView v = begin_segment(dsc, H_q, id.h, id.seg, page_cnt, a0, a1);
    if (((v.p_begin + 2 * tid) & (S - 1)) == 0) a0 = 0;
    if (((v.p_begin + 2 * tid + 1) & (S - 1)) == 0) a1 = 0;
    scan_segment(v, a0, a1, off, wtot); // barriers inside
    constexpr int U = 4; // independent loads per thread and step
    for (int t0 = tid; t0 < v.total; t0 += U * kSelectThreads) {
        float s[U];
        bool ranked[U]; // a survivor outside the window: the histogram counts only those
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int t = t0 + u * kSelectThreads;
            const bool in = t < v.total;
            const uint2 pr = in ? cand[flat_to_offset(v, off, t)] : make_uint2(0u, 0u);
            s[u] = __uint_as_float(pr.x);
            ranked[u] = in && !in_window(dsc, (int)pr.y);
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (ranked[u]) atomicAdd(&lh[ord_key(s[u]) >> 21], 1u);
    }
    __syncthreads();
    for (int i = tid; i < kHistBins; i += kSelectThreads)
        if (lh[i]) atomicAdd(&hist[(size_t)rh * kHistBins + i], lh[i]);
}

// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kSelectThreads) void select_local_kernel(
    const ReqDesc *__restrict__ desc_mem, const ReqDesc desc0, int desc_n, int B, int H_q, int mode, const uint2 *__restrict__ cand,
    const int32_t *__restrict__ page_cnt,
    const uint32_t *__restrict__ hist, const uint32_t *__restrict__ head_maxkey, float *__restrict__ head_M,
    int32_t *__restrict__ head_info, int32_t *__restrict__ seg_counts, float *__restrict__ loc_scores,
    int32_t *__restrict__ loc_ids, const uint32_t *__restrict__ tau, uint32_t *__restrict__ fail,
    uint32_t *__restrict__ any_fail, int redo)
{
    const Descs desc{desc_mem, desc0, desc_n};
    __shared__ uint32_t lh[kHistBins];
    __shared__ int32_t off[kMaxSegPages + 1];
    __shared__ ScanShared scan;
    __shared__ int32_t wtot[kSelWaves];
    __shared__ int32_t res[2];

    if (redo && *any_fail == 0u) return; // second run, and nothing was marked: the usual case
    const SegId id = seg_of_block(desc, B, H_q);
    const ReqDesc dsc = desc[id.r];
    const int rh = id.r * H_q + id.h;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (redo && fail[rh] == 0u) return; // second run: only the heads that the repair pass rewrote

    // issue every independent load first: the page counts, the maximum, the histogram
    int a0, a1;
    SegView v = begin_segment(dsc, H_q, id.h, id.seg, page_cnt, a0, a1);
    const float M = ord_float(head_maxkey[rh]);
    const bool bucket_rule = mode == 0 && dsc.k < dsc.n - dsc.nwin;
    if (bucket_rule) {
        for (int i = tid; i < kHistBins; i += kSelectThreads) lh[i] = hist[(size_t)rh * kHistBins + i];
        if (tid == 0) res[0] = -1;
        __syncthreads();
        block_find_bin(lh, kHistBins, dsc.k, wtot, res);
        // The histogram is complete from the bucket of the main pass's bound upwards (below it only
        // the sampled pages are counted).  If the k-th largest score does not lie in that part, the
        // bound - an estimate then - was too high and tokens are missing: every workgroup of the
        // head sees the same histogram, steps aside, and the head is marked for the repair pass.
        const int b_bound = dsc.sample_stride > 1 ? (int)(tau[rh] >> 21) : 0;
        if (!redo && (res[0] < 0 || res[0] < b_bound)) {
            if (id.seg == 0 && tid == 0) {
                fail[rh] = 1u;
                *any_fail = 1u; // (several heads may write the same 1)
            }
            return;
        }
    }
    Rule rule;
    rule.topk = bucket_rule;
    rule.b1 = bucket_rule ? (uint32_t)res[0] : 0u;
    rule.thr = mode == 1 ? M - dsc.beta : -INFINITY; // top-k with k >= n: every token
    if (id.seg == 0 && tid == 0) {
        if (mode == 1) head_M[rh] = M; // top-k: written by the finishing pass (a DIPR call has none)
        head_info[2 * rh] = bucket_rule ? res[0] : -1;
        head_info[2 * rh + 1] = bucket_rule ? res[1] : 0;
    }
    __syncthreads(); // wtot is reused below
    scan_segment(v, a0, a1, off, wtot);

    // Ordered placement into the segment's region, chunk by chunk in flat (= token) order: definite
    // tokens grow from the front, candidates from the back (so they end up in descending token order;
    // the finishing pass reads them backwards).
    const size_t loc = (size_t)dsc.score_off + (size_t)id.h * dsc.head_stride +
                       (size_t)id.seg * dsc.seg_pages * kPageTokens;
    const size_t last = loc + (size_t)v.np * kPageTokens - 1; // the region holds np * 64 elements
    int baseA = 0, baseC = 0, parity = 0;
    for (int c0 = 0; c0 < v.total; c0 += kSelChunk) {
        float sv[kSelE];
        int tok[kSelE];
        bool fa[kSelE], fc[kSelE];
#pragma unroll
        for (int e = 0; e < kSelE; ++e) {
            const int t = c0 + e * kSelectThreads + tid;
            const bool in = t < v.total;
            const size_t o = in ? flat_to_offset(v, off, t) : v.base;
            const uint2 pr = in ? cand[o] : make_uint2(0u, 0u);
            sv[e] = __uint_as_float(pr.x);
            tok[e] = (int)pr.y;
            rule.classify(sv[e], in, in_window(dsc, tok[e]), fa[e], fc[e]);
        }
        int exA[kSelE], exC[kSelE], totA, totC;
        chunk_ranks(scan, parity, fa, fc, exA, exC, totA, totC);
        parity ^= 1;
#pragma unroll
        for (int e = 0; e < kSelE; ++e) {
            if (fa[e]) { loc_scores[loc + baseA + exA[e]] = sv[e]; loc_ids[loc + baseA + exA[e]] = tok[e]; }
            if (fc[e]) { loc_scores[last - (baseC + exC[e])] = sv[e]; loc_ids[last - (baseC + exC[e])] = tok[e]; }
        }
        baseA += totA;
        baseC += totC;
    }
    if (tid == 0) {
        seg_counts[((size_t)rh * kMaxSegs + id.seg) * 2] = baseA;
        seg_counts[((size_t)rh * kMaxSegs + id.seg) * 2 + 1] = baseC;
    }
}

// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kSelectThreads) void select_finish_kernel(
    const ReqDesc *__restrict__ desc_mem, const ReqDesc desc0, int desc_n, int H_q, const int32_t *__restrict__ head_info,
    const int32_t *__restrict__ seg_counts, const float *__restrict__ loc_scores,
    const int32_t *__restrict__ loc_ids, uint32_t *__restrict__ hist, uint32_t *__restrict__ head_maxkey,
    int32_t *__restrict__ sel_ids, float *__restrict__ sel_scores, int32_t *__restrict__ counts,
    int32_t *__restrict__ out_ids, int32_t *__restrict__ out_counts, int64_t ids_stride,
    int32_t *__restrict__ status, float *__restrict__ head_M, uint32_t *__restrict__ fail,
    uint32_t *__restrict__ any_fail)
{
    const Descs desc{desc_mem, desc0, desc_n};
    __shared__ uint32_t lh[kHistBins];
    __shared__ float wred[kSelWaves];
    __shared__ ScanShared scan;
    __shared__ int32_t preA[kMaxSegs + 1], preC[kMaxSegs + 1], cntA[kMaxSegs];
    __shared__ int32_t wtot[kSelWaves];
    __shared__ int32_t res[2];

    const int rh = blockIdx.x;
    const int r = rh / H_q, h = rh % H_q;
    const ReqDesc dsc = desc[r];
    const int tid = threadIdx.x, lane = tid & 63;
    const size_t off = (size_t)dsc.score_off + (size_t)h * dsc.head_stride;
    int32_t *ids = sel_ids + off;
    float *ss = sel_scores + off;
    const float *ls = loc_scores + off;
    const int32_t *li = loc_ids + off;
    const size_t seg_region = (size_t)dsc.seg_pages * kPageTokens;
    const int nseg = dsc.nseg;

    if (tid < 64) {
        int a = 0, c = 0;
        if (lane < nseg) {
            a = seg_counts[((size_t)rh * kMaxSegs + lane) * 2];
            c = seg_counts[((size_t)rh * kMaxSegs + lane) * 2 + 1];
        }
        int ia = a, ic = c;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int ta = __shfl_up(ia, o), tc = __shfl_up(ic, o);
            if (lane >= o) { ia += ta; ic += tc; }
        }
        preA[lane] = ia - a; // exclusive
        preC[lane] = ic - c;
        cntA[lane] = a;
        if (lane == 63) { preA[64] = ia; preC[64] = ic; }
    }
    __syncthreads();
    const int totA = preA[64], totC = preC[64];

    // gather: element e of the concatenation lives in the last segment whose prefix is <= e
    auto find_seg = [&](const int32_t *pre, int e) {
        int lo = 0, hi = nseg; // answer in [lo, hi)
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (pre[mid] <= e) lo = mid; else hi = mid;
        }
        return lo;
    };
    float mx = -INFINITY; // maximum of the scores this thread enters into the final list
    for (int e = tid; e < totA; e += kSelectThreads) {
        const int s = find_seg(preA, e);
        const size_t src = (size_t)s * seg_region + (size_t)(e - preA[s]);
        const float x = ls[src];
        ids[e] = li[src];
        ss[e] = x;
        mx = fmaxf(mx, x);
    }
    const bool bucket_rule = head_info[2 * rh] >= 0;
    int count = totA;

    if (bucket_rule && totC <= kFinSets * kSelChunk) {
        // The usual case: the tie bucket's tokens fit in registers (kFinSets sets of four per thread,
        // in token order).  They are gathered once, refined from registers, and only the kept ones
        // are written.
        const uint32_t b1 = (uint32_t)head_info[2 * rh];
        const int cb = totC;
        int need = dsc.k + dsc.nwin - totA; // 1 <= need <= cb (totA counts the window's tokens too)
        float v[kFinSets][kSelE];
        int idv[kFinSets][kSelE];
        uint32_t key[kFinSets][kSelE];
        bool in[kFinSets][kSelE];
#pragma unroll
        for (int s = 0; s < kFinSets; ++s) {
#pragma unroll
            for (int e = 0; e < kSelE; ++e) {
                in[s][e] = false;
                v[s][e] = 0.f;
                idv[s][e] = 0;
                key[s][e] = 0u;
            }
        }
#pragma unroll
        for (int s = 0; s < kFinSets; ++s) {
            if (s * kSelChunk >= cb) break; // (uniform) the sets behind the last candidate stay empty
#pragma unroll
            for (int e = 0; e < kSelE; ++e) {
                const int i = s * kSelChunk + e * kSelectThreads + tid;
                in[s][e] = i < cb;
                const int sgm = in[s][e] ? find_seg(preC, i) : 0;
                const int np_s = min(dsc.n_pages, (sgm + 1) * dsc.seg_pages) - sgm * dsc.seg_pages;
                const size_t src =
                    (size_t)sgm * seg_region + (size_t)np_s * kPageTokens - 1 - (size_t)(i - preC[sgm]);
                v[s][e] = in[s][e] ? ls[src] : 0.f;
                idv[s][e] = in[s][e] ? li[src] : 0;
                key[s][e] = ord_key(v[s][e]);
            }
        }
        uint32_t T = 0u; // keep key > T, and the first `ties` tokens with key == T
        int ties = 0;
        if (need < cb) {
            for (int i = tid; i < kHistBins; i += kSelectThreads) lh[i] = 0u;
            __syncthreads();
#pragma unroll
            for (int s = 0; s < kFinSets; ++s) {
                if (s * kSelChunk >= cb) break;
#pragma unroll
                for (int e = 0; e < kSelE; ++e)
                    if (in[s][e]) atomicAdd(&lh[(key[s][e] >> 10) & 0x7FFu], 1u);
            }
            __syncthreads();
            block_find_bin(lh, 2048, need, wtot, res);
            const uint32_t b2 = (uint32_t)res[0];
            need -= res[1];
            __syncthreads();
            for (int i = tid; i < 1024; i += kSelectThreads) lh[i] = 0u;
            __syncthreads();
            const uint32_t pre = (b1 << 11) | b2; // key >> 10 of the threshold
#pragma unroll
            for (int s = 0; s < kFinSets; ++s) {
                if (s * kSelChunk >= cb) break;
#pragma unroll
                for (int e = 0; e < kSelE; ++e)
                    if (in[s][e] && (key[s][e] >> 10) == pre) atomicAdd(&lh[key[s][e] & 0x3FFu], 1u);
            }
            __syncthreads();
            block_find_bin(lh, 1024, need, wtot, res);
            T = (pre << 10) | (uint32_t)res[0];
            ties = need - res[1];
        }
        int baseG = 0, baseT = 0; // kept-above and tie tokens in the sets before this one
#pragma unroll
        for (int s = 0; s < kFinSets; ++s) {
            if (s * kSelChunk >= cb) break; // (uniform)
            bool fa[kSelE], fb[kSelE];
#pragma unroll
            for (int e = 0; e < kSelE; ++e) {
                fa[e] = in[s][e] && key[s][e] > T;
                fb[e] = in[s][e] && key[s][e] == T;
            }
            int exA[kSelE], exB[kSelE], tA, tB;
            chunk_ranks(scan, s & 1, fa, fb, exA, exB, tA, tB);
#pragma unroll
            for (int e = 0; e < kSelE; ++e) {
                const int tb = baseT + exB[e]; // ties before this element
                if (fa[e] || (fb[e] && tb < ties)) {
                    const int pos = totA + baseG + exA[e] + min(tb, ties);
                    ids[pos] = idv[s][e];
                    ss[pos] = v[s][e];
                    mx = fmaxf(mx, v[s][e]);
                }
            }
            baseG += tA;
            baseT += tB;
        }
        count = dsc.k + dsc.nwin;
    } else if (bucket_rule) {
        for (int e = tid; e < totC; e += kSelectThreads) {
            const int s = find_seg(preC, e);
            const int np_s = min(dsc.n_pages, (s + 1) * dsc.seg_pages) - s * dsc.seg_pages;
            const size_t src = (size_t)s * seg_region + (size_t)np_s * kPageTokens - 1 - (size_t)(e - preC[s]);
            const float x = ls[src];
            ids[totA + e] = li[src];
            ss[totA + e] = x;
            mx = fmaxf(mx, x); // the candidates dropped below are the smallest ones
        }
        __syncthreads(); // candidates visible to the whole workgroup
        const uint32_t b1 = (uint32_t)head_info[2 * rh];
        const int above1 = totA; // every window token and every token above bucket b1
        const int cb = totC;
        int need = dsc.k + dsc.nwin - above1; // 1 <= need <= cb (above1 counts the window's tokens too)
        int parity = 0;
        if (need < cb) {
            // refine over the candidates: key bits [20:10], then bits [9:0]
            const float *cs = ss + above1;
            for (int i = tid; i < kHistBins; i += kSelectThreads) lh[i] = 0u;
            __syncthreads();
            for (int i = tid; i < cb; i += kSelectThreads) atomicAdd(&lh[(ord_key(cs[i]) >> 10) & 0x7FFu], 1u);
            __syncthreads();
            block_find_bin(lh, 2048, need, wtot, res);
            const uint32_t b2 = (uint32_t)res[0];
            need -= res[1];
            __syncthreads();
            for (int i = tid; i < 1024; i += kSelectThreads) lh[i] = 0u;
            __syncthreads();
            const uint32_t pre = (b1 << 11) | b2; // key >> 10 of the threshold
            for (int i = tid; i < cb; i += kSelectThreads) {
                const uint32_t key = ord_key(cs[i]);
                if ((key >> 10) == pre) atomicAdd(&lh[key & 0x3FFu], 1u);
            }
            __syncthreads();
            block_find_bin(lh, 1024, need, wtot, res);
            const uint32_t T = (pre << 10) | (uint32_t)res[0];
            const int ties = need - res[1]; // tokens with key == T that are taken, smallest ids first
            // ordered in-place compaction of the candidates (writes never pass the chunk being read)
            int baseG = 0, baseT = 0;
            for (int c0 = 0; c0 < cb; c0 += kSelChunk) {
                float v[kSelE];
                int idv[kSelE];
                bool fa[kSelE], fb[kSelE];
#pragma unroll
                for (int e = 0; e < kSelE; ++e) {
                    const int i = c0 + e * kSelectThreads + tid;
                    v[e] = i < cb ? cs[i] : 0.f;
                    idv[e] = i < cb ? ids[above1 + i] : 0;
                    const uint32_t key = ord_key(v[e]);
                    fa[e] = i < cb && key > T;
                    fb[e] = i < cb && key == T;
                }
                int exA[kSelE], exB[kSelE], tA, tB;
                chunk_ranks(scan, parity, fa, fb, exA, exB, tA, tB); // barriers: this chunk is fully read
                parity ^= 1;
#pragma unroll
                for (int e = 0; e < kSelE; ++e) {
                    const int tb = baseT + exB[e]; // ties before this element
                    if (fa[e] || (fb[e] && tb < ties)) {
                        const int pos = above1 + baseG + exA[e] + min(tb, ties);
                        ids[pos] = idv[e];
                        ss[pos] = v[e];
                    }
                }
                baseG += tA;
                baseT += tB;
            }
        }
        count = dsc.k + dsc.nwin;
    }

#pragma unroll
    for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
    if (lane == 0) wred[tid >> 6] = mx;
    __syncthreads(); // list complete and visible to the whole workgroup
    if (tid == 0) {
        float M = wred[0]; // the largest score overall is the largest selected one
        for (int w = 1; w < kSelWaves; ++w) M = fmaxf(M, wred[w]);
        head_M[rh] = M;
        counts[rh] = count;
        if (out_counts) out_counts[rh] = count;
        if (out_ids && (int64_t)count > ids_stride) atomicOr(status, 1);
        head_maxkey[rh] = 0u; // leave the running maximum, the histogram and the repair mark clean for the next call
        fail[rh] = 0u;
        if (rh == 0) *any_fail = 0u;
    }
    if (out_ids) {
        const int m = (int)((int64_t)count < ids_stride ? (int64_t)count : ids_stride);
        int32_t *dst = out_ids + (size_t)rh * (size_t)ids_stride;
        for (int i = tid; i < m; i += kSelectThreads) dst[i] = ids[i];
    }
    for (int i = tid; i < kHistBins; i += kSelectThreads) hist[(size_t)rh * kHistBins + i] = 0u;
}

hipError_t launch_select_front(const Shape &sh, const DeviceViews &dv, int B, int mode, int total_segs,
                               hipStream_t st)
{
    const dim3 block(kSelectThreads);
    const dim3 seg_grid((unsigned)(total_segs * sh.n_q_heads));
    // (a DIPR call needs no statistics: its main pass raises the maximum itself)
    if (mode == 0)
        select_stats_kernel<<<seg_grid, block, 0, st>>>(dv.desc.mem, dv.desc.in, dv.desc.n, B, sh.n_q_heads, dv.cand,
                                                        dv.page_cnt, dv.hist);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    select_local_kernel<<<seg_grid, block, 0, st>>>(dv.desc.mem, dv.desc.in, dv.desc.n, B, sh.n_q_heads, mode, dv.cand, dv.page_cnt, dv.hist,
                                                    dv.head_maxkey, dv.head_M, dv.head_info, dv.seg_counts,
                                                    dv.loc_scores, dv.loc_ids, dv.tau, dv.fail, dv.any_fail, 0);
    return hipGetLastError();
}

hipError_t launch_select_back(const Shape &sh, const DeviceViews &dv, int B, int mode, int total_segs, bool redo,
                              int32_t *out_ids, int32_t *out_counts, int64_t ids_stride, hipStream_t st)
{
    const dim3 block(kSelectThreads);
    if (redo) {
        const dim3 seg_grid((unsigned)(total_segs * sh.n_q_heads));
        select_local_kernel<<<seg_grid, block, 0, st>>>(dv.desc.mem, dv.desc.in, dv.desc.n, B, sh.n_q_heads, mode, dv.cand, dv.page_cnt,
                                                        dv.hist, dv.head_maxkey, dv.head_M, dv.head_info,
                                                        dv.seg_counts, dv.loc_scores, dv.loc_ids, dv.tau, dv.fail, dv.any_fail,
                                                        1);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    select_finish_kernel<<<dim3((unsigned)(B * sh.n_q_heads)), block, 0, st>>>(
        dv.desc.mem, dv.desc.in, dv.desc.n, sh.n_q_heads, dv.head_info, dv.seg_counts, dv.loc_scores, dv.loc_ids, dv.hist,
        dv.head_maxkey, dv.sel_ids, dv.sel_scores, dv.counts, out_ids, out_counts, ids_stride, dv.status,
        dv.head_M, dv.fail, dv.any_fail);
    return hipGetLastError();
}

} // namespace alaya
