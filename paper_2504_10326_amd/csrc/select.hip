// Selection of the critical tokens of every (request, query head) from the survivors the main scoring
// pass wrote (every token that can possibly be selected is among them).
//   top-k (Sec. 6.1.1): the k largest scores; equal scores at the k-th place go to the smaller id.
//   DIPR  (Def. 2, 3) : every token with score >= max - beta.
//   window (Sec. 7.1) : window tokens are always selected; top-k neither counts nor ranks them.
// The coarse-grained index (Sec. 6.2) selects pages with the same kernel: the survivors then are (block score,
// page) pairs, and every selected page is also marked in the page mask that the main scoring pass reads.
// Everything is exact and order-deterministic: counting is integer (radix select on the
// order-preserving image of the score) and placement is an ordered compaction, so the selected list
// is the same on every run: ascending by token.
//
// One 1024-thread workgroup per (request, head).  The head's survivors sit in one block per main-pass
// workgroup; the blocks' counts are scanned in LDS (kSelBatch blocks at a time) and element t of the
// concatenation is found by a binary search over the prefix sums, so that all loads of a pass are
// independent and the flat order is ascending token order.
//   top-k: three counting passes find the exact 32-bit key T of the k-th largest score (11 + 11 + 10
//          bits, a histogram in LDS each) and the number of tokens with key == T that are kept
//          (`ties`, smallest ids first); one placement pass writes the selected tokens.  If fewer
//          than k tokens survived - possible only when the main pass filtered with an ESTIMATED bound -
//          the head is marked for the repair pass and left alone until the kernel runs again.
//   DIPR:  the maximum is known (the main pass raised it); one placement pass.
// The first 16384 survivors (the usual case: the bound leaves one to two times k) are read once and kept in
// registers for all passes; what lies beyond them is streamed from the blocks once per pass.
#include "alaya_internal.h"
#include <type_traits>

namespace alaya {

constexpr int kSelE = 4;                       // elements per thread per chunk
constexpr int kSelWaves = kSelectThreads / 64; // 16
constexpr int kSelChunk = kSelE * kSelectThreads;
constexpr int kRegSets = 4;                    // chunks of survivors kept in registers
static_assert(kSelE * kSelWaves == 64, "the cross-wave scan maps one (e, wave) pair to one lane of wave 0");
static_assert(kSelBatch == 4 * kSelectThreads, "the block-count scan takes four blocks per thread");

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
        const int ia = wave_scan(a), ib = wave_scan(b);
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
    const int inc = wave_scan(local);
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

// lh[bin] += 1 for every lane with `on`.  Atomics of many lanes on one LDS word are carried out one after the
// other.  When the scores crowd into one bucket (many equal keys) the lanes that share the first active lane's
// bucket are therefore counted with a ballot and added at once (crowded); when they are spread, that costs more
// vector instructions than the conflicts it saves (a counting pass over 3600 survivors: 2.4 us merging bucket
// after bucket three rounds deep, 1.5 us with every lane adding for itself), so a wavefront looks at the first
// survivors it counts in a pass (is_crowded) and goes on as they suggest.
__device__ __forceinline__ bool is_crowded(uint32_t bin, bool on)
{
    const unsigned long long act = __ballot(on);
    if (act == 0ull) return false;
    const uint32_t lb = (uint32_t)__builtin_amdgcn_readlane((int)bin, __ffsll((long long)act) - 1);
    return 8 * __popcll(__ballot(on && bin == lb)) >= 7 * __popcll(act) && __popcll(act) >= 16;
}

__device__ __forceinline__ void hist_add(uint32_t *lh, uint32_t bin, bool on, bool crowded)
{
    if (crowded) {
        const unsigned long long act = __ballot(on);
        if (act == 0ull) return;
        const int leader = __ffsll((long long)act) - 1;
        const uint32_t lb = (uint32_t)__builtin_amdgcn_readlane((int)bin, leader); // (leader is wave-uniform: no trip through LDS)
        const unsigned long long same = __ballot(on && bin == lb);
        if ((int)(threadIdx.x & 63) == leader) atomicAdd(&lh[lb], (uint32_t)__popcll(same));
        on = on && bin != lb;
    }
    if (on) atomicAdd(&lh[bin], 1u);
}

// Where one head's survivors are: its KV head's blocks, and its slot in their headers.
struct HeadBlocks {
    BlockArea area;
    int H_kv, G, kvh, g;
    __device__ __forceinline__ size_t block(int tile) const { return (size_t)tile * H_kv + kvh; }
    __device__ __forceinline__ uint2 header(int tile) const { return *area.hdr(tile, kvh * G + g); } // {count, start}
    __device__ __forceinline__ uint2 pair(int tile, int p) const { return *area.at(block(tile), p); } // p-th of the block
};

// The survivors of one head in a batch of consecutive blocks, addressed by a flat index.
struct Batch {
    int first_tile; // tile of the batch's first block
    int nb;         // blocks in the batch
    int total;      // survivors in the batch
};

// Loads the {count, start} headers of the batch's blocks (four blocks per thread), leaves the exclusive
// prefix sums of the counts in off[0 .. nb] and the starts in st[0 .. nb).  Three barriers.
__device__ __forceinline__ Batch load_batch(const HeadBlocks &hb, int first_tile, int nb, int32_t *off, int32_t *st,
                                            int32_t *wtot)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int a[4], s4[4];
    int sum = 0;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int i = 4 * tid + u;
        uint2 hd = make_uint2(0u, 0u);
        if (i < nb) hd = hb.header(first_tile + i);
        a[u] = (int)hd.x;
        s4[u] = (int)hd.y;
        sum += a[u];
    }
    const int inc = wave_scan(sum);
    __syncthreads(); // wtot, off, st: the readers of the batch before this one are done
    if (lane == 63) wtot[wave] = inc;
    __syncthreads();
    int pre = inc - sum;
    for (int w = 0; w < wave; ++w) pre += wtot[w];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int i = 4 * tid + u;
        if (i <= nb) off[i] = pre;
        if (i < nb) st[i] = s4[u];
        pre += a[u];
    }
    if (tid == kSelectThreads - 1 && nb == kSelBatch) off[nb] = pre;
    __syncthreads();
    Batch b;
    b.first_tile = first_tile;
    b.nb = nb;
    b.total = off[nb];
    return b;
}

// The last block of a batch whose prefix is <= t, searched among the blocks [lo, hi).
__device__ __forceinline__ int batch_block(const int32_t *off, int lo, int hi, int t)
{
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (off[mid] <= t) lo = mid; else hi = mid;
    }
    return lo;
}

// Flat index t of a batch -> the pair.
__device__ __forceinline__ uint2 batch_pair(const HeadBlocks &hb, const Batch &b, const int32_t *off, const int32_t *st, int t)
{
    const int lo = batch_block(off, 0, b.nb, t);
    return hb.pair(b.first_tile + lo, st[lo] + (t - off[lo]));
}

// The same for the 64 consecutive flat indices that the lanes of a wavefront hold (t - lane a multiple
// of 64): the block of the group's first index is known (gfirst, one entry per group of 64, so that the
// lookup is a broadcast), and the lanes search only the few blocks that the group spans.
__device__ __forceinline__ uint2 batch_pair_grouped(const HeadBlocks &hb, const Batch &b, const int32_t *off, const int32_t *st,
                                                    const int32_t *gfirst, int t)
{
    const int grp = t >> 6;
    const int lo = batch_block(off, gfirst[grp], min(b.nb, gfirst[grp + 1] + 1), t);
    return hb.pair(b.first_tile + lo, st[lo] + (t - off[lo]));
}

// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kSelectThreads) void select_kernel(
    const ReqDesc *__restrict__ desc_mem, const ReqDesc desc0, int desc_n, int H_q, int H_kv, int mode,
    const BlockArea area, uint32_t *__restrict__ head_maxkey,
    uint32_t *__restrict__ fail, uint32_t *__restrict__ any_fail, int redo, int batch_blocks,
    const int32_t *__restrict__ page_table, int32_t *__restrict__ sel_ids, int32_t *__restrict__ sel_rows,
    float *__restrict__ sel_scores, int32_t *__restrict__ counts,
    float *__restrict__ head_M, int32_t *__restrict__ out_ids, int32_t *__restrict__ out_counts, int64_t ids_stride,
    int32_t *__restrict__ status, uint32_t *__restrict__ repairs, uint32_t *__restrict__ pmask)
{
    const Descs desc{desc_mem, desc0, desc_n};
    __shared__ uint32_t lh[kHistBins];
    __shared__ int32_t off[kSelBatch + 1];
    __shared__ int32_t st[kSelBatch];
    __shared__ ScanShared scan;
    __shared__ int32_t wtot[kSelWaves];
    __shared__ float wred[kSelWaves];
    __shared__ int32_t res[2];
    __shared__ int32_t gfirst[kRegSets * kSelChunk / 64 + 1]; // register path: block of every 64th survivor

    if (redo && *any_fail == 0u) return; // second run: only the heads that the repair pass rewrote
    const int h = blockIdx.x % H_q;
    const int r = desc_n > 1 ? desc[blockIdx.x / H_q].flags >> 8 : 0; // (the largest requests first)
    const int rh = r * H_q + h;
    if (redo && fail[rh] == 0u) return;
    const int G = H_q / H_kv;
    const HeadBlocks hb{area, H_kv, G, h / G, h % G};
    const ReqDesc dsc = desc[r];
    const int tid = threadIdx.x, lane = tid & 63;
    int32_t *ids = sel_ids + (size_t)dsc.score_off + (size_t)h * dsc.head_stride;
    float *ss = sel_scores + (size_t)dsc.score_off + (size_t)h * dsc.head_stride;
    int32_t *rows = sel_rows + (size_t)dsc.score_off + (size_t)h * dsc.head_stride;
    const int nb_all = dsc.ntiles_b;
    const int n_batches = (nb_all + batch_blocks - 1) / batch_blocks;
    bool bucket_rule = mode == 0 && dsc.k < dsc.n - dsc.nwin;
    const float M_dipr = mode == 1 ? ord_float(head_maxkey[rh]) : 0.f;
    const float thr = mode == 1 ? M_dipr - dsc.beta : -INFINITY; // top-k with k >= n: every token

    // The survivors in registers, when they are few: set s, element e of a thread is flat index
    // s * 4096 + e * 1024 + tid of the (single) batch.
    uint32_t rbits[kRegSets][kSelE]; // score bits
    int rid[kRegSets][kSelE];        // token id
    int rrow[kRegSets][kSelE];       // the token's row in the V pool (asked for early: the counting passes hide the trip)
    // With all blocks in one batch (the usual case) the batch's prefix sums stay in LDS for the whole kernel and
    // the first reg_total survivors stay in registers; what lies beyond them is streamed once per pass.
    const bool single = n_batches == 1;
    Batch b0{0, 0, 0};
    int reg_total = 0;
    if (single) {
        b0 = load_batch(hb, dsc.tileb_start, nb_all, off, st, wtot);
        reg_total = min(b0.total, kRegSets * kSelChunk);
        const int ngrp = (reg_total + 63) >> 6;
        if (tid <= ngrp) gfirst[tid] = (tid << 6) < b0.total ? batch_block(off, 0, b0.nb, tid << 6) : b0.nb - 1;
        __syncthreads();
#pragma unroll
        for (int s = 0; s < kRegSets; ++s) {
#pragma unroll
            for (int e = 0; e < kSelE; ++e) { rbits[s][e] = 0u; rid[s][e] = 0; rrow[s][e] = 0; }
            if (s * kSelChunk >= reg_total) continue; // (uniform)
#pragma unroll
            for (int e = 0; e < kSelE; ++e) {
                const int t = s * kSelChunk + e * kSelectThreads + tid;
                if (t < reg_total) {
                    const uint2 pr = batch_pair_grouped(hb, b0, off, st, gfirst, t);
                    rbits[s][e] = pr.x;
                    rid[s][e] = (int)pr.y;
                }
            }
            if (sel_rows) {
#pragma unroll
                for (int e = 0; e < kSelE; ++e)
                    if (s * kSelChunk + e * kSelectThreads + tid < reg_total)
                        rrow[s][e] = page_table[dsc.pt_off + (rid[s][e] >> 6)] * kPageTokens + (rid[s][e] & 63);
            }
        }
    }

    // One counting pass: adds to lh[] the digit `(key >> shift) & mask` of every ranked survivor (outside
    // the window) whose bits from `pshift` up equal `prefix` (pshift = 32: all of them).  lh must be zero;
    // the barriers around the pass are the caller's.
    auto count_pass = [&](int shift, uint32_t mask, int pshift, uint32_t prefix) {
        auto digit = [&](uint32_t key) { return (key >> shift) & mask; };
        auto counted = [&](uint32_t key, int tok, bool in) {
            return in && !in_window(dsc, tok) && (pshift >= 32 || (key >> pshift) == prefix);
        };
        constexpr int U = 4; // independent loads per thread and step of the streamed part
        auto stream = [&](const Batch &b, int from) {
            for (int t0 = from + tid; t0 < b.total; t0 += U * kSelectThreads) {
                uint2 pr[U];
                bool in[U];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int t = t0 + u * kSelectThreads;
                    in[u] = t < b.total;
                    pr[u] = in[u] ? batch_pair(hb, b, off, st, t) : make_uint2(0u, 0u);
                }
                const uint32_t key0 = ord_key(__uint_as_float(pr[0].x));
                const bool crowded = is_crowded(digit(key0), counted(key0, (int)pr[0].y, in[0]));
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const uint32_t key = ord_key(__uint_as_float(pr[u].x));
                    hist_add(lh, digit(key), counted(key, (int)pr[u].y, in[u]), crowded);
                }
            }
        };
        if (single) {
            // (one decision per wavefront and pass, from its first survivors: two straight-line copies of the loop)
            auto all_sets = [&](auto crowded) {
#pragma unroll
                for (int s = 0; s < kRegSets; ++s) {
                    if (s * kSelChunk >= reg_total) continue;
#pragma unroll
                    for (int e = 0; e < kSelE; ++e) {
                        const uint32_t key = ord_key(__uint_as_float(rbits[s][e]));
                        hist_add(lh, digit(key), counted(key, rid[s][e], s * kSelChunk + e * kSelectThreads + tid < reg_total),
                                 decltype(crowded)::value);
                    }
                }
            };
            const uint32_t key0 = ord_key(__uint_as_float(rbits[0][0]));
            if (is_crowded(digit(key0), counted(key0, rid[0][0], tid < reg_total))) all_sets(std::true_type{});
            else all_sets(std::false_type{});
            stream(b0, reg_total);
            return;
        }
        for (int bi = 0; bi < n_batches; ++bi) {
            const int first = bi * batch_blocks;
            stream(load_batch(hb, dsc.tileb_start + first, min(batch_blocks, nb_all - first), off, st, wtot), 0);
        }
    };

    uint32_t T = 0u; // top-k: keep key > T, and the first `ties` ranked tokens with key == T
    int ties = 0;
    if (bucket_rule) {
        int need = dsc.k;
        for (int i = tid; i < kHistBins; i += kSelectThreads) lh[i] = 0u;
        if (tid == 0) res[0] = -1;
        __syncthreads();
        count_pass(21, 0x7FFu, 32, 0u);
        __syncthreads();
        block_find_bin(lh, kHistBins, need, wtot, res);
        if (res[0] < 0 && !(dsc.flags & 1)) {
            // Fewer than k ranked tokens survived: the bound - an estimate then - was too high.  Every
            // thread sees the same histogram; the head is marked for the repair pass and left alone.
            if (tid == 0) {
                fail[rh] = 1u;
                *any_fail = 1u; // (several heads may write the same 1)
            }
            return;
        }
        // (short_ok: the candidates were cut down on purpose - the coarse index - and all of them are taken)
        if (res[0] < 0) bucket_rule = false;
    }
    if (bucket_rule) {
        const uint32_t b1 = (uint32_t)res[0];
        int need = dsc.k - res[1];
        __syncthreads();
        for (int i = tid; i < kHistBins; i += kSelectThreads) lh[i] = 0u;
        __syncthreads();
        count_pass(10, 0x7FFu, 21, b1);
        __syncthreads();
        block_find_bin(lh, kHistBins, need, wtot, res);
        const uint32_t pre = (b1 << 11) | (uint32_t)res[0]; // key >> 10 of the threshold
        need -= res[1];
        __syncthreads();
        for (int i = tid; i < 1024; i += kSelectThreads) lh[i] = 0u;
        __syncthreads();
        count_pass(0, 0x3FFu, 10, pre);
        __syncthreads();
        block_find_bin(lh, 1024, need, wtot, res);
        T = (pre << 10) | (uint32_t)res[0];
        ties = need - res[1]; // tokens with key == T that are taken, smallest ids first
    }

    // Placement, chunk by chunk in flat (= token) order.
    int baseA = 0, baseT = 0, parity = 0;
    float mx = -INFINITY; // maximum of the scores this thread enters into the list
    auto place_chunk = [&](const uint32_t *bits, const int *tok, const bool *in, const int *vrow) {
        bool fa[kSelE], fb[kSelE];
#pragma unroll
        for (int e = 0; e < kSelE; ++e) {
            const float v = __uint_as_float(bits[e]);
            const bool win = in_window(dsc, tok[e]);
            if (bucket_rule) {
                const uint32_t key = ord_key(v);
                fa[e] = in[e] && (win || key > T);
                fb[e] = in[e] && !win && key == T;
            } else {
                fa[e] = in[e] && (win || v >= thr);
                fb[e] = false;
            }
        }
        int exA[kSelE], exB[kSelE], tA, tB;
        chunk_ranks(scan, parity, fa, fb, exA, exB, tA, tB);
        parity ^= 1;
#pragma unroll
        for (int e = 0; e < kSelE; ++e) {
            const int tb = baseT + exB[e]; // ties before this element
            if (fa[e] || (fb[e] && tb < ties)) {
                const int pos = baseA + exA[e] + min(tb, ties);
                const float v = __uint_as_float(bits[e]);
                ids[pos] = tok[e];
                ss[pos] = v;
                // where the gather finds the token's value row: physical page * 64 + slot
                if (sel_rows) rows[pos] = vrow ? vrow[e] : page_table[dsc.pt_off + (tok[e] >> 6)] * kPageTokens + (tok[e] & 63);
                if (out_ids && (int64_t)pos < ids_stride) out_ids[(size_t)rh * (size_t)ids_stride + pos] = tok[e];
                if (pmask) { // a selection of pages: bit g of the page's byte in the KV head's row of the mask
                    const size_t byte = (size_t)dsc.pm_off + (size_t)hb.kvh * dsc.pm_stride + tok[e];
                    atomicOr(&pmask[byte >> 2], 1u << (8 * (int)(byte & 3) + hb.g));
                }
                mx = fmaxf(mx, v);
            }
        }
        baseA += tA;
        baseT += tB;
    };
    auto place_streamed = [&](const Batch &b, int from) {
        for (int c0 = from; c0 < b.total; c0 += kSelChunk) {
            uint32_t bits[kSelE];
            int tok[kSelE];
            bool in[kSelE];
#pragma unroll
            for (int e = 0; e < kSelE; ++e) {
                const int t = c0 + e * kSelectThreads + tid;
                in[e] = t < b.total;
                const uint2 pr = in[e] ? batch_pair(hb, b, off, st, t) : make_uint2(0u, 0u);
                bits[e] = pr.x;
                tok[e] = (int)pr.y;
            }
            place_chunk(bits, tok, in, nullptr);
        }
    };
    if (single) {
#pragma unroll
        for (int s = 0; s < kRegSets; ++s) {
            if (s * kSelChunk >= reg_total) continue; // (uniform)
            bool in[kSelE];
#pragma unroll
            for (int e = 0; e < kSelE; ++e) in[e] = s * kSelChunk + e * kSelectThreads + tid < reg_total;
            place_chunk(rbits[s], rid[s], in, rrow[s]);
        }
        place_streamed(b0, reg_total);
    } else {
        for (int bi = 0; bi < n_batches; ++bi) {
            const int first = bi * batch_blocks;
            place_streamed(load_batch(hb, dsc.tileb_start + first, min(batch_blocks, nb_all - first), off, st, wtot), 0);
        }
    }
    const int count = baseA + min(baseT, ties);

#pragma unroll
    for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
    if (lane == 0) wred[tid >> 6] = mx;
    __syncthreads();
    if (tid == 0) {
        float M = wred[0]; // the largest score of the selected set (DIPR: of all scores, which is selected)
        for (int w = 1; w < kSelWaves; ++w) M = fmaxf(M, wred[w]);
        head_M[rh] = M;
        counts[rh] = count;
        if (out_counts) out_counts[rh] = count;
        if (out_ids && (int64_t)count > ids_stride) atomicOr(status, 1);
        head_maxkey[rh] = 0u; // leave the running maximum and the repair mark clean for the next call
        fail[rh] = 0u;
        if (redo) atomicAdd(repairs, 1u);
    }
}

hipError_t launch_select(const Shape &sh, const DeviceViews &dv, const SelectIO &io, int B, int mode, bool redo,
                         int batch_blocks, int32_t *out_ids, int32_t *out_counts, int64_t ids_stride, hipStream_t st)
{
    if (batch_blocks <= 0 || batch_blocks > kSelBatch) batch_blocks = kSelBatch;
    select_kernel<<<dim3((unsigned)(B * sh.n_q_heads)), dim3(kSelectThreads), 0, st>>>(
        io.desc.mem, io.desc.in, io.desc.n, sh.n_q_heads, sh.n_kv_heads, mode, io.area,
        dv.head_maxkey, dv.fail, dv.any_fail, redo ? 1 : 0, batch_blocks, dv.page_table, io.ids, io.rows,
        io.scores, io.counts, io.head_M, out_ids, out_counts, ids_stride, dv.status, dv.repairs, io.pmask);
    return hipGetLastError();
}

} // namespace alaya
