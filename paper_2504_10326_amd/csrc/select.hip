// Selection of the critical tokens of one (request, query head) from its fp32 scores.
//   top-k (Sec. 5.1.1): the k largest scores; equal scores at the k-th place go to the smaller id.
//   DIPR  (Def. 2, 3) : every token with score >= max - beta.
// One 1024-thread workgroup owns one head.  Everything is exact and order-deterministic: counting
// is integer (radix select on the order-preserving image of the score), and placement is an ordered
// compaction, so the selected list is the same on every run.
//
// top-k in four steps:
//   1. histogram of the top 11 key bits over all n scores (LDS atomics)
//   2. walk the histogram from the top: bucket b holds the k-th score; buckets above it are taken whole
//   3. one ordered pass over the scores: tokens above b go to the front of the list ("definite"),
//      tokens in b go behind them ("candidates"), each kept in ascending token order
//   4. radix-refine the remaining 21 bits over the candidates only, then compact them in place:
//      keep key > T, and the first `ties` tokens with key == T
// DIPR is step 3 alone with the predicate score >= max - beta.
#include "alaya_internal.h"

namespace alaya {

constexpr int kSelE = 4;                         // scores per thread per chunk
constexpr int kSelWaves = kSelectThreads / 64;   // 16
constexpr int kSelChunk = kSelectThreads * kSelE;
static_assert(kSelE * kSelWaves == 64, "the cross-wave scan maps one (e, wave) pair to one lane of wave 0");

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

// Walk a histogram from its top bin down (wave 0 only): find the bin holding the `need`-th largest
// element.  res[0] = bin, res[1] = elements in bins above it.
__device__ __forceinline__ void find_bin(const uint32_t *hist, int nbins, int need, int32_t *res)
{
    const int lane = threadIdx.x & 63;
    int above = 0;
    for (int top = nbins - 64; top >= 0; top -= 64) {
        const int bin = top + 63 - lane; // lane 0 takes the highest bin of this group
        const int c = (int)hist[bin];
        int inc = c;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int t = __shfl_up(inc, o);
            if (lane >= o) inc += t;
        }
        const unsigned long long hit = __ballot(above + inc >= need);
        if (hit) {
            const int first = __ffsll((long long)hit) - 1;
            if (lane == first) { res[0] = bin; res[1] = above + inc - c; }
            return;
        }
        above += __shfl(inc, 63);
    }
    if (lane == 0) { res[0] = 0; res[1] = above - (int)hist[0]; } // unreachable when need <= total
}

__global__ __launch_bounds__(kSelectThreads) void select_kernel(
    const ReqDesc *__restrict__ desc, int H_q, int mode, const float *__restrict__ scores,
    uint32_t *__restrict__ head_max, float *__restrict__ head_M, int32_t *__restrict__ sel_ids,
    float *__restrict__ sel_scores, int32_t *__restrict__ counts, int32_t *__restrict__ out_ids,
    int32_t *__restrict__ out_counts, int64_t ids_stride, int32_t *__restrict__ status)
{
    __shared__ uint32_t hist[2048];
    __shared__ ScanShared scan;
    __shared__ int32_t res[2];
    __shared__ float s_M;

    const int rh = blockIdx.x;
    const int r = rh / H_q, h = rh % H_q;
    const ReqDesc dsc = desc[r];
    const int n = dsc.n;
    const size_t off = (size_t)dsc.score_off + (size_t)h * dsc.n_pad;
    const float *s = scores + off;
    int32_t *ids = sel_ids + off;
    float *ss = sel_scores + off;
    const int tid = threadIdx.x;
    int parity = 0;

    // The scoring pass left the running maximum here; take it and leave the slot clean for the next call.
    if (tid == 0) {
        const uint32_t e = head_max[rh];
        const float M = ord_float(e);
        s_M = M;
        head_M[rh] = M;
        head_max[rh] = 0u;
    }
    __syncthreads();
    const float M = s_M;
    int count = 0;

    if (mode == 1 /* DIPR */ || dsc.k >= n) {
        // DIPR: threshold pass.  top-k with k >= n: every token (threshold -inf).
        const float thr = (mode == 1) ? (M - dsc.beta) : -INFINITY;
        int base = 0;
        for (int c0 = 0; c0 < n; c0 += kSelChunk) {
            float v[kSelE];
            bool fa[kSelE], fb[kSelE];
#pragma unroll
            for (int e = 0; e < kSelE; ++e) {
                const int j = c0 + e * kSelectThreads + tid;
                v[e] = j < n ? s[j] : 0.f;
                fa[e] = j < n && v[e] >= thr;
                fb[e] = false;
            }
            int exA[kSelE], exB[kSelE], totA, totB;
            chunk_ranks(scan, parity, fa, fb, exA, exB, totA, totB);
            parity ^= 1;
#pragma unroll
            for (int e = 0; e < kSelE; ++e)
                if (fa[e]) {
                    ids[base + exA[e]] = c0 + e * kSelectThreads + tid;
                    ss[base + exA[e]] = v[e];
                }
            base += totA;
        }
        count = base;
    } else {
        const int kk = dsc.k;
        // 1. histogram of the top 11 bits
        for (int i = tid; i < 2048; i += kSelectThreads) hist[i] = 0u;
        __syncthreads();
        for (int j = tid; j < n; j += kSelectThreads) atomicAdd(&hist[ord_key(s[j]) >> 21], 1u);
        __syncthreads();
        // 2. bucket of the k-th score
        if (tid < 64) find_bin(hist, 2048, kk, res);
        __syncthreads();
        const uint32_t b1 = (uint32_t)res[0];
        const int above1 = res[1];
        const int cb = (int)hist[b1];
        int need = kk - above1; // 1 <= need <= cb
        __syncthreads();
        // 3. ordered split into definite (front) and candidates (behind them)
        {
            int baseA = 0, baseC = above1;
            for (int c0 = 0; c0 < n; c0 += kSelChunk) {
                float v[kSelE];
                bool fa[kSelE], fb[kSelE];
#pragma unroll
                for (int e = 0; e < kSelE; ++e) {
                    const int j = c0 + e * kSelectThreads + tid;
                    v[e] = j < n ? s[j] : 0.f;
                    const uint32_t bin = ord_key(v[e]) >> 21;
                    fa[e] = j < n && bin > b1;
                    fb[e] = j < n && bin == b1;
                }
                int exA[kSelE], exB[kSelE], totA, totB;
                chunk_ranks(scan, parity, fa, fb, exA, exB, totA, totB);
                parity ^= 1;
#pragma unroll
                for (int e = 0; e < kSelE; ++e) {
                    const int j = c0 + e * kSelectThreads + tid;
                    if (fa[e]) { ids[baseA + exA[e]] = j; ss[baseA + exA[e]] = v[e]; }
                    if (fb[e]) { ids[baseC + exB[e]] = j; ss[baseC + exB[e]] = v[e]; }
                }
                baseA += totA;
                baseC += totB;
            }
        }
        __syncthreads(); // candidate writes visible to the whole workgroup
        if (need < cb) {
            // 4. refine over the candidates: bits [20:10], then bits [9:0]
            const float *cs = ss + above1;
            for (int i = tid; i < 2048; i += kSelectThreads) hist[i] = 0u;
            __syncthreads();
            for (int i = tid; i < cb; i += kSelectThreads) atomicAdd(&hist[(ord_key(cs[i]) >> 10) & 0x7FFu], 1u);
            __syncthreads();
            if (tid < 64) find_bin(hist, 2048, need, res);
            __syncthreads();
            const uint32_t b2 = (uint32_t)res[0];
            need -= res[1];
            __syncthreads();
            for (int i = tid; i < 1024; i += kSelectThreads) hist[i] = 0u;
            __syncthreads();
            const uint32_t pre = (b1 << 11) | b2; // key >> 10 of the threshold
            for (int i = tid; i < cb; i += kSelectThreads) {
                const uint32_t key = ord_key(cs[i]);
                if ((key >> 10) == pre) atomicAdd(&hist[key & 0x3FFu], 1u);
            }
            __syncthreads();
            if (tid < 64) find_bin(hist, 1024, need, res);
            __syncthreads();
            const uint32_t T = (pre << 10) | (uint32_t)res[0];
            const int ties = need - res[1]; // how many tokens with key == T are taken, smallest ids first
            // ordered in-place compaction of the candidates
            int baseG = 0, baseT = 0, kept = 0;
            for (int c0 = 0; c0 < cb; c0 += kSelChunk) {
                float v[kSelE];
                int id[kSelE];
                bool fa[kSelE], fb[kSelE];
#pragma unroll
                for (int e = 0; e < kSelE; ++e) {
                    const int i = c0 + e * kSelectThreads + tid;
                    v[e] = i < cb ? cs[i] : 0.f;
                    id[e] = i < cb ? ids[above1 + i] : 0;
                    const uint32_t key = ord_key(v[e]);
                    fa[e] = i < cb && key > T;
                    fb[e] = i < cb && key == T;
                }
                int exA[kSelE], exB[kSelE], totA, totB;
                chunk_ranks(scan, parity, fa, fb, exA, exB, totA, totB); // barriers: all reads of this chunk done
                parity ^= 1;
#pragma unroll
                for (int e = 0; e < kSelE; ++e) {
                    const int tb = baseT + exB[e]; // ties before this element
                    const bool keep = fa[e] || (fb[e] && tb < ties);
                    if (keep) {
                        const int pos = above1 + baseG + exA[e] + min(tb, ties);
                        ids[pos] = id[e];
                        ss[pos] = v[e];
                    }
                }
                baseG += totA;
                baseT += totB;
                kept = baseG + min(baseT, ties);
            }
            (void)kept;
        }
        count = kk;
    }

    __syncthreads(); // list complete and visible
    if (tid == 0) {
        counts[rh] = count;
        if (out_counts) out_counts[rh] = count;
        if (out_ids && (int64_t)count > ids_stride) atomicOr(status, 1);
    }
    if (out_ids) {
        const int m = (int)((int64_t)count < ids_stride ? (int64_t)count : ids_stride);
        int32_t *dst = out_ids + (size_t)rh * (size_t)ids_stride;
        for (int i = tid; i < m; i += kSelectThreads) dst[i] = ids[i];
    }
}

hipError_t launch_select(const Shape &sh, const DeviceViews &dv, int B, int mode, int32_t *out_ids,
                         int32_t *out_counts, int64_t ids_stride, hipStream_t st)
{
    select_kernel<<<dim3((unsigned)(B * sh.n_q_heads)), dim3(kSelectThreads), 0, st>>>(
        dv.desc, sh.n_q_heads, mode, dv.scores, dv.head_max, dv.head_M, dv.sel_ids, dv.sel_scores, dv.counts,
        out_ids, out_counts, ids_stride, dv.status);
    return hipGetLastError();
}

} // namespace alaya
