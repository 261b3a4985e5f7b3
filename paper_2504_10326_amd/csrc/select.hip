// Selection of the critical tokens of every (request, query head) from its fp32 scores.
//   top-k (Sec. 5.1.1): the k largest scores; equal scores at the k-th place go to the smaller id.
//   DIPR  (Def. 2, 3) : every token with score >= max - beta.
// Everything is exact and order-deterministic: counting is integer (radix select on the
// order-preserving image of the score) and placement is an ordered compaction, so the selected list
// is the same on every run.
//
// A head's n scores are cut into segments; one 1024-thread workgroup owns one segment.
//   count   per segment: how many tokens are "definite" (top-k: bucket above the bucket b of the k-th
//           score, which is read off the histogram the scoring pass left; DIPR: score >= max - beta)
//           and how many are "candidates" (top-k only: bucket == b)
//   place   per segment: prefix over the earlier segments' counts gives the write offsets; an ordered
//           compaction puts definite tokens at the front of the head's list and candidates behind them,
//           both in ascending token order
//   finish  per head: (top-k) radix-refine the remaining 21 key bits over the candidates only and
//           compact them in place - keep key > T and the first `ties` tokens with key == T; publish
//           the count, copy ids out if asked, and zero the head's histogram for the next call
#include "alaya_internal.h"

namespace alaya {

constexpr int kSelE = 4;                       // scores per thread per chunk
constexpr int kSelWaves = kSelectThreads / 64; // 16
static_assert(kSelE * kSelWaves == 64, "the cross-wave scan maps one (e, wave) pair to one lane of wave 0");
static_assert(kSelE * kSelectThreads == kSelChunkTokens, "chunk size");

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

// Walk a histogram from its top bin down (one wavefront): find the bin holding the `need`-th largest
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

// blockIdx -> (request, head, segment).  Heads are the fastest index.
struct SegId { int r, h, seg; };
__device__ __forceinline__ SegId seg_of_block(const ReqDesc *desc, int B, int H_q)
{
    const int h = blockIdx.x % H_q;
    const int gs = blockIdx.x / H_q;
    int r = 0;
    while (r + 1 < B && desc[r + 1].seg_start <= gs) ++r;
    return {r, h, gs - desc[r].seg_start};
}

// What a token's score means for the selection, given the head's threshold data.
struct Rule {
    int topk;     // 1: bucket rule, 0: threshold rule
    uint32_t b1;  // bucket of the k-th score
    float thr;    // threshold rule: definite iff score >= thr
    __device__ __forceinline__ void classify(float v, bool in, bool &definite, bool &candidate) const
    {
        if (topk) {
            const uint32_t bin = ord_key(v) >> 21;
            definite = in && bin > b1;
            candidate = in && bin == b1;
        } else {
            definite = in && v >= thr;
            candidate = false;
        }
    }
};

// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kSelectThreads) void select_count_kernel(
    const ReqDesc *__restrict__ desc, int B, int H_q, int mode, const float *__restrict__ scores,
    const float *__restrict__ tile_max, const uint32_t *__restrict__ hist, float *__restrict__ head_M,
    int32_t *__restrict__ head_info, int32_t *__restrict__ seg_counts)
{
    __shared__ uint32_t lh[kHistBins];
    __shared__ float wred[kSelWaves];
    __shared__ int32_t ired[2][kSelWaves];
    __shared__ int32_t res[2];

    const SegId id = seg_of_block(desc, B, H_q);
    const ReqDesc dsc = desc[id.r];
    const int rh = id.r * H_q + id.h;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = dsc.n;

    // the head's maximum score, from the scoring pass's per-tile maxima
    float m = -INFINITY;
    for (int t = tid; t < dsc.n_tiles; t += kSelectThreads)
        m = fmaxf(m, tile_max[(size_t)(dsc.tile_start + t) * H_q + id.h]);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o));
    if (lane == 0) wred[wave] = m;
    const bool bucket_rule = mode == 0 && dsc.k < n;
    if (bucket_rule)
        for (int i = tid; i < kHistBins; i += kSelectThreads) lh[i] = hist[(size_t)rh * kHistBins + i];
    __syncthreads();
    float M = wred[0];
#pragma unroll
    for (int w = 1; w < kSelWaves; ++w) M = fmaxf(M, wred[w]);
    if (bucket_rule && tid < 64) find_bin(lh, kHistBins, dsc.k, res);
    __syncthreads();

    Rule rule;
    rule.topk = bucket_rule;
    rule.b1 = bucket_rule ? (uint32_t)res[0] : 0u;
    rule.thr = mode == 1 ? M - dsc.beta : -INFINITY; // top-k with k >= n: every token
    if (id.seg == 0 && tid == 0) {
        head_M[rh] = M;
        head_info[2 * rh] = bucket_rule ? res[0] : -1;
        head_info[2 * rh + 1] = bucket_rule ? res[1] : 0;
    }

    const float *s = scores + (size_t)dsc.score_off + (size_t)id.h * dsc.head_stride;
    const int begin = id.seg * dsc.seg_len, end = min(n, begin + dsc.seg_len);
    int ca = 0, cc = 0;
    for (int c0 = begin; c0 < end; c0 += kSelChunkTokens) {
#pragma unroll
        for (int e = 0; e < kSelE; ++e) {
            const int j = c0 + e * kSelectThreads + tid;
            const bool in = j < end;
            const float v = in ? s[j] : 0.f;
            bool a, c;
            rule.classify(v, in, a, c);
            ca += a;
            cc += c;
        }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        ca += __shfl_xor(ca, o);
        cc += __shfl_xor(cc, o);
    }
    if (lane == 0) { ired[0][wave] = ca; ired[1][wave] = cc; }
    __syncthreads();
    if (tid < 2) {
        int t = 0;
#pragma unroll
        for (int w = 0; w < kSelWaves; ++w) t += ired[tid][w];
        seg_counts[((size_t)rh * kMaxSegs + id.seg) * 2 + tid] = t;
    }
}

// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kSelectThreads) void select_place_kernel(
    const ReqDesc *__restrict__ desc, int B, int H_q, int mode, const float *__restrict__ scores,
    const float *__restrict__ head_M, const int32_t *__restrict__ head_info,
    const int32_t *__restrict__ seg_counts, int32_t *__restrict__ sel_ids, float *__restrict__ sel_scores)
{
    __shared__ ScanShared scan;
    __shared__ int32_t base[2];

    const SegId id = seg_of_block(desc, B, H_q);
    const ReqDesc dsc = desc[id.r];
    const int rh = id.r * H_q + id.h;
    const int tid = threadIdx.x, lane = tid & 63;
    const int n = dsc.n;

    Rule rule;
    rule.topk = head_info[2 * rh] >= 0;
    rule.b1 = (uint32_t)head_info[2 * rh];
    rule.thr = mode == 1 ? head_M[rh] - dsc.beta : -INFINITY;
    const int above1 = head_info[2 * rh + 1];

    if (tid < 64) { // earlier segments of this head: at most kMaxSegs = 64 of them
        int a = 0, c = 0;
        if (lane < id.seg) {
            a = seg_counts[((size_t)rh * kMaxSegs + lane) * 2];
            c = seg_counts[((size_t)rh * kMaxSegs + lane) * 2 + 1];
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            a += __shfl_xor(a, o);
            c += __shfl_xor(c, o);
        }
        if (lane == 0) { base[0] = a; base[1] = above1 + c; }
    }
    __syncthreads();
    int baseA = base[0], baseC = base[1];

    const size_t off = (size_t)dsc.score_off + (size_t)id.h * dsc.head_stride;
    const float *s = scores + off;
    int32_t *ids = sel_ids + off;
    float *ss = sel_scores + off;
    const int begin = id.seg * dsc.seg_len, end = min(n, begin + dsc.seg_len);
    int parity = 0;
    for (int c0 = begin; c0 < end; c0 += kSelChunkTokens) {
        float v[kSelE];
        bool fa[kSelE], fb[kSelE];
#pragma unroll
        for (int e = 0; e < kSelE; ++e) {
            const int j = c0 + e * kSelectThreads + tid;
            const bool in = j < end;
            v[e] = in ? s[j] : 0.f;
            rule.classify(v[e], in, fa[e], fb[e]);
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

// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kSelectThreads) void select_finish_kernel(
    const ReqDesc *__restrict__ desc, int H_q, int mode, const int32_t *__restrict__ head_info,
    const int32_t *__restrict__ seg_counts, uint32_t *__restrict__ hist, int32_t *__restrict__ sel_ids,
    float *__restrict__ sel_scores, int32_t *__restrict__ counts, int32_t *__restrict__ out_ids,
    int32_t *__restrict__ out_counts, int64_t ids_stride, int32_t *__restrict__ status)
{
    __shared__ uint32_t lh[kHistBins];
    __shared__ ScanShared scan;
    __shared__ int32_t res[2];
    __shared__ int32_t tot[2];

    const int rh = blockIdx.x;
    const int r = rh / H_q, h = rh % H_q;
    const ReqDesc dsc = desc[r];
    const int tid = threadIdx.x, lane = tid & 63;
    const size_t off = (size_t)dsc.score_off + (size_t)h * dsc.head_stride;
    int32_t *ids = sel_ids + off;
    float *ss = sel_scores + off;

    if (tid < 64) {
        int a = 0, c = 0;
        if (lane < dsc.nseg) {
            a = seg_counts[((size_t)rh * kMaxSegs + lane) * 2];
            c = seg_counts[((size_t)rh * kMaxSegs + lane) * 2 + 1];
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            a += __shfl_xor(a, o);
            c += __shfl_xor(c, o);
        }
        if (lane == 0) { tot[0] = a; tot[1] = c; }
    }
    __syncthreads();
    const bool bucket_rule = head_info[2 * rh] >= 0;
    int count = tot[0];

    if (bucket_rule) {
        const uint32_t b1 = (uint32_t)head_info[2 * rh];
        const int above1 = head_info[2 * rh + 1]; // == tot[0]
        const int cb = tot[1];
        int need = dsc.k - above1; // 1 <= need <= cb
        int parity = 0;
        if (need < cb) {
            // refine over the candidates: key bits [20:10], then bits [9:0]
            const float *cs = ss + above1;
            for (int i = tid; i < kHistBins; i += kSelectThreads) lh[i] = 0u;
            __syncthreads();
            for (int i = tid; i < cb; i += kSelectThreads) atomicAdd(&lh[(ord_key(cs[i]) >> 10) & 0x7FFu], 1u);
            __syncthreads();
            if (tid < 64) find_bin(lh, 2048, need, res);
            __syncthreads();
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
            if (tid < 64) find_bin(lh, 1024, need, res);
            __syncthreads();
            const uint32_t T = (pre << 10) | (uint32_t)res[0];
            const int ties = need - res[1]; // tokens with key == T that are taken, smallest ids first
            // ordered in-place compaction of the candidates (writes never pass the chunk being read)
            int baseG = 0, baseT = 0;
            for (int c0 = 0; c0 < cb; c0 += kSelChunkTokens) {
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
                int exA[kSelE], exB[kSelE], totA, totB;
                chunk_ranks(scan, parity, fa, fb, exA, exB, totA, totB); // barriers: this chunk is fully read
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
                baseG += totA;
                baseT += totB;
            }
        }
        count = dsc.k;
    }

    __syncthreads(); // list complete and visible to the whole workgroup
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
    if (mode == 0) // the scoring pass of a top-k call filled this head's histogram: leave it clean
        for (int i = tid; i < kHistBins; i += kSelectThreads) hist[(size_t)rh * kHistBins + i] = 0u;
}

hipError_t launch_select(const Shape &sh, const DeviceViews &dv, int B, int mode, int total_segs, int32_t *out_ids,
                         int32_t *out_counts, int64_t ids_stride, hipStream_t st)
{
    const dim3 block(kSelectThreads);
    const dim3 seg_grid((unsigned)(total_segs * sh.n_q_heads));
    select_count_kernel<<<seg_grid, block, 0, st>>>(dv.desc, B, sh.n_q_heads, mode, dv.scores, dv.tile_max, dv.hist,
                                                    dv.head_M, dv.head_info, dv.seg_counts);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    select_place_kernel<<<seg_grid, block, 0, st>>>(dv.desc, B, sh.n_q_heads, mode, dv.scores, dv.head_M,
                                                    dv.head_info, dv.seg_counts, dv.sel_ids, dv.sel_scores);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    select_finish_kernel<<<dim3((unsigned)(B * sh.n_q_heads)), block, 0, st>>>(
        dv.desc, sh.n_q_heads, mode, dv.head_info, dv.seg_counts, dv.hist, dv.sel_ids, dv.sel_scores, dv.counts,
        out_ids, out_counts, ids_stride, dv.status);
    return hipGetLastError();
}

} // namespace alaya
