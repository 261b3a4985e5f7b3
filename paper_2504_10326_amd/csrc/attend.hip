// Attention over the selected tokens (gather of their value rows + softmax-weighted sum), the merge
// of partial results, and dense attention over the whole cache.
//
//   z_j = s_j * scale;  a = softmax over the selected set;  o = sum_j a_j v_j        (Eq. 1, restricted
//   to the critical tokens as in Sec. 2 "Sparse Attention").
// Partial results carry (m, l, acc) = (reference max, sum of exp(z - m), sum of exp(z - m) v) and are
// merged in a fixed order, as in the paper's data-centric engine (Sec. 7.2: partial attention computed
// where the vectors sit, then aggregated the FlashAttention way).  The sparse path knows its softmax
// reference before it starts: the selection leaves the maximum over the selected set in head_M, so no
// rescaling is needed on the way.
#include "alaya_internal.h"
#include "row_slice.h"
#include "score_page.h"

namespace alaya {

// ------------------------------------------------------------------------------------------------
// Sparse attend.  Grid: (request, head, split).  A wavefront takes 4 selected rows per step
// (16 lanes per 256-byte row), kAttendU steps in flight: 128 rows per workgroup and pass - the gather of
// 256-byte rows at random runs fastest with many small workgroups (6.1 TB/s at 128 rows each against
// 3.8 at 2048 on a 410 MB gather).  The head's selected tokens are one list (sel_rows / sel_scores,
// `counts` long, ascending by token), as the selection leaves them; sel_rows already holds the rows'
// places in the V pool, so that the loads of a pass are two deep (row number, row), not three.
// The grid has `splits` workgroups per head, sized for the longest list of the call; a head uses as many
// of them as give each about 128 rows, 256 in large calls (head_splits; small calls more, with fewer rows each,
// to fill the chip), the others leave at once.
constexpr int kAttendU = 8;

// min_splits carries two things: the least number of splits in its low 16 bits and log2 of the rows that a
// workgroup should get (7 or 8) above them.
__device__ __forceinline__ int head_splits(int cnt, int splits, int min_splits)
{
    const int sh = min_splits >> 16;
    return min(splits, max(min_splits & 0xFFFF, (cnt + (1 << sh) - 1) >> sh));
}

template <int DT, int D>
__global__ __launch_bounds__(kAttendThreads) void attend_kernel(
    const ReqDesc *__restrict__ desc_mem, const ReqDesc desc0, int desc_n, int H_q, int H_kv,
    const char *__restrict__ v_pool, const int32_t *__restrict__ rows_in, const float *__restrict__ scores_in,
    const int32_t *__restrict__ counts, const float *__restrict__ head_M, float scale, int splits, int min_splits,
    float *__restrict__ partials)
{
    const Descs desc{desc_mem, desc0, desc_n};
    using RS = RowSlice<DT, D>;
    constexpr int EPL = RS::EPL;
    constexpr size_t ROW_BYTES = (size_t)D * (DT == 0 ? 2 : 4);
    __shared__ float red[4][D + 1];

    const int sp = blockIdx.x % splits;
    const int rh = blockIdx.x / splits;
    const int r = rh / H_q, h = rh % H_q;
    const int kvh = h / (H_q / H_kv);
    const ReqDesc dsc = desc[r];
    const size_t off = (size_t)dsc.score_off + (size_t)h * dsc.head_stride;
    const int32_t *rows = rows_in + off;
    const float *ss = scores_in + off;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int cnt = counts[rh];
    const float M = head_M[rh]; // (asked for before the early exit: one trip to memory, not two)
    const int eff = head_splits(cnt, splits, min_splits);
    if (sp >= eff) return;
    int per = (cnt + eff - 1) / eff;
    per = (per + 15) & ~15;
    const int begin = min(cnt, sp * per), end = min(cnt, begin + per);

    const int sub = lane & 15, grp = lane >> 4;
    float acc[EPL];
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[e] = 0.f;
    float l = 0.f;

    for (int i0 = begin + wave * 4 + grp; i0 < end; i0 += 16 * kAttendU) {
        int row[kAttendU];
        float p[kAttendU];
#pragma unroll
        for (int u = 0; u < kAttendU; ++u) {
            const int i = i0 + u * 16;
            const bool ok = i < end;
            row[u] = ok ? rows[i] : -1;
            p[u] = ok ? __expf((ss[i] - M) * scale) : 0.f;
        }
        typename RS::Raw raw[kAttendU];
#pragma unroll
        for (int u = 0; u < kAttendU; ++u) {
            // row = physical page * 64 + slot; a page holds 64 rows of each of its H_kv heads
            const size_t at = ((size_t)(row[u] >> 6) * H_kv + kvh) * 64 + (row[u] & 63);
            if (row[u] >= 0) raw[u] = RS::load_raw(v_pool + at * ROW_BYTES, sub);
            else raw[u] = typename RS::Raw{};
        }
#pragma unroll
        for (int u = 0; u < kAttendU; ++u) {
            float v[EPL];
            RS::widen(raw[u], v);
            l += p[u];
#pragma unroll
            for (int e = 0; e < EPL; ++e) acc[e] = fmaf(p[u], v[e], acc[e]);
        }
    }
    // the four 16-lane groups of a wavefront hold different rows: add them up
#pragma unroll
    for (int e = 0; e < EPL; ++e) {
        acc[e] += __shfl_xor(acc[e], 16);
        acc[e] += __shfl_xor(acc[e], 32);
    }
    l += __shfl_xor(l, 16);
    l += __shfl_xor(l, 32);
    if (lane < 16) {
#pragma unroll
        for (int e = 0; e < EPL; ++e) red[wave][sub * EPL + e] = acc[e];
        if (lane == 0) red[wave][D] = l;
    }
    __syncthreads();
    float *dst = partials + (size_t)blockIdx.x * (D + 2);
    for (int c = threadIdx.x; c <= D; c += kAttendThreads) {
        const float t = ((red[0][c] + red[1][c]) + red[2][c]) + red[3][c];
        if (c < D) dst[2 + c] = t;
        else { dst[1] = t; dst[0] = t > 0.f ? M * scale : -INFINITY; }
    }
}

hipError_t launch_attend(const Shape &sh, const DeviceViews &dv, int B, float scale, int splits, int min_splits,
                         hipStream_t st)
{
    const dim3 grid((unsigned)(B * sh.n_q_heads * splits)), block(kAttendThreads);
#define ALAYA_ATTEND(DT, D)                                                                                  \
    attend_kernel<DT, D><<<grid, block, 0, st>>>(dv.desc.mem, dv.desc.in, dv.desc.n, sh.n_q_heads, sh.n_kv_heads, \
                                                 (const char *)dv.v_pool, dv.sel_rows, dv.sel_scores,        \
                                                 dv.counts, dv.head_M, scale, splits, min_splits, dv.partials)
    if (sh.dtype == 0 && sh.head_dim == 128) ALAYA_ATTEND(0, 128);
    else if (sh.dtype == 0 && sh.head_dim == 64) ALAYA_ATTEND(0, 64);
    else if (sh.dtype == 1 && sh.head_dim == 128) ALAYA_ATTEND(1, 128);
    else if (sh.dtype == 1 && sh.head_dim == 64) ALAYA_ATTEND(1, 64);
    else return hipErrorInvalidValue;
#undef ALAYA_ATTEND
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// Merge of partial results, fixed order.  Grid: (request, head); block: (output channel, slice).  The sparse
// path has at most kMaxSplits partials per head and one slice.  Dense attention has one partial per tile of the
// request, hundreds at 1M tokens: kCombineSlices slices take consecutive runs of them (one slice alone went
// through them eight at a time, 40 us at 1M tokens), and slice 0 adds the slices' sums up, in order.
constexpr int kCombineSlices = 8;

template <int D>
__global__ __launch_bounds__(D * kCombineSlices) void combine_kernel(const ReqDesc *__restrict__ desc_mem, const ReqDesc desc0, int desc_n, int B, int H_q,
                                                     const float *__restrict__ partials, int splits,
                                                     int per_request_tiles, int pages_per_tile,
                                                     const int32_t *__restrict__ counts, int min_splits,
                                                     float *__restrict__ out)
{
    const Descs desc{desc_mem, desc0, desc_n};
    __shared__ float sM[kCombineSlices], sL[kCombineSlices], sO[kCombineSlices][D];
    const int rh = blockIdx.x;
    const int r = rh / H_q, h = rh % H_q;
    const int ch = threadIdx.x, sl = threadIdx.y, S = blockDim.y;
    int np;
    size_t first, stride;
    if (per_request_tiles) {
        const ReqDesc dsc = desc[r];
        const int n_pages = (dsc.n + kPageTokens - 1) >> 6;
        np = (n_pages + pages_per_tile - 1) / pages_per_tile;
        first = ((size_t)dsc.tile_start * H_q + h) * (D + 2);
        stride = (size_t)H_q * (D + 2);
    } else {
        np = head_splits(counts[rh], splits, min_splits); // what the attend pass used of the head's slots
        first = (size_t)rh * splits * (D + 2);
        stride = D + 2;
    }
    const int per = (np + S - 1) / S;
    const int i_begin = min(np, sl * per), i_end = min(np, i_begin + per); // this slice's partials
    // loads are issued eight at a time so that their latencies overlap; the merge order stays fixed
    constexpr int U = 8;
    // The splits of a sparse call all subtracted the same maximum (or hold nothing): no rescaling, and
    // no need to look for the largest reference first.
    float M = -INFINITY;
    if (per_request_tiles) {
        for (int i0 = i_begin; i0 < i_end; i0 += U) {
            float mm[U];
#pragma unroll
            for (int u = 0; u < U; ++u) mm[u] = i0 + u < i_end ? partials[first + (size_t)(i0 + u) * stride] : -INFINITY;
#pragma unroll
            for (int u = 0; u < U; ++u) M = fmaxf(M, mm[u]);
        }
        if (S > 1) {
            if (ch == 0) sM[sl] = M;
            __syncthreads();
            for (int t = 0; t < S; ++t) M = fmaxf(M, sM[t]);
        }
    }
    float L = 0.f, o = 0.f;
    for (int i0 = i_begin; i0 < i_end; i0 += U) {
        float mm[U], ll[U], aa[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const bool ok = i0 + u < i_end;
            const float *p = partials + first + (size_t)(ok ? i0 + u : i_begin) * stride;
            mm[u] = ok ? p[0] : -INFINITY;
            ll[u] = p[1];
            aa[u] = p[2 + ch];
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const float w = mm[u] == -INFINITY ? 0.f : per_request_tiles ? __expf(mm[u] - M) : 1.f;
            L = fmaf(w, ll[u], L);
            o = fmaf(w, aa[u], o);
        }
    }
    if (S > 1) {
        if (ch == 0) sL[sl] = L;
        sO[sl][ch] = o;
        __syncthreads();
        if (sl != 0) return;
        for (int t = 1; t < S; ++t) { L += sL[t]; o += sO[t][ch]; }
    }
    out[(size_t)rh * D + ch] = o / L;
}

hipError_t launch_combine(const Shape &sh, const DeviceViews &dv, int B, int splits, int min_splits,
                          int per_request_tiles, int pages_per_tile, float *out, hipStream_t st)
{
    const dim3 grid((unsigned)(B * sh.n_q_heads));
    const unsigned slices = per_request_tiles ? kCombineSlices : 1;
    if (sh.head_dim == 128)
        combine_kernel<128><<<grid, dim3(128, slices), 0, st>>>(dv.desc.mem, dv.desc.in, dv.desc.n, B, sh.n_q_heads, dv.partials, splits,
                                                        per_request_tiles, pages_per_tile, dv.counts, min_splits, out);
    else if (sh.head_dim == 64)
        combine_kernel<64><<<grid, dim3(64, slices), 0, st>>>(dv.desc.mem, dv.desc.in, dv.desc.n, B, sh.n_q_heads, dv.partials, splits,
                                                      per_request_tiles, pages_per_tile, dv.counts, min_splits, out);
    else
        return hipErrorInvalidValue;
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// Dense attention, split over pages (Eq. 1 over every cached token).  Grid: (tile, KV head).  Each
// wavefront walks its pages: scores for 64 tokens x G heads with the scoring pass's own routine
// (lane = token), online softmax per head, probabilities through LDS, then the page's value rows with
// 16 lanes per row.  Keys and values are read once: non-temporal loads.  The four wavefronts' results
// are merged before the partial is written.
template <int DT, int D, int G>
__global__ __launch_bounds__(256) void full_partial_kernel(const ReqDesc *__restrict__ desc_mem, const ReqDesc desc0, int desc_n, int B,
                                                            const int32_t *__restrict__ page_table,
                                                            const void *__restrict__ qv,
                                                            const uint4 *__restrict__ k_pool,
                                                            const char *__restrict__ v_pool, float scale, int H_kv,
                                                            int ppt, float *__restrict__ partials)
{
    const Descs desc{desc_mem, desc0, desc_n};
    using RS = RowSlice<DT, D>;
    constexpr int EPL = RS::EPL;
    constexpr int E = DT == 0 ? 8 : 4;
    constexpr int NC = D / E;
    constexpr size_t ROW_BYTES = (size_t)D * (DT == 0 ? 2 : 4);
    __shared__ float ps[4][G][64];
    __shared__ float red[4][G][D + 2];

    const int kvh = blockIdx.x % H_kv;
    const int tile = blockIdx.x / H_kv;
    int r = 0;
    while (r + 1 < B && desc[r + 1].tile_start <= tile) ++r;
    const ReqDesc dsc = desc[r];
    const int H_q = H_kv * G;
    constexpr int QW = D * (DT == 0 ? 2 : 4) / 4;
    const uint4 *qh = (const uint4 *)((const uint32_t *)qv + ((size_t)r * H_q + kvh * G) * QW); // wave-uniform

    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63, sub = lane & 15, grp = lane >> 4;
    const int n_pages = (dsc.n + kPageTokens - 1) >> 6;
    const int ppw = ppt / 4;
    const int p_begin = (tile - dsc.tile_start) * ppt + wave * ppw;

    float m[G], l[G], acc[G][EPL];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        m[g] = -INFINITY;
        l[g] = 0.f;
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[g][e] = 0.f;
    }

    for (int it = 0; it < ppw; ++it) { // same trip count for all four wavefronts: barriers inside
        const int p = p_begin + it;
        const bool active = p < n_pages;
        const int phys = active ? page_table[dsc.pt_off + p] : 0;
        const size_t tile_off = ((size_t)phys * H_kv + kvh);
        if (active) {
            float s[G];
            score_page<DT, D, G>(k_pool + tile_off * (size_t)(NC * 64) + lane, qh, s);
            const bool valid = p * kPageTokens + lane < dsc.n;
#pragma unroll
            for (int g = 0; g < G; ++g) {
                float mp = valid ? s[g] : -INFINITY;
#pragma unroll
                for (int o = 32; o > 0; o >>= 1) mp = fmaxf(mp, __shfl_xor(mp, o));
                const float mn = fmaxf(m[g], mp); // finite: a page in range holds at least one token
                const float corr = m[g] == -INFINITY ? 0.f : __expf((m[g] - mn) * scale);
                const float pg = valid ? __expf((s[g] - mn) * scale) : 0.f;
                ps[wave][g][lane] = pg;
                l[g] = fmaf(l[g], corr, pg);
#pragma unroll
                for (int e = 0; e < EPL; ++e) acc[g][e] *= corr;
                m[g] = mn;
            }
        }
        __syncthreads();
        if (active) {
            const char *vbase = v_pool + tile_off * 64 * ROW_BYTES;
#pragma unroll 4
            for (int t4 = 0; t4 < 16; ++t4) {
                const int tok = t4 * 4 + grp;
                float v[EPL];
                RS::template load<true>(vbase + (size_t)tok * ROW_BYTES, sub, v);
                if (p * kPageTokens + tok >= dsc.n) { // unwritten tail of the last page: weight 0, but 0 * NaN is NaN
#pragma unroll
                    for (int e = 0; e < EPL; ++e) v[e] = 0.f;
                }
#pragma unroll
                for (int g = 0; g < G; ++g) {
                    const float pg = ps[wave][g][tok];
#pragma unroll
                    for (int e = 0; e < EPL; ++e) acc[g][e] = fmaf(pg, v[e], acc[g][e]);
                }
            }
        }
        __syncthreads();
    }

#pragma unroll
    for (int g = 0; g < G; ++g) {
        float lw = l[g];
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) lw += __shfl_xor(lw, o);
#pragma unroll
        for (int e = 0; e < EPL; ++e) {
            acc[g][e] += __shfl_xor(acc[g][e], 16);
            acc[g][e] += __shfl_xor(acc[g][e], 32);
        }
        if (lane < 16) {
#pragma unroll
            for (int e = 0; e < EPL; ++e) red[wave][g][2 + sub * EPL + e] = acc[g][e];
            if (lane == 0) { red[wave][g][0] = m[g]; red[wave][g][1] = lw; }
        }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < G * (D + 1); i += 256) {
        const int g = i / (D + 1), c = i % (D + 1); // c == D is the l slot
        float M = -INFINITY;
#pragma unroll
        for (int w = 0; w < 4; ++w) M = fmaxf(M, red[w][g][0]);
        float t = 0.f;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const float mw = red[w][g][0];
            const float wt = mw == -INFINITY ? 0.f : __expf((mw - M) * scale);
            t = fmaf(wt, c < D ? red[w][g][2 + c] : red[w][g][1], t);
        }
        float *dst = partials + ((size_t)tile * H_q + kvh * G + g) * (D + 2);
        if (c < D) dst[2 + c] = t;
        else { dst[1] = t; dst[0] = M == -INFINITY ? -INFINITY : M * scale; }
    }
}

template <int DT, int D>
static hipError_t launch_full_g(const Shape &sh, const DeviceViews &dv, int B, const void *q, float scale,
                                int total_tiles, int ppt, hipStream_t st)
{
    const int G = sh.n_q_heads / sh.n_kv_heads;
    const dim3 grid((unsigned)(total_tiles * sh.n_kv_heads)), block(256);
#define ALAYA_FULL(GG)                                                                                     \
    full_partial_kernel<DT, D, GG><<<grid, block, 0, st>>>(dv.desc.mem, dv.desc.in, dv.desc.n, B, dv.page_table, q,                   \
                                                           (const uint4 *)dv.k_pool, (const char *)dv.v_pool, \
                                                           scale, sh.n_kv_heads, ppt, dv.partials)
    switch (G) {
    case 1: ALAYA_FULL(1); break;
    case 2: ALAYA_FULL(2); break;
    case 4: ALAYA_FULL(4); break;
    case 8: ALAYA_FULL(8); break;
    default: return hipErrorInvalidValue;
    }
#undef ALAYA_FULL
    return hipGetLastError();
}

hipError_t launch_full_partial(const Shape &sh, const DeviceViews &dv, int B, const void *q, float scale,
                               int total_tiles, int ppt, hipStream_t st)
{
    if (sh.dtype == 0) {
        if (sh.head_dim == 128) return launch_full_g<0, 128>(sh, dv, B, q, scale, total_tiles, ppt, st);
        if (sh.head_dim == 64) return launch_full_g<0, 64>(sh, dv, B, q, scale, total_tiles, ppt, st);
    } else {
        if (sh.head_dim == 128) return launch_full_g<1, 128>(sh, dv, B, q, scale, total_tiles, ppt, st);
        if (sh.head_dim == 64) return launch_full_g<1, 64>(sh, dv, B, q, scale, total_tiles, ppt, st);
    }
    return hipErrorInvalidValue;
}

} // namespace alaya
