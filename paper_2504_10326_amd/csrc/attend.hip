// Attention over the selected tokens (gather of their value rows + softmax-weighted sum), the merge
// of partial results, and dense attention over the whole cache.
//
//   z_j = s_j * scale;  a = softmax over the selected set;  o = sum_j a_j v_j        (Eq. 1, restricted
//   to the critical tokens as in Sec. 2 "Sparse Attention").
// Partial results carry (m, l, acc) = (reference max, sum of exp(z - m), sum of exp(z - m) v) and are
// merged in a fixed order, as in the paper's data-centric engine (Sec. 6.2: partial attention computed
// where the vectors sit, then aggregated the FlashAttention way).  The sparse path knows its softmax
// reference before it starts: the selection leaves the maximum over the selected set in head_M (DIPR:
// the maximum of all scores, which is always selected; top-k: the maximum of the finished list), so no
// rescaling is needed on the way.
#include "alaya_internal.h"

namespace alaya {

__device__ __forceinline__ float bf16_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t u) { return __uint_as_float(u & 0xFFFF0000u); }
__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

// A value row is spread over 16 lanes; each lane owns EPL = D / 16 consecutive elements.
template <int DT, int D> struct RowSlice {
    static constexpr int EPL = D / 16;
    static constexpr int BYTES = EPL * (DT == 0 ? 2 : 4);
    // row: first byte of the token's value row; sub = lane % 16
    __device__ static __forceinline__ void load(const char *row, int sub, float *f)
    {
        const char *p = row + (size_t)sub * BYTES;
        if constexpr (DT == 0 && EPL == 8) {
            const uint4 c = *(const uint4 *)p;
            f[0] = bf16_lo(c.x); f[1] = bf16_hi(c.x); f[2] = bf16_lo(c.y); f[3] = bf16_hi(c.y);
            f[4] = bf16_lo(c.z); f[5] = bf16_hi(c.z); f[6] = bf16_lo(c.w); f[7] = bf16_hi(c.w);
        } else if constexpr (DT == 0 && EPL == 4) {
            const uint2 c = *(const uint2 *)p;
            f[0] = bf16_lo(c.x); f[1] = bf16_hi(c.x); f[2] = bf16_lo(c.y); f[3] = bf16_hi(c.y);
        } else if constexpr (DT == 1 && EPL == 8) {
            const float4 a = *(const float4 *)p, b = *(const float4 *)(p + 16);
            f[0] = a.x; f[1] = a.y; f[2] = a.z; f[3] = a.w; f[4] = b.x; f[5] = b.y; f[6] = b.z; f[7] = b.w;
        } else {
            const float4 a = *(const float4 *)p;
            f[0] = a.x; f[1] = a.y; f[2] = a.z; f[3] = a.w;
        }
    }
};

// ------------------------------------------------------------------------------------------------
// Sparse attend.  Grid: (request, head, split).  A wavefront takes 4 selected rows per step
// (16 lanes per 256-byte row), kAttendU steps in flight.
// SEG = false: the head's selected tokens are one list (sel_ids / sel_scores, `counts` long), as the
// finishing pass of a top-k call leaves them.
// SEG = true (DIPR): there is no finishing pass; the selected tokens are still where select_local put
// them, one list per selection segment (`ids_in` / `scores_in` = its arrays, seg_counts = the lengths).
// The kernel reads the concatenation of those lists through the segments' prefix sums, and does what
// is left of the finishing pass on the way: the true count, the ids for the caller, the overflow
// status, and the reset of the head's running maximum for the next call.
constexpr int kAttendU = 4;

struct AttendOut { // SEG only: what the caller asked to get back
    int32_t *out_ids, *out_counts;
    int64_t ids_stride;
    int32_t *status;
};

template <int DT, int D, bool SEG>
__global__ __launch_bounds__(kAttendThreads) void attend_kernel(
    const ReqDesc *__restrict__ desc_mem, const ReqDesc desc0, int desc_n, int H_q, int H_kv, const int32_t *__restrict__ page_table,
    const char *__restrict__ v_pool, const int32_t *__restrict__ ids_in, const float *__restrict__ scores_in,
    int32_t *__restrict__ counts, const float *__restrict__ head_M, float scale, int splits,
    float *__restrict__ partials, const int32_t *__restrict__ seg_counts, uint32_t *__restrict__ head_maxkey,
    const AttendOut ao)
{
    const Descs desc{desc_mem, desc0, desc_n};
    using RS = RowSlice<DT, D>;
    constexpr int EPL = RS::EPL;
    constexpr size_t ROW_BYTES = (size_t)D * (DT == 0 ? 2 : 4);
    __shared__ float red[4][D + 1];
    __shared__ int32_t pre[SEG ? kMaxSegs + 1 : 1]; // exclusive prefix sums of the segments' list lengths

    const int sp = blockIdx.x % splits;
    const int rh = blockIdx.x / splits;
    const int r = rh / H_q, h = rh % H_q;
    const int kvh = h / (H_q / H_kv);
    const ReqDesc dsc = desc[r];
    const size_t off = (size_t)dsc.score_off + (size_t)h * dsc.head_stride;
    const int32_t *ids = ids_in + off;
    const float *ss = scores_in + off;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int nseg = dsc.nseg;
    if (SEG) {
        static_assert(kMaxSegs == 64, "one segment per lane");
        if (threadIdx.x < 64) {
            const int a = lane < nseg ? seg_counts[((size_t)rh * kMaxSegs + lane) * 2] : 0;
            int ia = a;
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                const int t = __shfl_up(ia, o);
                if (lane >= o) ia += t;
            }
            pre[lane] = ia - a;
            if (lane == 63) pre[64] = ia;
        }
        __syncthreads();
    }
    const size_t seg_region = (size_t)dsc.seg_pages * kPageTokens;
    // position of element i of the head's list in ids / ss
    auto at = [&](int i) -> size_t {
        if (!SEG) return (size_t)i;
        int lo = 0, hi = nseg; // the last segment whose prefix is <= i
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (pre[mid] <= i) lo = mid; else hi = mid;
        }
        return (size_t)lo * seg_region + (size_t)(i - pre[lo]);
    };
    const int cnt = SEG ? pre[kMaxSegs] : counts[rh];
    int per = (cnt + splits - 1) / splits;
    per = (per + 15) & ~15;
    const int begin = min(cnt, sp * per), end = min(cnt, begin + per);
    const float M = head_M[rh];
    if (SEG) {
        if (ao.out_ids) {
            const int m = (int)((int64_t)end < ao.ids_stride ? (int64_t)end : ao.ids_stride);
            int32_t *dst = ao.out_ids + (size_t)rh * (size_t)ao.ids_stride;
            for (int i = begin + (int)threadIdx.x; i < m; i += kAttendThreads) dst[i] = ids[at(i)];
        }
        if (sp == 0 && threadIdx.x == 0) {
            counts[rh] = cnt;
            if (ao.out_counts) ao.out_counts[rh] = cnt;
            if (ao.out_ids && (int64_t)cnt > ao.ids_stride) atomicOr(ao.status, 1);
            head_maxkey[rh] = 0u; // clean for the next call (select_local, the last reader, is done)
        }
    }

    const int sub = lane & 15, grp = lane >> 4;
    float acc[EPL];
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[e] = 0.f;
    float l = 0.f;

    for (int i0 = begin + wave * 4 + grp; i0 < end; i0 += 16 * kAttendU) {
        int id[kAttendU];
        float p[kAttendU];
#pragma unroll
        for (int u = 0; u < kAttendU; ++u) {
            const int i = i0 + u * 16;
            const bool ok = i < end;
            const size_t src = ok ? at(i) : 0;
            id[u] = ok ? ids[src] : -1;
            p[u] = ok ? __expf((ss[src] - M) * scale) : 0.f;
        }
        const char *row[kAttendU];
#pragma unroll
        for (int u = 0; u < kAttendU; ++u) {
            const int t = id[u] < 0 ? 0 : id[u];
            const int phys = id[u] < 0 ? 0 : page_table[dsc.pt_off + (t >> 6)];
            row[u] = v_pool + (((size_t)phys * H_kv + kvh) * 64 + (t & 63)) * ROW_BYTES;
        }
        float v[kAttendU][EPL];
#pragma unroll
        for (int u = 0; u < kAttendU; ++u) {
            if (id[u] >= 0) {
                RS::load(row[u], sub, v[u]);
            } else {
#pragma unroll
                for (int e = 0; e < EPL; ++e) v[u][e] = 0.f;
            }
        }
#pragma unroll
        for (int u = 0; u < kAttendU; ++u) {
            l += p[u];
#pragma unroll
            for (int e = 0; e < EPL; ++e) acc[e] = fmaf(p[u], v[u][e], acc[e]);
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

hipError_t launch_attend(const Shape &sh, const DeviceViews &dv, int B, float scale, int splits, bool segmented,
                         int32_t *out_ids, int32_t *out_counts, int64_t ids_stride, hipStream_t st)
{
    const dim3 grid((unsigned)(B * sh.n_q_heads * splits)), block(kAttendThreads);
    const AttendOut ao{out_ids, out_counts, ids_stride, dv.status};
#define ALAYA_ATTEND(DT, D)                                                                                  \
    do {                                                                                                     \
        if (segmented)                                                                                       \
            attend_kernel<DT, D, true><<<grid, block, 0, st>>>(                                              \
                dv.desc.mem, dv.desc.in, dv.desc.n, sh.n_q_heads, sh.n_kv_heads, dv.page_table,              \
                (const char *)dv.v_pool, dv.loc_ids, dv.loc_scores, dv.counts, dv.head_M, scale, splits,     \
                dv.partials, dv.seg_counts, dv.head_maxkey, ao);                                             \
        else                                                                                                 \
            attend_kernel<DT, D, false><<<grid, block, 0, st>>>(                                             \
                dv.desc.mem, dv.desc.in, dv.desc.n, sh.n_q_heads, sh.n_kv_heads, dv.page_table,              \
                (const char *)dv.v_pool, dv.sel_ids, dv.sel_scores, dv.counts, dv.head_M, scale, splits,     \
                dv.partials, dv.seg_counts, dv.head_maxkey, ao);                                             \
    } while (0)
    if (sh.dtype == 0 && sh.head_dim == 128) ALAYA_ATTEND(0, 128);
    else if (sh.dtype == 0 && sh.head_dim == 64) ALAYA_ATTEND(0, 64);
    else if (sh.dtype == 1 && sh.head_dim == 128) ALAYA_ATTEND(1, 128);
    else if (sh.dtype == 1 && sh.head_dim == 64) ALAYA_ATTEND(1, 64);
    else return hipErrorInvalidValue;
#undef ALAYA_ATTEND
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// Merge of partial results, fixed order.  Grid: (request, head); one thread per output channel.
template <int D>
__global__ __launch_bounds__(D) void combine_kernel(const ReqDesc *__restrict__ desc_mem, const ReqDesc desc0, int desc_n, int B, int H_q,
                                                     const float *__restrict__ partials, int splits,
                                                     int per_request_tiles, int pages_per_tile,
                                                     float *__restrict__ out)
{
    const Descs desc{desc_mem, desc0, desc_n};
    const int rh = blockIdx.x;
    const int r = rh / H_q, h = rh % H_q;
    int np;
    size_t first, stride;
    if (per_request_tiles) {
        const ReqDesc dsc = desc[r];
        const int n_pages = (dsc.n + kPageTokens - 1) >> 6;
        np = (n_pages + pages_per_tile - 1) / pages_per_tile;
        first = ((size_t)dsc.tile_start * H_q + h) * (D + 2);
        stride = (size_t)H_q * (D + 2);
    } else {
        np = splits;
        first = (size_t)rh * splits * (D + 2);
        stride = D + 2;
    }
    // loads are issued eight at a time so that their latencies overlap; the merge order stays fixed
    constexpr int U = 8;
    // The splits of a sparse call all subtracted the same maximum (or hold nothing): no rescaling, and
    // no need to look for the largest reference first.
    float M = -INFINITY;
    for (int i0 = 0; per_request_tiles && i0 < np; i0 += U) {
        float mm[U];
#pragma unroll
        for (int u = 0; u < U; ++u) mm[u] = i0 + u < np ? partials[first + (size_t)(i0 + u) * stride] : -INFINITY;
#pragma unroll
        for (int u = 0; u < U; ++u) M = fmaxf(M, mm[u]);
    }
    float L = 0.f, o = 0.f;
    for (int i0 = 0; i0 < np; i0 += U) {
        float mm[U], ll[U], aa[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const bool ok = i0 + u < np;
            const float *p = partials + first + (size_t)(ok ? i0 + u : 0) * stride;
            mm[u] = ok ? p[0] : -INFINITY;
            ll[u] = p[1];
            aa[u] = p[2 + threadIdx.x];
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const float w = mm[u] == -INFINITY ? 0.f : per_request_tiles ? __expf(mm[u] - M) : 1.f;
            L = fmaf(w, ll[u], L);
            o = fmaf(w, aa[u], o);
        }
    }
    out[(size_t)rh * D + threadIdx.x] = o / L;
}

hipError_t launch_combine(const Shape &sh, const DeviceViews &dv, int B, int splits, int per_request_tiles,
                          int pages_per_tile, float *out, hipStream_t st)
{
    const dim3 grid((unsigned)(B * sh.n_q_heads));
    if (sh.head_dim == 128)
        combine_kernel<128><<<grid, dim3(128), 0, st>>>(dv.desc.mem, dv.desc.in, dv.desc.n, B, sh.n_q_heads, dv.partials, splits,
                                                        per_request_tiles, pages_per_tile, out);
    else if (sh.head_dim == 64)
        combine_kernel<64><<<grid, dim3(64), 0, st>>>(dv.desc.mem, dv.desc.in, dv.desc.n, B, sh.n_q_heads, dv.partials, splits,
                                                      per_request_tiles, pages_per_tile, out);
    else
        return hipErrorInvalidValue;
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// Dense attention, split over pages (Eq. 1 over every cached token).  Grid: (tile, KV head).  Each
// wavefront walks its pages: scores for 64 tokens x G heads as in the scoring pass (lane = token),
// online softmax per head, probabilities through LDS, then the page's value rows with 16 lanes per
// row.  The four wavefronts' results are merged before the partial is written.
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
    __shared__ float qs[G][D];
    __shared__ float ps[4][G][64];
    __shared__ float red[4][G][D + 2];

    const int kvh = blockIdx.x % H_kv;
    const int tile = blockIdx.x / H_kv;
    int r = 0;
    while (r + 1 < B && desc[r + 1].tile_start <= tile) ++r;
    const ReqDesc dsc = desc[r];
    const int H_q = H_kv * G;
    for (int i = threadIdx.x; i < G * D; i += 256) {
        const int g = i / D, c = i % D;
        const size_t qi = ((size_t)r * H_q + kvh * G + g) * D + c;
        qs[g][c] = DT == 0 ? bf16_to_f32(((const uint16_t *)qv)[qi]) : ((const float *)qv)[qi];
    }
    __syncthreads();

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
            const uint4 *base = k_pool + tile_off * (size_t)(NC * 64) + lane;
            uint4 kc[NC];
#pragma unroll
            for (int c = 0; c < NC; ++c) kc[c] = base[c * 64];
            float s[G];
#pragma unroll
            for (int g = 0; g < G; ++g) s[g] = 0.f;
#pragma unroll
            for (int c = 0; c < NC; ++c) {
                float kf[E];
                if constexpr (DT == 0) {
                    kf[0] = bf16_lo(kc[c].x); kf[1] = bf16_hi(kc[c].x); kf[2] = bf16_lo(kc[c].y); kf[3] = bf16_hi(kc[c].y);
                    kf[4] = bf16_lo(kc[c].z); kf[5] = bf16_hi(kc[c].z); kf[6] = bf16_lo(kc[c].w); kf[7] = bf16_hi(kc[c].w);
                } else {
                    kf[0] = __uint_as_float(kc[c].x); kf[1] = __uint_as_float(kc[c].y);
                    kf[2] = __uint_as_float(kc[c].z); kf[3] = __uint_as_float(kc[c].w);
                }
#pragma unroll
                for (int e = 0; e < E; ++e)
#pragma unroll
                    for (int g = 0; g < G; ++g) s[g] = fmaf(kf[e], qs[g][c * E + e], s[g]);
            }
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
                RS::load(vbase + (size_t)tok * ROW_BYTES, sub, v);
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
