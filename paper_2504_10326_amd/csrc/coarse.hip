// The coarse-grained index (Sec. 6.2 "Query Optimizer", index types; Table 4: top-k and filter queries):
// adjacent tokens are grouped into blocks, each block is represented by a few vectors, only the inner
// products of the query with the representatives are computed during retrieval, and the critical blocks
// are selected for the attention computation.  Here a block is a page of 64 tokens and its
// representatives are two vectors per KV head, the channel-wise minimum lo and maximum hi of its keys;
//   u[h][b] = sum_c max(q_hc * lo_bc, q_hc * hi_bc)
// is an upper bound of every q_h . k in block b.  The P blocks with the largest u are the critical blocks
// of head h (equal u: the smaller block), and the top-k query then runs over their tokens only.
//
//   reps_kernel          keeps lo and hi of the pages that an append touched (the index is maintained at
//                        Session.update, so a query never builds it)
//   coarse_score_kernel  u for every (page, head), written in the survivor-block format of the scoring
//                        pass with the page in the place of the token, so that the selection kernel picks
//                        the P best pages with the very code that picks the k best tokens
//   page_mask_kernel     turns each head's chosen pages into one byte per (KV head, page), bit g = chosen
//                        by head g of the group: what the main scoring pass needs to skip a page's keys
#include "alaya_internal.h"
#include "row_slice.h"

namespace alaya {

// ------------------------------------------------------------------------------------------------
// Representatives of one page of one KV head: thread = channel, a loop over the page's tokens.
//   K pool [page][kvh][D/E][64][E]      rep pool [page][kvh][2][D] (lo row, hi row), storage dtype
template <int DT>
__device__ __forceinline__ void rep_page(const void *__restrict__ k_pool, void *__restrict__ rep_pool, int phys, int kvh,
                                         int H_kv, int D, int ntok)
{
    constexpr int E = DT == 0 ? 8 : 4;
    const int c = threadIdx.x;
    if (c >= D) return;
    const size_t tile = ((size_t)phys * H_kv + kvh) * (size_t)(64 * D);
    const size_t col = tile + (size_t)(c / E) * 64 * E + (c % E);
    float mn = INFINITY, mx = -INFINITY;
    for (int j = 0; j < ntok; ++j) {
        float x;
        if (DT == 0) x = bf16_to_f32(((const uint16_t *)k_pool)[col + (size_t)j * E]);
        else x = ((const float *)k_pool)[col + (size_t)j * E];
        mn = fminf(mn, x);
        mx = fmaxf(mx, x);
    }
    const size_t row = ((size_t)phys * H_kv + kvh) * 2 * (size_t)D + c;
    if (DT == 0) { // the minimum and maximum of bf16 values are bf16 values: the upper halves are exact
        ((uint16_t *)rep_pool)[row] = (uint16_t)(__float_as_uint(mn) >> 16);
        ((uint16_t *)rep_pool)[row + D] = (uint16_t)(__float_as_uint(mx) >> 16);
    } else {
        ((float *)rep_pool)[row] = mn;
        ((float *)rep_pool)[row + D] = mx;
    }
}

// the pages first .. first + count - 1 of one sequence, which now holds n_new tokens
template <int DT>
__global__ __launch_bounds__(128) void reps_range_kernel(const int32_t *__restrict__ pt_row, const void *__restrict__ k_pool,
                                                         void *__restrict__ rep_pool, int first, int64_t n_new, int H_kv, int D)
{
    const int kvh = blockIdx.x % H_kv;
    const int p = first + blockIdx.x / H_kv;
    const int64_t in_page = n_new - (int64_t)p * kPageTokens;
    rep_page<DT>(k_pool, rep_pool, pt_row[p], kvh, H_kv, D, (int)(in_page < kPageTokens ? in_page : kPageTokens));
}

// the last page of each of B sequences after a decode step's append: desc[b].n = the length BEFORE it
template <int DT>
__global__ __launch_bounds__(128) void reps_step_kernel(const ReqDesc *__restrict__ desc_mem, const ReqDesc desc0, int desc_n,
                                                        const int32_t *__restrict__ page_table, const void *__restrict__ k_pool,
                                                        void *__restrict__ rep_pool, int H_kv, int D)
{
    const Descs desc{desc_mem, desc0, desc_n};
    const int kvh = blockIdx.x % H_kv;
    const ReqDesc d = desc[blockIdx.x / H_kv];
    const int p = d.n >> 6;
    rep_page<DT>(k_pool, rep_pool, page_table[d.pt_off + p], kvh, H_kv, D, (d.n & 63) + 1);
}

hipError_t launch_reps_range(const Shape &sh, const int32_t *pt_row, const void *k_pool, void *rep_pool, int first,
                             int count, int64_t n_new, hipStream_t st)
{
    if (count <= 0) return hipSuccess;
    const dim3 grid((unsigned)(count * sh.n_kv_heads)), block(128);
    if (sh.dtype == 0) reps_range_kernel<0><<<grid, block, 0, st>>>(pt_row, k_pool, rep_pool, first, n_new, sh.n_kv_heads, sh.head_dim);
    else reps_range_kernel<1><<<grid, block, 0, st>>>(pt_row, k_pool, rep_pool, first, n_new, sh.n_kv_heads, sh.head_dim);
    return hipGetLastError();
}

hipError_t launch_reps_step(const Shape &sh, const DeviceViews &dv, void *rep_pool, int B, hipStream_t st)
{
    const dim3 grid((unsigned)(B * sh.n_kv_heads)), block(128);
    if (sh.dtype == 0)
        reps_step_kernel<0><<<grid, block, 0, st>>>(dv.desc.mem, dv.desc.in, dv.desc.n, dv.page_table, dv.k_pool, rep_pool,
                                                     sh.n_kv_heads, sh.head_dim);
    else
        reps_step_kernel<1><<<grid, block, 0, st>>>(dv.desc.mem, dv.desc.in, dv.desc.n, dv.page_table, dv.k_pool, rep_pool,
                                                     sh.n_kv_heads, sh.head_dim);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// Block scores.  Grid: (tile of 256 pages, KV head); descriptors are the PAGE-LEVEL ones (n = pages that
// hold a visible token, tileb_start / ntiles_b = tiles of 256 pages).  16 lanes per representative row,
// four pages per wavefront step; the lane's slice of the G queries stays in registers.
template <int DT, int D, int G>
__global__ __launch_bounds__(256) void coarse_score_kernel(const ReqDesc *__restrict__ desc_mem, const ReqDesc desc0, int desc_n, int B,
                                                            const int32_t *__restrict__ page_table, const void *__restrict__ qv,
                                                            const char *__restrict__ rep_pool, const BlockArea area,
                                                            int H_kv)
{
    const Descs desc{desc_mem, desc0, desc_n};
    using RS = RowSlice<DT, D>;
    constexpr int EPL = RS::EPL;
    constexpr size_t ROW_BYTES = (size_t)D * (DT == 0 ? 2 : 4);
    __shared__ float ustage[G][256];

    const int kvh = blockIdx.x % H_kv;
    const int tile = blockIdx.x / H_kv;
    int r = 0;
    while (r + 1 < B && desc[r + 1].tileb_start <= tile) ++r;
    const ReqDesc dsc = desc[r];
    const int H_q = H_kv * G;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, sub = lane & 15, grp = lane >> 4;
    float q[G][EPL];
#pragma unroll
    for (int g = 0; g < G; ++g)
        RS::load((const char *)qv + ((size_t)r * H_q + kvh * G + g) * ROW_BYTES, sub, q[g]);
    const int p_tile = (tile - dsc.tileb_start) * 256;
    const int n_pages = dsc.n; // page-level descriptor: n counts pages
#pragma unroll 4
    for (int it = 0; it < 16; ++it) {
        const int pi = wave * 64 + it * 4 + grp; // page inside the tile
        const int p = p_tile + pi;
        float u[G];
#pragma unroll
        for (int g = 0; g < G; ++g) u[g] = 0.f;
        if (p < n_pages) {
            const int phys = page_table[dsc.pt_off + p];
            const char *row = rep_pool + ((size_t)phys * H_kv + kvh) * 2 * ROW_BYTES;
            float lo[EPL], hi[EPL];
            RS::load(row, sub, lo);
            RS::load(row + ROW_BYTES, sub, hi);
#pragma unroll
            for (int g = 0; g < G; ++g)
#pragma unroll
                for (int e = 0; e < EPL; ++e) u[g] += fmaxf(q[g][e] * lo[e], q[g][e] * hi[e]);
        }
#pragma unroll
        for (int g = 0; g < G; ++g) {
            float x = u[g];
            x += __shfl_xor(x, 1);
            x += __shfl_xor(x, 2);
            x += __shfl_xor(x, 4);
            x += __shfl_xor(x, 8);
            if (sub == 0) ustage[g][pi] = x;
        }
    }
    __syncthreads();
    const int cnt = min(256, n_pages - p_tile); // pages of this tile: every one is handed on
    if (threadIdx.x < G)
        *area.hdr((int)(blockIdx.x / H_kv), (int)(blockIdx.x % H_kv) * G + (int)threadIdx.x) =
            make_uint2((uint32_t)cnt, (uint32_t)(threadIdx.x * cnt));
    if ((int)threadIdx.x < cnt) {
#pragma unroll
        for (int g = 0; g < G; ++g)
            *area.at(blockIdx.x, g * cnt + (int)threadIdx.x) = make_uint2(__float_as_uint(ustage[g][threadIdx.x]), (uint32_t)(p_tile + threadIdx.x));
    }
}

hipError_t launch_coarse_score(const Shape &sh, const DeviceViews &dv, const DescArgs &pdesc, int B, const void *q,
                               const void *rep_pool, int total_tiles, const BlockArea &area, hipStream_t st)
{
    if (total_tiles <= 0) return hipSuccess;
    const int G = sh.n_q_heads / sh.n_kv_heads;
    const dim3 grid((unsigned)(total_tiles * sh.n_kv_heads)), block(256);
#define ALAYA_COARSE(DT, D, GG)                                                                               \
    coarse_score_kernel<DT, D, GG><<<grid, block, 0, st>>>(pdesc.mem, pdesc.in, pdesc.n, B, dv.page_table, q,  \
                                                           (const char *)rep_pool, area,                      \
                                                           sh.n_kv_heads)
#define ALAYA_COARSE_G(DT, D)                                                                                 \
    switch (G) {                                                                                              \
    case 1: ALAYA_COARSE(DT, D, 1); break;                                                                    \
    case 2: ALAYA_COARSE(DT, D, 2); break;                                                                    \
    case 4: ALAYA_COARSE(DT, D, 4); break;                                                                    \
    case 8: ALAYA_COARSE(DT, D, 8); break;                                                                    \
    default: return hipErrorInvalidValue;                                                                     \
    }
    if (sh.dtype == 0 && sh.head_dim == 128) { ALAYA_COARSE_G(0, 128) }
    else if (sh.dtype == 0 && sh.head_dim == 64) { ALAYA_COARSE_G(0, 64) }
    else if (sh.dtype == 1 && sh.head_dim == 128) { ALAYA_COARSE_G(1, 128) }
    else if (sh.dtype == 1 && sh.head_dim == 64) { ALAYA_COARSE_G(1, 64) }
    else return hipErrorInvalidValue;
#undef ALAYA_COARSE_G
#undef ALAYA_COARSE
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// Chosen pages -> one byte per (KV head, page).  Grid: (request, head); the mask was zeroed before.
__global__ __launch_bounds__(256) void page_mask_kernel(const ReqDesc *__restrict__ desc_mem, const ReqDesc desc0, int desc_n,
                                                         const ReqDesc *__restrict__ tdesc_mem, const ReqDesc tdesc0, int H_q,
                                                         int H_kv, const int32_t *__restrict__ pg_ids,
                                                         const int32_t *__restrict__ pg_counts, uint32_t *__restrict__ pmask)
{
    const Descs pdesc{desc_mem, desc0, desc_n};   // page-level: where the chosen pages are
    const Descs tdesc{tdesc_mem, tdesc0, desc_n}; // token-level: where the request's mask is
    const int rh = blockIdx.x;
    const int r = rh / H_q, h = rh % H_q;
    const int G = H_q / H_kv, kvh = h / G, g = h % G;
    const ReqDesc pd = pdesc[r], td = tdesc[r];
    const int32_t *ids = pg_ids + (size_t)pd.score_off + (size_t)h * pd.head_stride;
    const int cnt = pg_counts[rh];
    for (int i = threadIdx.x; i < cnt; i += 256) {
        const size_t byte = (size_t)td.pm_off + (size_t)kvh * td.pm_stride + ids[i];
        atomicOr(&pmask[byte >> 2], 1u << (8 * (byte & 3) + g));
    }
}

hipError_t launch_page_mask(const Shape &sh, const DeviceViews &dv, const DescArgs &pdesc, int B, const int32_t *pg_ids,
                            const int32_t *pg_counts, uint32_t *pmask, hipStream_t st)
{
    page_mask_kernel<<<dim3((unsigned)(B * sh.n_q_heads)), dim3(256), 0, st>>>(
        pdesc.mem, pdesc.in, pdesc.n, dv.desc.mem, dv.desc.in, sh.n_q_heads, sh.n_kv_heads, pg_ids, pg_counts, pmask);
    return hipGetLastError();
}

} // namespace alaya
