// The coarse-grained index (Sec. 6.2 "Query Optimizer", index types; Table 4: top-k and filter queries):
// adjacent tokens are grouped into blocks, each block is represented by a few vectors, only the inner
// products of the query with the representatives are computed during retrieval, and the critical blocks
// are selected for the attention computation.  Here a block is a page of 64 tokens and its
// representatives are two vectors per KV head, the channel-wise minimum lo and maximum hi of its keys;
//   u[h][b] = sum_c max(q_hc * lo_bc, q_hc * hi_bc) = sum_c max(q_hc, 0) * hi_bc + min(q_hc, 0) * lo_bc
// is an upper bound of every q_h . k in block b.  The P blocks with the largest u are the critical blocks
// of head h (equal u: the smaller block), and the top-k query then runs over their tokens only.
//
//   reps_kernel          keeps lo and hi of the pages that an append touched (the index is maintained at
//                        Session.update, so a query never builds it)
//   coarse_score_kernel  u for every (page, head), written in the survivor-block format of the scoring
//                        pass with the page in the place of the token, so that the selection kernel picks
//                        the P best pages with the very code that picks the k best tokens; clears the page mask
//   select_kernel        (select.hip) also marks each head's chosen pages in one byte per (KV head, page),
//                        bit g = chosen by head g of the group: what the main scoring pass needs to skip a
//                        page's keys
#include "alaya_internal.h"
#include "row_slice.h"
#include "score_page.h"

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
    // (eight tokens at a time, so that their loads are on their way together; a token beyond the page's last
    // one repeats the last one, which changes neither extreme)
    for (int j0 = 0; j0 < ntok; j0 += 8) {
        float x[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int j = min(j0 + u, ntok - 1);
            if (DT == 0) x[u] = bf16_to_f32(((const uint16_t *)k_pool)[col + (size_t)j * E]);
            else x[u] = ((const float *)k_pool)[col + (size_t)j * E];
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            mn = fminf(mn, x[u]);
            mx = fmaxf(mx, x[u]);
        }
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
// The sum of x over the 16 lanes of a row (lanes 16 r .. 16 r + 15), in every one of them: four additions whose
// second operand comes through the DPP rotation of the row.
__device__ __forceinline__ float row16_sum(float x)
{
    x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x128, 0xf, 0xf, false)); // row_ror:8
    x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x124, 0xf, 0xf, false)); // row_ror:4
    x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x122, 0xf, 0xf, false)); // row_ror:2
    x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x121, 0xf, 0xf, false)); // row_ror:1
    return x;
}

// Block scores.  Grid: (tile of 256 pages, KV head, quarter of the tile), one wavefront each; descriptors are
// the PAGE-LEVEL ones (n = pages that hold a visible token, tileb_start / ntiles_b = tiles of 256 pages).
// 16 lanes per representative row, four pages per step; the lane's slice of the G queries stays in
// registers, split by sign.  The wavefront reads the page table entries of its 64 pages with one load and then has the rows
// of many pages on their way at once: taken page after page, every page cost two trips to memory in a row.
// It also clears the bytes of its pages in the page mask, which the selection of the pages fills afterwards.
template <int DT, int D, int G>
__global__ __launch_bounds__(64) void coarse_score_kernel(const ReqDesc *__restrict__ desc_mem, const ReqDesc desc0, int desc_n, int B,
                                                           const int32_t *__restrict__ page_table, const void *__restrict__ qv,
                                                           const char *__restrict__ rep_pool, const BlockArea area,
                                                           uint8_t *__restrict__ pmask, int H_kv)
{
    const Descs desc{desc_mem, desc0, desc_n};
    using RS = RowSlice<DT, D>;
    constexpr size_t ROW_BYTES = (size_t)D * (DT == 0 ? 2 : 4);
    constexpr int UN = RS::WORDS == 8 ? 8 : 16; // pages (x 4) whose rows are in flight together
    __shared__ float ustage[G][64];

    const int quarter = blockIdx.x & 3;
    const int blk = blockIdx.x >> 2; // (tile, KV head): the survivor block
    const int kvh = blk % H_kv;
    const int tile = blk / H_kv;
    int r = 0;
    while (r + 1 < B && desc[r + 1].tileb_start <= tile) ++r;
    const ReqDesc dsc = desc[r];
    const int H_q = H_kv * G;
    const int lane = threadIdx.x, sub = lane & 15, grp = lane >> 4;
    const int p_tile = (tile - dsc.tileb_start) * 256;
    const int n_pages = dsc.n; // page-level descriptor: n counts pages
    const int cnt = min(256, n_pages - p_tile); // pages of this tile: every one is handed on
    if (quarter == 0 && lane < G) *area.hdr(tile, kvh * G + lane) = make_uint2((uint32_t)cnt, (uint32_t)(lane * cnt));
    const int j = quarter * 64 + lane; // this lane's page inside the tile
    if (quarter * 64 >= cnt) return;   // (uniform)
    int phys_l = 0;                    // (beyond the last page: physical page 0, read and not used)
    if (j < cnt) {
        phys_l = page_table[dsc.pt_off + p_tile + j];
        pmask[(size_t)dsc.pm_off + (size_t)kvh * dsc.pm_stride + p_tile + j] = 0;
    }
    // The positive and the negative part of the lane's slice of each query (bf16: as packed pairs, so that two
    // channels take one dot instruction per part).
    constexpr int W = RS::WORDS;
    uint32_t qp[G][W], qn[G][W];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        const typename RS::Raw qr = RS::load_raw((const char *)qv + ((size_t)r * H_q + kvh * G + g) * ROW_BYTES, sub);
#pragma unroll
        for (int w = 0; w < W; ++w) {
            const uint32_t x = qr.w[w];
            if constexpr (DT == 0) {
                const uint32_t neg = ((x & 0x8000u) ? 0xFFFFu : 0u) | ((x & 0x80000000u) ? 0xFFFF0000u : 0u);
                qn[g][w] = x & neg;
                qp[g][w] = x & ~neg;
            } else {
                qn[g][w] = __float_as_uint(fminf(__uint_as_float(x), 0.f));
                qp[g][w] = __float_as_uint(fmaxf(__uint_as_float(x), 0.f));
            }
        }
    }
#pragma unroll 1
    for (int it0 = 0; it0 < 16; it0 += UN) {
        typename RS::Raw lo[UN], hi[UN];
#pragma unroll
        for (int i = 0; i < UN; ++i) {
            const int phys = __shfl(phys_l, (it0 + i) * 4 + grp);
            const char *row = rep_pool + ((size_t)phys * H_kv + kvh) * 2 * ROW_BYTES;
            lo[i] = RS::load_raw(row, sub);
            hi[i] = RS::load_raw(row + ROW_BYTES, sub);
        }
#pragma unroll
        for (int i = 0; i < UN; ++i) {
#pragma unroll
            for (int g = 0; g < G; ++g) {
                float x = 0.f;
#pragma unroll
                for (int w = 0; w < W; ++w) {
                    if constexpr (DT == 0) {
                        x = dot2_bf16(hi[i].w[w], qp[g][w], x);
                        x = dot2_bf16(lo[i].w[w], qn[g][w], x);
                    } else {
                        x = fmaf(__uint_as_float(hi[i].w[w]), __uint_as_float(qp[g][w]), x);
                        x = fmaf(__uint_as_float(lo[i].w[w]), __uint_as_float(qn[g][w]), x);
                    }
                }
                x = row16_sum(x);
                if (sub == 0) ustage[g][(it0 + i) * 4 + grp] = x;
            }
        }
    }
    __syncthreads();
    if (j < cnt) {
#pragma unroll
        for (int g = 0; g < G; ++g)
            *area.at(blk, g * cnt + j) = make_uint2(__float_as_uint(ustage[g][lane]), (uint32_t)(p_tile + j));
    }
}

hipError_t launch_coarse_score(const Shape &sh, const DeviceViews &dv, const DescArgs &pdesc, int B, const void *q,
                               const void *rep_pool, int total_tiles, const BlockArea &area, uint8_t *pmask, hipStream_t st)
{
    if (total_tiles <= 0) return hipSuccess;
    const int G = sh.n_q_heads / sh.n_kv_heads;
    const dim3 grid((unsigned)(total_tiles * sh.n_kv_heads * 4)), block(64);
#define ALAYA_COARSE(DT, D, GG)                                                                               \
    coarse_score_kernel<DT, D, GG><<<grid, block, 0, st>>>(pdesc.mem, pdesc.in, pdesc.n, B, dv.page_table, q,  \
                                                           (const char *)rep_pool, area, pmask,               \
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

} // namespace alaya
