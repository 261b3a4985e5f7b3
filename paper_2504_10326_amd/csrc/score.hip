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

namespace alaya {

__device__ __forceinline__ float bf16_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t u) { return __uint_as_float(u & 0xFFFF0000u); }
__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

// Unpack one 16-byte chunk into floats: 8 bf16 or 4 fp32.
template <int DT> struct Chunk;
template <> struct Chunk<0> {
    static constexpr int E = 8;
    __device__ static __forceinline__ void unpack(const uint4 &c, float *f)
    {
        f[0] = bf16_lo(c.x); f[1] = bf16_hi(c.x); f[2] = bf16_lo(c.y); f[3] = bf16_hi(c.y);
        f[4] = bf16_lo(c.z); f[5] = bf16_hi(c.z); f[6] = bf16_lo(c.w); f[7] = bf16_hi(c.w);
    }
};
template <> struct Chunk<1> {
    static constexpr int E = 4;
    __device__ static __forceinline__ void unpack(const uint4 &c, float *f)
    {
        f[0] = __uint_as_float(c.x); f[1] = __uint_as_float(c.y);
        f[2] = __uint_as_float(c.z); f[3] = __uint_as_float(c.w);
    }
};

// ------------------------------------------------------------------------------------------------
// Append: one thread moves one 16-byte slice of one token's key and of its value.
//   k, v   [t][H_kv][D] token-major (what the model emits)
//   K pool [page][kvh][D/E][64][E]      V pool [page][kvh][64][D]
template <int DT>
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
    const int E = sh.dtype == 0 ? 8 : 4;
    const int NC = sh.head_dim / E;
    const int64_t total = t * sh.n_kv_heads * NC;
    int64_t blocks = (total + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    if (blocks < 1) blocks = 1;
    if (sh.dtype == 0)
        append_kernel<0><<<dim3((unsigned)blocks), dim3(256), 0, st>>>(pt_row, (uint4 *)k_pool, (uint4 *)v_pool,
                                                                       (const uint4 *)k, (const uint4 *)v, n_old, t,
                                                                       sh.n_kv_heads, NC);
    else
        append_kernel<1><<<dim3((unsigned)blocks), dim3(256), 0, st>>>(pt_row, (uint4 *)k_pool, (uint4 *)v_pool,
                                                                       (const uint4 *)k, (const uint4 *)v, n_old, t,
                                                                       sh.n_kv_heads, NC);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// Scoring.  Grid: one workgroup per (tile, KV head); KV head is the fastest index so that with
// 8 KV heads each head's stream stays on one XCD (workgroups are dealt to XCDs round-robin).
// A tile is kScoreWaves * pages_per_wave consecutive pages of one request; each wavefront scores
// pages_per_wave pages in a row.
//
// The query stays in scalar registers: its address is wave-uniform, so the compiler fetches it with
// scalar loads and feeds it to the vector ALU as the scalar operand.  bf16 uses the packed
// dot-product instruction (two bf16 products and the fp32 accumulate in one op, both operands used
// as stored); fp32 uses fused multiply-add.
//
// Epilogue, no global float atomics and nothing to reset:
//   tile_max[tile][head]   maximum score of the tile (the heads' global maxima are reduced from these)
//   hist[request, head][.] (top-k only) counts per top-11-bit bucket of the order-preserving score
//                          image, gathered in LDS and flushed with integer atomics (exact, order-free)
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;

__device__ __forceinline__ float dot2_bf16(uint32_t a, uint32_t b, float c)
{
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a), __builtin_bit_cast(bf16x2_t, b), c,
                                           false);
}

template <int DT, int D, int G>
__global__ __launch_bounds__(256) void score_kernel(const ReqDesc *__restrict__ desc, int B,
                                                     const int32_t *__restrict__ page_table,
                                                     const uint32_t *__restrict__ qw, const uint4 *__restrict__ k_pool,
                                                     float *__restrict__ scores, float *__restrict__ tile_max,
                                                     uint32_t *__restrict__ hist, int H_kv, int ppw, int want_hist)
{
    constexpr int NC = D * (DT == 0 ? 2 : 4) / 16; // 16-byte chunks per key
    constexpr int QW = D * (DT == 0 ? 2 : 4) / 4;  // 32-bit words per query head
    // two 16-bit counters per word: a workgroup scores at most 4 * 64 * 64 = 16384 tokens per head
    __shared__ uint32_t lhist[G][kHistBins / 2];
    __shared__ float wmax[kScoreWaves][G];

    const int kvh = blockIdx.x % H_kv;
    const int tile = blockIdx.x / H_kv;
    int r = 0;
    while (r + 1 < B && desc[r + 1].tile_start <= tile) ++r;
    const ReqDesc dsc = desc[r];
    const int H_q = H_kv * G;

    if (want_hist) {
        for (int i = threadIdx.x; i < G * (kHistBins / 2); i += 256) (&lhist[0][0])[i] = 0u;
        __syncthreads();
    }

    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    const int n_pages = (dsc.n + kPageTokens - 1) >> 6;
    const int p_begin = ((tile - dsc.tile_start) * kScoreWaves + wave) * ppw;
    const int p_end = min(p_begin + ppw, n_pages);
    const uint32_t *qh = qw + ((size_t)r * H_q + kvh * G) * QW; // wave-uniform: scalar loads

    float lmax[G];
#pragma unroll
    for (int g = 0; g < G; ++g) lmax[g] = -INFINITY;

    for (int p = p_begin; p < p_end; ++p) {
        const int phys = page_table[dsc.pt_off + p];
        const uint4 *base = k_pool + ((size_t)phys * H_kv + kvh) * (size_t)(NC * 64) + lane;
        uint4 kc[NC];
#pragma unroll
        for (int c = 0; c < NC; ++c) kc[c] = base[c * 64];
        float acc[G];
#pragma unroll
        for (int g = 0; g < G; ++g) acc[g] = 0.f;
#pragma unroll
        for (int c = 0; c < NC; ++c) {
#pragma unroll
            for (int g = 0; g < G; ++g) {
                const uint32_t *qg = qh + g * QW + c * 4;
                if constexpr (DT == 0) {
                    acc[g] = dot2_bf16(kc[c].x, qg[0], acc[g]);
                    acc[g] = dot2_bf16(kc[c].y, qg[1], acc[g]);
                    acc[g] = dot2_bf16(kc[c].z, qg[2], acc[g]);
                    acc[g] = dot2_bf16(kc[c].w, qg[3], acc[g]);
                } else {
                    acc[g] = fmaf(__uint_as_float(kc[c].x), __uint_as_float(qg[0]), acc[g]);
                    acc[g] = fmaf(__uint_as_float(kc[c].y), __uint_as_float(qg[1]), acc[g]);
                    acc[g] = fmaf(__uint_as_float(kc[c].z), __uint_as_float(qg[2]), acc[g]);
                    acc[g] = fmaf(__uint_as_float(kc[c].w), __uint_as_float(qg[3]), acc[g]);
                }
            }
        }
        const int j = p * kPageTokens + lane;
        if (j < dsc.n) {
#pragma unroll
            for (int g = 0; g < G; ++g) {
                scores[dsc.score_off + (size_t)(kvh * G + g) * dsc.head_stride + j] = acc[g];
                lmax[g] = fmaxf(lmax[g], acc[g]);
                if (want_hist) {
                    const uint32_t bin = ord_key(acc[g]) >> 21;
                    atomicAdd(&lhist[g][bin >> 1], 1u << ((bin & 1u) * 16u));
                }
            }
        }
    }

#pragma unroll
    for (int g = 0; g < G; ++g) {
        float m = lmax[g];
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o));
        if (lane == 0) wmax[wave][g] = m;
    }
    __syncthreads();
    if (threadIdx.x < G) {
        float m = wmax[0][threadIdx.x];
#pragma unroll
        for (int w = 1; w < kScoreWaves; ++w) m = fmaxf(m, wmax[w][threadIdx.x]);
        tile_max[(size_t)tile * H_q + kvh * G + threadIdx.x] = m; // -inf if the tile's pages were all out of range
    }
    if (want_hist) {
        uint32_t *gh = hist + ((size_t)r * H_q + kvh * G) * kHistBins;
        for (int i = threadIdx.x; i < G * (kHistBins / 2); i += 256) {
            const uint32_t v = (&lhist[0][0])[i];
            if (v & 0xFFFFu) atomicAdd(&gh[2 * i], v & 0xFFFFu);
            if (v >> 16) atomicAdd(&gh[2 * i + 1], v >> 16);
        }
    }
}

template <int DT, int D>
static hipError_t launch_score_g(const Shape &sh, const DeviceViews &dv, int B, const void *q, int total_tiles,
                                 int ppw, int want_hist, hipStream_t st)
{
    const int G = sh.n_q_heads / sh.n_kv_heads;
    const dim3 grid((unsigned)(total_tiles * sh.n_kv_heads)), block(256);
#define ALAYA_SCORE(GG)                                                                                       \
    score_kernel<DT, D, GG><<<grid, block, 0, st>>>(dv.desc, B, dv.page_table, (const uint32_t *)q,           \
                                                    (const uint4 *)dv.k_pool, dv.scores, dv.tile_max, dv.hist, \
                                                    sh.n_kv_heads, ppw, want_hist)
    switch (G) {
    case 1: ALAYA_SCORE(1); break;
    case 2: ALAYA_SCORE(2); break;
    case 4: ALAYA_SCORE(4); break;
    case 8: ALAYA_SCORE(8); break;
    default: return hipErrorInvalidValue;
    }
#undef ALAYA_SCORE
    return hipGetLastError();
}

hipError_t launch_score(const Shape &sh, const DeviceViews &dv, int B, const void *q, int total_tiles, int ppw,
                        int want_hist, hipStream_t st)
{
    if (sh.dtype == 0) {
        if (sh.head_dim == 128) return launch_score_g<0, 128>(sh, dv, B, q, total_tiles, ppw, want_hist, st);
        if (sh.head_dim == 64) return launch_score_g<0, 64>(sh, dv, B, q, total_tiles, ppw, want_hist, st);
    } else {
        if (sh.head_dim == 128) return launch_score_g<1, 128>(sh, dv, B, q, total_tiles, ppw, want_hist, st);
        if (sh.head_dim == 64) return launch_score_g<1, 64>(sh, dv, B, q, total_tiles, ppw, want_hist, st);
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

} // namespace alaya
