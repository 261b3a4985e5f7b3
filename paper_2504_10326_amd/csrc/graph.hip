// The fine-grained index (Sec. 6.2 "Query Optimizer", index types) and the DIPRS query on it (Sec. 6.1.3
// "DIPR Query Processing", Algorithm 1).
//
// Index: the exact M-nearest-neighbour graph of a sequence's keys under the inner product, one graph per
// KV head (shared by the query heads of the group, as Sec. 7.2 "GQA-based index sharing" shares one graph
// among a query group).  The paper builds RoarGraph with a GPU nearest-neighbour stage (Sec. 7.2 "Index
// Construction Acceleration"); any graph index serves Algorithm 1, and the exact graph needs nothing but the keys:
//   knn_kernel    K K^T on the matrix cores (v_mfma_f32_32x32x16_bf16; the K pool keeps 8 consecutive
//                 channels of a token in one 16-byte word: the operand of the instruction as it is), the M
//                 best of every row kept on the way (equal product: smaller token first)
//   norm_kernel   the entry point of each KV head's graph: its key of largest norm
// Query: diprs_kernel, one wavefront per query head, walks Algorithm 1 in the paper's order - the list C
// is visited entry by entry, the neighbours of an entry are examined in the order of its list - so that the
// list C and the answer are the ones the sequential algorithm gives.  The neighbours of one entry are scored
// by the lanes side by side (lane = neighbour); what the sequential order decides (who is still under the
// capacity threshold l0, what the best inner product was when a neighbour's turn came) is recovered with a
// prefix count and a prefix maximum over the lanes.  Scores are fp32, one fused multiply-add per channel in
// channel order.
#include "alaya_internal.h"
#include "row_slice.h"

#include <algorithm>

namespace alaya {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_g;
typedef __attribute__((ext_vector_type(16))) float f32x16_g;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4_g;

// 16-byte word holding channels [8c, 8c + 8) of token j of KV head kvh (bf16 pool, D = 128: 16 words per token)
__device__ __forceinline__ const uint4 *key_word(const uint4 *__restrict__ k_pool, const int32_t *__restrict__ pt_row,
                                                 int H_kv, int kvh, int NC, int j, int c)
{
    const int phys = pt_row[j >> 6];
    return k_pool + ((size_t)phys * H_kv + kvh) * (size_t)(NC * 64) + (size_t)c * 64 + (j & 63);
}

// ------------------------------------------------------------------------------------------------
// Entry point of a KV head's graph: the key of largest squared norm (equal norms: smaller token).  Grid:
// (KV heads, slices of the sequence); best[kvh] = (ordered norm << 32) | ~token, zero on entry, raised with
// a 64-bit atomic maximum (one per workgroup).
template <int D>
__global__ __launch_bounds__(256) void norm_kernel(const uint4 *__restrict__ k_pool, const int32_t *__restrict__ pt_row,
                                                   int H_kv, int n, unsigned long long *__restrict__ best)
{
    constexpr int NC = D / 8;
    __shared__ unsigned long long red[256];
    const int kvh = blockIdx.x;
    unsigned long long mine = 0ull;
    for (int j = blockIdx.y * 256 + threadIdx.x; j < n; j += 256 * gridDim.y) {
        float acc = 0.f;
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            const uint4 w = *key_word(k_pool, pt_row, H_kv, kvh, NC, j, c);
            const uint32_t ww[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float lo = bf16_lo(ww[e]), hi = bf16_hi(ww[e]);
                acc = fmaf(lo, lo, acc);
                acc = fmaf(hi, hi, acc);
            }
        }
        const unsigned long long key = ((unsigned long long)ord_key(acc) << 32) | (0xFFFFFFFFu - (uint32_t)j);
        mine = key > mine ? key : mine;
    }
    red[threadIdx.x] = mine;
    __syncthreads();
    for (int o = 128; o > 0; o >>= 1) {
        if ((int)threadIdx.x < o && red[threadIdx.x + o] > red[threadIdx.x]) red[threadIdx.x] = red[threadIdx.x + o];
        __syncthreads();
    }
    if (threadIdx.x == 0 && red[0] != 0ull) atomicMax(best + kvh, red[0]);
}

// ------------------------------------------------------------------------------------------------
// The exact M-nearest-neighbour graph in one pass: K K^T on the matrix cores, the M best of every row kept on
// the way, no similarity matrix in memory.  Grid: (strips of 128 rows, KV heads).  Wavefront w of a workgroup
// owns rows [32 w, 32 w + 32) of the strip: their keys stay in its registers as the A operand, and it walks all
// columns 32 at a time (the 32 keys of a step are staged in LDS once for the four wavefronts).  The matrix
// instruction leaves a lane 16 entries of one column of its result; the step's keys go in as its first operand
// and the wavefront's rows as the second, so that this column is a ROW of K K^T: lanes l and l + 32 own row l
// of the wavefront, 16 of the step's 32 columns each (in groups of four, alternating), with a list of their
// own for it in LDS, its length and the row's bar in registers - no atomics, no lane depends on another.  A product above the bar - the M-th best of the row when its lists were last
// tidied - is appended.  Columns come in ascending order, so a later key with the same product as the M-th
// best loses the tie: the test is a strict "greater".  When one of a row's two lists cannot take another
// step's worth, the wavefront tidies the row: both lists sorted together (bitonic, two entries per lane; keys
// are (ordered product, ~column), a total order), cut to M, dealt back to the two lists, the bar raised.
constexpr int kKnnRows = 128; // rows per workgroup
constexpr int kKnnSub = 64;   // entries per list; a row has two
static_assert(kKnnSub <= 64 && kKnnSub >= 32 + 16, "a list is sorted as one entry per lane, and holds M / 2 entries plus a step's 16");

__device__ __forceinline__ unsigned long long shfl_xor_u64(unsigned long long v, int m)
{
    const uint32_t lo = (uint32_t)__shfl_xor((int)(uint32_t)v, m), hi = (uint32_t)__shfl_xor((int)(uint32_t)(v >> 32), m);
    return ((unsigned long long)hi << 32) | lo;
}

// Sorts the 128 keys held two per lane (element lane + 64 * slot) into descending order.
__device__ __forceinline__ void sort128_desc(unsigned long long &k0, unsigned long long &k1, int lane)
{
#pragma unroll
    for (int k = 2; k <= 128; k <<= 1) {
#pragma unroll
        for (int j = k >> 1; j > 0; j >>= 1) {
            if (j == 64) { // partner: the lane's own other slot; k == 128, descending throughout
                const unsigned long long hi = k0 > k1 ? k0 : k1, lo = k0 > k1 ? k1 : k0;
                k0 = hi;
                k1 = lo;
            } else {
                const unsigned long long p0 = shfl_xor_u64(k0, j), p1 = shfl_xor_u64(k1, j);
                const bool first = (lane & j) == 0;                  // this element is the lower index of the pair
                const bool desc0 = (lane & k) == 0;                  // element index = lane (slot 0): direction of its run
                const bool desc1 = ((lane + 64) & k) == 0;           // element index = lane + 64 (slot 1)
                const bool take_max0 = first == desc0, take_max1 = first == desc1;
                k0 = take_max0 ? (k0 > p0 ? k0 : p0) : (k0 < p0 ? k0 : p0);
                k1 = take_max1 ? (k1 > p1 ? k1 : p1) : (k1 < p1 ? k1 : p1);
            }
        }
    }
}

constexpr int kKnnAhead = 8;      // steps per round: a round's keys are loaded during the round before
constexpr int kKnnPtLds = 3584;   // page-table entries that fit beside the lists (229 thousand tokens)

// A workgroup barrier that orders LDS traffic only.  (__syncthreads also waits for every global load in
// flight - here the keys fetched several steps ahead - which would undo the prefetch.)
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

template <int D>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1))) void knn_kernel(const uint4 *__restrict__ k_pool, const int32_t *__restrict__ pt_row,
                                                  int H_kv, int n, int M, int32_t *__restrict__ nbr_all)
{
    constexpr int NC = D / 8, STEPS = D / 16, LA = kKnnAhead;
    extern __shared__ __attribute__((aligned(16))) unsigned long long knn_lds[];
    unsigned long long *lists = knn_lds;                                     // [kKnnRows][2][kKnnSub]
    u32x4_g *stage = (u32x4_g *)(lists + (size_t)kKnnRows * 2 * kKnnSub);    // [2][NC][32]
    int32_t *pt_lds = (int32_t *)(stage + 2 * NC * 32);                      // [kKnnPtLds]

    const int kvh = blockIdx.y;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int half = lane >> 5, l32 = lane & 31;
    const int r0 = blockIdx.x * kKnnRows;          // first row of the strip
    int32_t *nbr = nbr_all + (size_t)kvh * (size_t)n * M;
    const int n_pages = (n + kPageTokens - 1) / kPageTokens;
    const bool pt_near = n_pages <= kKnnPtLds; // (uniform) the page table is read from LDS: one latency less per key

    if (pt_near)
        for (int i = tid; i < n_pages; i += 256) pt_lds[i] = pt_row[i];
    // A operand: this wavefront's 32 rows
    u32x4_g a[STEPS];
    const int arow = r0 + wave * 32 + l32;
#pragma unroll
    for (int s = 0; s < STEPS; ++s)
        a[s] = arow < n ? *(const u32x4_g *)key_word(k_pool, pt_row, H_kv, kvh, NC, arow, 2 * s + half) : u32x4_g{0u, 0u, 0u, 0u};
    __syncthreads();
    // staging: thread t brings the words (t / 32) and (t / 32 + 8) of column t % 32 of a step
    const int scol = tid & 31, sw = tid >> 5;
    // (columns beyond n are not skipped but clamped, and never selected: straight-line loads keep the count of
    // loads in flight exact, so that a step waits only for the keys it needs)
    auto fetch = [&](int cb, u32x4_g &x, u32x4_g &y) {
        const int col = min(cb * 32 + scol, n - 1);
        const int phys = pt_near ? pt_lds[col >> 6] : pt_row[col >> 6];
        const u32x4_g *kp = (const u32x4_g *)k_pool + ((size_t)phys * H_kv + kvh) * (size_t)(NC * 64) + (col & 63);
        x = kp[(size_t)sw * 64];
        y = kp[(size_t)(sw + 8) * 64];
    };
    const int steps = ((n + 31) / 32 + LA - 1) / LA * LA; // (whole rounds of LA steps; the extra ones find no column < n)
    // A round is LA steps.  Its keys were asked for a round ago and are awaited once, at its start; the next
    // round's are asked for at once and travel while this round computes.  (A ring of loads that wraps around
    // the loop would do with fewer registers, but the compiler cannot tell how old a load is once the loop has
    // turned, and waits for all of them at every step.)
    u32x4_g cx[LA], cy[LA], nx[LA], ny[LA];
#pragma unroll
    for (int u = 0; u < LA; ++u) fetch(u, nx[u], ny[u]);

    // this lane's row, its list, and what it knows of the row
    const int myrow = r0 + wave * 32 + l32;
    unsigned long long *mylist = lists + ((size_t)(wave * 32 + l32) * 2 + half) * kKnnSub;
    int cnt = 0;
    float bar = -INFINITY;

    // Tidying a row: of the entries of its two lists the M best stay, dealt back to the two lists (in no
    // particular order: only the final pass sorts), and the bar becomes the M-th best product.  That product is
    // found bit by bit from the top - ballots and counts, no sorting network, no shuffles; equal products at the
    // bar (they differ in their columns) are settled the same way on the low halves of the keys.  Returns what
    // the row's two lanes keep: their new lengths and the new bar.
    auto tidy = [&](int r, int &len_a, int &len_b, float &new_bar) {
        const int ca = __builtin_amdgcn_readlane(cnt, r), cb = __builtin_amdgcn_readlane(cnt, 32 + r);
        unsigned long long *la = lists + (size_t)(wave * 32 + r) * 2 * kKnnSub;
        const unsigned long long k0 = lane < ca ? la[lane] : 0ull, k1 = lane < cb ? la[kKnnSub + lane] : 0ull;
        const uint32_t s0 = (uint32_t)(k0 >> 32), s1 = (uint32_t)(k1 >> 32); // (0: no entry; below every product)
        bool keep0 = k0 != 0ull, keep1 = k1 != 0ull;
        new_bar = -INFINITY;
        if (ca + cb > M) { // (uniform)
            uint32_t T = 0u;
            int need = M;
#pragma unroll 1
            for (int bit = 31; bit >= 0; --bit) {
                const uint32_t cand = T | (1u << bit), top = ~((1u << bit) - 1u);
                const int c = __popcll(__ballot((s0 & top) == cand)) + __popcll(__ballot((s1 & top) == cand));
                if (c >= need) T = cand; else need -= c;
            }
            // T: the M-th best product; `need` of the entries equal to it stay: those with the smallest columns
            const bool eq0 = s0 == T, eq1 = s1 == T;
            const int n_eq = __popcll(__ballot(eq0)) + __popcll(__ballot(eq1));
            uint32_t L = 0u; // of the entries at T, those with low half >= L stay
            if (n_eq != need) {
                const uint32_t l0 = (uint32_t)k0, l1 = (uint32_t)k1;
#pragma unroll 1
                for (int bit = 31; bit >= 0; --bit) {
                    const uint32_t cand = L | (1u << bit), top = ~((1u << bit) - 1u);
                    const int c = __popcll(__ballot(eq0 && (l0 & top) == cand)) + __popcll(__ballot(eq1 && (l1 & top) == cand));
                    if (c >= need) L = cand; else need -= c;
                }
            }
            keep0 = s0 > T || (eq0 && (uint32_t)k0 >= L);
            keep1 = s1 > T || (eq1 && (uint32_t)k1 >= L);
            new_bar = ord_float(T);
        }
        const unsigned long long b0 = __ballot(keep0), b1 = __ballot(keep1);
        const unsigned long long lt = (1ull << lane) - 1ull;
        const int n0 = __popcll(b0), p0 = __popcll(b0 & lt), p1 = n0 + __popcll(b1 & lt);
        if (keep0) la[(size_t)(p0 & 1) * kKnnSub + (p0 >> 1)] = k0;
        if (keep1) la[(size_t)(p1 & 1) * kKnnSub + (p1 >> 1)] = k1;
        const int kept = n0 + __popcll(b1);
        len_a = (kept + 1) >> 1;
        len_b = kept >> 1;
    };

    for (int cb0 = 0; cb0 < steps; cb0 += LA) {
#pragma unroll
        for (int u = 0; u < LA; ++u) { cx[u] = nx[u]; cy[u] = ny[u]; }
#pragma unroll
        for (int u = 0; u < LA; ++u) fetch(cb0 + LA + u, nx[u], ny[u]);
        stage[sw * 32 + scol] = cx[0]; // (the round's first step; the last round's barrier has passed)
        stage[(sw + 8) * 32 + scol] = cy[0];
        lds_barrier();
#pragma unroll
        for (int u = 0; u < LA; ++u) {
            const int cb = cb0 + u;
            const u32x4_g *cur = stage + (size_t)(u & 1) * NC * 32;
            f32x16_g c = {0.f};
#pragma unroll
            for (int s = 0; s < STEPS; ++s) {
                const u32x4_g b = cur[(2 * s + half) * 32 + l32];
                c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_g, b), __builtin_bit_cast(bf16x8_g, a[s]), c, 0, 0, 0);
            }
            if (u + 1 < LA) { // the next step's keys go to the other half of the staging area
                u32x4_g *nxt = stage + (size_t)((u + 1) & 1) * NC * 32;
                nxt[sw * 32 + scol] = cx[u + 1 < LA ? u + 1 : 0];
                nxt[(sw + 8) * 32 + scol] = cy[u + 1 < LA ? u + 1 : 0];
            }
            // c[i]: the product of this lane's row with the step's column 8 (i / 4) + 4 (lane / 32) + i % 4.
            // Which of the 16 pass: compares only; the appends - rare once the bars have risen - are done in
            // a loop of their own, which most steps skip or leave after one turn.
            const int col0 = cb * 32 + 4 * half;
            uint32_t pass = 0u;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int col = col0 + 8 * (i >> 2) + (i & 3);
                pass |= (c[i] > bar && col < n && col != myrow ? 1u : 0u) << i;
            }
            if (myrow >= n) pass = 0u;
            while (__ballot(pass != 0u) != 0ull) {
                if (pass != 0u) {
                    const int i = __ffs(pass) - 1;
                    pass &= pass - 1u;
                    float ci = c[0];
#pragma unroll
                    for (int t = 1; t < 16; ++t) ci = i == t ? c[t] : ci;
                    mylist[cnt] = ((unsigned long long)ord_key(ci) << 32) | (0xFFFFFFFFu - (uint32_t)(col0 + 8 * (i >> 2) + (i & 3)));
                    ++cnt;
                }
            }
            // tidy the rows one of whose lists could not take another step (16 entries at most per list and step)
            unsigned long long full = __ballot(cnt > kKnnSub - 16);
            full = (full | (full >> 32)) & 0xFFFFFFFFull;
            while (full) {
                const int r = __ffsll((long long)full) - 1;
                full &= full - 1;
                int len_a, len_b;
                float new_bar;
                tidy(r, len_a, len_b, new_bar);
                if (l32 == r) {
                    cnt = half ? len_b : len_a;
                    bar = new_bar;
                }
            }
            lds_barrier(); // the next step's keys are staged; everyone is done with this step's
        }
    }
    // what is left: sort every row's two lists together and write the first M entries
    for (int r = 0; r < 32; ++r) {
        const int row = r0 + wave * 32 + r;
        if (row >= n) break;
        const int ca = __builtin_amdgcn_readlane(cnt, r), cb = __builtin_amdgcn_readlane(cnt, 32 + r);
        const unsigned long long *la = lists + (size_t)(wave * 32 + r) * 2 * kKnnSub;
        unsigned long long k0 = lane < ca ? la[lane] : 0ull, k1 = lane < cb ? la[kKnnSub + lane] : 0ull;
        sort128_desc(k0, k1, lane);
        if (lane < M) nbr[(size_t)row * M + lane] = k0 == 0ull ? -1 : (int32_t)(0xFFFFFFFFu - (uint32_t)(k0 & 0xFFFFFFFFull));
    }
}

hipError_t launch_graph_knn(const Shape &sh, const void *k_pool, const int32_t *pt_row, int n, int M, int32_t *nbr, hipStream_t st)
{
    if (sh.dtype != 0 || sh.head_dim != 128 || M < 1 || M > 64 || n < 1) return hipErrorInvalidValue;
    const size_t lds = (size_t)kKnnRows * 2 * kKnnSub * 8 + 2 * 16 * 32 * 16 + kKnnPtLds * 4;
    static bool prepared = false;
    if (!prepared) {
        const hipError_t e = hipFuncSetAttribute((const void *)knn_kernel<128>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        prepared = true;
    }
    knn_kernel<128><<<dim3((unsigned)((n + kKnnRows - 1) / kKnnRows), (unsigned)sh.n_kv_heads), dim3(256), lds, st>>>(
        (const uint4 *)k_pool, pt_row, sh.n_kv_heads, n, M, nbr);
    return hipGetLastError();
}

hipError_t launch_graph_norm(const Shape &sh, const void *k_pool, const int32_t *pt_row, int n, unsigned long long *best,
                             hipStream_t st)
{
    if (sh.dtype != 0 || sh.head_dim != 128) return hipErrorInvalidValue;
    const hipError_t e = launch_fill_u32((uint32_t *)best, 2 * (size_t)sh.n_kv_heads, 0u, st);
    if (e != hipSuccess) return e;
    const unsigned slices = (unsigned)std::max(1, std::min(256, n / 1024));
    norm_kernel<128><<<dim3((unsigned)sh.n_kv_heads, slices), dim3(256), 0, st>>>((const uint4 *)k_pool, pt_row, sh.n_kv_heads, n, best);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// DIPRS.  Grid: one 64-thread workgroup (one wavefront) per query head.
//   nbr       [H_kv][n_idx][M] neighbour lists (-1 = none)
//   k0s       [H_kv] entry point of each KV head's graph
//   clist     [H_q][cap] the list C as (score bits, token) pairs, in the order in which it grew
//   visited   [H_q][words] one bit per token, zero on entry; used only when the bits do not fit the LDS
//   Mp        M rounded up to a power of two: 64 / Mp entries of C are visited side by side
//   lds       how the workgroup's dynamic LDS is divided (DiprsLds, chosen by the launcher)
// The answer - the window's tokens, then every entry of C within beta of the best - goes to the
// selected-token arrays that the gather kernel reads.
//
// A visit is a chain of dependent reads (list entry -> neighbour list -> visited bits -> key rows), so the
// walk is bound by latency, and everything that can be kept close is: the visited bits, the sequence's row
// of the page table and the first tokens of C sit in LDS (as far as they fit: gfx950 has 160 KB), the
// neighbour lists of the next entries are fetched while this visit's keys are scored, and with M <= 32
// several consecutive entries of C are visited at once (lane = (entry, neighbour), which is the sequential
// order; a key that two of those entries share goes to the earlier one, as it would one after the other).
struct DiprsLds {
    int vis_words; // visited bits kept in LDS (0: in global memory)
    int pt_pages;  // page-table entries kept in LDS (0: read from global memory)
    int list;      // leading entries of C mirrored in LDS
};

template <int D>
__global__ __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(1, 2))) void diprs_kernel(const ReqDesc dsc, int H_q, int H_kv, const uint4 *__restrict__ k_pool,
                                                   const int32_t *__restrict__ page_table, const uint32_t *__restrict__ qw,
                                                   const int32_t *__restrict__ nbr, int n_idx, int M, int Mp,
                                                   const int32_t *__restrict__ k0s, int l0, float beta,
                                                   uint2 *clist, int64_t cap, uint32_t *visited,
                                                   int64_t vis_words, int32_t *__restrict__ sel_ids,
                                                   float *__restrict__ sel_scores, int32_t *__restrict__ sel_rows,
                                                   int32_t *__restrict__ counts, float *__restrict__ head_M,
                                                   int32_t *__restrict__ c_lens, int32_t *__restrict__ out_ids,
                                                   int32_t *__restrict__ out_counts, int64_t ids_stride,
                                                   int32_t *__restrict__ status, const DiprsLds lds)
{
    constexpr int NC = D / 8;
    extern __shared__ __attribute__((aligned(16))) uint32_t dyn_lds[];
    __shared__ __attribute__((aligned(16))) int32_t kk[64];
    uint32_t *vis_lds = dyn_lds;
    int32_t *pt_lds = (int32_t *)(dyn_lds + lds.vis_words);
    int32_t *c_lds = pt_lds + lds.pt_pages;
    const int kListLds = lds.list;
    const int h = blockIdx.x, lane = threadIdx.x;
    const int G = H_q / H_kv, kvh = h / G;
    const int32_t *pt_row = page_table + dsc.pt_off;
    const uint32_t *q = qw + (size_t)h * (D / 2);
    uint2 *C = clist + (size_t)h * cap;
    uint32_t *vis = visited + (size_t)h * vis_words;
    int32_t *ids = sel_ids + (size_t)dsc.score_off + (size_t)h * dsc.head_stride;
    float *ss = sel_scores + (size_t)dsc.score_off + (size_t)h * dsc.head_stride;
    int32_t *rows = sel_rows + (size_t)dsc.score_off + (size_t)h * dsc.head_stride;
    const int32_t *adj = nbr + (size_t)kvh * n_idx * M;
    const unsigned long long lt_mask = (1ull << lane) - 1ull;
    const bool lds_bits = lds.vis_words > 0, lds_pt = lds.pt_pages > 0; // (uniform)
    for (int i = lane; i < lds.vis_words; i += 64) vis_lds[i] = 0u;
    for (int i = lane; i < lds.pt_pages; i += 64) pt_lds[i] = pt_row[i];
    auto page_of = [&](int j) { return lds_pt ? pt_lds[j >> 6] : pt_row[j >> 6]; };

    // q . k_j in fp32: one fused multiply-add per channel, channels in order
    auto score = [&](int j) {
        // all sixteen loads of the key first (a barrier for the instruction scheduler keeps them together:
        // issued one by one, each behind the use of the one before, they cost sixteen memory latencies)
        uint4 w[NC];
        const uint4 *kp = k_pool + ((size_t)page_of(j) * H_kv + kvh) * (size_t)(NC * 64) + (j & 63);
#pragma unroll
        for (int c = 0; c < NC; ++c) w[c] = kp[(size_t)c * 64];
        __builtin_amdgcn_sched_barrier(0);
        float acc = 0.f;
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            const uint32_t kw[4] = {w[c].x, w[c].y, w[c].z, w[c].w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const uint32_t qq = q[c * 4 + e];
                acc = fmaf(bf16_lo(qq), bf16_lo(kw[e]), acc);
                acc = fmaf(bf16_hi(qq), bf16_hi(kw[e]), acc);
            }
        }
        return acc;
    };
    auto row_of = [&](int j) { return page_of(j) * kPageTokens + (j & 63); };
    auto wave_max = [&](float x) {
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) x = fmaxf(x, __shfl_xor(x, o));
        return x;
    };
    // The list and the global visited bits were written by this wavefront a moment ago (the bits with atomics
    // that are carried out in the L2): they are read back past the L1.
    auto c_token = [&](int i) {
        return i < kListLds ? c_lds[i]
                            : (int)(__hip_atomic_load((const unsigned long long *)&C[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >> 32);
    };
    auto seen = [&](int k) {
        const uint32_t w = lds_bits ? vis_lds[k >> 5] : __hip_atomic_load(&vis[k >> 5], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return (w & (1u << (k & 31))) != 0u;
    };
    auto mark = [&](int k) { // (tryAppend marks k as visited whether or not it appends it)
        if (lds_bits) atomicOr(&vis_lds[k >> 5], 1u << (k & 31));
        else atomicOr(&vis[k >> 5], 1u << (k & 31));
    };

    // The window (Sec. 7.1): always attended, seeds the best so far, takes no part in the walk.
    float best = -INFINITY;
    int n_sel = 0;
    for (int t0 = 0; t0 < dsc.nwin; t0 += 64) {
        const int t = t0 + lane;
        const bool on = t < dsc.nwin;
        const int j = t < dsc.w0 ? t : dsc.n - dsc.nwin + t; // first w0 tokens, then the last ones
        float s = -INFINITY;
        if (on) {
            s = score(j);
            ids[t] = j;
            ss[t] = s;
            rows[t] = row_of(j);
            if (out_ids && (int64_t)t < ids_stride) out_ids[(size_t)h * ids_stride + t] = j;
        }
        best = fmaxf(best, wave_max(s));
    }
    n_sel = dsc.nwin;

    // start key: the graph's entry point, or - if that is a window token - the first token behind the initial window
    int len = 0;
    int k0 = k0s[kvh];
    if (in_window(dsc, k0)) k0 = dsc.w0 < min(dsc.n - dsc.w1, n_idx) ? dsc.w0 : -1;
    if (k0 >= 0) {
        const float s0 = score(k0); // (every lane the same)
        if (lane == 0) {
            C[0] = make_uint2(__float_as_uint(s0), (uint32_t)k0);
            c_lds[0] = k0;
            mark(k0);
        }
        best = fmaxf(best, s0);
        len = 1;
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");

    const int E = 64 / Mp;                       // entries of C visited side by side
    const int ent = lane / Mp, t = lane % Mp;    // this lane's entry among them, and its neighbour
    auto neighbour = [&](int idx) { return adj[(size_t)c_token(idx) * M + t]; };
    int nb = ent < len && t < M ? neighbour(ent) : -1;
    int cnt = 0;
    for (int i = 0; i < len; i += cnt) { // len never exceeds the number of indexed tokens: every key enters C at most once
        const int len0 = len;
        cnt = min(E, len0 - i); // this round visits the entries i .. i + cnt - 1
        const int k = nb;
        // the neighbour lists of the entries after these, as far as the list is known already
        const int idx_next = i + cnt + ent;
        nb = idx_next < len0 && t < M ? neighbour(idx_next) : -1;
        bool fresh = k >= 0 && k < n_idx && !in_window(dsc, k);
        if (fresh) fresh = !seen(k);
        if (E > 1) { // a key shared with an earlier entry of this round is that entry's
            kk[lane] = fresh ? k : -1;
            const int lim = ent * Mp; // lanes below this one's entry
            bool dup = false;
            // (all sixteen 16-byte reads are issued at once: a loop of dependent LDS reads would cost more
            // than the round's memory latency)
            int4 v[16];
#pragma unroll
            for (int u = 0; u < 16; ++u) v[u] = ((const int4 *)kk)[u];
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int u = 0; u < 16; ++u) {
                dup |= (4 * u + 0 < lim && v[u].x == k) | (4 * u + 1 < lim && v[u].y == k) | (4 * u + 2 < lim && v[u].z == k) |
                       (4 * u + 3 < lim && v[u].w == k);
            }
            fresh = fresh && !dup;
        }
        if (fresh) mark(k);
        const float s = fresh ? score(k) : -INFINITY;
        const unsigned long long U = __ballot(fresh);
        if (U != 0ull) {
            // what the sequential order decides: the best inner product when this neighbour's turn comes ...
            float pm = s;
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                const float x = __shfl_up(pm, o);
                if (lane >= o) pm = fmaxf(pm, x);
            }
            float before = __shfl_up(pm, 1);
            before = lane == 0 ? best : fmaxf(best, before);
            // ... and whether the list is still at or under the capacity threshold
            const int r = __popcll(U & lt_mask);
            const bool app = fresh && (len + r <= l0 || s >= before - beta);
            const unsigned long long A = __ballot(app);
            const int at = len + __popcll(A & lt_mask);
            if (app && at < cap) { // (at < cap always: a key enters C once)
                C[at] = make_uint2(__float_as_uint(s), (uint32_t)k);
                if (at < kListLds) c_lds[at] = k;
            }
            len = min(len + __popcll(A), (int)cap);
            best = fmaxf(best, wave_max(app ? s : -INFINITY));
            // (entries beyond the LDS mirror are read back from global memory: their stores must have arrived)
            if (len > kListLds) __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
            // entries of the next round that this round appended
            if (idx_next >= len0 && idx_next < len && t < M) nb = neighbour(idx_next);
        }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
    // the answer: every c in C with q.c >= best - beta
    const float thr = best - beta;
    for (int i0 = 0; i0 < len; i0 += 64) {
        const int i = i0 + lane;
        const unsigned long long raw =
            i < len ? __hip_atomic_load((const unsigned long long *)&C[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0ull;
        const uint2 pr = make_uint2((uint32_t)raw, (uint32_t)(raw >> 32)); // .x = score bits (low word), .y = token
        const float s = __uint_as_float(pr.x);
        const bool take = i < len && s >= thr;
        const unsigned long long T = __ballot(take);
        if (take) {
            const int pos = n_sel + __popcll(T & lt_mask);
            ids[pos] = (int)pr.y;
            ss[pos] = s;
            rows[pos] = row_of((int)pr.y);
            if (out_ids && (int64_t)pos < ids_stride) out_ids[(size_t)h * ids_stride + pos] = (int)pr.y;
        }
        n_sel += __popcll(T);
    }
    if (lane == 0) {
        counts[h] = n_sel;
        head_M[h] = best;
        c_lens[h] = len;
        if (out_counts) out_counts[h] = n_sel;
        if (out_ids && (int64_t)n_sel > ids_stride) atomicOr(status, 1);
    }
}

hipError_t launch_diprs(const Shape &sh, const DeviceViews &dv, const void *q, const int32_t *nbr, int n_idx, int M,
                        const int32_t *k0s, int l0, float beta, uint2 *clist, int64_t cap, uint32_t *visited,
                        int64_t vis_words, int32_t *c_lens, int32_t *out_ids, int32_t *out_counts, int64_t ids_stride,
                        int lds_limit, hipStream_t st)
{
    if (sh.dtype != 0 || sh.head_dim != 128 || M < 1 || M > 64) return hipErrorInvalidValue;
    int Mp = 1;
    while (Mp < M) Mp <<= 1;
    // Divide the workgroup's LDS: the visited bits first, then the page-table row, the rest mirrors the list.
    static int max_lds = 0; // what a workgroup of this kernel may have, asked for once
    if (max_lds == 0) {
        int dev = 0, v = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&v, hipDeviceAttributeMaxSharedMemoryPerBlock, dev) != hipSuccess)
            v = 64 << 10;
        if (v > (64 << 10) &&
            hipFuncSetAttribute((const void *)diprs_kernel<128>, hipFuncAttributeMaxDynamicSharedMemorySize, v - 1024) != hipSuccess) {
            (void)hipGetLastError();
            v = 64 << 10;
        }
        max_lds = v;
    }
    int64_t budget = (lds_limit > 0 && lds_limit < max_lds ? lds_limit : max_lds) - 1024; // (the static part and slack)
    const ReqDesc &d = dv.desc.in;
    DiprsLds lds{0, 0, 0};
    const int64_t bits = ((int64_t)n_idx + 31) / 32 * 4;
    if (bits + 8192 <= budget) { lds.vis_words = (int)(bits / 4); budget -= bits; }
    if ((int64_t)d.n_pages * 4 + 4096 <= budget) { lds.pt_pages = d.n_pages; budget -= (int64_t)d.n_pages * 4; }
    lds.list = (int)std::min<int64_t>(budget / 4, (int64_t)n_idx + 1);
    if (lds.list < 1) lds.list = 1; // (entry 0 is always mirrored)
    const size_t dyn = ((size_t)lds.vis_words + lds.pt_pages + lds.list) * 4;
    if (lds.vis_words == 0) {
        const hipError_t e = launch_fill_u32(visited, (size_t)sh.n_q_heads * vis_words, 0u, st);
        if (e != hipSuccess) return e;
    }
    diprs_kernel<128><<<dim3((unsigned)sh.n_q_heads), dim3(64), dyn, st>>>(
        dv.desc.in, sh.n_q_heads, sh.n_kv_heads, (const uint4 *)dv.k_pool, dv.page_table, (const uint32_t *)q, nbr, n_idx, M, Mp,
        k0s, l0, beta, clist, cap, visited, vis_words, dv.sel_ids, dv.sel_scores, dv.sel_rows, dv.counts, dv.head_M, c_lens,
        out_ids, out_counts, ids_stride, dv.status, lds);
    return hipGetLastError();
}

} // namespace alaya
