// Internal declarations shared by the host side (api.hip) and the kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace alaya {

constexpr int kPageTokens = 64;      // one page == one wavefront of tokens
constexpr int kScoreWaves = 4;       // wavefronts per scoring workgroup
constexpr int kMaxPagesPerWave = 4;  // pages one wavefront of the main pass scores in a row, at most
constexpr int kSelectThreads = 1024;
constexpr int kAttendThreads = 256;
constexpr int kMaxSplits = 64;
constexpr int kSampScoresMinStride = 8; // sample strides from which the sample pass hands its scores to the main pass
constexpr int kHistBins = 2048;      // top 11 bits of the order-preserving score image
constexpr int kRepairGrid = 512;     // workgroups of the (normally idle) repair scoring pass, at most
constexpr int kMaxSlots = 64;        // addresses one head's sample-pass maxima are spread over
constexpr int kHeadStride = 512;     // 8-byte words of a block's dense part: its first kHeadStride survivors
constexpr int kSelBatch = 4096;      // survivor blocks whose prefix sums the selection holds in LDS at a time
constexpr int kMaxReqBlocks = 1 << 16; // survivor blocks of one request per KV head, at most

// Elements added to each head's row in the per-head arrays so that rows of different heads, touched
// at the same offset at the same time, do not all start on the same memory channel.
constexpr int kScorePad = 1088; // 17 * 256 bytes

// Per-request descriptor, built on the host for every attention call and copied to the device.
struct ReqDesc {
    int32_t pt_off;        // first entry of this sequence's row in the device page table
    int32_t n;             // tokens the query sees (the cached ones, or a prefix of them)
    int32_t head_stride;   // elements between consecutive heads in the selected-token arrays
    int32_t k;             // top-k: tokens to retrieve outside the window, already clamped (0 in DIPR mode)
    float beta;            // DIPR margin (raw inner-product units)
    int32_t tile_start;    // first sample-pass tile / full-attention tile of this request (prefix sum)
    int64_t score_off;     // offset (elements) of this request's block in the selected-token arrays
    int32_t n_pages;       // pages of this request
    int32_t tileb_start;   // first main-pass tile (= survivor block per KV head) of this request (prefix sum)
    int32_t ntiles_b;      // main-pass tiles of this request
    int32_t sample_stride; // S: the sample pass scores pages 0, S, 2S, ...; 1 = no sample, no pruning
    int32_t w0, w1;        // window: tokens j < w0 and j >= n - w1 are always selected
    int32_t nwin;          // tokens in the window: min(n, w0 + w1)
    int32_t k_est;         // top-k: rank in the sample that the ESTIMATED bound is read at; 0 = guaranteed bound only
    int32_t xf, xb;        // the sample pass also scores the pages [0, xf) and [xb, n_pages): DIPR with a window,
                           // whose tokens seed the maximum (Sec. 7.1); a decode step, whose newest token that
                           // pass writes.  Only the every-S-th pages enter top-k's histogram.
    int32_t hist_cap;      // top-k: what one sample-pass workgroup (four sampled pages) may add to one bucket, at most
    int32_t pm_stride;     // coarse index: bytes between the KV heads' rows of this request's page mask
    int64_t pm_off;        // coarse index: first byte of this request's page mask; without it: this request's first
                           // entry in the sample pass's score area (DeviceViews::samp), in pages
    int32_t flags;         // bit 0 (short_ok): top-k, fewer than k candidates is no failure, all of them are taken (coarse
                           // index without a bound); bits 8..: the request whose heads the i-th group of selection
                           // workgroups takes, this descriptor being the i-th (requests with the most to select go
                           // first, so that the chip's second round is short)
    int32_t est_cand;      // coarse index: tokens in the pages a head chose (64 P); > 0: the rank that the estimated bound is
                           // read at follows the share of them that the head's sample really holds
};
// (The descriptor of a one-request call travels in the kernel arguments, that is in scalar registers: at 104
// bytes instead of 96 the main scoring pass, which then kept its queries in scalar registers too, ran 15 to 25 %
// slower.  Keep it at 96.)
static_assert(sizeof(ReqDesc) == 96, "ReqDesc layout");

// How the kernels get at the request descriptors.  A call of one request carries its descriptor in
// the kernel arguments, which saves the host-to-device copy (a 4 us blit ahead of the first kernel of
// every step); calls of more requests read the copy in the scratch memory.  (One only: indexing an array
// in the arguments makes the compiler treat the descriptor as varying from lane to lane.)
constexpr int kInlineDescs = 1;
struct DescArgs { // host side: what the launchers hand to every kernel as (mem, in, n)
    const ReqDesc *mem; // device copy, [n]; valid when n > 1
    ReqDesc in;         // valid when n == 1
    int32_t n;          // requests in this call
};
struct Descs { // device side, built from those three kernel arguments
    const ReqDesc *__restrict__ mem;
    const ReqDesc &in;
    int n;
    __device__ __forceinline__ ReqDesc operator[](int r) const { return n == 1 ? in : mem[r]; }
};

// The decode step's append, carried out by the sample pass (alaya_decode_step): the wavefront that
// scores the page holding a request's newest token first writes that token's key and value rows.
struct FusedAppend {
    uint4 *k_pool, *v_pool; // the pools, writable
    const uint4 *k, *v;     // [B][H_kv][D] new rows; k == nullptr: nothing to append
};

// A window token is always selected, and top-k neither counts nor ranks it.
__device__ __forceinline__ bool in_window(const ReqDesc &d, int j) { return j < d.w0 || j >= d.n - d.w1; }

// Device views handed to the launchers.
// Where the survivor blocks lie.  One block per main-pass workgroup = (tile, KV head), block = tile * H_kv + kvh: the
// survivors of the tile as (score bits, token id) pairs, head after head of the group, each head's ascending by token,
// and a header {count, start} per head.
//   A block seldom holds more than a few hundred survivors but may hold every token it covers, and the blocks'
// writes, a KiB each, are mixed into the stream of key reads: they cost the less the closer together they land.  So
// every block has a dense part of kHeadStride words next to its neighbours', and the survivors beyond those, if any,
// go to a second area with room for the rest of a full block.  (Blocks of full size next to each other, 33 KiB
// apart, made the main pass of the batched workload 2 % slower.)
//   The headers lie apart, one row per query head with the tiles side by side: the selection reads the headers of
// one head's tiles, which this way are consecutive words (a header inside every block cost it one memory
// transaction per tile).
struct BlockArea {
    uint2 *hdrs;         // [query head = kvh * G + g][n_tiles]
    uint2 *head;         // [block][kHeadStride]
    uint2 *rest;         // [block][rest_stride]: the block's survivors from the kHeadStride-th on
    int64_t rest_stride; // 0 when no block can hold more than kHeadStride
    int64_t n_tiles;
#ifdef __HIPCC__
    __device__ __forceinline__ uint2 *hdr(int tile, int q_head) const { return hdrs + (size_t)q_head * (size_t)n_tiles + tile; }
    __device__ __forceinline__ uint2 *at(size_t block, int p) const
    {
        return p < kHeadStride ? head + block * (size_t)kHeadStride + p : rest + block * (size_t)rest_stride + (p - kHeadStride);
    }
#endif
};
// 8-byte words that n_tiles tiles of n_kv_heads blocks each, of at most `full` survivors for G heads, take
inline int64_t block_area_words(int64_t n_tiles, int n_kv_heads, int G, int64_t full)
{
    return n_tiles * n_kv_heads * (G + kHeadStride + (full > kHeadStride ? full - kHeadStride : 0));
}
inline BlockArea make_block_area(uint2 *mem, int64_t n_tiles, int n_kv_heads, int G, int64_t full)
{
    const int64_t n_blocks = n_tiles * n_kv_heads;
    uint2 *head = mem + n_blocks * G;
    return BlockArea{mem, head, head + n_blocks * kHeadStride, full > kHeadStride ? full - kHeadStride : 0, n_tiles};
}

struct DeviceViews {
    DescArgs desc;             // the call's request descriptors
    FusedAppend fused;         // set for the duration of a decode-step call, all null otherwise
    const int32_t *page_table; // [max_seqs][max_pages_per_seq]   (the cache's own memory)
    const void *k_pool;
    const void *v_pool;
    // Everything below lives in the scratch memory of the call.
    // Scoring output: the survivor blocks (see BlockArea).
    uint2 *blocks;             // the memory that the call's BlockArea is laid out in
    BlockArea area;            // of the call's token-level blocks
    // what attention reads: [head][head_stride] inside the request's block at score_off
    float *sel_scores;
    int32_t *sel_ids;
    int32_t *sel_rows;         // the same tokens as rows of the V pool: physical page * 64 + slot in the page
    uint32_t *hist;            // [max_batch * n_q_heads][kHistBins] bucket counts of the sample (top-k); zero between calls
    uint32_t *head_maxkey;     // [max_batch * n_q_heads] DIPR: running maximum (ordered key); zero between calls
    uint32_t *sample_max;      // [max_batch * n_q_heads][kMaxSlots] maxima of the sample pass (DIPR); zero between calls
    uint32_t *fail;            // [max_batch * n_q_heads] 1: the estimated bound lost tokens, repair this head; zero between calls
    uint32_t *any_fail;        // one word: some head of the call is marked
    uint32_t *tau;             // [max_batch * n_q_heads] the bound the main pass filters with (ordered key)
    uint32_t *tau_safe;        // [max_batch * n_q_heads] the guaranteed lower bound of the selection threshold
    float *head_M;             // [max_batch * n_q_heads]: maximum score over the selected set
    int32_t *counts;           // [max_batch * n_q_heads]: size of the selected set
    float *partials;           // attend / full-attention partial results
    int32_t *status;           // device status word
    uint32_t *repairs;         // heads that took the repair path since the counter was last read (inspection)
    const uint8_t *pmask;      // coarse index: one byte per (KV head, page), bit g = head g of the group chose the page
    // Scores of the sample pass's every-S-th pages (S >= kSampScoresMinStride, no coarse index), which the main pass
    // takes over instead of reading those pages' keys again: [entry][KV head][G][64] floats, entry = the request's
    // pm_off + page / S.
    float *samp;
};

struct Shape {
    int dtype;      // alaya_dtype
    int head_dim;
    int n_q_heads;
    int n_kv_heads;
};

#ifdef __HIPCC__
// Inclusive prefix sum over the 64 lanes of a wavefront with data-parallel-primitive moves (no trip through LDS,
// which is what a shuffle is on this chip): shifts by 1, 2, 4, 8 inside each row of 16 lanes - a lane without
// a source adds 0 - then the last lane of row 0 / 2 is added to row 1 / 3, then lane 31 to rows 2 and 3.
__device__ __forceinline__ int wave_scan(int v)
{
    v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, false); // row_shr:1
    v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, false); // row_shr:2
    v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, false); // row_shr:4
    v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xf, 0xf, false); // row_shr:8
    v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xa, 0xf, false); // row_bcast:15 into rows 1 and 3
    v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xc, 0xf, false); // row_bcast:31 into rows 2 and 3
    return v;
}
#endif

// Launchers (one per kernel family).  Each returns the hipError_t of its launch.
hipError_t launch_append(const Shape &sh, const int32_t *page_table_row, void *k_pool, void *v_pool,
                         const void *k, const void *v, int64_t n_old, int64_t t, hipStream_t st);

// one token for each of B sequences; dv.desc[b] holds the page-table row offset and the old length
hipError_t launch_append_step(const Shape &sh, const DeviceViews &dv, void *k_pool, void *v_pool, const void *k,
                              const void *v, int B, hipStream_t st);

// Sample pass: statistics of every S-th page (histogram for top-k, maximum for DIPR) and, in a decode
// step, the append of the newest token.  total_tiles may be 0 (nothing to launch).
// coarse: only the pages marked in dv.pmask are scored, and a head counts only tokens of pages it chose itself.
hipError_t launch_sample(const Shape &sh, const DeviceViews &dv, int B, const void *q, int total_tiles, int mode,
                         bool coarse, hipStream_t st);
// The bound of every head from the sample's statistics; mode: 0 top-k, 1 DIPR.
hipError_t launch_tau(const Shape &sh, const DeviceViews &dv, int B, int mode, hipStream_t st);
// Main pass: every page against dv.tau (repair = false), or - only for the workgroups with a head marked
// in dv.fail - against dv.tau_safe for the marked heads (repair = true).  cp = pages per wavefront.
// ev0 / ev1: optional events that take the kernel's own begin and end times.
// coarse: only the pages marked in dv.pmask (and those that hold window tokens) are read, and a head keeps
// only tokens of pages it chose itself.
hipError_t launch_score(const Shape &sh, const DeviceViews &dv, int B, const void *q, int total_tiles, int cp,
                        bool repair, int mode, bool coarse, hipStream_t st, hipEvent_t ev0 = nullptr,
                        hipEvent_t ev1 = nullptr);

// Selection: one workgroup per (request, head).  redo: only the heads marked in dv.fail (after the repair pass).
// What is selected from, and where the result goes, may differ from the views' own (the page level of the
// coarse index runs the same kernel over block scores).
struct SelectIO {
    DescArgs desc;          // descriptors of this level
    BlockArea area;         // survivor blocks
    int32_t *ids;           // selected ids, [head][head_stride] at score_off
    float *scores;          // their scores
    int32_t *rows;          // their V-pool rows, or null (not wanted)
    int32_t *counts;        // [request * head]
    float *head_M;          // [request * head]
    uint32_t *pmask;        // selection of pages: the page mask (cleared), where each head marks its pages; else null
};
hipError_t launch_select(const Shape &sh, const DeviceViews &dv, const SelectIO &io, int B, int mode, bool redo,
                         int batch_blocks, int32_t *out_ids, int32_t *out_counts, int64_t ids_stride, hipStream_t st);

// Coarse-grained index (coarse.hip).
hipError_t launch_reps_range(const Shape &sh, const int32_t *pt_row, const void *k_pool, void *rep_pool, int first,
                             int count, int64_t n_new, hipStream_t st);
hipError_t launch_reps_step(const Shape &sh, const DeviceViews &dv, void *rep_pool, int B, hipStream_t st);
hipError_t launch_coarse_score(const Shape &sh, const DeviceViews &dv, const DescArgs &pdesc, int B, const void *q,
                               const void *rep_pool, int total_tiles, const BlockArea &area, uint8_t *pmask, hipStream_t st);

hipError_t launch_attend(const Shape &sh, const DeviceViews &dv, int B, float scale, int splits, int min_splits,
                         hipStream_t st);

// partial layout: [slot][head_dim + 2] = {m (already times scale), l, acc[head_dim]}
// sparse: slot = (b * n_q_heads + h) * splits + s           (per_request_tiles == 0)
// full  : slot = (tile_start[b] + t) * n_q_heads + h        (per_request_tiles == 1)
// sparse: a head's first head_splits(count) slots hold partials, as in the attend pass (min_splits: the least
// number of splits | log2 of the rows per workgroup << 16)
hipError_t launch_combine(const Shape &sh, const DeviceViews &dv, int B, int splits, int min_splits,
                          int per_request_tiles, int pages_per_tile, float *out, hipStream_t st);

hipError_t launch_full_partial(const Shape &sh, const DeviceViews &dv, int B, const void *q, float scale,
                               int total_tiles, int pages_per_tile, hipStream_t st);

hipError_t launch_fill_u32(uint32_t *p, size_t n, uint32_t v, hipStream_t st);

// Fine-grained index and DIPRS (graph.hip).
hipError_t launch_graph_knn(const Shape &sh, const void *k_pool, const int32_t *pt_row, int n, int M, int32_t *nbr, hipStream_t st);
hipError_t launch_graph_norm(const Shape &sh, const void *k_pool, const int32_t *pt_row, int n, unsigned long long *best,
                             hipStream_t st);
hipError_t launch_diprs(const Shape &sh, const DeviceViews &dv, const void *q, const int32_t *nbr, int n_idx, int M,
                        const int32_t *k0s, int l0, float beta, uint2 *clist, int64_t cap, uint32_t *visited,
                        int64_t vis_words, int32_t *c_lens, int32_t *out_ids, int32_t *out_counts, int64_t ids_stride,
                        int lds_limit, hipStream_t st);

// Inspection (tests, measurement): the survivors' scores scattered into dense rows
// out[score_off + head * head_stride + token]; the number of survivors of the call added to *total.
hipError_t launch_debug_scatter(const Shape &sh, const DeviceViews &dv, int B, int total_tiles, float *out,
                                unsigned long long *total, hipStream_t st);

// ---- device helpers ---------------------------------------------------------------------------

// Order-preserving map float -> uint32 (larger float <=> larger unsigned).  0 is below every float.
__device__ __forceinline__ uint32_t ord_key(float x)
{
    uint32_t b = __float_as_uint(x);
    if (b == 0x80000000u) b = 0u; // -0 and +0 are one score
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}
__device__ __forceinline__ float ord_float(uint32_t k)
{
    uint32_t b = (k & 0x80000000u) ? (k & 0x7FFFFFFFu) : ~k;
    return __uint_as_float(b);
}

// 16-byte load of data that is read once: marked non-temporal so that the stream does not push the
// small, re-read structures (survivor blocks, page table, queries) out of the caches.  Measured on a
// 2 GiB key pool: 6.8 against 6.0 TB/s for the bare read stream.
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4_nt;
__device__ __forceinline__ uint4 load_stream(const uint4 *p)
{
    const u32x4_nt t = __builtin_nontemporal_load((const u32x4_nt *)p);
    return make_uint4(t.x, t.y, t.z, t.w);
}

} // namespace alaya
