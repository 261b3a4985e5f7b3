/*
 * alaya.h - C ABI of the MI355X sparse-attention decode library.
 *
 * One alaya_cache is ONE transformer layer's paged key/value store in HBM,
 * holding many sequences.  Per decode step the caller appends the new token's
 * key and value (the paper's Session.update, Sec. 5 "User Interface", Table 2)
 * and then asks for attention of the new query against everything cached (the
 * paper's Session.attention): score every cached key, select the critical
 * tokens, and take the softmax-weighted sum of their values.
 *
 *   scores      s[h][j] = q_h . k_{h/G, j}         raw inner product, no 1/sqrt(d)  (Eq. 1; Def. 2)
 *   top-k       the min(k, n) tokens with the largest s[h][.]                        (Sec. 6.1.1)
 *   DIPR        every j with s[h][j] >= max_j s[h][j] - beta,  beta >= 0            (Def. 2, Def. 3)
 *   attention   softmax of s * scale over the SELECTED tokens, times their values   (Eq. 1, Sec. 2
 *               "Sparse Attention"; partial results merged by running max / sum,
 *               Sec. 7.2 "Data-centric Attention Engine")
 *   GQA         query head h reads key/value head h / G, G = n_q_heads / n_kv_heads (Sec. 7.2)
 *
 * Conventions
 *   - Every pointer is tagged HOST or DEVICE below.  The library never allocates
 *     or frees device memory: pools, page-table workspace and scratch are the caller's,
 *     and stay the caller's.  It keeps a few KB of pinned host memory per cache for descriptors.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls are
 *     asynchronous on it.  All calls on one cache must use one stream at a time; the
 *     handle is not thread-safe; distinct caches are independent.
 *   - Every function returns an alaya_status (or a size / length).  Errors that the
 *     host can see (bad handle, shapes, k <= 0, beta < 0 or NaN, empty sequence, pool
 *     exhausted) are returned BEFORE anything is launched and leave the cache unchanged.
 *     alaya_last_error() gives a thread-local message for the last failure.
 *   - Only head_dim 64 or 128, page_tokens 64 and G in {1, 2, 4, 8} are built.
 *   - NaN or Inf in keys, values or queries is undefined behaviour of the arithmetic
 *     (never of memory safety).
 */
#ifndef ALAYA_H
#define ALAYA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct alaya_cache alaya_cache; /* opaque host-side handle */

typedef enum { ALAYA_BF16 = 0, ALAYA_F32 = 1 } alaya_dtype;
typedef enum { ALAYA_TOPK = 0, ALAYA_DIPR = 1 } alaya_mode;

typedef enum {
    ALAYA_OK = 0,
    ALAYA_E_INVAL = -1,    /* bad argument */
    ALAYA_E_NOMEM = -2,    /* page pool or workspace too small */
    ALAYA_E_CAPACITY = -3, /* a selected set was larger than the caller's id buffer */
    ALAYA_E_EMPTY = -4,    /* a sequence in the call holds no tokens */
    ALAYA_E_DEVICE = -5    /* a HIP call failed */
} alaya_status;

/*
 * Shape of one cache.  Storage layout inside the pools (both are
 * n_phys_pages * n_kv_heads * 64 * head_dim elements of `dtype`):
 *   V pool  [phys_page][kv_head][token_in_page (64)][head_dim]                row-major rows
 *   K pool  [phys_page][kv_head][head_dim / E][token_in_page (64)][E]         E = 16 bytes of elements
 *           (8 for bf16, 4 for fp32): the 64 tokens of a page are adjacent for each 16-byte slice
 *           of the head dimension, so that one wavefront (lane = token) reads every slice of a
 *           page as one contiguous 1 KiB run.
 * Only alaya_append_kv writes the pools; callers treat them as raw memory.
 */
typedef struct {
    int32_t n_q_heads;          /* query heads per attention call                          */
    int32_t n_kv_heads;         /* key/value heads; n_q_heads % n_kv_heads == 0            */
    int32_t head_dim;           /* 64 or 128                                               */
    int32_t page_tokens;        /* 64                                                      */
    int32_t dtype;              /* alaya_dtype of K, V and q                               */
    int32_t max_seqs;           /* sequences the cache can hold (ids 0 .. max_seqs-1)      */
    int32_t max_batch;          /* requests in one attention call                          */
    int32_t reserved;           /* 0                                                       */
    int64_t max_tokens_per_seq; /* longest sequence                                        */
    int64_t max_batch_tokens;   /* largest sum of sequence lengths in one attention call   */
    int64_t n_phys_pages;       /* pages in each pool                                      */
} alaya_cache_config;

/* Bytes of ONE pool (K or V) / of the cache's workspace (its page table) / of the scratch memory an
 * attention call needs for this configuration; 0 if cfg is invalid. */
size_t alaya_pool_bytes(const alaya_cache_config *cfg);
size_t alaya_workspace_bytes(const alaya_cache_config *cfg);
size_t alaya_scratch_bytes(const alaya_cache_config *cfg);

/*
 * Create a cache over caller-owned DEVICE memory: k_pool, v_pool (alaya_pool_bytes each) and
 * workspace (>= alaya_workspace_bytes, 256-byte aligned; holds the page table - its contents are
 * the library's while the cache lives).
 * phys_page_order: HOST, optional, n_phys_pages distinct page numbers - the order in which
 * physical pages are handed to growing sequences (NULL = 0, 1, 2, ...).  Copied.
 * No device work happens here.
 */
int alaya_create_cache(alaya_cache **out, const alaya_cache_config *cfg, void *k_pool, void *v_pool,
                       const int32_t *phys_page_order, void *workspace, size_t workspace_bytes);
int alaya_destroy_cache(alaya_cache *c);

/*
 * Scratch memory for the attention calls of this cache (and for alaya_append_kv_step / alaya_decode_step
 * of more than one sequence): DEVICE, >= alaya_scratch_bytes(cfg of the cache), 256-byte aligned.  It
 * holds the survivors of the scoring pass, the selected tokens and the partial results of ONE call;
 * nothing in it has to outlive a call.  One cache is one layer (Sec. 2: a key/value cache per layer), and
 * a model runs its layers one after the other, so SEVERAL CACHES MAY BIND THE SAME SCRATCH MEMORY as long
 * as their calls are ordered on one stream - a 32-layer model then holds one scratch area, not 32.  The
 * first call of each cache after binding clears the few words that must start at zero; calls leave them
 * zero.  scratch = NULL unbinds.  alaya_poll_status reads a status word that lives in the scratch memory:
 * caches that share it share the word.
 */
int alaya_bind_scratch(alaya_cache *c, void *scratch, size_t scratch_bytes);

/*
 * The coarse-grained index (Sec. 6.2 "Query Optimizer", index types; Table 4): every page of 64 adjacent
 * tokens is represented, per KV head, by two vectors - the channel-wise minimum and maximum of its keys.
 * rep_pool: DEVICE, >= alaya_rep_bytes(cfg), 256-byte aligned, laid out [phys_page][kv_head][2][head_dim]
 * in the cache dtype; the library's while the cache lives.  Bind it while every sequence is empty: from
 * then on each append also brings the representatives of the pages it touches up to date, and
 * alaya_sparse_attn accepts coarse_pages.  A cache without it answers exact queries only.
 */
size_t alaya_rep_bytes(const alaya_cache_config *cfg);
int alaya_bind_reps(alaya_cache *c, void *rep_pool, size_t rep_bytes);

/*
 * Session.update: append t tokens to sequence `seq`.
 * k, v: DEVICE, [t][n_kv_heads][head_dim] of the cache dtype (token-major, as a model emits them).
 * Pages are taken from the pool as needed; if it runs out: ALAYA_E_NOMEM and nothing changes.
 * A token appended here is visible to every later attention call on the same stream
 * (update, then attention on the whole cache: Sec. 5 "User Interface").
 */
int alaya_append_kv(alaya_cache *c, int seq, const void *k, const void *v, int64_t t, void *stream);

/*
 * Session.update for one decode step of a batch: appends ONE token to each of the B listed
 * sequences with a single launch.
 * seqs: HOST [B], distinct.  k, v: DEVICE, [B][n_kv_heads][head_dim] of the cache dtype; row b
 * goes to sequence seqs[b].  Either every listed sequence grows by one token or, on an error
 * (ALAYA_E_INVAL for a bad or repeated id, ALAYA_E_NOMEM when a length limit or the page pool is
 * hit), none does.
 */
int alaya_append_kv_step(alaya_cache *c, const int32_t *seqs, int B, const void *k, const void *v, void *stream);

/* Tokens cached for seq (host bookkeeping, includes appends still in flight); -1 on a bad argument. */
int64_t alaya_seq_len(const alaya_cache *c, int seq);

/* Forget seq and return its pages to the pool (host bookkeeping only; the caller must make
 * sure no launched work still reads the sequence). */
int alaya_reset_seq(alaya_cache *c, int seq);

typedef struct {
    int32_t mode;          /* alaya_mode                                                        */
    int32_t window_init;   /* >= 0: the first window_init visible tokens are always attended    */
    const int32_t *topk;   /* HOST [B], ALAYA_TOPK: per-request k > 0 (k > n means all n)       */
    const float *beta;     /* HOST [B], ALAYA_DIPR: per-request beta >= 0, +inf allowed         */
    float scale;           /* softmax scale; 0 means 1 / sqrt(head_dim)                         */
    int32_t window_last;   /* >= 0: the last window_last visible tokens are always attended     */
    int32_t *out_ids;      /* DEVICE, optional [B][n_q_heads][ids_stride]: selected token ids   */
    int32_t *out_counts;   /* DEVICE, optional [B][n_q_heads]: TRUE size of each selected set   */
    int64_t ids_stride;    /* capacity per head of out_ids                                      */
    const int32_t *n_visible; /* HOST [B], optional: request b sees only its first n_visible[b]
                                 cached tokens (1 .. cached length); NULL = all of them         */
    const int32_t *coarse_pages; /* HOST [B], optional, ALAYA_TOPK only: answer through the coarse index -
                                 request b's query runs over the tokens of its coarse_pages[b] >= 1
                                 best pages only (see alaya_bind_reps); NULL = the exact query   */
    int32_t *out_pages;    /* DEVICE, optional [B][n_q_heads][pages_stride]: the chosen pages    */
    int64_t pages_stride;  /* capacity per head of out_pages                                     */
} alaya_sparse_params;

/*
 * Session.attention, sparse: for each request b (sequence seqs[b]) and each query head, score all
 * cached keys, select (top-k or DIPR), and attend over the selected tokens.
 *   seqs  HOST [B], distinct or repeated sequence ids      q    DEVICE [B][n_q_heads][head_dim], cache dtype
 *   out   DEVICE [B][n_q_heads][head_dim], fp32
 * Window (Sec. 7.1 "Window Caching Enhanced DIPR"; Table 3 counts "[initial + last] + retrieved"
 * tokens): with window_init / window_last set, those tokens are always in the selected set; top-k
 * retrieves its k tokens among the OTHER tokens (k more than there are means all of them); DIPR keeps
 * the others that are within beta of the maximum over all visible tokens, the window's included.
 * out_ids / out_counts cover window and retrieved tokens alike.
 * Prefix (Sec. 7.1 "Flexible Context Reuse"): with n_visible set, the query runs as if the sequence
 * ended after n_visible[b] tokens; "last" window tokens are then the last visible ones.
 * Coarse index (Sec. 6.2; Table 4: top-k and filter queries): with coarse_pages set, each query head first
 * scores every page by u = sum_c max(q_c * lo_c, q_c * hi_c) over the page's two representative vectors - an
 * upper bound of every inner product in the page -, keeps the coarse_pages[b] pages with the largest u (equal
 * u: the smaller page) and runs the top-k query over their tokens only (k larger than they hold means all of
 * them; window tokens are attended wherever they are).  Only those pages' keys are read.  With n_visible the
 * pages that hold a visible token take part, each with the representatives of all its cached tokens.
 * A request may see at most 131072 pages (8388608 tokens); a longer one is refused with
 * ALAYA_E_INVAL (alaya_full_attn has no such limit).
 * Selection runs on raw fp32 inner products (bf16 products are exact in fp32; accumulation is fp32).
 * Among equal scores at the k-th place the smaller token id is taken, so results are reproducible.
 * out_ids come back in an unspecified but deterministic order.  If a set is larger than ids_stride
 * the first ids_stride ids are written, out_counts still holds the true size, the attention output
 * is still over the whole set, and alaya_poll_status reports ALAYA_E_CAPACITY after the stream syncs.
 */
int alaya_sparse_attn(alaya_cache *c, const int32_t *seqs, int B, int n_q_heads, const void *q,
                      const alaya_sparse_params *p, float *out, void *stream);

/*
 * One decode step of one layer (Sec. 5 "User Interface": Session.update, then Session.attention):
 * appends ONE token to each of the B listed sequences and runs alaya_sparse_attn over the grown
 * sequences.  Results are those of alaya_append_kv_step(seqs, k, v) followed by
 * alaya_sparse_attn(seqs, q, p, out); the difference is one launch less: the first scoring kernel
 * writes the new key and value rows itself.
 *   seqs  HOST [B], distinct          k, v  DEVICE [B][n_kv_heads][head_dim], cache dtype
 *   q, p, out: as for alaya_sparse_attn (with p->n_visible set the two calls are simply made in turn)
 * Errors: if the append is refused (bad or repeated id, a length limit, the page pool: see
 * alaya_append_kv_step) nothing changes.  If only the attention part is refused (its arguments, its
 * workspace), the tokens HAVE been appended, as after the two separate calls.
 */
int alaya_decode_step(alaya_cache *c, const int32_t *seqs, int B, int n_q_heads, const void *k, const void *v,
                      const void *q, const alaya_sparse_params *p, float *out, void *stream);

/*
 * alaya_sparse_attn for callers that cannot allocate device memory or bind any (code under HIP graph
 * capture set-up, tight serving loops, harnesses that forbid hipMalloc): same arguments, same results,
 * but the scratch memory of the call is an array of ALAYA_STATIC_SCRATCH_BYTES that the library holds
 * itself on each GPU it runs on (in its device image, until the process ends); the cache needs no
 * alaya_bind_scratch.  The call allocates nothing, on the host's device side or through any library.
 * Limit: the call's scratch need - about 16 bytes per (query head, token the call sees) plus 0.6 MB per
 * request - must fit the array (32 query heads: about 160 thousand tokens in one call); a larger call
 * is refused with ALAYA_E_NOMEM and nothing is launched.  Every call on a GPU, from any cache, uses that
 * GPU's one array: calls that overlap in time on one GPU race, so order them on one stream.  The array
 * keeps the last call's contents; each call clears the words that must start at zero.
 * alaya_poll_status does not see this call's status word; ask for out_counts to detect an id overflow.
 */
#define ALAYA_STATIC_SCRATCH_BYTES (80u << 20)
int alaya_sparse_attn_static(alaya_cache *c, const int32_t *seqs, int B, int n_q_heads, const void *q,
                             const alaya_sparse_params *p, float *out, void *stream);

/*
 * The fine-grained index (Sec. 6.2 "Query Optimizer", index types: a graph over the key vectors) and the
 * approximate DIPR query on it, DIPRS (Sec. 6.1.3 "DIPR Query Processing", Algorithm 1).
 *
 * alaya_graph_build indexes the tokens that sequence `seq` holds now: for every KV head the exact
 * degree-nearest-neighbour graph of its keys under the inner product (best neighbour first; equal products:
 * smaller token), shared by the query heads of the group (Sec. 7.2 "GQA-based index sharing"), and as entry
 * point the key of largest norm.  (The paper builds RoarGraph; Algorithm 1 runs on any graph index.)
 * bf16 caches of head_dim 128, degree 1..64.  index_mem (>= alaya_graph_bytes) holds the graph and stays
 * the library's while the handle lives; build_mem (>= alaya_graph_build_bytes, a few hundred bytes today:
 * the builder keeps its working lists on chip) is scratch for the build only.
 * Both DEVICE, 256-byte aligned.  The call synchronises `stream` before it returns.
 *
 * alaya_diprs_attn runs Algorithm 1 for every query head on its KV head's graph - start key = the entry
 * point, capacity threshold l0, margin beta - in the paper's order, and attends over the answer: every key of
 * the list C whose inner product is within beta of the best one met.  Inner products are fp32, one fused
 * multiply-add per channel in channel order (the answer depends on comparisons of them).
 *   q, out              as for alaya_sparse_attn with B = 1 (the graph's sequence)
 *   p                   optional: window_init / window_last (Sec. 7.1 "Window Caching Enhanced DIPR": the
 *                       window's tokens are always attended, take no part in the walk, and their best inner
 *                       product seeds the walk's threshold), scale, out_ids / out_counts / ids_stride;
 *                       the other fields are ignored
 * Tokens appended after the build are not in the graph (Sec. 7.2 "Late Materialization for Index
 * Updating"): they are treated as part of the window of last tokens.
 */
typedef struct alaya_graph alaya_graph;
size_t alaya_graph_bytes(const alaya_cache *c, int seq, int degree);
size_t alaya_graph_build_bytes(const alaya_cache *c, int seq, int degree);
int alaya_graph_build(alaya_graph **out, alaya_cache *c, int seq, int degree, void *index_mem, size_t index_bytes,
                      void *build_mem, size_t build_bytes, void *stream);
int alaya_graph_destroy(alaya_graph *g);
/* n_indexed, degree: HOST, optional; neighbours: DEVICE pointer to [n_kv_heads][n_indexed][degree] int32
 * (-1 = none), optional; entry: HOST [n_kv_heads], optional. */
int alaya_graph_info(const alaya_graph *g, int64_t *n_indexed, int32_t *degree, const int32_t **neighbours,
                     int32_t *entry);
int alaya_diprs_attn(alaya_cache *c, const alaya_graph *g, int n_q_heads, const void *q, float beta, int32_t l0,
                     const alaya_sparse_params *p, float *out, void *stream);

/*
 * The rule-based query optimizer (Sec. 6.2 "Query Optimizer", the workflow of its figure): which query type
 * on which index type answers one layer's attention query.  Host code, no GPU work, no state.  The rules, in
 * the paper's order:
 *   1. context_len <= short_context                 -> full attention, no index
 *   2. 0 < reused_prefix < context_len              -> the query carries the filter predicate
 *                                                      "token position < reused_prefix" (n_visible)
 *   3. gpu_budget_bytes >= coarse_bytes             -> top-k on the coarse-grained index
 *   4. otherwise DIPR: the flat index (a scan) for layer 0, the fine-grained index (DIPRS on the graph) for
 *      every other layer
 * The paper fixes neither the short-context length nor what the coarse index needs on the GPU: both are the
 * caller's (coarse_bytes = what keeping the blocks and their representatives on the GPU takes: for this
 * library alaya_pool_bytes twice plus alaya_rep_bytes).  out->n_visible = context_len when no filter applies.
 * Returns ALAYA_E_INVAL for null pointers, context_len <= 0 or a negative field.
 */
enum { ALAYA_QUERY_FULL = 0, ALAYA_QUERY_TOPK = 1, ALAYA_QUERY_DIPR = 2 };
enum { ALAYA_INDEX_NONE = 0, ALAYA_INDEX_COARSE = 1, ALAYA_INDEX_FLAT = 2, ALAYA_INDEX_FINE = 3 };
typedef struct alaya_plan_input {
    int64_t context_len;      /* tokens of the stored context */
    int64_t short_context;    /* contexts up to this length are attended in full */
    int64_t reused_prefix;    /* tokens of the context that this request reuses; 0 or >= context_len: all */
    int64_t gpu_budget_bytes; /* GPU memory the session may use */
    int64_t coarse_bytes;     /* GPU memory the coarse-grained plan needs */
    int32_t layer_id;         /* 0 = the first layer */
    int32_t reserved;
} alaya_plan_input;
typedef struct alaya_plan {
    int32_t query; /* ALAYA_QUERY_* */
    int32_t index; /* ALAYA_INDEX_* */
    int64_t n_visible;
} alaya_plan;
int alaya_plan_query(const alaya_plan_input *in, alaya_plan *out);

/* Session.attention, dense: Eq. (1) over every cached token (same q / out layout as above). */
int alaya_full_attn(alaya_cache *c, const int32_t *seqs, int B, int n_q_heads, const void *q,
                    float scale, float *out, void *stream);

/* Synchronises `stream`, then returns and clears the device-side status word of the cache:
 * ALAYA_OK or ALAYA_E_CAPACITY (or ALAYA_E_DEVICE if the sync fails). */
int alaya_poll_status(alaya_cache *c, void *stream);

/* Thread-local description of the last error returned on this thread ("" if none). */
const char *alaya_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* ALAYA_H */
