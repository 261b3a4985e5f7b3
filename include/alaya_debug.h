/*
 * alaya_debug.h - measurement, tuning and inspection hooks of the MI355X sparse-attention library.
 *
 * None of these is part of the paper-defined interface (include/alaya.h); they exist for the tests,
 * for bench.py and for launch-shape sweeps.  Same conventions as alaya.h.
 */
#ifndef ALAYA_DEBUG_H
#define ALAYA_DEBUG_H

#include "alaya.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Kernel timing with HIP events recorded on the call's own stream.
 * alaya_set_profiling(c, 1) makes every later call bracket each of its kernels with events;
 * alaya_kernel_times synchronises them and returns, per kernel slot, the summed duration in
 * milliseconds and the number of launches since profiling was (re)enabled.
 * Slots: 0 score (the main scoring pass; its events are attached to the kernel's dispatch, so the
 * figure is the kernel's own run time), 1 select (the selection kernel and, for calls with an
 * estimated bound, the two repair launches), 2 attend, 3 combine, 4 full-attention partial, 5 append
 * (the append kernel; an alaya_decode_step has none: its sample pass writes the new rows), 6 sample
 * (statistics of the sampled pages + the threshold bound), 7 coarse (calls through the coarse index:
 * block scores, selection of the pages, page mask).  Slots other than 0 span from an event
 * before their first launch to one after their last, dispatch gaps included.
 * sum_ms, launches: HOST arrays of n_slots entries (n_slots <= ALAYA_N_KERNEL_SLOTS).
 */
#define ALAYA_N_KERNEL_SLOTS 8
int alaya_set_profiling(alaya_cache *c, int enabled);
int alaya_kernel_times(alaya_cache *c, double *sum_ms, int64_t *launches, int n_slots);

/* Launch-shape knobs for measurement sweeps and tests; each <= 0 keeps the built-in choice.
 * score_pages_per_wave: pages one wavefront scores in a row in the main scoring pass (1..16; rounded
 * down to a power of two that the kernel is built for: at most 4, at most 16 / G).
 * attend_splits: workgroups that share one head's selected set (1..64).
 * select_batch_blocks: survivor blocks whose prefix sums the selection holds at a time (1..4096;
 * small values drive the multi-batch path on small inputs).
 * write_all_scores: 1 makes the scoring pass keep every score instead of only those that can still
 * be selected (results are identical either way; it exists so that tests can read all scores). */
int alaya_set_tuning(alaya_cache *c, int score_pages_per_wave, int attend_splits, int select_batch_blocks,
                     int write_all_scores);

/* Test hook for the estimated threshold bound of top-k calls (k >= 512 on 64 pages or more).  Such
 * calls filter the main scoring pass with a bound that is only very likely to be low enough, check it
 * afterwards against the number of tokens that survived, and repair the heads where it was not
 * (results are exact either way).  mode 0, 1: estimate whenever the shapes allow (default);
 * 2: with an estimate so high that every head needs the repair; -1: never estimate. */
int alaya_debug_estimate(alaya_cache *c, int mode);

/* Inspection hook: synchronises `stream` and returns how many (token, score) pairs the main scoring
 * pass of the last alaya_sparse_attn / alaya_decode_step call kept, summed over requests and heads;
 * -1 on error.  With out != NULL (DEVICE) it also scatters their fp32 scores into dense rows: requests
 * follow each other, each block being n_q_heads rows of (n rounded up to a whole page + ALAYA_SCORE_PAD)
 * floats; the score of token j of head h is element j of row h; elements of tokens that were not kept
 * are left as they are.  Valid until the next call on the cache or on its scratch memory. */
#define ALAYA_SCORE_PAD 1088
int64_t alaya_debug_scores(alaya_cache *c, float *out, void *stream);

/* Inspection hook: synchronises `stream` and returns how many (request, head) selections took the repair path
 * of the estimated bound since the counter was last read (it lives in the scratch memory), then clears it;
 * -1 on error. */
int64_t alaya_debug_repairs(alaya_cache *c, void *stream);

/* Test hook: the walk of alaya_diprs_attn keeps its visited bits, the page-table row and the head of the list C
 * in on-chip memory as far as they fit; `bytes` > 0 lowers what it may use (so that small tests reach the
 * paths that large contexts take), 0 restores the default.  Results do not depend on it. */
int alaya_debug_diprs_lds(alaya_cache *c, int bytes);

/* Inspection hook: the list C that the last alaya_diprs_attn call grew for query head `head`, in the order in
 * which it grew: synchronises `stream`, copies the first min(length, cap) tokens to ids (HOST, optional) and
 * returns the length; -1 on error.  Valid until the next call on the cache or its scratch memory. */
int64_t alaya_debug_diprs_list(alaya_cache *c, int head, int32_t *ids, int64_t cap, void *stream);

/* How the last alaya_sparse_attn call split its pages (one page = 64 tokens of one sequence, scored
 * for every KV head): *sampled pages were scored by the sample pass for the threshold bound,
 * *main_pass pages whose keys the main scoring kernel read (all but those of the sample pass whose scores that pass
 * handed over).  HOST pointers. */
int alaya_debug_pages(const alaya_cache *c, int64_t *sampled, int64_t *main_pass);

#ifdef __cplusplus
}
#endif
#endif /* ALAYA_DEBUG_H */
