// The rule-based query optimizer (Sec. 6.2 "Query Optimizer", the workflow of its figure): host code only.
#include "../../include/alaya.h"

extern "C" int alaya_plan_query(const alaya_plan_input *in, alaya_plan *out)
{
    if (!in || !out) return ALAYA_E_INVAL;
    if (in->context_len <= 0 || in->short_context < 0 || in->reused_prefix < 0 || in->gpu_budget_bytes < 0 ||
        in->coarse_bytes < 0 || in->layer_id < 0)
        return ALAYA_E_INVAL;
    out->n_visible = in->context_len;
    // 1. the context length: short contexts are attended in full
    if (in->context_len <= in->short_context) {
        out->query = ALAYA_QUERY_FULL;
        out->index = ALAYA_INDEX_NONE;
        return ALAYA_OK;
    }
    // 2. partial reuse of a stored context: a filter predicate on the token position
    if (in->reused_prefix > 0 && in->reused_prefix < in->context_len) out->n_visible = in->reused_prefix;
    // 3. the GPU memory budget: if the blocks fit, top-k on the coarse-grained index
    if (in->gpu_budget_bytes >= in->coarse_bytes) {
        out->query = ALAYA_QUERY_TOPK;
        out->index = ALAYA_INDEX_COARSE;
        return ALAYA_OK;
    }
    // 4. otherwise DIPR; the first layer needs many tokens and scans, the others walk the graph
    out->query = ALAYA_QUERY_DIPR;
    out->index = in->layer_id == 0 ? ALAYA_INDEX_FLAT : ALAYA_INDEX_FINE;
    return ALAYA_OK;
}
