// PriorFilter of Alg. 2 as one call: C_SA over the whole population, then the k best per subgraph.
//
// The same kernels as pruner_draft_score followed by pruner_topk, with one saving: when the population takes the
// selection's large route and the draft kernel runs at its full load width, the draft kernel counts the first
// selection digit of every score while it still holds the score in a register, and the selection skips its first
// pass over the score array.  The result is the same as that of the two separate calls, bit for bit.
#include "common.h"

namespace pruner {

size_t prior_filter_workspace_bytes(int64_t n, int32_t n_sg, int32_t k)
{
    return round_up(draft_workspace_bytes(n_sg), 256) + topk_workspace_bytes(n, n_sg, k);
}

}  // namespace pruner

using namespace pruner;

extern "C" int pruner_prior_filter(const pruner_subgraph* sg, int32_t n_sg, const int64_t* seg_off, const uint16_t* tiles,
                                   int64_t tiles_pitch, int32_t flags, int32_t k, float* score, int32_t* idx_out, float* val_out,
                                   void* workspace, size_t workspace_bytes, void* stream, void* scored_event)
{
    if (!sg || !seg_off || n_sg < 1 || n_sg > PRUNER_MAX_SUBGRAPHS) return PRUNER_EINVAL;
    if (!workspace || !aligned(workspace, 256)) return PRUNER_EWORKSPACE;
    const size_t draft_bytes = round_up(draft_workspace_bytes(n_sg), 256);
    if (workspace_bytes < draft_bytes) return PRUNER_EWORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    char* ws = static_cast<char*>(workspace);

    // every refusal happens before the first launch
    int rc0 = draft_check(sg, n_sg, seg_off, tiles, tiles_pitch, flags, score, nullptr, ws, draft_bytes);
    if (rc0) return rc0;
    if (!idx_out || !aligned(idx_out, 4) || (val_out && !aligned(val_out, 4))) return PRUNER_EINVAL;

    // The selection's tables are prepared first and travel with the draft tables in one launch, which also clears the
    // histograms the draft kernel adds to.
    TopkCtx ctx;
    Upload pending;
    int rc = topk_prepare(seg_off, n_sg, k, ws + draft_bytes, workspace_bytes - draft_bytes, st, &ctx, &pending);
    if (rc) return rc;
    bool counted = false;
    rc = draft_launch(sg, n_sg, seg_off, tiles, tiles_pitch, flags, score, nullptr, ws, draft_bytes, st,
                      ctx.large ? ctx.d_hist : nullptr, ctx.large ? ctx.d_block_max : nullptr, ctx.copies, &counted, &pending);
    if (rc) return rc;
    if (scored_event && hipEventRecord(static_cast<hipEvent_t>(scored_event), st) != hipSuccess) return PRUNER_EHIP;
    return topk_finish(ctx, score, seg_off, idx_out, val_out, ctx.large && counted, st);
}
