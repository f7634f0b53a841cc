// d3tom_merge_layer: the whole merge layer of one denoising step in one call (Algorithm 1, the block guarded
// by "l = l* and the decider set is not empty": importance map, TopK at the step's keep ratio, cosine
// assignment, aggregation and removal), with the kept counts computed on the device from per-sample keep
// ratios, so that no host integer sits between the importance map and the merge.  Host-side sequencing of
// the same kernels the four separate entry points launch, sharing one workspace.
#include "internal.hpp"

namespace d3tom {
struct LayerWs { size_t imp, merge, slot, total; };
static LayerWs layer_ws_layout(int B, int max_N, int max_V, int H, int dh, int max_D) {
    LayerWs w;
    size_t o = 0;
    auto take = [&](size_t bytes) { const size_t at = o; o += align_up(bytes, 256); return at; };
    w.imp = take(importance_ws_bytes(B, max_N, max_V, H, dh, max_D));
    w.merge = take(merge_ws_bytes(B, max_V));
    w.slot = take((size_t)B * max_V * 4);
    w.total = o;
    return w;
}
}  // namespace d3tom

using namespace d3tom;

extern "C" size_t d3tom_merge_layer_workspace_bytes(int B, int max_N, int max_V, int H, int dh, int max_D) {
    if (B < 1 || max_N < 1 || max_V < 1 || H < 1 || dh < 1 || max_D < 1) return 0;
    return layer_ws_layout(B, max_N, max_V, H, dh, max_D).total;
}

extern "C" int d3tom_merge_layer(const void* q, const void* k, const void* x, const void* sim, int d, int d_sim, int dt,
                                 int B, const int32_t* seq_off, int H, int dh, float scale,
                                 const int32_t* dec_idx, const int32_t* dec_off, int min_D, int max_D,
                                 const int32_t* vis_start, const int32_t* vis_count, const int32_t* vis_off,
                                 const double* keep_ratio, int max_N, int max_V, int min_keep, int max_keep, int mode,
                                 float* scores, int32_t* keep_k, int32_t* kept_off, int32_t* kept_idx, int32_t* out_off,
                                 void* y, int32_t* assign, int32_t* counts, int32_t* src_pos,
                                 void* ws, size_t ws_bytes, void* stream) {
    if (!x || !y || !vis_off || !keep_ratio || !keep_k || !kept_off || !kept_idx || !out_off) return D3TOM_ERR_INVALID_ARG;
    int rc = importance_check(q, k, dt, B, seq_off, H, dh, scale, dec_idx, dec_off, min_D, max_D, vis_start, vis_count,
                              vis_off, max_N, max_V, scores);
    if (rc != D3TOM_OK) return rc;
    if (min_keep < 1 || max_keep < min_keep || max_keep > max_V) return D3TOM_ERR_INVALID_ARG;
    if (max_V > D3TOM_MAX_VISUAL) return D3TOM_ERR_UNSUPPORTED;
    if (mode != D3TOM_MERGE_MEAN && mode != D3TOM_MERGE_SUM) return D3TOM_ERR_INVALID_ARG;
    if (!ws) return D3TOM_ERR_INVALID_ARG;
    const LayerWs w = layer_ws_layout(B, max_N, max_V, H, dh, max_D);
    if (ws_bytes < w.total || (((uintptr_t)ws) & 255u)) return D3TOM_ERR_WORKSPACE_TOO_SMALL;
    char* base = (char*)ws;
    rc = importance_run(q, k, dt, B, seq_off, H, dh, scale, dec_idx, dec_off, max_D, vis_start, vis_count, vis_off, max_N,
                        max_V, scores, base + w.imp, stream);
    if (rc != D3TOM_OK) return rc;
    // The selection leaves most of the chip idle: its launch carries workgroups that stream the visual rows of the
    // similarity features and leave their norms, so that the rows are in the memory-side cache when the cosine kernel
    // gathers them and the merge needs no norms launch; the selecting workgroup writes the pruned list and the token
    // table.  (Giving half of the rows to the second importance launch was measured and lost: that kernel slows down
    // by more than the selection gains.)
    MergePrep prep;
    prep.feat = sim ? sim : x;
    prep.d = sim ? d_sim : d;
    prep.dt = dt;
    prep.vis_start = vis_start;
    prep.vis_count = vis_count;
    merge_prep_targets(base + w.merge, B, max_V, &prep);
    bool prepared = false;
    rc = topk_run(scores, B, vis_off, nullptr, nullptr, max_V, kept_idx, (int32_t*)(base + w.slot), keep_ratio, seq_off, keep_k,
                  kept_off, out_off, stream, &prep, &prepared);
    if (rc != D3TOM_OK) return rc;
    // launch sizes from the host-known bounds on the kept counts; workgroups beyond a sample's real sizes exit at once
    return merge_run(x, y, nullptr, nullptr, sim, d, d_sim, dt, B, seq_off, vis_start, vis_count, vis_off, kept_idx, kept_off,
                     max_N, max_V, max_keep, max_V - min_keep, max_N, mode, out_off, assign, counts, src_pos,
                     base + w.merge, merge_ws_bytes(B, max_V), stream, prepared, max_N - max_V + max_keep);
}
