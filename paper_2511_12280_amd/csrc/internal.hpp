// Entry-point bodies shared between the C ABI functions of different source files (not part of the C ABI).
#pragma once
#include "common.hpp"

namespace d3tom {

// d3tom_importance after its argument and workspace checks
int importance_check(const void* q, const void* k, int dt, int B, const int32_t* seq_off, int H, int dh, float scale,
                     const int32_t* dec_idx, const int32_t* dec_off, int min_D, int max_D,
                     const int32_t* vis_start, const int32_t* vis_count, const int32_t* score_off,
                     int max_N, int max_V, const float* scores);
int importance_run(const void* q, const void* k, int dt, int B, const int32_t* seq_off, int H, int dh, float scale,
                   const int32_t* dec_idx, const int32_t* dec_off, int max_D,
                   const int32_t* vis_start, const int32_t* vis_count, const int32_t* score_off,
                   int max_N, int max_V, float* scores, void* ws, void* stream);
size_t importance_ws_bytes(int B, int max_N, int max_V, int H, int dh, int max_D);

// Rows the kernels after the selection will gather: the visual block of every sample in a row-major tensor
// (base == nullptr: none).  The selection keeps one compute unit per sample busy; the other compute units
// stream these rows meanwhile, so that they are in the memory-side cache when the merge reads them.
struct RowPrefetch {
    const void* base = nullptr;
    int row_bytes = 0;                       // a multiple of 16, base 16-byte aligned
    const int32_t* vis_start = nullptr;
    const int32_t* vis_count = nullptr;
};

// d3tom_select_topk; with keep_ratio != nullptr the kept counts are computed on the device from the ratios and
// written, with their prefix sums and the output row offsets, to keep_k / kept_off / out_off
int topk_run(const float* scores, int B, const int32_t* score_off, const int32_t* keep_k, const int32_t* kept_off, int max_V,
             int32_t* kept_idx, int32_t* slot_of, const double* keep_ratio, const int32_t* seq_off, int32_t* keep_k_out,
             int32_t* kept_off_out, int32_t* out_off_out, void* stream, RowPrefetch prefetch = RowPrefetch());

// d3tom_merge / d3tom_merge_kv
int merge_run(const void* x0, void* y0, const void* x1, void* y1, const void* sim, int d, int d_sim, int dt,
              int B, const int32_t* seq_off, const int32_t* vis_start, const int32_t* vis_count,
              const int32_t* vis_off, const int32_t* kept_idx, const int32_t* kept_off,
              int max_N, int max_V, int max_keep, int max_pruned, int max_out, int mode,
              const int32_t* out_off, int32_t* assign, int32_t* counts, int32_t* src_pos,
              void* ws, size_t ws_bytes, void* stream);
size_t merge_ws_bytes(int B, int max_V);

}  // namespace d3tom
