// Entry-point bodies shared between the C ABI functions of different source files (not part of the C ABI).
#pragma once
#include "common.hpp"

namespace d3tom {

struct MergePrep;

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

// Sum of squares of one row of d elements (bf16 or float32, 16-byte aligned, d a multiple of the elements per 16
// bytes), computed by one wave: lane-strided 16-byte chunks, eight loads in flight per lane, elements added in
// storage order inside a lane, lanes combined by wave_sum.  Every lane returns the total.  One definition, so that
// every kernel that needs a row norm gets the same bits.
template <typename T>
__device__ __forceinline__ float row_sum_squares(const T* __restrict__ row, int d, int lane) {
    constexpr int EPC = 16 / sizeof(T);       // elements per 16-byte chunk
    float ss = 0.f;
    const int nch = d / EPC;
    for (int c0 = 0; c0 < nch; c0 += 64 * 8) {
        uint4 w8[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int c = c0 + u * 64 + lane;
            w8[u] = (c < nch) ? *reinterpret_cast<const uint4*>(row + (size_t)c * EPC) : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const uint4 w = w8[u];
            if constexpr (sizeof(T) == 2) {
                const uint32_t ww[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
                for (int e = 0; e < 4; ++e) { const float a = bf16_lo(ww[e]), c2 = bf16_hi(ww[e]); ss += a * a; ss += c2 * c2; }
            } else {
                const float a0 = __uint_as_float(w.x), a1 = __uint_as_float(w.y), a2 = __uint_as_float(w.z), a3 = __uint_as_float(w.w);
                ss += a0 * a0; ss += a1 * a1; ss += a2 * a2; ss += a3 * a3;
            }
        }
    }
    return wave_sum(ss);
}
__device__ __forceinline__ float reciprocal_norm(float sum_squares) { return 1.0f / fmaxf(sqrtf(sum_squares), 1e-15f); }

// Table entry of a visual token: (order-preserving integer image of its best value so far) << 32 | (2^32-1 - slot).
// Unsigned comparison of entries = (value, then lower slot); 0 = nothing yet (below every real entry); a kept
// token holds the largest high word with its own slot and is never a target of an update.
typedef unsigned long long table_t;
__device__ __forceinline__ uint32_t value_key(float f) {       // ascending uint order == ascending float order
    const uint32_t u = __float_as_uint(f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ table_t table_entry(float value, int slot) {
    return ((table_t)value_key(value) << 32) | (table_t)(0xFFFFFFFFu - (uint32_t)slot);
}
__device__ __forceinline__ table_t table_entry_kept(int slot) {
    return ((table_t)0xFFFFFFFFu << 32) | (table_t)(0xFFFFFFFFu - (uint32_t)slot);
}

// What the merge needs before its cosine kernel, when the selection launch prepares it (the one-call merge layer):
// the selection keeps one compute unit per sample busy, so the launch carries further workgroups that stream the
// visual rows of the similarity features (one wave per row) and leave 1 / norm of EVERY visual row in rnorm, indexed
// by token; the rows are then in the memory-side cache when the cosine kernel gathers them, and the separate norms
// launch is not needed.  The selecting workgroup writes the ascending pruned list and the initial token table
// (0 for a pruned token, its own slot at the largest value for a kept one) while it emits the kept list.
struct MergePrep {
    const void* feat = nullptr;              // similarity features [sum N, d], 16-byte aligned rows
    int d = 0, dt = 0;
    const int32_t* vis_start = nullptr;
    const int32_t* vis_count = nullptr;
    float* rnorm = nullptr;                  // [B, max_V]
    int32_t* pruned = nullptr;               // [B, max_V]
    table_t* table = nullptr;                // [B, VP]
    int VP = 0;
};
// the arrays above inside a merge workspace
void merge_prep_targets(void* merge_ws, int B, int max_V, MergePrep* prep);

// Whether the preparing launch is used for a batch: only where the streaming workgroups can form their rows
// (per-sample offsets, 16-byte reads) and where it pays: rows that overflow the memory-side cache (256 MB, shared
// with everything else the step touches) would be gone again before the cosine kernel wants them, and reading every
// row then costs more than the norms of the kept rows alone.
constexpr size_t MERGE_PREP_MAX_BYTES = (size_t)160 << 20;
inline bool merge_prep_usable(const MergePrep* q, int B, int max_V, const int32_t* seq_off) {
    if (!q || !q->feat || !seq_off || !q->vis_start || !q->vis_count || !q->rnorm || !q->pruned || !q->table) return false;
    if (q->VP < max_V || (q->dt != D3TOM_BF16 && q->dt != D3TOM_F32) || q->d < 1) return false;
    const size_t row_bytes = (size_t)q->d * (q->dt == D3TOM_BF16 ? 2 : 4);
    if (row_bytes % 16 != 0 || (((uintptr_t)q->feat) & 15u) != 0) return false;
    return (size_t)B * max_V * row_bytes <= MERGE_PREP_MAX_BYTES;
}

// The streaming job of the preparing launch: 1 / norm of the visual rows of sample b, one wave per row, waves
// wave_id, wave_id + nwaves, ... (rows clamped to the sample)
__device__ __forceinline__ void stream_row_norms(const MergePrep& prep, int max_V, int b, const int32_t* __restrict__ seq_off,
                                                 int wave_id, int nwaves, int lane) {
    const int n = seq_off[b + 1] - seq_off[b];
    const int vs = min(max(prep.vis_start[b], 0), n);
    const int cnt = min(min(max(prep.vis_count[b], 0), n - vs), max_V);
    float* rn = prep.rnorm + (size_t)b * max_V;
    for (int r = wave_id; r < cnt; r += nwaves) {
        const size_t row = (size_t)(seq_off[b] + vs + r) * prep.d;
        const float ss = (prep.dt == D3TOM_BF16) ? row_sum_squares(static_cast<const uint16_t*>(prep.feat) + row, prep.d, lane)
                                                 : row_sum_squares(static_cast<const float*>(prep.feat) + row, prep.d, lane);
        if (lane == 0) rn[r] = reciprocal_norm(ss);
    }
}

// d3tom_select_topk; with a usable prep the launch prepares the merge and *prepared says so; with keep_ratio != nullptr the kept counts are computed on the device from the ratios and
// written, with their prefix sums and the output row offsets, to keep_k / kept_off / out_off
int topk_run(const float* scores, int B, const int32_t* score_off, const int32_t* keep_k, const int32_t* kept_off, int max_V,
             int32_t* kept_idx, int32_t* slot_of, const double* keep_ratio, const int32_t* seq_off, int32_t* keep_k_out,
             int32_t* kept_off_out, int32_t* out_off_out, void* stream, const MergePrep* prep = nullptr,
             bool* prepared = nullptr);

// d3tom_merge / d3tom_merge_kv; prepared: the selection launch has filled the workspace as MergePrep describes;
// out_rows_hint: output rows per sample to expect when max_out is only a loose bound (tuning only)
int merge_run(const void* x0, void* y0, const void* x1, void* y1, const void* sim, int d, int d_sim, int dt,
              int B, const int32_t* seq_off, const int32_t* vis_start, const int32_t* vis_count,
              const int32_t* vis_off, const int32_t* kept_idx, const int32_t* kept_off,
              int max_N, int max_V, int max_keep, int max_pruned, int max_out, int mode,
              const int32_t* out_off, int32_t* assign, int32_t* counts, int32_t* src_pos,
              void* ws, size_t ws_bytes, void* stream, bool prepared = false, int out_rows_hint = 0);
size_t merge_ws_bytes(int B, int max_V);

}  // namespace d3tom
