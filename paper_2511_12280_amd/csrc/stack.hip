// d3tom_stack_step: one denoising step of Algorithm 1's inner loop, hidden states through all blocks with
// the merge layer inside block l*: full-length blocks before it, the merge between that block's attention
// and its feed-forward part, every later block on the shortened sequence.  Host-side sequencing only: every
// stage is one of the library's kernels, enqueued on the caller's stream.
#include "common.hpp"

namespace d3tom {
int linear_run(const void* a, const void* w, int M, int N, int K, int epilogue, const void* residual, void* out,
               int out_chunk, int tm_override, hipStream_t st);
int rmsnorm_run(const void* x, const void* gain, int rows, int d, float eps, void* y, hipStream_t st);
int rope_run(void* q, void* k, const int32_t* pos, int rows, int H, int dh, float theta, hipStream_t st);
int linear_split_plan(int M, int N, int K);
int linear_partial_run(const void* a, const void* w, int M, int N, int K, int ksplit, float* partial, hipStream_t st);
int add_norm_run(const float* part, int nsplit, const void* residual, const void* gain, int rows, int d, float eps,
                 void* h, void* y, hipStream_t st);
// float32 partial products of a split projection: the plan only splits while the 256 x 128 tiles of the result
// number at most 64, i.e. at most 2 Mi elements per slice, 4 slices
constexpr size_t STACK_PARTIAL_BYTES = (size_t)4 * 64 * 256 * 128 * sizeof(float);

enum { LIN_PLAIN = 0, LIN_RESIDUAL = 1, LIN_SWIGLU = 2 };

// Device metadata of the single sample, written by one small kernel (the merge-layer entry points read
// their per-sample sizes from device arrays).
enum MetaSlot {
    META_SEQ_OFF = 0,      // {0, N}
    META_VIS_START = 2,    // {vis_start}
    META_VIS_COUNT = 3,    // {V}
    META_VIS_OFF = 4,      // {0, V}
    META_KEEP_K = 6,       // {k}
    META_KEPT_OFF = 7,     // {0, k}
    META_OUT_OFF = 9,      // {0, N_m}
    META_DEC_OFF = 11,     // {0, D}
    META_INTS = 64
};

__global__ void stack_meta_kernel(int32_t* meta, int32_t* pos, int N, int vis_start, int V, int k, int D) {
    const int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t < N) pos[t] = t;
    if (t == 0) {
        meta[META_SEQ_OFF] = 0; meta[META_SEQ_OFF + 1] = N;
        meta[META_VIS_START] = vis_start; meta[META_VIS_COUNT] = V;
        meta[META_VIS_OFF] = 0; meta[META_VIS_OFF + 1] = V;
        meta[META_KEEP_K] = k;
        meta[META_KEPT_OFF] = 0; meta[META_KEPT_OFF + 1] = k;
        meta[META_OUT_OFF] = 0; meta[META_OUT_OFF + 1] = N - (V - k);
        meta[META_DEC_OFF] = 0; meta[META_DEC_OFF + 1] = D;
    }
}

__global__ void stack_copy_i32_kernel(const int32_t* __restrict__ src, int32_t* __restrict__ dst, int n) {
    const int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t < n) dst[t] = src[t];
}

struct StackWs {
    size_t meta, pos, h, hm, nrm, qkv, att, act, part, scores, kept, slot, assign, sub, sub_bytes, total;
};
StackWs stack_ws_layout(int N, int d, int H, int F, int V, int max_D) {
    StackWs w;
    size_t o = 0;
    auto take = [&](size_t bytes) { const size_t at = o; o += align_up(bytes, 256); return at; };
    const size_t act_row = (size_t)N * d * 2;
    w.meta = take(META_INTS * 4);
    w.pos = take((size_t)N * 4);
    w.h = take(act_row); w.hm = take(act_row); w.nrm = take(act_row);
    w.qkv = take(3 * act_row);             // q, k, v of the current length, back to back
    w.att = take(act_row);
    w.act = take((size_t)N * F * 2);
    w.part = take(STACK_PARTIAL_BYTES);
    w.scores = take((size_t)(V > 0 ? V : 1) * 4);
    w.kept = take((size_t)(V > 0 ? V : 1) * 4);
    w.slot = take((size_t)(V > 0 ? V : 1) * 4);
    w.assign = take((size_t)(V > 0 ? V : 1) * 4);
    const int dh = d / H;
    size_t sub = 256;
    const size_t s_imp = d3tom_workspace_bytes(D3TOM_OP_IMPORTANCE, 1, N, V > 0 ? V : 1, H, dh, max_D > 0 ? max_D : 1);
    const size_t s_mrg = d3tom_workspace_bytes(D3TOM_OP_MERGE, 1, N, V > 0 ? V : 1, H, dh, 1);
    if (s_imp > sub) sub = s_imp;
    if (s_mrg > sub) sub = s_mrg;
    w.sub_bytes = sub;
    w.sub = take(sub);
    w.total = o;
    return w;
}
}  // namespace d3tom

extern "C" size_t d3tom_stack_workspace_bytes(int N, int d, int H, int F, int V, int max_D) {
    if (N < 1 || d < 1 || H < 1 || F < 1 || d % H != 0) return 0;
    return d3tom::stack_ws_layout(N, d, H, F, V, max_D).total;
}

extern "C" int d3tom_stack_step(const void* x, int N, int d, int H, int F, int L, const d3tom_block_weights* blocks,
                                int merge_layer, const int32_t* dec_idx, int D, int vis_start, int V, int keep_k, int mode,
                                float eps, float theta, void* y, int32_t* src_pos, float* scores_out, int32_t* kept_idx_out,
                                int32_t* assign_out, int* n_out, void* ws, size_t ws_bytes, void* stream) {
    using namespace d3tom;
    hipStream_t st = (hipStream_t)stream;
    if (!x || !y || !blocks || !ws || N < 1 || d < 1 || H < 1 || F < 1 || L < 1) return D3TOM_ERR_INVALID_ARG;
    if (d % H != 0 || !aligned16(x) || !aligned16(y)) return D3TOM_ERR_INVALID_ARG;
    if (D < 0 || (D > 0 && !dec_idx)) return D3TOM_ERR_INVALID_ARG;
    if (mode != D3TOM_MERGE_MEAN && mode != D3TOM_MERGE_SUM) return D3TOM_ERR_INVALID_ARG;
    const bool merging = (D > 0) && merge_layer >= 1 && merge_layer <= L;
    if (merging) {
        if (V < 1 || vis_start < 0 || vis_start + V > N || keep_k < 1 || keep_k > V) return D3TOM_ERR_INVALID_ARG;
        if (D > D3TOM_MAX_DECIDERS || V > D3TOM_MAX_VISUAL) return D3TOM_ERR_UNSUPPORTED;
    }
    const int dh = d / H;
    if (dh != 64 && dh != 128) return D3TOM_ERR_UNSUPPORTED;
    if (d % 64 != 0 || F % 64 != 0) return D3TOM_ERR_UNSUPPORTED;
    {   // every operand of a projection is addressed with 32-bit byte offsets: check here, before anything is enqueued
        const size_t lim = (size_t)1 << 31, wide = (size_t)(d > F ? d : F);
        if ((size_t)N * wide * 2 >= lim || (size_t)3 * d * d * 2 >= lim || (size_t)2 * F * d * 2 >= lim) return D3TOM_ERR_UNSUPPORTED;
        if (d > 8192) return D3TOM_ERR_UNSUPPORTED;              // row-wise kernels keep a row in registers
    }
    for (int l = 0; l < L; ++l) {
        const d3tom_block_weights& b = blocks[l];
        if (!b.attn_norm || !b.w_qkv || !b.w_o || !b.ffn_norm || !b.w_gate_up || !b.w_down) return D3TOM_ERR_INVALID_ARG;
    }
    const StackWs w = stack_ws_layout(N, d, H, F, merging ? V : 0, merging ? D : 0);
    if (ws_bytes < w.total || (((uintptr_t)ws) & 255u)) return D3TOM_ERR_WORKSPACE_TOO_SMALL;
    char* base = (char*)ws;
    int32_t* meta = (int32_t*)(base + w.meta);
    int32_t* pos = (int32_t*)(base + w.pos);
    void *h = base + w.h, *hm = base + w.hm, *nrm = base + w.nrm, *qkv = base + w.qkv;
    void *att = base + w.att, *act = base + w.act;
    float* part = (float*)(base + w.part);
    float* scores = (float*)(base + w.scores);
    int32_t* kept = (int32_t*)(base + w.kept);
    int32_t* slot = (int32_t*)(base + w.slot);
    int32_t* asg = (int32_t*)(base + w.assign);
    void* sub = base + w.sub;
    const float scale = 1.0f / sqrtf((float)dh);
    const int N_m = merging ? N - (V - keep_k) : N;
    if (n_out) *n_out = N_m;

    D3TOM_LAUNCH(STACK_META, st, (stack_meta_kernel<<<ceil_div(N, 256), 256, 0, st>>>(meta, pos, N, vis_start, V, keep_k, D)));

    const void* cur = x;          // hidden state entering the block (the input itself is never written)
    int n = N;                    // its row count
    int32_t* cu = meta + META_SEQ_OFF;
    int status;
#define D3TOM_TRY(call) do { status = (call); if (status != D3TOM_OK) return status; } while (0)
    // A projection whose result is short and narrow (output and down projection of the shortened sequence) is
    // cut along the contraction; the row-wise kernel that adds its slices and the residual also writes the
    // normalised rows the next sub-block starts from, so `nrm` may already be filled when a sub-block begins.
    bool nrm_ready = false;
    for (int l = 1; l <= L; ++l) {
        const d3tom_block_weights& b = blocks[l - 1];
        const bool last = (l == L);
        const bool merge_here = merging && l == merge_layer;
        if (!nrm_ready) D3TOM_TRY(rmsnorm_run(cur, b.attn_norm, n, d, eps, nrm, st));
        // q | k | v in one projection, written as three [n, d] matrices back to back
        void* qq = qkv;
        void* kk = (char*)qkv + (size_t)n * d * 2;
        void* vv = (char*)qkv + (size_t)2 * n * d * 2;
        D3TOM_TRY(linear_run(nrm, b.w_qkv, n, 3 * d, d, LIN_PLAIN, nullptr, qkv, d, 0, st));
        D3TOM_TRY(rope_run(qq, kk, pos, n, H, dh, theta, st));
        D3TOM_TRY(d3tom_attend(qq, kk, vv, D3TOM_BF16, 1, cu, n, H, dh, scale, att, sub, w.sub_bytes, st));
        // post-attention hidden state = residual + attention output projection; in place, except that the
        // caller's input is never written
        void* post = (cur == x) ? h : const_cast<void*>(cur);
        bool ffn_nrm_ready = false;
        const int ks_o = linear_split_plan(n, d, d);
        if (ks_o > 1) {
            D3TOM_TRY(linear_partial_run(att, b.w_o, n, d, d, ks_o, part, st));
            D3TOM_TRY(add_norm_run(part, ks_o, cur, merge_here ? nullptr : b.ffn_norm, n, d, eps, post, nrm, st));
            ffn_nrm_ready = !merge_here;
        } else {
            D3TOM_TRY(linear_run(att, b.w_o, n, d, d, LIN_RESIDUAL, cur, post, 0, 0, st));
        }
        void* ht = post;
        if (merge_here) {
            D3TOM_TRY(d3tom_importance(qq, kk, D3TOM_BF16, 1, meta + META_SEQ_OFF, H, dh, scale, dec_idx, meta + META_DEC_OFF,
                                       D, D, meta + META_VIS_START, meta + META_VIS_COUNT, meta + META_VIS_OFF, N, V,
                                       scores, sub, w.sub_bytes, st));
            D3TOM_TRY(d3tom_select_topk(scores, 1, meta + META_VIS_OFF, meta + META_KEEP_K, meta + META_KEPT_OFF, V, kept,
                                        slot, sub, w.sub_bytes, st));
            void* merged = (post == h) ? hm : h;
            D3TOM_TRY(d3tom_merge(post, nullptr, d, d, D3TOM_BF16, 1, meta + META_SEQ_OFF, meta + META_VIS_START,
                                  meta + META_VIS_COUNT, meta + META_VIS_OFF, kept, meta + META_KEPT_OFF, N, V, keep_k,
                                  V - keep_k, N_m, mode, meta + META_OUT_OFF, merged, asg, nullptr, pos, sub, w.sub_bytes,
                                  st));
            // from here on every stage sees the shortened sequence; pos holds the original positions
            ht = merged;
            n = N_m;
            cu = meta + META_OUT_OFF;
            if (scores_out)
                D3TOM_LAUNCH(STACK_META, st, (stack_copy_i32_kernel<<<ceil_div(V, 256), 256, 0, st>>>((const int32_t*)scores, (int32_t*)scores_out, V)));
            if (kept_idx_out)
                D3TOM_LAUNCH(STACK_META, st, (stack_copy_i32_kernel<<<ceil_div(keep_k, 256), 256, 0, st>>>(kept, kept_idx_out, keep_k)));
            if (assign_out)
                D3TOM_LAUNCH(STACK_META, st, (stack_copy_i32_kernel<<<ceil_div(V, 256), 256, 0, st>>>(asg, assign_out, V)));
        }
        if (!ffn_nrm_ready) D3TOM_TRY(rmsnorm_run(ht, b.ffn_norm, n, d, eps, nrm, st));
        D3TOM_TRY(linear_run(nrm, b.w_gate_up, n, 2 * F, d, LIN_SWIGLU, nullptr, act, 0, 0, st));
        void* outp = last ? y : ht;                  // in place, except that the last block writes the caller's y
        const int ks_d = linear_split_plan(n, d, F);
        if (ks_d > 1) {
            D3TOM_TRY(linear_partial_run(act, b.w_down, n, d, F, ks_d, part, st));
            D3TOM_TRY(add_norm_run(part, ks_d, ht, last ? nullptr : blocks[l].attn_norm, n, d, eps, outp, nrm, st));
            nrm_ready = !last;
        } else {
            D3TOM_TRY(linear_run(act, b.w_down, n, d, F, LIN_RESIDUAL, ht, outp, 0, 0, st));
            nrm_ready = false;
        }
        cur = outp;
    }
#undef D3TOM_TRY
    if (src_pos)
        D3TOM_LAUNCH(STACK_META, st, (stack_copy_i32_kernel<<<ceil_div(N_m, 256), 256, 0, st>>>(pos, src_pos, N_m)));
    return D3TOM_OK;
}
