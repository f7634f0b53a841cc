// d3tom_stack_step: one denoising step of Algorithm 1's inner loop, hidden states through all blocks with
// the merge layer inside block l*: full-length blocks before it, the merge between that block's attention
// and its feed-forward part, every later block on the shortened sequence.  Host-side sequencing only: every
// stage is one of the library's kernels, enqueued on the caller's stream.
#include "common.hpp"

namespace d3tom {
int linear_run(const void* a, const void* w, int M, int N, int K, int epilogue, const void* residual, void* out,
               int out_chunk, int tm_override, hipStream_t st, const float2* rope_cs = nullptr, int rope_dh = 0);
int rope_table_run(const int32_t* pos, int rows, int dh, float theta, float2* table, hipStream_t st);
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

// Per-sample sizes of the batch, host-known; passed to the metadata kernel by value.
constexpr int STACK_MAX_BATCH = D3TOM_STACK_MAX_BATCH;
struct BatchSizes {
    int B;
    int N[STACK_MAX_BATCH], vs[STACK_MAX_BATCH], V[STACK_MAX_BATCH], k[STACK_MAX_BATCH], D[STACK_MAX_BATCH];
};

// Device metadata of the batch (the merge-layer entry points read their per-sample sizes from device arrays):
// eight int32 arrays of STACK_MAX_BATCH + 1 entries each.
enum MetaSlot { META_SEQ_OFF = 0, META_VIS_START, META_VIS_COUNT, META_VIS_OFF, META_KEEP_K, META_KEPT_OFF, META_OUT_OFF,
                META_DEC_OFF, META_ARRAYS };
constexpr int META_STRIDE = STACK_MAX_BATCH + 1;
constexpr int META_INTS = META_ARRAYS * META_STRIDE;

// prefix sums of the per-sample sizes (one thread: at most 64 samples) and the position of every token inside
// its sample
__global__ void stack_meta_kernel(int32_t* meta, int32_t* pos, BatchSizes sz, int sum_N) {
    const int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t < sum_N) {
        int off = 0, b = 0;
        while (b < sz.B - 1 && t >= off + sz.N[b]) { off += sz.N[b]; ++b; }
        pos[t] = t - off;
    }
    if (t == 0) {
        int so = 0, vo = 0, ko = 0, oo = 0, dof = 0;
        for (int b = 0; b < sz.B; ++b) {
            meta[META_SEQ_OFF * META_STRIDE + b] = so;
            meta[META_VIS_START * META_STRIDE + b] = sz.vs[b];
            meta[META_VIS_COUNT * META_STRIDE + b] = sz.V[b];
            meta[META_VIS_OFF * META_STRIDE + b] = vo;
            meta[META_KEEP_K * META_STRIDE + b] = sz.k[b];
            meta[META_KEPT_OFF * META_STRIDE + b] = ko;
            meta[META_OUT_OFF * META_STRIDE + b] = oo;
            meta[META_DEC_OFF * META_STRIDE + b] = dof;
            so += sz.N[b]; vo += sz.V[b]; ko += sz.k[b]; oo += sz.N[b] - (sz.V[b] - sz.k[b]); dof += sz.D[b];
        }
        meta[META_SEQ_OFF * META_STRIDE + sz.B] = so;
        meta[META_VIS_OFF * META_STRIDE + sz.B] = vo;
        meta[META_KEPT_OFF * META_STRIDE + sz.B] = ko;
        meta[META_OUT_OFF * META_STRIDE + sz.B] = oo;
        meta[META_DEC_OFF * META_STRIDE + sz.B] = dof;
    }
}

__global__ void stack_copy_i32_kernel(const int32_t* __restrict__ src, int32_t* __restrict__ dst, int n) {
    const int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t < n) dst[t] = src[t];
}

struct StackWs {
    size_t meta, pos, rope, h, hm, nrm, qkv, att, act, part, scores, kept, slot, assign, sub, sub_bytes, total;
};
// sum_N / max_N: total and largest token count; sum_V / max_V likewise for the visual blocks
StackWs stack_ws_layout(int B, int sum_N, int max_N, int d, int H, int F, int sum_V, int max_V, int max_D) {
    StackWs w;
    size_t o = 0;
    auto take = [&](size_t bytes) { const size_t at = o; o += align_up(bytes, 256); return at; };
    const size_t act_row = (size_t)sum_N * d * 2;
    const size_t vis = (size_t)(sum_V > 0 ? sum_V : 1) * 4;
    w.meta = take(META_INTS * 4);
    w.pos = take((size_t)sum_N * 4);
    w.rope = take((size_t)sum_N * (d / H / 2) * sizeof(float2));      // (cos, sin) of every token's rotary angles
    w.h = take(act_row); w.hm = take(act_row); w.nrm = take(act_row);
    w.qkv = take(3 * act_row);             // q, k, v of the current length, back to back
    w.att = take(act_row);
    w.act = take((size_t)sum_N * F * 2);
    w.part = take(STACK_PARTIAL_BYTES);
    w.scores = take(vis); w.kept = take(vis); w.slot = take(vis); w.assign = take(vis);
    const int dh = d / H;
    size_t sub = 256;
    const size_t s_imp = d3tom_workspace_bytes(D3TOM_OP_IMPORTANCE, B, max_N, max_V > 0 ? max_V : 1, H, dh, max_D > 0 ? max_D : 1);
    const size_t s_mrg = d3tom_workspace_bytes(D3TOM_OP_MERGE, B, max_N, max_V > 0 ? max_V : 1, H, dh, 1);
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
    return d3tom::stack_ws_layout(1, N, N, d, H, F, V, V, max_D).total;
}

extern "C" size_t d3tom_stack_batch_workspace_bytes(int B, int sum_N, int max_N, int d, int H, int F, int sum_V, int max_V, int max_D) {
    if (B < 1 || B > D3TOM_STACK_MAX_BATCH || sum_N < 1 || max_N < 1 || max_N > sum_N || d < 1 || H < 1 || F < 1 || d % H != 0) return 0;
    return d3tom::stack_ws_layout(B, sum_N, max_N, d, H, F, sum_V, max_V, max_D).total;
}

extern "C" int d3tom_stack_step_batch(const void* x, int B, const int32_t* N_h, int d, int H, int F, int L,
                                      const d3tom_block_weights* blocks, int merge_layer, const int32_t* dec_idx, const int32_t* D_h,
                                      const int32_t* vis_start_h, const int32_t* V_h, const int32_t* keep_h, int mode,
                                      float eps, float theta, void* y, int32_t* src_pos, float* scores_out, int32_t* kept_idx_out,
                                      int32_t* assign_out, int* n_out, void* ws, size_t ws_bytes, void* stream) {
    using namespace d3tom;
    hipStream_t st = (hipStream_t)stream;
    if (!x || !y || !blocks || !ws || !N_h || !D_h || B < 1 || d < 1 || H < 1 || F < 1 || L < 1) return D3TOM_ERR_INVALID_ARG;
    if (B > STACK_MAX_BATCH) return D3TOM_ERR_UNSUPPORTED;
    if (d % H != 0 || !aligned16(x) || !aligned16(y)) return D3TOM_ERR_INVALID_ARG;
    if (mode != D3TOM_MERGE_MEAN && mode != D3TOM_MERGE_SUM) return D3TOM_ERR_INVALID_ARG;
    BatchSizes sz;
    sz.B = B;
    int sum_N = 0, max_N = 0, sum_D = 0, min_D = 0x7FFFFFFF, max_D = 0;
    for (int b = 0; b < B; ++b) {
        if (N_h[b] < 1 || D_h[b] < 0) return D3TOM_ERR_INVALID_ARG;
        sz.N[b] = N_h[b]; sz.D[b] = D_h[b];
        sz.vs[b] = 0; sz.V[b] = 0; sz.k[b] = 0;
        sum_N += N_h[b]; max_N = N_h[b] > max_N ? N_h[b] : max_N;
        sum_D += D_h[b]; min_D = D_h[b] < min_D ? D_h[b] : min_D; max_D = D_h[b] > max_D ? D_h[b] : max_D;
    }
    if (sum_D > 0 && !dec_idx) return D3TOM_ERR_INVALID_ARG;
    const bool layer_ok = merge_layer >= 1 && merge_layer <= L;
    // Algorithm 1 skips the merge of a step whose decider set is empty; inside one batch all samples take the same path
    if (layer_ok && max_D > 0 && min_D == 0) return D3TOM_ERR_NO_DECIDERS;
    const bool merging = layer_ok && max_D > 0;
    int sum_V = 0, max_V = 0, max_keep = 0, max_pruned = 0, max_out = max_N, sum_out = sum_N;
    if (merging) {
        if (!vis_start_h || !V_h || !keep_h) return D3TOM_ERR_INVALID_ARG;
        max_out = 0; sum_out = 0;
        for (int b = 0; b < B; ++b) {
            const int V = V_h[b], vs = vis_start_h[b], k = keep_h[b];
            if (V < 1 || vs < 0 || vs + V > N_h[b] || k < 1 || k > V) return D3TOM_ERR_INVALID_ARG;
            if (D_h[b] > D3TOM_MAX_DECIDERS || V > D3TOM_MAX_VISUAL) return D3TOM_ERR_UNSUPPORTED;
            sz.vs[b] = vs; sz.V[b] = V; sz.k[b] = k;
            sum_V += V; max_V = V > max_V ? V : max_V; max_keep = k > max_keep ? k : max_keep;
            max_pruned = (V - k) > max_pruned ? (V - k) : max_pruned;
            const int out = N_h[b] - (V - k);
            max_out = out > max_out ? out : max_out; sum_out += out;
        }
    }
    const int dh = d / H;
    if (dh != 64 && dh != 128) return D3TOM_ERR_UNSUPPORTED;
    if (d % 64 != 0 || F % 64 != 0) return D3TOM_ERR_UNSUPPORTED;
    {   // every operand of a projection is addressed with 32-bit byte offsets: check here, before anything is enqueued
        const size_t lim = (size_t)1 << 31, wide = (size_t)(d > F ? d : F);
        if ((size_t)sum_N * wide * 2 >= lim || (size_t)3 * d * d * 2 >= lim || (size_t)2 * F * d * 2 >= lim) return D3TOM_ERR_UNSUPPORTED;
        if (d > 8192) return D3TOM_ERR_UNSUPPORTED;              // row-wise kernels keep a row in registers
    }
    for (int l = 0; l < L; ++l) {
        const d3tom_block_weights& b = blocks[l];
        if (!b.attn_norm || !b.w_qkv || !b.w_o || !b.ffn_norm || !b.w_gate_up || !b.w_down) return D3TOM_ERR_INVALID_ARG;
    }
    const StackWs w = stack_ws_layout(B, sum_N, max_N, d, H, F, merging ? sum_V : 0, merging ? max_V : 0, merging ? max_D : 0);
    if (ws_bytes < w.total || (((uintptr_t)ws) & 255u)) return D3TOM_ERR_WORKSPACE_TOO_SMALL;
    char* base = (char*)ws;
    int32_t* meta = (int32_t*)(base + w.meta);
    int32_t* pos = (int32_t*)(base + w.pos);
    float2* rope_cs = (float2*)(base + w.rope);
    void *h = base + w.h, *hm = base + w.hm, *nrm = base + w.nrm, *qkv = base + w.qkv;
    void *att = base + w.att, *act = base + w.act;
    float* part = (float*)(base + w.part);
    float* scores = (float*)(base + w.scores);
    int32_t* kept = (int32_t*)(base + w.kept);
    int32_t* slot = (int32_t*)(base + w.slot);
    int32_t* asg = (int32_t*)(base + w.assign);
    void* sub = base + w.sub;
    const float scale = 1.0f / sqrtf((float)dh);
    if (n_out)
        for (int b = 0; b < B; ++b) n_out[b] = merging ? N_h[b] - (V_h[b] - keep_h[b]) : N_h[b];
    auto M = [&](int slot_id) { return meta + slot_id * META_STRIDE; };

    D3TOM_LAUNCH(STACK_META, st, (stack_meta_kernel<<<ceil_div(sum_N, 256), 256, 0, st>>>(meta, pos, sz, sum_N)));
    {   // rotary angles of the tokens at their positions; renewed after the merge, when the positions change
        const int rc = rope_table_run(pos, sum_N, dh, theta, rope_cs, st);
        if (rc != D3TOM_OK) return rc;
    }

    const void* cur = x;          // hidden state entering the block (the input itself is never written)
    int n = sum_N;                // its row count
    int longest = max_N;          // longest sample at the current length
    int32_t* cu = M(META_SEQ_OFF);
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
        // the rotation of q and k happens in the projection's epilogue
        D3TOM_TRY(linear_run(nrm, b.w_qkv, n, 3 * d, d, LIN_PLAIN, nullptr, qkv, d, 0, st, rope_cs, dh));
        D3TOM_TRY(d3tom_attend(qq, kk, vv, D3TOM_BF16, B, cu, longest, H, dh, scale, att, sub, w.sub_bytes, st));
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
            D3TOM_TRY(d3tom_importance(qq, kk, D3TOM_BF16, B, M(META_SEQ_OFF), H, dh, scale, dec_idx, M(META_DEC_OFF),
                                       min_D, max_D, M(META_VIS_START), M(META_VIS_COUNT), M(META_VIS_OFF), max_N, max_V,
                                       scores, sub, w.sub_bytes, st));
            D3TOM_TRY(d3tom_select_topk(scores, B, M(META_VIS_OFF), M(META_KEEP_K), M(META_KEPT_OFF), max_V, kept,
                                        slot, sub, w.sub_bytes, st));
            void* merged = (post == h) ? hm : h;
            D3TOM_TRY(d3tom_merge(post, nullptr, d, d, D3TOM_BF16, B, M(META_SEQ_OFF), M(META_VIS_START),
                                  M(META_VIS_COUNT), M(META_VIS_OFF), kept, M(META_KEPT_OFF), max_N, max_V, max_keep,
                                  max_pruned, max_out, mode, M(META_OUT_OFF), merged, asg, nullptr, pos, sub, w.sub_bytes,
                                  st));
            // from here on every stage sees the shortened sequences; pos holds the original positions
            ht = merged;
            D3TOM_TRY(rope_table_run(pos, sum_out, dh, theta, rope_cs, st));
            n = sum_out;
            longest = max_out;
            cu = M(META_OUT_OFF);
            const int sum_k = sum_out - (sum_N - sum_V);
            if (scores_out)
                D3TOM_LAUNCH(STACK_META, st, (stack_copy_i32_kernel<<<ceil_div(sum_V, 256), 256, 0, st>>>((const int32_t*)scores, (int32_t*)scores_out, sum_V)));
            if (kept_idx_out)
                D3TOM_LAUNCH(STACK_META, st, (stack_copy_i32_kernel<<<ceil_div(sum_k, 256), 256, 0, st>>>(kept, kept_idx_out, sum_k)));
            if (assign_out)
                D3TOM_LAUNCH(STACK_META, st, (stack_copy_i32_kernel<<<ceil_div(sum_V, 256), 256, 0, st>>>(asg, assign_out, sum_V)));
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
        D3TOM_LAUNCH(STACK_META, st, (stack_copy_i32_kernel<<<ceil_div(n, 256), 256, 0, st>>>(pos, src_pos, n)));
    return D3TOM_OK;
}

extern "C" int d3tom_stack_step(const void* x, int N, int d, int H, int F, int L, const d3tom_block_weights* blocks,
                                int merge_layer, const int32_t* dec_idx, int D, int vis_start, int V, int keep_k, int mode,
                                float eps, float theta, void* y, int32_t* src_pos, float* scores_out, int32_t* kept_idx_out,
                                int32_t* assign_out, int* n_out, void* ws, size_t ws_bytes, void* stream) {
    if (D < 0) return D3TOM_ERR_INVALID_ARG;
    const int32_t N1 = N, D1 = D, vs1 = vis_start, V1 = V, k1 = keep_k;
    return d3tom_stack_step_batch(x, 1, &N1, d, H, F, L, blocks, merge_layer, dec_idx, &D1, &vs1, &V1, &k1, mode, eps, theta, y,
                                  src_pos, scores_out, kept_idx_out, assign_out, n_out, ws, ws_bytes, stream);
}
