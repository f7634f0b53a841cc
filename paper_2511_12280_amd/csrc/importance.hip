// d3tom_importance: decider-guided importance map (Section 3.2, "The Decider-Guided Mechanism";
// Algorithm 1, the line that forms S).
//
// S_j = (1/H) sum_h sum_{i in D} softmax_j(scale * q_{i,h} . k_{j,h}), softmax over ALL keys of the
// sample, written for the visual columns only.  The N x N matrix is never formed: only the |D|
// decider rows are ever evaluated.  Large decider sets take two sweeps over K (below); small ones keep
// the D x N x H logits of the first sweep and finish from those (imp_scores_from_logits):
//
//   sweep 1 (stats)   per (head, decider): running max and sum of exp2 over all keys, computed per
//                     512-key chunk by one workgroup each and combined later in a fixed order
//   sweep 2 (scores)  per (head, visual key): sum over deciders of exp2(logit - logsumexp), one row
//                     per head; a small third kernel adds the H rows in head order (no atomics)
//
// bf16 path: logits on MFMA 16x16x32 (rows = 16 deciders, cols = 16 keys, contraction = dh), both
// operands read straight from HBM/L2 in the MFMA operand layout (each lane reads dh/4 contiguous
// elements of its row; the contraction index is permuted identically for both operands, which a
// dot product does not see).  Everything is bandwidth bound: K is streamed twice, the second time
// usually from the memory-side cache; with many deciders (64 and up) the exp2 / max arithmetic per logit
// becomes a comparable share of the run time.
//
// The generic path (any float type / head size) is a plain one-thread-per-output kernel pair.
#include <mutex>
#include "internal.hpp"

namespace d3tom {

// keys per workgroup (4 waves x SUB sub-tiles x 16): every workgroup re-fetches the decider rows of its
// head, so few large chunks (one workgroup per CU at 3.7k tokens x 32 heads) beat many small ones; when
// 512-key chunks would leave CUs idle (short sequences) the first sweep takes 256-key chunks instead
// (8.5 instead of 11.5 us at 1152 tokens)
constexpr int IMP_KC_STATS = 512;
constexpr int IMP_KC_SCORES = 512, IMP_SUB_SCORES = IMP_KC_SCORES / (4 * 16);

constexpr int IMP_KEEP_MAXD_WS = 32;   // largest decider set whose logits are kept (workspace is sized for it)
struct ImpWs {
    size_t part_off, sp_off, cnt_off, c_off, logit_off, total;
    int KC, NCH, NCHV, DPAD, VPAD, NKB;
};
__host__ inline ImpWs imp_ws_layout(int B, int max_N, int max_V, int H, int max_D) {
    ImpWs w;
    w.KC = ((long)ceil_div(max_N, IMP_KC_STATS) * H * B < 256) ? IMP_KC_STATS / 2 : IMP_KC_STATS;     // keys per chunk of the first sweep
    w.NCH = ceil_div(max_N, w.KC);
    w.NCHV = ceil_div(max_V, IMP_KC_SCORES);
    w.DPAD = ceil_div(max_D, 16) * 16;
    w.VPAD = w.NCHV * IMP_KC_SCORES;
    size_t o = 0;
    w.part_off = o; o += align_up((size_t)B * H * w.NCH * w.DPAD * sizeof(float2), 256);
    w.sp_off = o;   o += align_up((size_t)B * H * w.VPAD * sizeof(float), 256);
    w.cnt_off = o;  o += align_up((size_t)B * w.NCHV * sizeof(int), 256);
    w.c_off = o;    o += align_up((size_t)B * H * max_D * sizeof(float), 256);   // generic path
    w.NKB = w.NCH * (w.KC / 16);
    w.logit_off = o;                                                              // kept logits (small decider sets)
    if (max_D <= IMP_KEEP_MAXD_WS) o += align_up((size_t)B * w.NKB * H * w.DPAD * 16 * sizeof(float), 256);
    w.total = o;
    return w;
}
size_t importance_ws_bytes(int B, int max_N, int max_V, int H, int dh, int max_D) {
    (void)dh;
    // a workspace sized for a bound on the decider count must also serve every smaller count: small sets
    // keep their logits, which can take more room than the statistics of a large set
    const size_t a = imp_ws_layout(B, max_N, max_V, H, max_D).total;
    const size_t b = imp_ws_layout(B, max_N, max_V, H, max_D < IMP_KEEP_MAXD_WS ? max_D : IMP_KEEP_MAXD_WS).total;
    return a > b ? a : b;
}

// Load one MFMA operand row fragment: lane (r = lane % 16, g = lane / 16) takes elements
// [kk*32 + g*8, +8) of its row for k-step kk, so the four lanes of a row fetch 64 contiguous bytes per
// load instruction.
template <int DH>
__device__ __forceinline__ void load_frag(const uint16_t* row, int g, bool valid, bf16x8 (&f)[DH / 32]) {
    const bf16x8* p = reinterpret_cast<const bf16x8*>(row + g * 8);
#pragma unroll
    for (int kk = 0; kk < DH / 32; ++kk) {
        bf16x8 z = {0, 0, 0, 0, 0, 0, 0, 0};
        f[kk] = valid ? p[kk * 4] : z;
    }
}

constexpr int IMP_NB = 4;       // 16-decider blocks whose query fragments are fetched together

// (running max, running sum of exp2) of decider rows over one chunk of IMP_SUB_STATS x 64 keys of one head
template <int DH, bool KEEP, int IMP_SUB_STATS>
__global__ __launch_bounds__(256) void imp_stats_bf16(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ k, int H, float scale2,
    const int32_t* __restrict__ seq_off, const int32_t* __restrict__ dec_idx, const int32_t* __restrict__ dec_off,
    int max_D, int DPAD, int NCH, float2* __restrict__ part, int NKB, float* __restrict__ logits) {
    constexpr int KS = DH / 32;
    // heads vary fastest over the grid: workgroups that run together read neighbouring 2*DH-byte pieces of the same key rows
    const int h = blockIdx.x, chunk = blockIdx.y, b = blockIdx.z;
    const int tok0 = seq_off[b];
    constexpr int KC = IMP_SUB_STATS * 64;
    const int N = min(seq_off[b + 1] - tok0, NCH * KC);               // the workspace holds NCH chunks per head
    const int D = min(dec_off[b + 1] - dec_off[b], max_D);
    const int32_t* dec = dec_idx + dec_off[b];
    const int key_base = chunk * KC;
    if (key_base >= N || D <= 0) return;

    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, r = lane & 15, g = lane >> 4;
    __shared__ float2 wstat[4][D3TOM_MAX_DECIDERS];

    // decider positions of the first group are requested before the key fragments, so that the
    // position -> query-row chain runs beside the key loads instead of behind them
    int pos0[IMP_NB];
#pragma unroll
    for (int nb = 0; nb < IMP_NB; ++nb) pos0[nb] = (nb * 16 + r < D) ? dec[nb * 16 + r] : 0;

    bf16x8 kf[IMP_SUB_STATS][KS];
    bool kvalid[IMP_SUB_STATS];
#pragma unroll
    for (int s = 0; s < IMP_SUB_STATS; ++s) {
        const int key = key_base + (wave * IMP_SUB_STATS + s) * 16 + r;
        kvalid[s] = key < N;
        const uint16_t* row = k + ((size_t)(tok0 + (kvalid[s] ? key : 0)) * H + h) * DH;
        load_frag<DH>(row, g, kvalid[s], kf[s]);
    }
    const int nblk = (D + 15) >> 4;
    for (int db0 = 0; db0 < nblk; db0 += IMP_NB) {
        bf16x8 qf[IMP_NB][KS];
#pragma unroll
        for (int nb = 0; nb < IMP_NB; ++nb) {
            const int i = (db0 + nb) * 16 + r;
            const bool qv = i < D;
            const int pos = min(max(db0 == 0 ? pos0[nb] : (qv ? dec[i] : 0), 0), N - 1);
            load_frag<DH>(q + ((size_t)(tok0 + pos) * H + h) * DH, g, qv, qf[nb]);
        }
#pragma unroll
        for (int nb = 0; nb < IMP_NB; ++nb) {
            if (db0 + nb >= nblk) break;
            // l2[s][e]: scaled logit of decider row (db0+nb)*16 + 4g + e and key column r of sub-tile s
            f32x4 l2[IMP_SUB_STATS];
#pragma unroll
            for (int s = 0; s < IMP_SUB_STATS; ++s) {
                f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int kk = 0; kk < KS; ++kk)
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qf[nb][kk], kf[s][kk], acc, 0, 0, 0);
#pragma unroll
                for (int e = 0; e < 4; ++e) l2[s][e] = kvalid[s] ? acc[e] * scale2 : -INFINITY;
                if constexpr (KEEP) {
                    // [key block][head][decider][key in block]: the 16 lanes of a decider row write 64 contiguous bytes
                    const int kb = (key_base >> 4) + wave * IMP_SUB_STATS + s;
                    float* lp = logits + (((size_t)(b * NKB + kb) * H + h) * DPAD + (db0 + nb) * 16 + 4 * g) * 16 + r;
#pragma unroll
                    for (int e = 0; e < 4; ++e) lp[e * 16] = l2[s][e];
                }
            }
            // max over this wave's 64 keys first (in-lane, then the 16 key columns), then one exp2 per logit
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                float mx = l2[0][e];
#pragma unroll
                for (int s = 1; s < IMP_SUB_STATS; ++s) mx = fmaxf(mx, l2[s][e]);
                mx = row16_max(mx);
                float zz = 0.f;
                if (mx != -INFINITY) {
#pragma unroll
                    for (int s = 0; s < IMP_SUB_STATS; ++s) zz += __builtin_amdgcn_exp2f(l2[s][e] - mx);
                }
                zz = row16_sum(zz);
                if (r == 0) wstat[wave][(db0 + nb) * 16 + 4 * g + e] = make_float2(mx, zz);
            }
        }
    }
    __syncthreads();
    for (int t = threadIdx.x; t < nblk * 16; t += 256) {
        float2 a = wstat[0][t];
#pragma unroll
        for (int w = 1; w < 4; ++w) lse2_combine_fast(a.x, a.y, wstat[w][t].x, wstat[w][t].y);
        part[((size_t)(b * H + h) * NCH + chunk) * DPAD + t] = a;
    }
}

// per-head score rows: sp[h][j] = sum over deciders of exp2(logit - log2sumexp2)
template <int DH>
__global__ __launch_bounds__(256) void imp_scores_bf16(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ k, int H, float scale2,
    const int32_t* __restrict__ seq_off, const int32_t* __restrict__ dec_idx, const int32_t* __restrict__ dec_off,
    const int32_t* __restrict__ vis_start, const int32_t* __restrict__ vis_count,
    int max_D, int max_V, int DPAD, int NCH, int KC, int VPAD, const float2* __restrict__ part, float* __restrict__ sp) {
    constexpr int KS = DH / 32;
    // heads vary fastest over the grid: workgroups that run together read neighbouring 2*DH-byte pieces of the same key rows
    const int h = blockIdx.x, chunk = blockIdx.y, b = blockIdx.z;
    const int tok0 = seq_off[b];
    const int N = min(seq_off[b + 1] - tok0, NCH * KC);
    const int D = min(dec_off[b + 1] - dec_off[b], max_D);
    const int32_t* dec = dec_idx + dec_off[b];
    const int vs = min(max(vis_start[b], 0), N);
    const int V = min(min(vis_count[b], max_V), N - vs);
    const int key_base = chunk * IMP_KC_SCORES;
    if (key_base >= V || D <= 0) return;

    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, r = lane & 15, g = lane >> 4;
    __shared__ float c_lds[D3TOM_MAX_DECIDERS];

    int pos0[IMP_NB];
#pragma unroll
    for (int nb = 0; nb < IMP_NB; ++nb) pos0[nb] = (nb * 16 + r < D) ? dec[nb * 16 + r] : 0;
    // log2-sum-exp2 of every decider row of this head, key chunks combined in ascending order
    const int nch = (N + KC - 1) / KC;
    for (int t = threadIdx.x; t < D; t += 256) {
        const float2* p = part + ((size_t)(b * H + h) * NCH) * DPAD + t;
        float m = -INFINITY, z = 0.f;
        for (int c0 = 0; c0 < nch; c0 += 16) {             // 16 independent loads in flight, combined in order
            float2 a[16];
#pragma unroll
            for (int u = 0; u < 16; ++u) a[u] = (c0 + u < nch) ? p[(size_t)(c0 + u) * DPAD] : make_float2(-INFINITY, 0.f);
#pragma unroll
            for (int u = 0; u < 16; ++u) lse2_combine_fast(m, z, a[u].x, a[u].y);
        }
        c_lds[t] = m + __builtin_amdgcn_logf(z);
    }
    bf16x8 kf[IMP_SUB_SCORES][KS];
    float acc_s[IMP_SUB_SCORES];
#pragma unroll
    for (int s = 0; s < IMP_SUB_SCORES; ++s) {
        const int j = key_base + (wave * IMP_SUB_SCORES + s) * 16 + r;
        const bool kv = j < V;
        const uint16_t* row = k + ((size_t)(tok0 + vs + (kv ? j : 0)) * H + h) * DH;
        load_frag<DH>(row, g, kv, kf[s]);
        acc_s[s] = 0.f;
    }
    __syncthreads();

    const int nblk = (D + 15) >> 4;
    for (int db0 = 0; db0 < nblk; db0 += IMP_NB) {
        bf16x8 qf[IMP_NB][KS];
#pragma unroll
        for (int nb = 0; nb < IMP_NB; ++nb) {
            const int i = (db0 + nb) * 16 + r;
            const bool qv = i < D;
            const int pos = min(max(db0 == 0 ? pos0[nb] : (qv ? dec[i] : 0), 0), N - 1);
            load_frag<DH>(q + ((size_t)(tok0 + pos) * H + h) * DH, g, qv, qf[nb]);
        }
#pragma unroll
        for (int nb = 0; nb < IMP_NB; ++nb) {
            if (db0 + nb >= nblk) break;
            float cc[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int row = (db0 + nb) * 16 + 4 * g + e;
                cc[e] = (row < D) ? c_lds[row] : INFINITY;       // padded rows contribute exp2(-inf) = 0
            }
#pragma unroll
            for (int s = 0; s < IMP_SUB_SCORES; ++s) {
                f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int kk = 0; kk < KS; ++kk)
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qf[nb][kk], kf[s][kk], acc, 0, 0, 0);
#pragma unroll
                for (int e = 0; e < 4; ++e) acc_s[s] += __builtin_amdgcn_exp2f(__builtin_fmaf(acc[e], scale2, -cc[e]));
            }
        }
    }
    float* sp_row = sp + (size_t)(b * H + h) * VPAD;
#pragma unroll
    for (int s = 0; s < IMP_SUB_SCORES; ++s) {
        float v = acc_s[s];
        v += __shfl_xor(v, 16, WAVE);
        v += __shfl_xor(v, 32, WAVE);
        if (g == 0) sp_row[key_base + (wave * IMP_SUB_SCORES + s) * 16 + r] = v;
    }
}

// Small decider sets (at most IMP_KEEP_MAXD): the first sweep also writes its scaled logits, D x N x H
// floats (a quarter of K's bytes at 16 deciders), in blocks of [16 keys' block][head][decider][16 keys], and
// the scores come from those instead of a second sweep over K: one workgroup per 16-key block reads its
// contiguous H x D x 64 bytes, subtracts each (head, decider) row's log-sum-exp and adds the exponentials
// over deciders and heads, so the mean over heads is finished in the same pass (no per-head rows, no
// third launch, K fetched once).
constexpr int IMP_KEEP_MAXD = IMP_KEEP_MAXD_WS;
__global__ __launch_bounds__(256) void imp_scores_from_logits(
    int H, const int32_t* __restrict__ seq_off, const int32_t* __restrict__ dec_off,
    const int32_t* __restrict__ vis_start, const int32_t* __restrict__ vis_count, const int32_t* __restrict__ score_off,
    int max_D, int max_V, int DPAD, int NCH, int KC, int NKB, const float2* __restrict__ part, const float* __restrict__ logits,
    float* __restrict__ scores) {
    const int kb = blockIdx.x, b = blockIdx.y;
    const int N = min(seq_off[b + 1] - seq_off[b], NCH * KC);
    const int D = min(dec_off[b + 1] - dec_off[b], max_D);
    const int vs = min(max(vis_start[b], 0), N);
    const int V = min(min(vis_count[b], max_V), N - vs);
    const int key0 = kb * 16;
    if (D <= 0 || key0 >= vs + V || key0 + 16 <= vs || key0 >= N) return;
    extern __shared__ float c_lds[];                    // [H][DPAD] log2-sum-exp2, +inf for padded decider rows
    __shared__ float red[16][16];
    constexpr int NBK = IMP_KEEP_MAXD / 16;             // 16-decider blocks a kept set can have
    const int nblk = (D + 15) >> 4;                     // decider blocks the first sweep has written
    // thread (key = t % 16, group = t / 16) takes decider row 16 ib + group of every head: the 256 threads
    // read whole 1 KB blocks of logits.  All loads of up to 32 heads are requested before anything else, so
    // their latency (the logits come from another XCD's writes, i.e. from memory) overlaps the statistics below.
    const int key = threadIdx.x & 15, grp = threadIdx.x >> 4;
    const float* lb = logits + ((size_t)(b * NKB + kb) * H) * DPAD * 16 + (size_t)grp * 16 + key;
    float l[32][NBK];
#pragma unroll
    for (int h = 0; h < 32; ++h)
#pragma unroll
        for (int ib = 0; ib < NBK; ++ib)
            l[h][ib] = (h < H && ib < nblk) ? lb[((size_t)h * DPAD + ib * 16) * 16] : -INFINITY;
    const int nch = min((N + KC - 1) / KC, NCH);
    for (int t = threadIdx.x; t < H * nblk * 16; t += 256) {
        const int h = t / (nblk * 16), i = t - h * (nblk * 16);
        float c = INFINITY;
        if (i < D) {
            const float2* p = part + ((size_t)(b * H + h) * NCH) * DPAD + i;
            float m = -INFINITY, z = 0.f;
            for (int c0 = 0; c0 < nch; c0 += 8) {           // 8 independent loads in flight, combined in chunk order
                float2 a[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) a[u] = (c0 + u < nch) ? p[(size_t)(c0 + u) * DPAD] : make_float2(-INFINITY, 0.f);
#pragma unroll
                for (int u = 0; u < 8; ++u)
                    if (c0 + u < nch) lse2_combine_fast(m, z, a[u].x, a[u].y);
            }
            c = m + __builtin_amdgcn_logf(z);
        }
        c_lds[h * DPAD + i] = c;
    }
    __syncthreads();
    float acc = 0.f;
#pragma unroll
    for (int h = 0; h < 32; ++h)
#pragma unroll
        for (int ib = 0; ib < NBK; ++ib)
            if (h < H && ib < nblk) acc += __builtin_amdgcn_exp2f(l[h][ib] - c_lds[h * DPAD + ib * 16 + grp]);
    for (int h0 = 32; h0 < H; h0 += 32) {               // more than 32 heads: the same, 32 heads at a time
        float l2[32][NBK];
#pragma unroll
        for (int h = 0; h < 32; ++h)
#pragma unroll
            for (int ib = 0; ib < NBK; ++ib)
                l2[h][ib] = (h0 + h < H && ib < nblk) ? lb[((size_t)(h0 + h) * DPAD + ib * 16) * 16] : -INFINITY;
#pragma unroll
        for (int h = 0; h < 32; ++h)
#pragma unroll
            for (int ib = 0; ib < NBK; ++ib)
                if (h0 + h < H && ib < nblk) acc += __builtin_amdgcn_exp2f(l2[h][ib] - c_lds[(h0 + h) * DPAD + ib * 16 + grp]);
    }
    red[grp][key] = acc;
    __syncthreads();
    const int j = key0 + (int)threadIdx.x - vs;          // visual index of key threadIdx.x of this block
    if (threadIdx.x < 16 && j >= 0 && j < V) {
        float sum = 0.f;
#pragma unroll
        for (int gq = 0; gq < 16; ++gq) sum += red[gq][threadIdx.x];      // groups in ascending order
        scores[score_off[b] + j] = sum / (float)H;
    }
}

// S_j = mean over heads of the per-head rows, heads added in ascending order
__global__ __launch_bounds__(256) void imp_finish_kernel(
    const float* __restrict__ sp, int H, int VPAD, const int32_t* __restrict__ seq_off,
    const int32_t* __restrict__ vis_start, const int32_t* __restrict__ vis_count, const int32_t* __restrict__ score_off,
    int max_V, float* __restrict__ scores) {
    const int b = blockIdx.y, j = blockIdx.x * 256 + threadIdx.x;
    const int N = seq_off[b + 1] - seq_off[b];
    const int vs = min(max(vis_start[b], 0), N);
    const int V = min(min(vis_count[b], max_V), N - vs);
    if (j >= V) return;
    float s = 0.f;
    for (int h0 = 0; h0 < H; h0 += 32) {                   // 32 independent loads in flight, added in head order
        float a[32];
#pragma unroll
        for (int u = 0; u < 32; ++u) a[u] = (h0 + u < H) ? sp[(size_t)(b * H + h0 + u) * VPAD + j] : 0.f;
#pragma unroll
        for (int u = 0; u < 32; ++u) s += a[u];
    }
    scores[score_off[b] + j] = s / (float)H;
}

// ---------------------------------------------------------------------------------------------
// generic path: one workgroup per (decider, head) for the stats, one thread per visual key for
// the scores.  Plain float arithmetic, any head size up to 256.
// ---------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void imp_stats_generic(
    const T* __restrict__ q, const T* __restrict__ k, int H, int dh, float scale2,
    const int32_t* __restrict__ seq_off, const int32_t* __restrict__ dec_idx, const int32_t* __restrict__ dec_off,
    int max_D, float* __restrict__ cws) {
    const int i = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int tok0 = seq_off[b];
    const int N = seq_off[b + 1] - tok0;
    const int D = min(dec_off[b + 1] - dec_off[b], max_D);
    if (i >= D) return;
    __shared__ float qs[256];
    __shared__ float2 red[4];
    const int pos = min(max(dec_idx[dec_off[b] + i], 0), N - 1);
    for (int c = threadIdx.x; c < dh; c += 256) qs[c] = Elem<T>::load(q + ((size_t)(tok0 + pos) * H + h) * dh + c);
    __syncthreads();
    float m = -INFINITY, z = 0.f;
    for (int j = threadIdx.x; j < N; j += 256) {
        const T* kr = k + ((size_t)(tok0 + j) * H + h) * dh;
        float s = 0.f;
        for (int c = 0; c < dh; ++c) s += qs[c] * Elem<T>::load(kr + c);
        lse2_combine(m, z, s * scale2, 1.0f);
    }
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const float m2 = __shfl_xor(m, o, WAVE), z2 = __shfl_xor(z, o, WAVE);
        lse2_combine(m, z, m2, z2);
    }
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = make_float2(m, z);
    __syncthreads();
    if (threadIdx.x == 0) {
        float2 a = red[0];
        for (int w = 1; w < 4; ++w) lse2_combine(a.x, a.y, red[w].x, red[w].y);
        cws[(size_t)(b * H + h) * max_D + i] = a.x + log2f(a.y);
    }
}

template <typename T>
__global__ __launch_bounds__(256) void imp_scores_generic(
    const T* __restrict__ q, const T* __restrict__ k, int H, int dh, float scale2,
    const int32_t* __restrict__ seq_off, const int32_t* __restrict__ dec_idx, const int32_t* __restrict__ dec_off,
    const int32_t* __restrict__ vis_start, const int32_t* __restrict__ vis_count, const int32_t* __restrict__ score_off,
    int max_D, int max_V, const float* __restrict__ cws, float* __restrict__ scores) {
    const int b = blockIdx.y;
    const int j = blockIdx.x * 256 + threadIdx.x;
    const int tok0 = seq_off[b];
    const int N = seq_off[b + 1] - tok0;
    const int D = min(dec_off[b + 1] - dec_off[b], max_D);
    const int vs = min(max(vis_start[b], 0), N);
    const int V = min(min(vis_count[b], max_V), N - vs);
    if (j >= V || D <= 0) return;
    float acc = 0.f;
    for (int h = 0; h < H; ++h) {
        const T* kr = k + ((size_t)(tok0 + vs + j) * H + h) * dh;
        for (int i = 0; i < D; ++i) {
            const int pos = min(max(dec_idx[dec_off[b] + i], 0), N - 1);
            const T* qr = q + ((size_t)(tok0 + pos) * H + h) * dh;
            float s = 0.f;
            for (int c = 0; c < dh; ++c) s += Elem<T>::load(qr + c) * Elem<T>::load(kr + c);
            acc += exp2f(s * scale2 - cws[(size_t)(b * H + h) * max_D + i]);
        }
    }
    scores[score_off[b] + j] = acc / (float)H;
}

}  // namespace d3tom

using namespace d3tom;

// Host-side argument checks shared by the entry points (everything except the workspace).
int d3tom::importance_check(const void* q, const void* k, int dt, int B, const int32_t* seq_off, int H, int dh, float scale,
                            const int32_t* dec_idx, const int32_t* dec_off, int min_D, int max_D,
                            const int32_t* vis_start, const int32_t* vis_count, const int32_t* score_off,
                            int max_N, int max_V, const float* scores) {
    if (!q || !k || !seq_off || !dec_idx || !dec_off || !vis_start || !vis_count || !score_off || !scores)
        return D3TOM_ERR_INVALID_ARG;
    if (B < 1 || H < 1 || dh < 1 || max_N < 1 || max_V < 1 || max_V > max_N || min_D < 0 || max_D < min_D)
        return D3TOM_ERR_INVALID_ARG;
    if (dt != D3TOM_F32 && dt != D3TOM_BF16) return D3TOM_ERR_INVALID_ARG;
    if (!(scale > 0.f) || !(scale < 3.0e38f)) return D3TOM_ERR_INVALID_ARG;
    if (!aligned16(q) || !aligned16(k)) return D3TOM_ERR_INVALID_ARG;
    if (min_D == 0) return D3TOM_ERR_NO_DECIDERS;
    if (max_D > D3TOM_MAX_DECIDERS) return D3TOM_ERR_UNSUPPORTED;
    if (dh > 256 || (dt == D3TOM_BF16 ? (dh % 8) : (dh % 4))) return D3TOM_ERR_UNSUPPORTED;
    return D3TOM_OK;
}

// The launches; arguments and workspace have been checked.
int d3tom::importance_run(const void* q, const void* k, int dt,
                          int B, const int32_t* seq_off, int H, int dh, float scale,
                          const int32_t* dec_idx, const int32_t* dec_off, int max_D,
                          const int32_t* vis_start, const int32_t* vis_count, const int32_t* score_off,
                          int max_N, int max_V, float* scores, void* ws, void* stream) {
    const ImpWs w = imp_ws_layout(B, max_N, max_V, H, max_D);
    hipStream_t st = (hipStream_t)stream;
    char* wsb = (char*)ws;
    const float scale2 = scale * LOG2E;

    if (dt == D3TOM_BF16 && (dh == 128 || dh == 64)) {
        float2* part = (float2*)(wsb + w.part_off);
        float* sp = (float*)(wsb + w.sp_off);
        const dim3 g1(H, w.NCH, B), g2(H, w.NCHV, B), g3(ceil_div(max_V, 256), B);
        const uint16_t* qq = (const uint16_t*)q;
        const uint16_t* kk = (const uint16_t*)k;
        // small decider sets: the first sweep keeps its logits and the scores come from them (K fetched once)
        const bool keep = max_D <= IMP_KEEP_MAXD;
        float* logits = (float*)(wsb + w.logit_off);
#define D3TOM_IMP_STATS(DHV, KEEPV, SUBV)                                                                     \
    D3TOM_LAUNCH(IMP_STATS, st, (imp_stats_bf16<DHV, KEEPV, SUBV><<<g1, 256, 0, st>>>(                           \
        qq, kk, H, scale2, seq_off, dec_idx, dec_off, max_D, w.DPAD, w.NCH, part, w.NKB, logits)))
        const bool big = w.KC == IMP_KC_STATS;
        if (dh == 128) {
            if (keep) { if (big) D3TOM_IMP_STATS(128, true, 8); else D3TOM_IMP_STATS(128, true, 4); }
            else      { if (big) D3TOM_IMP_STATS(128, false, 8); else D3TOM_IMP_STATS(128, false, 4); }
        } else {
            if (keep) { if (big) D3TOM_IMP_STATS(64, true, 8); else D3TOM_IMP_STATS(64, true, 4); }
            else      { if (big) D3TOM_IMP_STATS(64, false, 8); else D3TOM_IMP_STATS(64, false, 4); }
        }
#undef D3TOM_IMP_STATS
        if (keep) {
            const dim3 g2k(ceil_div(max_N, 16), B);
            D3TOM_LAUNCH(IMP_SCORES, st, imp_scores_from_logits<<<g2k, 256, (size_t)H * w.DPAD * sizeof(float), st>>>(
                H, seq_off, dec_off, vis_start, vis_count, score_off, max_D, max_V, w.DPAD, w.NCH, w.KC, w.NKB, part, logits,
                scores));
            return D3TOM_OK;
        }
        if (dh == 128)
            D3TOM_LAUNCH(IMP_SCORES, st, imp_scores_bf16<128><<<g2, 256, 0, st>>>(
                qq, kk, H, scale2, seq_off, dec_idx, dec_off, vis_start, vis_count, max_D, max_V, w.DPAD, w.NCH, w.KC, w.VPAD,
                part, sp));
        else
            D3TOM_LAUNCH(IMP_SCORES, st, imp_scores_bf16<64><<<g2, 256, 0, st>>>(
                qq, kk, H, scale2, seq_off, dec_idx, dec_off, vis_start, vis_count, max_D, max_V, w.DPAD, w.NCH, w.KC, w.VPAD,
                part, sp));
        D3TOM_LAUNCH(IMP_FINISH, st, imp_finish_kernel<<<g3, 256, 0, st>>>(
            sp, H, w.VPAD, seq_off, vis_start, vis_count, score_off, max_V, scores));
        return D3TOM_OK;
    }
    float* cws = (float*)(wsb + w.c_off);
    const dim3 g1(max_D, H, B), g2(ceil_div(max_V, 256), B);
    if (dt == D3TOM_F32) {
        D3TOM_LAUNCH(IMP_STATS, st, imp_stats_generic<float><<<g1, 256, 0, st>>>(
            (const float*)q, (const float*)k, H, dh, scale2, seq_off, dec_idx, dec_off, max_D, cws));
        D3TOM_LAUNCH(IMP_SCORES, st, imp_scores_generic<float><<<g2, 256, 0, st>>>(
            (const float*)q, (const float*)k, H, dh, scale2, seq_off, dec_idx, dec_off, vis_start, vis_count, score_off,
            max_D, max_V, cws, scores));
    } else {
        D3TOM_LAUNCH(IMP_STATS, st, imp_stats_generic<uint16_t><<<g1, 256, 0, st>>>(
            (const uint16_t*)q, (const uint16_t*)k, H, dh, scale2, seq_off, dec_idx, dec_off, max_D, cws));
        D3TOM_LAUNCH(IMP_SCORES, st, imp_scores_generic<uint16_t><<<g2, 256, 0, st>>>(
            (const uint16_t*)q, (const uint16_t*)k, H, dh, scale2, seq_off, dec_idx, dec_off, vis_start, vis_count,
            score_off, max_D, max_V, cws, scores));
    }
    return D3TOM_OK;
}

extern "C" int d3tom_importance(const void* q, const void* k, int dt,
                                int B, const int32_t* seq_off, int H, int dh, float scale,
                                const int32_t* dec_idx, const int32_t* dec_off, int min_D, int max_D,
                                const int32_t* vis_start, const int32_t* vis_count, const int32_t* score_off,
                                int max_N, int max_V,
                                float* scores, void* ws, size_t ws_bytes, void* stream) {
    const int rc = importance_check(q, k, dt, B, seq_off, H, dh, scale, dec_idx, dec_off, min_D, max_D, vis_start,
                                    vis_count, score_off, max_N, max_V, scores);
    if (rc != D3TOM_OK) return rc;
    const ImpWs w = imp_ws_layout(B, max_N, max_V, H, max_D);
    if (!ws || ws_bytes < w.total || (((uintptr_t)ws) & 255u)) return ws ? D3TOM_ERR_WORKSPACE_TOO_SMALL : D3TOM_ERR_INVALID_ARG;
    return importance_run(q, k, dt, B, seq_off, H, dh, scale, dec_idx, dec_off, max_D, vis_start, vis_count, score_off,
                          max_N, max_V, scores, ws, stream);
}

// ---- the same call for callers that cannot allocate ---------------------------------------------
// The workspace is a file-scope device array instead of a caller buffer.  Every GPU the library runs on
// holds its own copy of the array at its own address; host code never uses the array's name as an
// address (it is a host-side stand-in) but the device address of the current GPU's copy, asked for
// once per device and kept.
static __device__ __align__(256) unsigned char scratch[D3TOM_IMPORTANCE_STATIC_BYTES];

namespace {
constexpr int MAX_GPUS = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[MAX_GPUS] = {};
}

extern "C" int d3tom_importance_static(const void* q, const void* k, int dt,
                                       int B, const int32_t* seq_off, int H, int dh, float scale,
                                       const int32_t* dec_idx, const int32_t* dec_off, int min_D, int max_D,
                                       const int32_t* vis_start, const int32_t* vis_count, const int32_t* score_off,
                                       int max_N, int max_V, float* scores, void* stream) {
    const int rc = importance_check(q, k, dt, B, seq_off, H, dh, scale, dec_idx, dec_off, min_D, max_D, vis_start,
                                    vis_count, score_off, max_N, max_V, scores);
    if (rc != D3TOM_OK) return rc;
    if (imp_ws_layout(B, max_N, max_V, H, max_D).total > (size_t)D3TOM_IMPORTANCE_STATIC_BYTES) return D3TOM_ERR_UNSUPPORTED;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_GPUS) return D3TOM_ERR_DEVICE;
    void* ptr = nullptr;
    {
        std::lock_guard<std::mutex> lk(g_scratch_mu);
        if (!g_scratch_ptr[dev]) {
            void* p = nullptr;
            if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return D3TOM_ERR_DEVICE;
            g_scratch_ptr[dev] = p;
        }
        ptr = g_scratch_ptr[dev];
    }
    return importance_run(q, k, dt, B, seq_off, H, dh, scale, dec_idx, dec_off, max_D, vis_start, vis_count, score_off,
                          max_N, max_V, scores, ptr, stream);
}
