// d3tom_attend: bidirectional (unmasked) attention over the shortened sequence (Section 3.2: the
// shortened tensor runs through the later layers; Section 4.3: the 2 n^2 d term of FLOPs_layer).
//
// bf16 path — flash-style, MFMA 32x32x16, written "transposed" so that everything per query stays
// inside one lane:
//     S^T = K Q^T      A = K tile (LDS, row-major), B = Q^T (registers, loaded once per workgroup)
//     P^T = exp2(S^T * scale*log2e - m)            in registers, the MFMA accumulator layout
//     O^T += V^T P^T   A = V^T tile (LDS, transposed while it is stored), B = P^T straight from the
//                      accumulator registers of the first product (no LDS round trip for P)
// In the accumulator layout a lane owns ONE query column (lane % 32) and 16 of the 32 key rows, so
// the running max / sum of the online softmax need one cross-lane exchange (lane ^ 32) per tile and
// the rescale of O^T is a per-lane scalar.  The contraction index of the second product (keys) is
// fed in the order the accumulator holds it; V^T is read from LDS in that same order.
//
// Workgroup = 4 waves x 32 queries of one head, 64 keys per LDS stage, global loads of the next
// stage overlap the MFMAs of the current one.  Softmax state and accumulators are float32.
//
// The generic path (float32 or any head size) is one workgroup per (query, head) with a chunked
// online softmax in plain float arithmetic.
#include "common.hpp"

namespace d3tom {

constexpr int ATT_BQ = 128;     // queries per workgroup
constexpr int ATT_BK = 64;      // keys per stage

template <int DH>
__global__ __launch_bounds__(256) void attend_bf16_kernel(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
    const int32_t* __restrict__ cu, int H, float scale2, uint16_t* __restrict__ o) {
    constexpr int KS = DH / 16;            // k-steps of the first product
    constexpr int DT = DH / 32;            // 32-dim tiles of O^T
    constexpr int K_LD = DH + 8;           // padded K row (elements)
    constexpr int V_LD = ATT_BK + 8;       // padded V^T row (elements)
    constexpr int K_CH = ATT_BK * (DH / 8) / 256;           // 16-byte chunks per thread, K tile
    constexpr int V_BLK = (ATT_BK / 4) * (DH / 8);          // 4-key x 8-dim blocks in a V tile
    constexpr int V_PT = (V_BLK + 255) / 256;

    const int qt = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int tok0 = cu[b];
    const int n = cu[b + 1] - tok0;
    if (qt * ATT_BQ >= n) return;

    __shared__ __attribute__((aligned(16))) uint16_t Ks[ATT_BK * K_LD];
    __shared__ __attribute__((aligned(16))) uint16_t Vt[DH * V_LD];

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int c = lane & 31, g = lane >> 5;
    const size_t rs = (size_t)H * DH;                      // token stride (elements)
    const uint16_t* kb = k + (size_t)tok0 * rs + (size_t)h * DH;
    const uint16_t* vb = v + (size_t)tok0 * rs + (size_t)h * DH;

    // Q^T fragments: lane (query c, g) holds dims kk*16 + 8g .. +7
    const int qrow = qt * ATT_BQ + wave * 32 + c;
    const bool qvalid = qrow < n;
    bf16x8 qf[KS];
    {
        const uint16_t* qp = q + (size_t)(tok0 + (qvalid ? qrow : 0)) * rs + (size_t)h * DH + g * 8;
#pragma unroll
        for (int kk = 0; kk < KS; ++kk) {
            bf16x8 z = {0, 0, 0, 0, 0, 0, 0, 0};
            qf[kk] = qvalid ? *reinterpret_cast<const bf16x8*>(qp + kk * 16) : z;
        }
    }
    f32x16 ot[DT];
#pragma unroll
    for (int t = 0; t < DT; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e) ot[t][e] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;

    uint4 k_reg[K_CH], v_reg[V_PT][4];
    auto load_tile = [&](int key0) {
#pragma unroll
        for (int i = 0; i < K_CH; ++i) {
            const int ch = tid + 256 * i, row = ch / (DH / 8), cc = ch % (DH / 8);
            const int key = key0 + row;
            k_reg[i] = (key < n) ? *reinterpret_cast<const uint4*>(kb + (size_t)key * rs + cc * 8) : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < V_PT; ++i) {
            const int blk = tid + 256 * i;
            if (blk < V_BLK) {
                const int kg = blk / (DH / 8), dg = blk % (DH / 8);
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) {
                    const int key = key0 + kg * 4 + jj;
                    v_reg[i][jj] = (key < n) ? *reinterpret_cast<const uint4*>(vb + (size_t)key * rs + dg * 8) : make_uint4(0, 0, 0, 0);
                }
            }
        }
    };
    auto store_tile = [&]() {
#pragma unroll
        for (int i = 0; i < K_CH; ++i) {
            const int ch = tid + 256 * i, row = ch / (DH / 8), cc = ch % (DH / 8);
            *reinterpret_cast<uint4*>(&Ks[row * K_LD + cc * 8]) = k_reg[i];
        }
#pragma unroll
        for (int i = 0; i < V_PT; ++i) {
            const int blk = tid + 256 * i;
            if (blk < V_BLK) {
                const int kg = blk / (DH / 8), dg = blk % (DH / 8);
                const uint32_t w0[4] = {v_reg[i][0].x, v_reg[i][0].y, v_reg[i][0].z, v_reg[i][0].w};
                const uint32_t w1[4] = {v_reg[i][1].x, v_reg[i][1].y, v_reg[i][1].z, v_reg[i][1].w};
                const uint32_t w2[4] = {v_reg[i][2].x, v_reg[i][2].y, v_reg[i][2].z, v_reg[i][2].w};
                const uint32_t w3[4] = {v_reg[i][3].x, v_reg[i][3].y, v_reg[i][3].z, v_reg[i][3].w};
#pragma unroll
                for (int p = 0; p < 4; ++p) {               // dims 8dg + 2p, 8dg + 2p + 1
                    uint2 lo, hi;
                    lo.x = (w0[p] & 0xFFFFu) | (w1[p] << 16);
                    lo.y = (w2[p] & 0xFFFFu) | (w3[p] << 16);
                    hi.x = (w0[p] >> 16) | (w1[p] & 0xFFFF0000u);
                    hi.y = (w2[p] >> 16) | (w3[p] & 0xFFFF0000u);
                    *reinterpret_cast<uint2*>(&Vt[(dg * 8 + 2 * p) * V_LD + kg * 4]) = lo;
                    *reinterpret_cast<uint2*>(&Vt[(dg * 8 + 2 * p + 1) * V_LD + kg * 4]) = hi;
                }
            }
        }
    };

    const int ntile = (n + ATT_BK - 1) / ATT_BK;
    load_tile(0);
    for (int it = 0; it < ntile; ++it) {
        const int key0 = it * ATT_BK;
        __syncthreads();                    // previous stage fully consumed
        store_tile();
        __syncthreads();
        if (it + 1 < ntile) load_tile(key0 + ATT_BK);

        // S^T = K Q^T for two 32-key tiles
        f32x16 st[2];
#pragma unroll
        for (int kt = 0; kt < 2; ++kt) {
#pragma unroll
            for (int e = 0; e < 16; ++e) st[kt][e] = 0.f;
#pragma unroll
            for (int kk = 0; kk < KS; ++kk) {
                const bf16x8 af = *reinterpret_cast<const bf16x8*>(&Ks[(kt * 32 + c) * K_LD + kk * 16 + g * 8]);
                st[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af, qf[kk], st[kt], 0, 0, 0);
            }
        }
        // online softmax (base 2); element e of st[kt]: key kt*32 + (e/4)*8 + 4g + e%4, query c
        float tmax = -INFINITY;
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int key = key0 + kt * 32 + (e >> 2) * 8 + g * 4 + (e & 3);
                const float s2 = (key < n) ? st[kt][e] * scale2 : -INFINITY;
                st[kt][e] = s2;
                tmax = fmaxf(tmax, s2);
            }
        tmax = fmaxf(tmax, __shfl_xor(tmax, 32, WAVE));
        const float m_new = fmaxf(m_run, tmax);            // finite: every stage holds >= 1 valid key
        const float alpha = exp2f(m_run - m_new);
        float psum = 0.f;
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const float p = exp2f(st[kt][e] - m_new);
                st[kt][e] = p;
                psum += p;
            }
        psum += __shfl_xor(psum, 32, WAVE);
        l_run = l_run * alpha + psum;
        m_run = m_new;
#pragma unroll
        for (int t = 0; t < DT; ++t)
#pragma unroll
            for (int e = 0; e < 16; ++e) ot[t][e] *= alpha;
        // O^T += V^T P^T
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
            for (int hh = 0; hh < 2; ++hh) {
                bf16x8 pf;
#pragma unroll
                for (int j = 0; j < 8; ++j) pf[j] = (__bf16)st[kt][hh * 8 + j];
                const int kofs = kt * 32 + hh * 16 + g * 4;          // keys kofs..+3 and kofs+8..+11
#pragma unroll
                for (int t = 0; t < DT; ++t) {
                    const uint16_t* vr = &Vt[(t * 32 + c) * V_LD + kofs];
                    const bf16x4 v0 = *reinterpret_cast<const bf16x4*>(vr);
                    const bf16x4 v1 = *reinterpret_cast<const bf16x4*>(vr + 8);
                    const bf16x8 vf = {v0[0], v0[1], v0[2], v0[3], v1[0], v1[1], v1[2], v1[3]};
                    ot[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf, ot[t], 0, 0, 0);
                }
            }
    }
    if (!qvalid) return;
    const float inv = 1.0f / l_run;
    uint16_t* op = o + (size_t)(tok0 + qrow) * rs + (size_t)h * DH;
#pragma unroll
    for (int t = 0; t < DT; ++t)
#pragma unroll
        for (int e4 = 0; e4 < 4; ++e4) {
            uint2 w;
            w.x = pack_bf16x2(ot[t][e4 * 4 + 0] * inv, ot[t][e4 * 4 + 1] * inv);
            w.y = pack_bf16x2(ot[t][e4 * 4 + 2] * inv, ot[t][e4 * 4 + 3] * inv);
            *reinterpret_cast<uint2*>(op + t * 32 + e4 * 8 + g * 4) = w;
        }
}

// generic: one workgroup per (query, head), keys in chunks of 256, plain float online softmax
template <typename T>
__global__ __launch_bounds__(256) void attend_generic_kernel(
    const T* __restrict__ q, const T* __restrict__ k, const T* __restrict__ v, const int32_t* __restrict__ cu,
    int H, int dh, float scale2, T* __restrict__ o) {
    const int i = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int tok0 = cu[b];
    const int n = cu[b + 1] - tok0;
    if (i >= n) return;
    __shared__ float qs[256];
    __shared__ float ps[256];
    __shared__ float red[8];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const size_t rs = (size_t)H * dh;
    for (int cidx = tid; cidx < dh; cidx += 256) qs[cidx] = Elem<T>::load(q + (size_t)(tok0 + i) * rs + (size_t)h * dh + cidx);
    __syncthreads();
    float m_run = -INFINITY, l_run = 0.f, acc = 0.f;
    for (int j0 = 0; j0 < n; j0 += 256) {
        const int j = j0 + tid;
        float s2 = -INFINITY;
        if (j < n) {
            const T* kr = k + (size_t)(tok0 + j) * rs + (size_t)h * dh;
            float s = 0.f;
            for (int cidx = 0; cidx < dh; ++cidx) s += qs[cidx] * Elem<T>::load(kr + cidx);
            s2 = s * scale2;
        }
        float wm = wave_max(s2);
        if (lane == 0) red[wave] = wm;
        __syncthreads();
        const float cmax = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
        const float m_new = fmaxf(m_run, cmax);
        const float alpha = exp2f(m_run - m_new);
        const float p = (j < n) ? exp2f(s2 - m_new) : 0.f;
        ps[tid] = p;
        float wsum = wave_sum(p);
        if (lane == 0) red[4 + wave] = wsum;
        __syncthreads();
        l_run = l_run * alpha + (red[4] + red[5] + red[6] + red[7]);
        m_run = m_new;
        if (tid < dh) {
            acc *= alpha;
            const int cnt = min(256, n - j0);
            const T* vr = v + (size_t)(tok0 + j0) * rs + (size_t)h * dh + tid;
            for (int t = 0; t < cnt; ++t) acc += ps[t] * Elem<T>::load(vr + (size_t)t * rs);
        }
        __syncthreads();
    }
    if (tid < dh) Elem<T>::store(o + (size_t)(tok0 + i) * rs + (size_t)h * dh + tid, acc / l_run);
}

}  // namespace d3tom

using namespace d3tom;

extern "C" int d3tom_attend(const void* q, const void* k, const void* v, int dt,
                            int B, const int32_t* cu_seqlens, int max_seqlen, int H, int dh, float scale,
                            void* o, void* ws, size_t ws_bytes, void* stream) {
    (void)ws; (void)ws_bytes;
    if (!q || !k || !v || !o || !cu_seqlens) return D3TOM_ERR_INVALID_ARG;
    if (B < 1 || max_seqlen < 1 || H < 1 || dh < 1) return D3TOM_ERR_INVALID_ARG;
    if (dt != D3TOM_F32 && dt != D3TOM_BF16) return D3TOM_ERR_INVALID_ARG;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o)) return D3TOM_ERR_INVALID_ARG;
    if (dh > 256 || (dt == D3TOM_BF16 ? (dh % 8) : (dh % 4))) return D3TOM_ERR_UNSUPPORTED;
    hipStream_t st = (hipStream_t)stream;
    const float scale2 = scale * LOG2E;
    if (dt == D3TOM_BF16 && (dh == 128 || dh == 64)) {
        const dim3 g(ceil_div(max_seqlen, ATT_BQ), H, B);
        if (dh == 128)
            D3TOM_LAUNCH(ATTEND, st, attend_bf16_kernel<128><<<g, 256, 0, st>>>(
                (const uint16_t*)q, (const uint16_t*)k, (const uint16_t*)v, cu_seqlens, H, scale2, (uint16_t*)o));
        else
            D3TOM_LAUNCH(ATTEND, st, attend_bf16_kernel<64><<<g, 256, 0, st>>>(
                (const uint16_t*)q, (const uint16_t*)k, (const uint16_t*)v, cu_seqlens, H, scale2, (uint16_t*)o));
    } else {
        const dim3 g(max_seqlen, H, B);
        if (dt == D3TOM_F32)
            D3TOM_LAUNCH(ATTEND, st, attend_generic_kernel<float><<<g, 256, 0, st>>>(
                (const float*)q, (const float*)k, (const float*)v, cu_seqlens, H, dh, scale2, (float*)o));
        else
            D3TOM_LAUNCH(ATTEND, st, attend_generic_kernel<uint16_t><<<g, 256, 0, st>>>(
                (const uint16_t*)q, (const uint16_t*)k, (const uint16_t*)v, cu_seqlens, H, dh, scale2, (uint16_t*)o));
    }
    return D3TOM_OK;
}
