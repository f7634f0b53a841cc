// d3tom_attend: bidirectional (unmasked) attention over the shortened sequence (Section 3.2: the
// shortened tensor runs through the later layers; Section 4.3: the 2 n^2 d term of FLOPs_layer).
//
// bf16 path — flash-style, MFMA 32x32x16, written "transposed" so that everything per query stays
// inside one lane:
//     S^T = K Q^T      A = K tile (LDS, row-major), B = Q^T (registers, loaded once per workgroup)
//     P^T = exp2(S^T * scale*log2e - m)            in registers, the MFMA accumulator layout
//     O^T += V^T P^T   A = V^T, read from the row-major V tile in LDS with the transposing LDS read
//                      (ds_read_b64_tr_b16), B = P^T straight from the accumulator registers of the
//                      first product (no LDS round trip for P)
// In the accumulator layout a lane owns ONE query column (lane % 32) and 16 of the 32 key rows, so
// the running max / sum of the online softmax need one cross-lane exchange (lane ^ 32) per tile and
// the rescale of O^T is a per-lane scalar.  The contraction index of the second product (keys) is
// fed in the order the accumulator holds it; V^T is read from LDS in that same order.
//
// Workgroup = 4 waves x 32 queries of one head, 64 keys per LDS stage.  K and V tiles go HBM/L2 -> LDS
// with direct loads (global_load_lds, no register staging) into a two-stage ring, so the loads of the
// next stage overlap the MFMAs of the current one and one s_barrier per stage suffices; rows are
// unpadded and their 16-byte chunks XOR-swizzled by the row index instead.  Softmax state and
// accumulators are float32; two workgroups fit a CU.
//
// The generic path (float32 or any head size) is one workgroup per (query, head) with a chunked
// online softmax in plain float arithmetic.
#include "common.hpp"

namespace d3tom {

constexpr int ATT_BQ = 128;     // queries per workgroup
constexpr int ATT_BK = 64;      // keys per stage
constexpr int ATT_NS = 2;       // LDS ring depth

typedef __attribute__((address_space(3))) void* att_lds_ptr_t;
typedef const __attribute__((address_space(1))) void* att_glb_ptr_t;
typedef __attribute__((__vector_size__(4 * sizeof(short)))) short att_short4;

// 4 keys x 16 dims of a row-major LDS tile, transposed on the way to the registers: within each group
// of 16 lanes, lanes 4j..4j+3 point at 4 x 4 consecutive elements of row j, and lane i receives
// column i of that 4 x 16 block (ds_read_b64_tr_b16).
__device__ __forceinline__ att_short4 lds_read_tr16(const char* p) {
    typedef __attribute__((address_space(3))) att_short4* lp;
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((lp)p);
}

template <int N>
__device__ __forceinline__ void att_wait_and_barrier() {
    if constexpr (N == 0) asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
    else {
        static_assert(N == 8, "add the wait count");
        asm volatile("s_waitcnt vmcnt(8) lgkmcnt(0)\n\ts_barrier" ::: "memory");
    }
}

template <int DH>
__global__ __launch_bounds__(256, 2) void attend_bf16_kernel(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
    const int32_t* __restrict__ cu, int H, int nB, int nqt, float scale2, uint16_t* __restrict__ o) {
    constexpr int KS = DH / 16;                 // k-steps of the first product
    constexpr int DT = DH / 32;                 // 32-dim tiles of O^T
    constexpr int ROWB = DH * 2;                // bytes per K / V row in LDS (unpadded, chunks swizzled)
    constexpr int NCHK = DH / 8;                // 16-byte chunks per row
    constexpr int RPI = 64 / NCHK;              // rows covered by one wave-wide direct load (1 KB)
    constexpr int LD = ATT_BK / (4 * RPI);      // direct loads per wave, per operand, per stage
    constexpr int TILE = ATT_BK * ROWB;         // bytes of one K (or V) tile
    constexpr int STAGE = 2 * TILE;
    extern __shared__ __attribute__((aligned(16))) char ring[];

    // Workgroup ids are dealt round-robin to the 8 XCDs; all query tiles of one (sample, head) are given
    // ids of the same residue so that the head's K and V are fetched into one XCD's L2 only.
    const int xcd = blockIdx.x & 7, li = blockIdx.x >> 3;
    const int hb = (li / nqt) * 8 + xcd, qt = li % nqt;         // hb = sample * H + head
    if (hb >= H * nB) return;
    const int h = hb % H, b = hb / H;
    const int tok0 = cu[b];
    const int n = cu[b + 1] - tok0;
    if (qt * ATT_BQ >= n) return;

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
    float m_run = -INFINITY, l_run = 0.f;       // running max of the RAW logits, running sum of exp2

    // direct loads: lane -> (row, chunk position); the chunk fetched into position p of row r is
    // p ^ (r & 15) for K (operand reads walk 16+ consecutive rows) and p ^ ((r & 3) * 4) for V
    // (transposing reads touch 4 consecutive rows per 16-lane group)
    const int ld_row = wave * (ATT_BK / 4) + lane / NCHK;       // + i * RPI
    const int ld_pos = lane % NCHK;
    auto issue = [&](int key0, int stage) {
        char* sb = ring + stage * STAGE;
#pragma unroll
        for (int i = 0; i < LD; ++i) {
            const int r = ld_row + i * RPI;
            const int key = min(key0 + r, n - 1);                // rows past the end re-read the last key (masked)
            const int kc = (ld_pos ^ (r & 15)) & (NCHK - 1);
            const int vc = (ld_pos ^ ((r & 3) * 4)) & (NCHK - 1);
            __builtin_amdgcn_global_load_lds((att_glb_ptr_t)(kb + (size_t)key * rs + kc * 8),
                                             (att_lds_ptr_t)(sb + (wave * (ATT_BK / 4) + i * RPI) * ROWB), 16, 0, 0);
            __builtin_amdgcn_global_load_lds((att_glb_ptr_t)(vb + (size_t)key * rs + vc * 8),
                                             (att_lds_ptr_t)(sb + TILE + (wave * (ATT_BK / 4) + i * RPI) * ROWB), 16, 0, 0);
        }
    };
    // transposing-read geometry of this lane: 16-lane group -> (g, dim half), lane in group -> (row j, 4-dim quad t)
    const int tr_j = (lane & 15) >> 2, tr_t = lane & 3, tr_half = (lane >> 4) & 1;

    const int ntile = (n + ATT_BK - 1) / ATT_BK;
    issue(0, 0);
    for (int it = 0; it < ntile; ++it) {
        const int key0 = it * ATT_BK;
        att_wait_and_barrier<0>();                             // stage `it` has landed; stage it-1 is free
        if (it + 1 < ntile) issue(key0 + ATT_BK, (it + 1) % ATT_NS);
        const char* sb = ring + (it % ATT_NS) * STAGE;

        // S^T = K Q^T for two 32-key tiles
        f32x16 st[2];
#pragma unroll
        for (int kt = 0; kt < 2; ++kt) {
#pragma unroll
            for (int e = 0; e < 16; ++e) st[kt][e] = 0.f;
            const int r = kt * 32 + c;
            const char* krow = sb + r * ROWB;
#pragma unroll
            for (int kk = 0; kk < KS; ++kk) {
                const bf16x8 af = *reinterpret_cast<const bf16x8*>(krow + ((((kk * 2 + g) ^ (r & 15)) & (NCHK - 1)) << 4));
                st[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af, qf[kk], st[kt], 0, 0, 0);
            }
        }
        // online softmax in base 2 on the raw logits; element e of st[kt]: key kt*32 + (e/4)*8 + 4g + e%4, query c
        if (key0 + ATT_BK > n) {
#pragma unroll
            for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int key = key0 + kt * 32 + (e >> 2) * 8 + g * 4 + (e & 3);
                    if (key >= n) st[kt][e] = -INFINITY;
                }
        }
        float tmax = st[0][0];
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
            for (int e = 0; e < 16; ++e) tmax = fmaxf(tmax, st[kt][e]);
        tmax = fmaxf(tmax, __shfl_xor(tmax, 32, WAVE));
        const float m_new = fmaxf(m_run, tmax);            // finite: every stage holds >= 1 valid key
        const float ms = m_new * scale2;
        float psum = 0.f;
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(st[kt][e], scale2, -ms));
                st[kt][e] = p;
                psum += p;
            }
        psum += __shfl_xor(psum, 32, WAVE);
        if (__builtin_amdgcn_ballot_w64(m_new > m_run) != 0) {      // some query of this wave moved its max
            const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * scale2);
            l_run *= alpha;
#pragma unroll
            for (int t = 0; t < DT; ++t)
#pragma unroll
                for (int e = 0; e < 16; ++e) ot[t][e] *= alpha;
        }
        l_run += psum;
        m_run = m_new;
        // O^T += V^T P^T
        const char* vt = sb + TILE;
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
            for (int hh = 0; hh < 2; ++hh) {
                bf16x8 pf;
#pragma unroll
                for (int j = 0; j < 8; ++j) pf[j] = (__bf16)st[kt][hh * 8 + j];
                // k-slots j = 0..3 of lane (., g): keys kofs + j; j = 4..7: keys kofs + 8 + (j - 4)
                const int key_a = kt * 32 + hh * 16 + g * 4 + tr_j;
                const int key_b = key_a + 8;
                const char* ra = vt + key_a * ROWB + tr_t % 2 * 8;
                const char* rb = vt + key_b * ROWB + tr_t % 2 * 8;
                const int sw_a = (key_a & 3) * 4, sw_b = (key_b & 3) * 4;
#pragma unroll
                for (int t = 0; t < DT; ++t) {
                    const int chunk = t * 4 + tr_half * 2 + (tr_t >> 1);
                    const att_short4 va = lds_read_tr16(ra + (((chunk ^ sw_a) & (NCHK - 1)) << 4));
                    const att_short4 vb2 = lds_read_tr16(rb + (((chunk ^ sw_b) & (NCHK - 1)) << 4));
                    union { short s[8]; bf16x8 b; } u;
                    u.s[0] = va[0]; u.s[1] = va[1]; u.s[2] = va[2]; u.s[3] = va[3];
                    u.s[4] = vb2[0]; u.s[5] = vb2[1]; u.s[6] = vb2[2]; u.s[7] = vb2[3];
                    ot[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(u.b, pf, ot[t], 0, 0, 0);
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
        const int nqt = ceil_div(max_seqlen, ATT_BQ);
        const dim3 g((unsigned)(8 * ceil_div(H * B, 8) * nqt));
        const size_t lds = (size_t)ATT_NS * 2 * ATT_BK * dh * 2;
        static bool attr_set = false;
        if (!attr_set) {
            if (hipFuncSetAttribute((const void*)attend_bf16_kernel<128>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                    ATT_NS * 2 * ATT_BK * 128 * 2) != hipSuccess ||
                hipFuncSetAttribute((const void*)attend_bf16_kernel<64>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                    ATT_NS * 2 * ATT_BK * 64 * 2) != hipSuccess)
                return D3TOM_ERR_DEVICE;
            attr_set = true;
        }
        if (dh == 128)
            D3TOM_LAUNCH(ATTEND, st, attend_bf16_kernel<128><<<g, 256, lds, st>>>(
                (const uint16_t*)q, (const uint16_t*)k, (const uint16_t*)v, cu_seqlens, H, B, nqt, scale2, (uint16_t*)o));
        else
            D3TOM_LAUNCH(ATTEND, st, attend_bf16_kernel<64><<<g, 256, lds, st>>>(
                (const uint16_t*)q, (const uint16_t*)k, (const uint16_t*)v, cu_seqlens, H, B, nqt, scale2, (uint16_t*)o));
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
