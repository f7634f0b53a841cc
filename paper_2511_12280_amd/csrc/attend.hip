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
// with direct loads (buffer_load ... lds, no register staging; rows past the end of the sample load as
// zeros through the buffer bounds check) into a two-stage ring; rows are unpadded and their 16-byte
// chunks XOR-swizzled by the row index instead.  Per tile a wave requests all 16 K fragments before the
// first MFMA, runs the two accumulation chains of S^T interleaved, requests the V^T fragments of the
// first 32 keys and starts the direct loads of the next stage, then does the softmax arithmetic while
// those are in flight (measured on gfx950: direct loads overlap vector-ALU work but not MFMAs), and
// finally the 16 MFMAs of the second product.  Softmax state and accumulators are float32; two
// workgroups fit a CU.  A wave raises its priority (s_setprio) for its MFMA bursts: the SIMD's arbiter
// otherwise favours the older of its two waves, and while that one issues softmax arithmetic back to back
// the other's next MFMA waits although the matrix core is idle (measured: 3-5 % at 1.2k-2k keys).
//
// The generic path (float32 or any head size) is one workgroup per (query, head) with a chunked
// online softmax in plain float arithmetic.
#include "common.hpp"
#include <type_traits>

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

// all of this wave's direct loads have landed and all its LDS reads are done; then meet the other waves
__device__ __forceinline__ void att_wait_and_barrier() {
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

#if defined(__HIP_DEVICE_COMPILE__)
// buffer resource over [p, p + bytes), built from values the compiler can see are wave-uniform
__device__ __forceinline__ __amdgpu_buffer_rsrc_t att_uniform_rsrc(const void* p, uint32_t bytes) {
    const uint64_t a = (uint64_t)p;
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)a), hi = __builtin_amdgcn_readfirstlane((uint32_t)(a >> 32));
    return __builtin_amdgcn_make_buffer_rsrc((void*)(((uint64_t)hi << 32) | lo), 0, (int)__builtin_amdgcn_readfirstlane(bytes), 0x00020000);
}
// One wave-wide direct load HBM/L2 -> LDS: lane i fetches 16 bytes at byte offset `voff` of the buffer
// (zeros when that is past the end of the buffer) into LDS byte lds_base + 16 i.  Issued from inline
// assembly on purpose: the waits for these loads are placed by hand (att_wait_and_barrier), and the
// compiler, when it sees such a load, makes every later transposing LDS read wait for all of them.
__device__ __forceinline__ void att_direct_load(__amdgpu_buffer_rsrc_t rsrc, int voff, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                 :: "s"(lds_base), "v"(voff), "s"(rsrc) : "memory", "m0");
}
// the two lanes (l, l ^ 32) that share a query column combine their values: after the swap of the upper
// half of one copy with the lower half of the other, the two results hold {own, partner} in some order
__device__ __forceinline__ float att_pair_max(float x) {
    typedef unsigned att_u2 __attribute__((ext_vector_type(2)));
    const att_u2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float att_pair_sum(float x) {
    typedef unsigned att_u2 __attribute__((ext_vector_type(2)));
    const att_u2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
#endif

// Size-weighted attention: key row j of sample b stands for w_j original tokens (the member counts of the
// merge); its logit gets + log2(w_j) in the base-2 softmax, which is attention over the sequence with the row
// written w_j times.  The weights are described the way the merge reports them: `counts` per kept slot; key
// rows vis_start[b] .. vis_start[b] + (kept_off[b+1] - kept_off[b]) - 1 are the merged rows, every other row
// weighs 1.
struct KeyWeights {
    const int32_t* counts;
    const int32_t* kept_off;
    const int32_t* vis_start;
};
__device__ __forceinline__ float key_log2_weight(const KeyWeights& kw, int b, int j) {
    const int r = j - kw.vis_start[b];
    const int k0 = kw.kept_off[b], kn = kw.kept_off[b + 1] - k0;
    return (r >= 0 && r < kn) ? __log2f((float)max(kw.counts[k0 + r], 1)) : 0.f;
}
constexpr int ATT_WKEYS = 3584;     // longest sample of the weighted tiled kernel: its log2 weights sit in LDS, and two
                                    // workgroups (64 KB ring + weights each) still fit the 160 KB of a CU

template <int DH, bool WGT>
__global__ __launch_bounds__(256, 2) void attend_bf16_kernel(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
    const int32_t* __restrict__ cu, int H, int nB, int nqt, float scale2, uint16_t* __restrict__ o, KeyWeights kw) {
#if defined(__HIP_DEVICE_COMPILE__)
    constexpr int KS = DH / 16;                 // k-steps of the first product
    constexpr int DT = DH / 32;                 // 32-dim tiles of O^T
    constexpr int ROWB = DH * 2;                // bytes per K / V row in LDS (unpadded, chunks swizzled)
    constexpr int NCHK = DH / 8;                // 16-byte chunks per row
    constexpr int RPI = 64 / NCHK;              // rows covered by one wave-wide direct load (1 KB)
    constexpr int LD = ATT_BK / (4 * RPI);      // direct loads per wave, per operand, per stage
    constexpr int TILE = ATT_BK * ROWB;         // bytes of one K (or V) tile
    constexpr int STAGE = 2 * TILE;
    extern __shared__ __attribute__((aligned(16))) char ring[];
    __shared__ __attribute__((aligned(16))) float lw_s[WGT ? ATT_WKEYS + ATT_BK : 4];

    const int xcd = blockIdx.x & 7, li = blockIdx.x >> 3;
    const int hb = (li / nqt) * 8 + xcd, qt = li % nqt;         // hb = sample * H + head
    if (hb >= H * nB) return;
    const int h = hb % H, b = hb / H;
    const int tok0 = cu[b];
    const int n = min(cu[b + 1] - tok0, WGT ? ATT_WKEYS : 0x7FFFFFFF);
    if (qt * ATT_BQ >= n) return;

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    if constexpr (WGT) {
        for (int j = tid; j < ((n + ATT_BK - 1) / ATT_BK) * ATT_BK; j += 256) lw_s[j] = (j < n) ? key_log2_weight(kw, b, j) : 0.f;
        __syncthreads();
    }
    const int c = lane & 31, g = lane >> 5;
    const size_t rs = (size_t)H * DH;                      // token stride (elements)
    const uint16_t* kb = k + (size_t)tok0 * rs + (size_t)h * DH;
    const uint16_t* vb = v + (size_t)tok0 * rs + (size_t)h * DH;
    // this head's K / V rows of this sample; a row index >= n is past the end and loads as zeros
    const uint32_t span = (uint32_t)(((size_t)(n - 1) * rs + DH) * 2);
    const __amdgpu_buffer_rsrc_t rk = att_uniform_rsrc(kb, span), rv = att_uniform_rsrc(vb, span);
    const int row_bytes = (int)(rs * 2);

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
    // p ^ (r mod NCHK) for K (operand reads walk 16+ consecutive rows) and p ^ ((r & 3) * 4) for V
    // (transposing reads touch 4 consecutive rows per 16-lane group)
    const int ld_pos = lane % NCHK;
    int k_off[LD], v_off[LD];                   // byte offsets inside the head's K / V for key0 = 0
#pragma unroll
    for (int i = 0; i < LD; ++i) {
        const int r = wave * (ATT_BK / 4) + lane / NCHK + i * RPI;
        k_off[i] = r * row_bytes + (((ld_pos ^ (r & 15)) & (NCHK - 1)) << 4);
        v_off[i] = r * row_bytes + (((ld_pos ^ ((r & 3) * 4)) & (NCHK - 1)) << 4);
    }
    const uint32_t ring0 = (uint32_t)(size_t)(att_lds_ptr_t)ring;
    const uint32_t wave_lds = __builtin_amdgcn_readfirstlane(ring0 + wave * (ATT_BK / 4) * ROWB);
    auto issue = [&](int key0, int stage) {
        const int kofs = key0 * row_bytes;
#pragma unroll
        for (int i = 0; i < LD; ++i) {
            att_direct_load(rk, k_off[i] + kofs, wave_lds + stage * STAGE + i * RPI * ROWB);
            att_direct_load(rv, v_off[i] + kofs, wave_lds + stage * STAGE + TILE + i * RPI * ROWB);
        }
    };
    // K operand fragments: lane (key row c, g) reads chunk (2 kk + g) of its row, swizzled by the row
    int k_addr[KS];
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) k_addr[kk] = c * ROWB + ((((kk * 2 + g) ^ (c & 15)) & (NCHK - 1)) << 4);
    // transposing-read geometry of this lane: 16-lane group -> (g, dim half), lane in group -> (row j, 4-dim quad t)
    const int tr_j = (lane & 15) >> 2, tr_t = lane & 3, tr_half = (lane >> 4) & 1;
    int v_addr[DT];
#pragma unroll
    for (int t = 0; t < DT; ++t) {
        const int chunk = t * 4 + tr_half * 2 + (tr_t >> 1);
        v_addr[t] = TILE + (g * 4 + tr_j) * ROWB + (tr_t % 2) * 8 + (((chunk ^ (tr_j * 4)) & (NCHK - 1)) << 4);
    }

    const int ntile = (n + ATT_BK - 1) / ATT_BK;
    // one 64-key tile out of ring stage STG (a compile-time constant so that every LDS offset folds
    // into the instruction)
    auto tile = [&](auto stg_c, int it) {
        constexpr int STG = decltype(stg_c)::value;
        const int key0 = it * ATT_BK;
        att_wait_and_barrier();                             // stage STG has landed; the other stage is free
        const char* sb = ring + STG * STAGE;

        // all K fragments of the tile are requested before the first MFMA
        bf16x8 kf[2][KS];
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
            for (int kk = 0; kk < KS; ++kk)
                kf[kt][kk] = *reinterpret_cast<const bf16x8*>(sb + k_addr[kk] + kt * 32 * ROWB);
        __builtin_amdgcn_sched_barrier(0);
        // S^T = K Q^T for two 32-key blocks, the two accumulation chains interleaved
        f32x16 st[2];
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
            for (int e = 0; e < 16; ++e) st[kt][e] = 0.f;
        __builtin_amdgcn_s_setprio(3);
#pragma unroll
        for (int kk = 0; kk < KS; ++kk) {
            st[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[0][kk], qf[kk], st[0], 0, 0, 0);
            st[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[1][kk], qf[kk], st[1], 0, 0, 0);
        }
        __builtin_amdgcn_s_setprio(0);
        __builtin_amdgcn_sched_barrier(0);
        // V^T fragments of the first 32 keys are requested now and land during the softmax arithmetic
        att_short4 vf[2][2][DT][2];                 // [kt][hh][t][a/b]
        auto read_v = [&](int kt) {
#pragma unroll
            for (int hh = 0; hh < 2; ++hh)
#pragma unroll
                for (int t = 0; t < DT; ++t) {
                    const char* pa = sb + v_addr[t] + (kt * 32 + hh * 16) * ROWB;
                    vf[kt][hh][t][0] = lds_read_tr16(pa);
                    vf[kt][hh][t][1] = lds_read_tr16(pa + 8 * ROWB);
                }
        };
        read_v(0);
        __builtin_amdgcn_sched_barrier(0);
        // the loads of the next stage start here, beside the softmax arithmetic: direct loads and MFMAs
        // slow each other down, direct loads and vector-ALU work do not
        if (it + 1 < ntile) issue(key0 + ATT_BK, STG ^ 1);
        __builtin_amdgcn_sched_barrier(0);
        // online softmax in base 2 on the raw logits; element e of st[kt]: key kt*32 + (e/4)*8 + 4g + e%4, query c
        if constexpr (WGT) {
            // weighted: the maximum is taken on scale2 * logit + log2 w (m_run lives in that scaled domain)
#pragma unroll
            for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                for (int e4 = 0; e4 < 4; ++e4) {
                    const f32x4 w4 = *reinterpret_cast<const f32x4*>(&lw_s[key0 + kt * 32 + e4 * 8 + g * 4]);
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int key = key0 + kt * 32 + e4 * 8 + g * 4 + e;
                        const float t = __builtin_fmaf(st[kt][e4 * 4 + e], scale2, w4[e]);
                        st[kt][e4 * 4 + e] = (key < n) ? t : -INFINITY;
                    }
                }
            float tmax = st[0][0];
#pragma unroll
            for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                for (int e = 0; e < 16; ++e) tmax = fmaxf(tmax, st[kt][e]);
            tmax = att_pair_max(tmax);
            const float m_new = fmaxf(m_run, tmax);
            float psum = 0.f;
#pragma unroll
            for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const float p = __builtin_amdgcn_exp2f(st[kt][e] - m_new);
                    st[kt][e] = p;
                    psum += p;
                }
            if (__builtin_amdgcn_ballot_w64(m_new > m_run) != 0) {
                const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
                l_run *= alpha;
#pragma unroll
                for (int t = 0; t < DT; ++t)
#pragma unroll
                    for (int e = 0; e < 16; ++e) ot[t][e] *= alpha;
            }
            l_run += psum;
            m_run = m_new;
        } else {
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
        tmax = att_pair_max(tmax);
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
        if (__builtin_amdgcn_ballot_w64(m_new > m_run) != 0) {      // some query of this wave moved its max
            const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * scale2);
            l_run *= alpha;
#pragma unroll
            for (int t = 0; t < DT; ++t)
#pragma unroll
                for (int e = 0; e < 16; ++e) ot[t][e] *= alpha;
        }
        l_run += psum;                               // per-lane partial; the two halves meet after the last tile
        m_run = m_new;
        }
        __builtin_amdgcn_sched_barrier(0);
        read_v(1);
        __builtin_amdgcn_sched_barrier(0);
        // O^T += V^T P^T
        __builtin_amdgcn_s_setprio(3);
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
            for (int hh = 0; hh < 2; ++hh) {
                bf16x8 pf;
#pragma unroll
                for (int j = 0; j < 8; ++j) pf[j] = (__bf16)st[kt][hh * 8 + j];
#pragma unroll
                for (int t = 0; t < DT; ++t) {
                    const att_short4 va = vf[kt][hh][t][0], vb2 = vf[kt][hh][t][1];
                    typedef __attribute__((__vector_size__(8 * sizeof(short)))) short att_short8;
                    const att_short8 v8 = __builtin_shufflevector(va, vb2, 0, 1, 2, 3, 4, 5, 6, 7);
                    ot[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, v8), pf, ot[t], 0, 0, 0);
                }
            }
        __builtin_amdgcn_s_setprio(0);
    };
    // The query fragments must have arrived before the first direct load is issued: otherwise the
    // compiler's own wait for them would sit inside the loop, where it would also wait for the direct
    // loads of the next stage.
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) asm volatile("" :: "v"(qf[kk]));
    issue(0, 0);
    for (int it = 0; it < ntile; it += 2) {
        tile(std::integral_constant<int, 0>{}, it);
        if (it + 1 < ntile) tile(std::integral_constant<int, 1>{}, it + 1);
    }
    l_run = att_pair_sum(l_run);
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
#endif
}
// ---- short sequences: the keys are split across the four waves -------------------------------------
// With a few hundred keys the kernel above is one short serial chain per workgroup (8 stages at 493 keys)
// on half of the CUs.  Here a workgroup owns 32 queries of one head and its four waves take the 32-key
// tiles w, w + 4, w + 8, ... with the same transposed products as above; each wave has a private K and V
// tile in LDS, filled by its own direct loads, so the waves never meet inside the loop (no s_barrier, only
// waits for the wave's own loads: K of the next tile is requested as soon as the K fragments are in
// registers, V of the next tile as soon as the V fragments are).  At the end the four partial results
// (running max, sum, O^T) meet in LDS and wave t combines and stores the 32 output dims t*32 ..
// Four times the K/V traffic per query of the kernel above, which is why it is only used while the whole
// sample is short.
constexpr int ATS_BK = 32;      // keys per wave tile
constexpr int ATS_MAX_KEYS = 512;

template <int N>
__device__ __forceinline__ void att_wait_loads() { asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory"); }

template <int DH, bool WGT>
__global__ __launch_bounds__(256, 2) void attend_bf16_short_kernel(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
    const int32_t* __restrict__ cu, int H, int nB, int nqt, float scale2, uint16_t* __restrict__ o, KeyWeights kw) {
#if defined(__HIP_DEVICE_COMPILE__)
    constexpr int KS = DH / 16;
    constexpr int DT = DH / 32;
    constexpr int ROWB = DH * 2;
    constexpr int NCHK = DH / 8;
    constexpr int RPI = 64 / NCHK;              // rows per wave-wide direct load
    constexpr int LD = ATS_BK / RPI;            // direct loads per operand tile
    constexpr int TILE = ATS_BK * ROWB;         // bytes of one K (or V) tile
    constexpr int WREG = 2 * TILE;              // bytes of a wave's private region (K tile, V tile)
    static_assert(WREG == DT * 16 * 64 * 4, "a wave's region also holds its partial O^T");
    extern __shared__ __attribute__((aligned(16))) char ring[];
    __shared__ float part_m[4][32], part_l[4][32];
    __shared__ __attribute__((aligned(16))) float lw_s[WGT ? ATS_MAX_KEYS : 4];

    const int xcd = blockIdx.x & 7, li = blockIdx.x >> 3;
    const int hb = (li / nqt) * 8 + xcd, qt = li % nqt;
    if (hb >= H * nB) return;
    const int h = hb % H, b = hb / H;
    const int tok0 = cu[b];
    const int n = min(cu[b + 1] - tok0, ATS_MAX_KEYS);
    if (qt * 32 >= n) return;

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    if constexpr (WGT) {
        for (int j = tid; j < ATS_MAX_KEYS; j += 256) lw_s[j] = (j < n) ? key_log2_weight(kw, b, j) : 0.f;
        __syncthreads();
    }
    const int c = lane & 31, g = lane >> 5;
    const size_t rs = (size_t)H * DH;
    const uint16_t* kb = k + (size_t)tok0 * rs + (size_t)h * DH;
    const uint16_t* vb = v + (size_t)tok0 * rs + (size_t)h * DH;
    const uint32_t span = (uint32_t)(((size_t)(n - 1) * rs + DH) * 2);      // rows past the end load as zeros
    const __amdgpu_buffer_rsrc_t rk = att_uniform_rsrc(kb, span), rv = att_uniform_rsrc(vb, span);
    const int row_bytes = (int)(rs * 2);

    const int qrow = qt * 32 + c;
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

    // direct loads of a 32-key tile: same chunk swizzles as in the kernel above
    const int ld_pos = lane % NCHK;
    int k_off[LD], v_off[LD];
#pragma unroll
    for (int i = 0; i < LD; ++i) {
        const int r = lane / NCHK + i * RPI;
        k_off[i] = r * row_bytes + (((ld_pos ^ (r & 15)) & (NCHK - 1)) << 4);
        v_off[i] = r * row_bytes + (((ld_pos ^ ((r & 3) * 4)) & (NCHK - 1)) << 4);
    }
    char* wreg = ring + wave * WREG;
    const uint32_t wave_lds = __builtin_amdgcn_readfirstlane((uint32_t)(size_t)(att_lds_ptr_t)ring + wave * WREG);
    auto issue_k = [&](int key0) {
        const int kofs = key0 * row_bytes;
#pragma unroll
        for (int i = 0; i < LD; ++i) att_direct_load(rk, k_off[i] + kofs, wave_lds + i * RPI * ROWB);
    };
    auto issue_v = [&](int key0) {
        const int kofs = key0 * row_bytes;
#pragma unroll
        for (int i = 0; i < LD; ++i) att_direct_load(rv, v_off[i] + kofs, wave_lds + TILE + i * RPI * ROWB);
    };
    int k_addr[KS];
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) k_addr[kk] = c * ROWB + ((((kk * 2 + g) ^ (c & 15)) & (NCHK - 1)) << 4);
    const int tr_j = (lane & 15) >> 2, tr_t = lane & 3, tr_half = (lane >> 4) & 1;
    int v_addr[DT];
#pragma unroll
    for (int t = 0; t < DT; ++t) {
        const int chunk = t * 4 + tr_half * 2 + (tr_t >> 1);
        v_addr[t] = TILE + (g * 4 + tr_j) * ROWB + (tr_t % 2) * 8 + (((chunk ^ (tr_j * 4)) & (NCHK - 1)) << 4);
    }

    const int ntile = (n + ATS_BK - 1) / ATS_BK;
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) asm volatile("" :: "v"(qf[kk]));      // Q has arrived before the first direct load
    if (wave < ntile) { issue_k(wave * ATS_BK); issue_v(wave * ATS_BK); }
    for (int it = wave; it < ntile; it += 4) {
        const int key0 = it * ATS_BK;
        const bool more = it + 4 < ntile;
        att_wait_loads<LD>();                                  // K of this tile has landed (V may still be on its way)
        bf16x8 kf[KS];
#pragma unroll
        for (int kk = 0; kk < KS; ++kk) kf[kk] = *reinterpret_cast<const bf16x8*>(wreg + k_addr[kk]);
        __builtin_amdgcn_sched_barrier(0);
        f32x16 st;
#pragma unroll
        for (int e = 0; e < 16; ++e) st[e] = 0.f;
        __builtin_amdgcn_s_setprio(3);
#pragma unroll
        for (int kk = 0; kk < KS; ++kk) st = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[kk], qf[kk], st, 0, 0, 0);
        __builtin_amdgcn_s_setprio(0);
        __builtin_amdgcn_sched_barrier(0);
        // the K fragments are in registers (the MFMAs above consumed them): the K tile is free
        if (more) issue_k(key0 + 4 * ATS_BK);
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (WGT) {
            // weighted: maximum and exponent on scale2 * logit + log2 w (m_run lives in that scaled domain)
#pragma unroll
            for (int e4 = 0; e4 < 4; ++e4) {
                const f32x4 w4 = *reinterpret_cast<const f32x4*>(&lw_s[min(key0 + e4 * 8 + g * 4, ATS_MAX_KEYS - 4)]);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int key = key0 + e4 * 8 + g * 4 + e;
                    const float t = __builtin_fmaf(st[e4 * 4 + e], scale2, w4[e]);
                    st[e4 * 4 + e] = (key < n) ? t : -INFINITY;
                }
            }
            float tmax = st[0];
#pragma unroll
            for (int e = 1; e < 16; ++e) tmax = fmaxf(tmax, st[e]);
            tmax = att_pair_max(tmax);
            const float m_new = fmaxf(m_run, tmax);
            float psum = 0.f;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const float p = __builtin_amdgcn_exp2f(st[e] - m_new);
                st[e] = p;
                psum += p;
            }
            if (__builtin_amdgcn_ballot_w64(m_new > m_run) != 0) {
                const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
                l_run *= alpha;
#pragma unroll
                for (int t = 0; t < DT; ++t)
#pragma unroll
                    for (int e = 0; e < 16; ++e) ot[t][e] *= alpha;
            }
            l_run += psum;
            m_run = m_new;
        } else {
        if (key0 + ATS_BK > n) {
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int key = key0 + (e >> 2) * 8 + g * 4 + (e & 3);
                    if (key >= n) st[e] = -INFINITY;
                }
            }
            float tmax = st[0];
#pragma unroll
            for (int e = 1; e < 16; ++e) tmax = fmaxf(tmax, st[e]);
            tmax = att_pair_max(tmax);
            const float m_new = fmaxf(m_run, tmax);                // finite: every tile holds >= 1 valid key
            const float ms = m_new * scale2;
            float psum = 0.f;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(st[e], scale2, -ms));
                st[e] = p;
                psum += p;
            }
            if (__builtin_amdgcn_ballot_w64(m_new > m_run) != 0) {
                const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * scale2);
                l_run *= alpha;
#pragma unroll
                for (int t = 0; t < DT; ++t)
#pragma unroll
                    for (int e = 0; e < 16; ++e) ot[t][e] *= alpha;
            }
            l_run += psum;
            m_run = m_new;
        }
        __builtin_amdgcn_sched_barrier(0);
        // V of this tile: everything older than the K loads just issued has landed
        if (more) att_wait_loads<LD>(); else att_wait_loads<0>();
        att_short4 vf[2][DT][2];
#pragma unroll
        for (int hh = 0; hh < 2; ++hh)
#pragma unroll
            for (int t = 0; t < DT; ++t) {
                const char* pa = wreg + v_addr[t] + hh * 16 * ROWB;
                vf[hh][t][0] = lds_read_tr16(pa);
                vf[hh][t][1] = lds_read_tr16(pa + 8 * ROWB);
            }
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_setprio(3);
#pragma unroll
        for (int hh = 0; hh < 2; ++hh) {
            bf16x8 pf;
#pragma unroll
            for (int j = 0; j < 8; ++j) pf[j] = (__bf16)st[hh * 8 + j];
#pragma unroll
            for (int t = 0; t < DT; ++t) {
                typedef __attribute__((__vector_size__(8 * sizeof(short)))) short att_short8;
                const att_short8 v8 = __builtin_shufflevector(vf[hh][t][0], vf[hh][t][1], 0, 1, 2, 3, 4, 5, 6, 7);
                ot[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, v8), pf, ot[t], 0, 0, 0);
            }
        }
        __builtin_amdgcn_s_setprio(0);
        __builtin_amdgcn_sched_barrier(0);
        // the V fragments are in registers: the V tile is free
        if (more) issue_v(key0 + 4 * ATS_BK);
    }
    // the four partial results meet in LDS (every wave's own region is free: it has no load in flight)
    l_run = att_pair_sum(l_run);
    float* po = reinterpret_cast<float*>(wreg);
#pragma unroll
    for (int t = 0; t < DT; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e) po[(t * 16 + e) * 64 + lane] = ot[t][e];
    if (g == 0) { part_m[wave][c] = m_run; part_l[wave][c] = l_run; }
    __syncthreads();
    if (wave >= DT || !qvalid) return;
    float m = part_m[0][c];
#pragma unroll
    for (int w2 = 1; w2 < 4; ++w2) m = fmaxf(m, part_m[w2][c]);
    float f[4], l = 0.f;
#pragma unroll
    for (int w2 = 0; w2 < 4; ++w2) {
        const float mw = part_m[w2][c];
        f[w2] = (mw == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f((mw - m) * (WGT ? 1.0f : scale2));
        l += part_l[w2][c] * f[w2];
    }
    const float inv = 1.0f / l;
    float acc[16];
#pragma unroll
    for (int e = 0; e < 16; ++e) {
        float a2 = 0.f;
#pragma unroll
        for (int w2 = 0; w2 < 4; ++w2)
            a2 += reinterpret_cast<const float*>(ring + w2 * WREG)[(wave * 16 + e) * 64 + lane] * f[w2];
        acc[e] = a2 * inv;
    }
    uint16_t* op = o + (size_t)(tok0 + qrow) * rs + (size_t)h * DH + wave * 32;
#pragma unroll
    for (int e4 = 0; e4 < 4; ++e4) {
        uint2 w2;
        w2.x = pack_bf16x2(acc[e4 * 4 + 0], acc[e4 * 4 + 1]);
        w2.y = pack_bf16x2(acc[e4 * 4 + 2], acc[e4 * 4 + 3]);
        *reinterpret_cast<uint2*>(op + e4 * 8 + g * 4) = w2;
    }
#endif
}

// generic: one workgroup per (query, head), keys in chunks of 256, plain float online softmax
template <typename T>
__global__ __launch_bounds__(256) void attend_generic_kernel(
    const T* __restrict__ q, const T* __restrict__ k, const T* __restrict__ v, const int32_t* __restrict__ cu,
    int H, int dh, float scale2, T* __restrict__ o, KeyWeights kw) {
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
            if (kw.counts) s2 += key_log2_weight(kw, b, j);
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

static int attend_run(const void* q, const void* k, const void* v, int dt,
                      int B, const int32_t* cu_seqlens, int max_seqlen, int H, int dh, float scale,
                      const int32_t* counts, const int32_t* kept_off, const int32_t* vis_start, void* o, void* stream) {
    if (!q || !k || !v || !o || !cu_seqlens) return D3TOM_ERR_INVALID_ARG;
    if (B < 1 || max_seqlen < 1 || H < 1 || dh < 1) return D3TOM_ERR_INVALID_ARG;
    if (!(scale > 0.f) || !(scale < 3.0e38f)) return D3TOM_ERR_INVALID_ARG;      // the running max is taken on raw logits
    if (dt != D3TOM_F32 && dt != D3TOM_BF16) return D3TOM_ERR_INVALID_ARG;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o)) return D3TOM_ERR_INVALID_ARG;
    if (dh > 256 || (dt == D3TOM_BF16 ? (dh % 8) : (dh % 4))) return D3TOM_ERR_UNSUPPORTED;
    const bool wgt = counts != nullptr;
    const KeyWeights kw{counts, kept_off, vis_start};
    hipStream_t st = (hipStream_t)stream;
    const float scale2 = scale * LOG2E;
    // the tiled kernel addresses one sample's K / V rows with 32-bit byte offsets
    const bool fits32 = ((size_t)max_seqlen + ATT_BK) * (size_t)H * (size_t)dh * 2 < ((size_t)1 << 31);
    const bool mfma = dt == D3TOM_BF16 && (dh == 128 || dh == 64) && fits32;
    // the weighted MFMA kernels keep a sample's log2 weights in LDS
    if (wgt && mfma && max_seqlen > ATT_WKEYS) return D3TOM_ERR_UNSUPPORTED;
    // short samples and too few 128-query tiles to fill the chip: keys split across the waves (measured
    // crossover with the tiled kernel: ~550 keys at 32 heads)
    if (mfma && max_seqlen <= ATS_MAX_KEYS && (long)ceil_div(max_seqlen, ATT_BQ) * H * B <= 512) {
        const int nqt = ceil_div(max_seqlen, 32);
        const dim3 g((unsigned)(8 * ceil_div(H * B, 8) * nqt));
        const size_t lds = (size_t)4 * 2 * ATS_BK * dh * 2;
        static PerDeviceOnce lds_setup_s;
        if (!lds_setup_s.run([] {
                return raise_dynamic_lds(attend_bf16_short_kernel<128, false>, 4 * 2 * ATS_BK * 128 * 2) &&
                       raise_dynamic_lds(attend_bf16_short_kernel<64, false>, 4 * 2 * ATS_BK * 64 * 2) &&
                       raise_dynamic_lds(attend_bf16_short_kernel<128, true>, 4 * 2 * ATS_BK * 128 * 2) &&
                       raise_dynamic_lds(attend_bf16_short_kernel<64, true>, 4 * 2 * ATS_BK * 64 * 2);
            }))
            return D3TOM_ERR_DEVICE;
#define D3TOM_ATT(KERNEL)                                                                                            \
    D3TOM_LAUNCH(ATTEND, st, (KERNEL<<<g, 256, lds, st>>>((const uint16_t*)q, (const uint16_t*)k, (const uint16_t*)v, \
                                                           cu_seqlens, H, B, nqt, scale2, (uint16_t*)o, kw)))
        if (dh == 128) { if (wgt) D3TOM_ATT((attend_bf16_short_kernel<128, true>)); else D3TOM_ATT((attend_bf16_short_kernel<128, false>)); }
        else           { if (wgt) D3TOM_ATT((attend_bf16_short_kernel<64, true>));  else D3TOM_ATT((attend_bf16_short_kernel<64, false>)); }
    } else if (mfma) {
        const int nqt = ceil_div(max_seqlen, ATT_BQ);
        const dim3 g((unsigned)(8 * ceil_div(H * B, 8) * nqt));
        const size_t lds = (size_t)ATT_NS * 2 * ATT_BK * dh * 2;
        static PerDeviceOnce lds_setup;
        if (!lds_setup.run([] {
                return raise_dynamic_lds(attend_bf16_kernel<128, false>, ATT_NS * 2 * ATT_BK * 128 * 2) &&
                       raise_dynamic_lds(attend_bf16_kernel<64, false>, ATT_NS * 2 * ATT_BK * 64 * 2) &&
                       raise_dynamic_lds(attend_bf16_kernel<128, true>, ATT_NS * 2 * ATT_BK * 128 * 2) &&
                       raise_dynamic_lds(attend_bf16_kernel<64, true>, ATT_NS * 2 * ATT_BK * 64 * 2);
            }))
            return D3TOM_ERR_DEVICE;
        if (dh == 128) { if (wgt) D3TOM_ATT((attend_bf16_kernel<128, true>)); else D3TOM_ATT((attend_bf16_kernel<128, false>)); }
        else           { if (wgt) D3TOM_ATT((attend_bf16_kernel<64, true>));  else D3TOM_ATT((attend_bf16_kernel<64, false>)); }
#undef D3TOM_ATT
    } else {
        const dim3 g(max_seqlen, H, B);
        if (dt == D3TOM_F32)
            D3TOM_LAUNCH(ATTEND, st, attend_generic_kernel<float><<<g, 256, 0, st>>>(
                (const float*)q, (const float*)k, (const float*)v, cu_seqlens, H, dh, scale2, (float*)o, kw));
        else
            D3TOM_LAUNCH(ATTEND, st, attend_generic_kernel<uint16_t><<<g, 256, 0, st>>>(
                (const uint16_t*)q, (const uint16_t*)k, (const uint16_t*)v, cu_seqlens, H, dh, scale2, (uint16_t*)o, kw));
    }
    return D3TOM_OK;
}

extern "C" int d3tom_attend(const void* q, const void* k, const void* v, int dt,
                            int B, const int32_t* cu_seqlens, int max_seqlen, int H, int dh, float scale,
                            void* o, void* ws, size_t ws_bytes, void* stream) {
    (void)ws; (void)ws_bytes;
    return attend_run(q, k, v, dt, B, cu_seqlens, max_seqlen, H, dh, scale, nullptr, nullptr, nullptr, o, stream);
}

extern "C" int d3tom_attend_weighted(const void* q, const void* k, const void* v, int dt,
                                     int B, const int32_t* cu_seqlens, int max_seqlen, int H, int dh, float scale,
                                     const int32_t* counts, const int32_t* kept_off, const int32_t* vis_start,
                                     void* o, void* ws, size_t ws_bytes, void* stream) {
    (void)ws; (void)ws_bytes;
    if (!counts || !kept_off || !vis_start) return D3TOM_ERR_INVALID_ARG;
    return attend_run(q, k, v, dt, B, cu_seqlens, max_seqlen, H, dh, scale, counts, kept_off, vis_start, o, stream);
}
