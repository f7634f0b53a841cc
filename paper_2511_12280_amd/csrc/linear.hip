// d3tom_linear: out = a w^T for the projections of a transformer block (the per-layer 4 n d^2 and 3 n d m
// terms of the cost model in Section 4.3), bf16 operands, float32 accumulation on MFMA 32x32x16, with the
// element-wise tail of the projection folded into the epilogue:
//   PLAIN     out = a w^T, optionally written as several [rows, out_chunk] matrices (q | k | v)
//   RESIDUAL  out = residual + a w^T                      (the block's two skip connections)
//   SWIGLU    out = silu(a w_gate^T) * (a w_up^T)         (w holds the F gate rows, then the F up rows)
//   ROPE      (inside the stack only) PLAIN for the stacked q | k | v weight with the rotary embedding of the q and k
//             sections folded in: a 128-column tile holds whole heads, so both channels of a rotation pair are in
//             the tile; the projection is rounded to bf16 first (the value the separate rotary kernel would have
//             read), turned by the token's angle from a per-step table, and rounded again
//   PARTIAL   (inside the stack only) the contraction is cut into gridDim.y slices and every slice writes
//             its float32 products to its own [rows, n] matrix; the row-wise kernel that follows adds the
//             slices, the residual, rounds once and normalises.  Used where a short sequence leaves the
//             output and down projections with too few tall tiles to fill the chip.
// One rounding to bf16, at the store (ROPE: one for the projection, one for the rotated value).
//
// Workgroup tile: (TM*64) rows x 128 columns of a w^T.  Eight waves with two jobs: waves 0..3 (2 x 2, wave
// tile (TM*32) x 64) only feed the matrix cores, waves 4..7 only move data.  Both operands are
// contraction-contiguous, so both tiles travel HBM/L2 -> LDS with direct loads (16 bytes per lane, no
// register staging) into a ring of 64-element k-stages, one s_barrier per stage.  A wave that issues such a
// load waits for room in the CU's single vector-memory queue (64 bytes per clock); kept in the computing
// waves, that wait stalled their MFMA stream (measured: 6-20 % slower), so the loads have waves of their own.
// The 16-byte chunk stored at position p of tile row r is chunk p ^ ((r >> 1) & 7), which makes the MFMA
// operand reads bank-conflict free.
// For SWIGLU the 128 tile columns are 64 gate rows and the 64 up rows of the same output columns, so the
// epilogue finds both factors of an output element in the same tile.
//
// Workgroup ids are dealt round-robin to the 8 XCDs; each XCD owns a contiguous range of column tiles
// (its private L2 sees only its share of w) and walks it in panels of a few column tiles, row tile
// fastest, so that the workgroups running together share operand rows.
#include "common.hpp"
#include "direct_load.hpp"

namespace d3tom {

enum { LIN_PLAIN = 0, LIN_RESIDUAL = 1, LIN_SWIGLU = 2, LIN_PARTIAL = 3, LIN_ROPE = 4 };
constexpr int LIN_BN = 128;
constexpr int LIN_BK = 64;
constexpr int LIN_PAD = 136;      // floats per row of the epilogue staging tile (see the epilogue)

template <int TM> struct LinCfg {
    static constexpr int BM = TM * 64;
    static constexpr int NS = (TM == 4) ? 3 : 4;                       // ring stages
    static constexpr int STAGE = (BM + LIN_BN) * 128;                  // bytes per stage
    static constexpr int LDS = (NS * STAGE > BM * LIN_PAD * 4) ? NS * STAGE : BM * LIN_PAD * 4;
};

template <int TM, int EPI>
__global__ __launch_bounds__(512) void linear_bf16_kernel(
    const uint16_t* __restrict__ a, const uint16_t* __restrict__ w, int M, int N, int K,
    const uint16_t* residual, uint16_t* out, int out_chunk, int NRT, int NCT, int cpx, int PC, int col0, int col_end,
    const float2* __restrict__ rope_cs, int rope_dh) {
#if defined(__HIP_DEVICE_COMPILE__)
    using C = LinCfg<TM>;
    constexpr int BM = C::BM, NS = C::NS, STAGE = C::STAGE;
    constexpr int A_LD = BM / 32;                       // direct loads per wave and stage, a tile (8 rows each)
    constexpr int B_LD = LIN_BN / 32;
    constexpr int LPS = A_LD + B_LD;
    extern __shared__ __attribute__((aligned(16))) char ring[];

    // tile of this workgroup
    const int xcd = blockIdx.x & 7, li = blockIdx.x >> 3;
    const int panel = li / (NRT * PC), within = li % (NRT * PC);
    const int cl = panel * PC + within % PC;            // column tile inside this XCD's range
    const int rt = within / PC, ct = xcd * cpx + cl;
    if (cl >= cpx || ct >= NCT) return;

    constexpr int NT = 512;
    const int tid = threadIdx.x, wave = (tid >> 6) & 3, lane = tid & 63;
    const bool loader = tid >> 8;                       // waves 4..7 only move data, waves 0..3 only compute
    const int wm = wave >> 1, wn = wave & 1;
    const int c = lane & 31, g = lane >> 5;
    // out columns per tile and rows of w behind the 128 tile columns
    constexpr int OUT_BN = (EPI == LIN_SWIGLU) ? 64 : 128;
    const int n_out = (EPI == LIN_SWIGLU) ? N / 2 : N;  // SWIGLU: N counts gate and up rows

    const __amdgpu_buffer_rsrc_t rs_a = make_uniform_rsrc(a, (uint32_t)((size_t)M * K * 2));
    const __amdgpu_buffer_rsrc_t rs_w = make_uniform_rsrc(w, (uint32_t)((size_t)N * K * 2));
    // byte offset of this lane inside its operand for each of its direct loads; rows past the end re-read
    // row 0 (their results are never stored); the k-slice moves through the scalar offset
    int a_off[A_LD], b_off[B_LD];
#pragma unroll
    for (int i = 0; i < A_LD; ++i) {
        const int row = wave * (BM / 4) + i * 8 + (lane >> 3);
        const int cg = (lane & 7) ^ ((row >> 1) & 7);
        const int m = rt * BM + row;
        a_off[i] = ((m < M) ? m : 0) * K * 2 + cg * 16;
    }
#pragma unroll
    for (int i = 0; i < B_LD; ++i) {
        const int row = wave * (LIN_BN / 4) + i * 8 + (lane >> 3);
        const int cg = (lane & 7) ^ ((row >> 1) & 7);
        int n;
        if constexpr (EPI == LIN_SWIGLU) {
            const int o = col0 + ct * 64 + (row & 63);
            n = (o < col_end) ? o + (row >> 6) * n_out : 0;
        } else {
            n = col0 + ct * LIN_BN + row;
            n = (n < col_end) ? n : 0;
        }
        b_off[i] = n * K * 2 + cg * 16;
    }
    const int nkt = (K / LIN_BK) / (int)gridDim.y;         // k-stages of this workgroup's slice of the contraction
    const int kt0 = (int)blockIdx.y * nkt;
    const uint32_t ring0 = (uint32_t)(size_t)(lds_ptr_t)ring;
    const uint32_t a_lds = __builtin_amdgcn_readfirstlane(ring0 + wave * (BM / 4) * 128);
    const uint32_t b_lds = __builtin_amdgcn_readfirstlane(ring0 + BM * 128 + wave * (LIN_BN / 4) * 128);
    auto issue_part = [&](int kt, int stage, int n0, int n1) {
#pragma unroll
        for (int i = 0; i < A_LD; ++i)
            if (i >= n0 && i < n1)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_a, (lds_ptr_t)(size_t)(a_lds + stage * STAGE + i * 8 * 128), 16,
                                                         a_off[i], (kt0 + kt) * (LIN_BK * 2), 0, 0);
#pragma unroll
        for (int i = 0; i < B_LD; ++i)
            if (A_LD + i >= n0 && A_LD + i < n1)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_w, (lds_ptr_t)(size_t)(b_lds + stage * STAGE + i * 8 * 128), 16,
                                                         b_off[i], (kt0 + kt) * (LIN_BK * 2), 0, 0);
    };

    f32x16 acc[TM][2];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    int a_row[TM], b_row[2], a_sw[TM], b_sw[2];
#pragma unroll
    for (int i = 0; i < TM; ++i) { const int Rr = wm * (TM * 32) + i * 32 + c; a_row[i] = Rr * 128; a_sw[i] = (Rr >> 1) & 7; }
#pragma unroll
    for (int j = 0; j < 2; ++j) { const int Rr = wn * 64 + j * 32 + c; b_row[j] = BM * 128 + Rr * 128; b_sw[j] = (Rr >> 1) & 7; }

    // one stage: feed stage kt to the MFMAs, operand fragments read one k-step ahead
    auto stage = [&](int kt) {
        const char* sb = ring + (kt % NS) * STAGE;
        bf16x8 af[2][TM], bfr[2][2];
        auto read_frags = [&](int kk, int buf) {
#pragma unroll
            for (int i = 0; i < TM; ++i)
                af[buf][i] = *reinterpret_cast<const bf16x8*>(sb + a_row[i] + (((kk * 2 + g) ^ a_sw[i]) << 4));
#pragma unroll
            for (int j = 0; j < 2; ++j)
                bfr[buf][j] = *reinterpret_cast<const bf16x8*>(sb + b_row[j] + (((kk * 2 + g) ^ b_sw[j]) << 4));
        };
        read_frags(0, 0);
#pragma unroll
        for (int kk = 0; kk < LIN_BK / 16; ++kk) {
            if (kk + 1 < LIN_BK / 16) read_frags(kk + 1, (kk + 1) & 1);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[kk & 1][i], bfr[kk & 1][j], acc[i][j], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    if (loader) {
#pragma unroll
        for (int st = 0; st < NS - 1; ++st)
            if (st < nkt) issue_part(st, st, 0, LPS);
        for (int kt = 0; kt < nkt; ++kt) {
            // stage kt has landed (the NS-2 stages behind it may still be in flight), then everyone meets
            if (kt + NS - 2 <= nkt - 1) wait_loads_and_barrier<(NS - 2) * LPS>();
            else wait_loads_and_barrier<0>();
            // the consumers are past stage kt-1: its slot takes stage kt+NS-1
            if (kt + NS - 1 < nkt) issue_part(kt + NS - 1, (kt + NS - 1) % NS, 0, LPS);
        }
    } else {
        for (int kt = 0; kt < nkt; ++kt) {
            wait_loads_and_barrier<0>();
            stage(kt);
        }
    }

    // epilogue: the float32 tile goes through LDS (the ring is free now) so that every thread ends up with
    // 8 consecutive columns of one row: 16-byte stores, residual rows read the same way.  Rows are padded
    // to LIN_PAD floats: the two half-waves of an accumulator store (rows 4 apart) then fall into different
    // bank halves.
    __syncthreads();
    float* tile = reinterpret_cast<float*>(ring);
    if (!loader) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int row = wm * (TM * 32) + i * 32 + (e >> 2) * 8 + g * 4 + (e & 3);
                    tile[row * LIN_PAD + wn * 64 + j * 32 + c] = acc[i][j][e];
                }
    }
    __syncthreads();
    if constexpr (EPI == LIN_ROPE) {
        // A unit is an 8-column group of the first half of a head together with its partner group half a head
        // further: the two share their angles, so one thread rotates both (one table read for 16 outputs).  Heads
        // start at multiples of their size, so a 128-column tile holds whole heads.
        const int half = rope_dh >> 1, gph = half >> 3;                // 8-column groups in half a head: 8 or 4
        constexpr int UPR = OUT_BN / 16;                               // units per tile row
        for (int u = tid; u < BM * UPR; u += NT) {
            const int row = u / UPR, un = u % UPR;
            const int hd = un / gph, gi = un - hd * gph;
            const int tc = hd * rope_dh + gi * 8;                      // tile column of the first-half group
            const int m = rt * BM + row, col = col0 + ct * OUT_BN + tc;
            if (m >= M || col >= col_end) continue;
            const float* pa = tile + row * LIN_PAD + tc;
            const float4 a0 = *reinterpret_cast<const float4*>(pa), a1 = *reinterpret_cast<const float4*>(pa + 4);
            const float4 b0 = *reinterpret_cast<const float4*>(pa + half), b1 = *reinterpret_cast<const float4*>(pa + half + 4);
            float va[8] = {a0.x, a0.y, a0.z, a0.w, a1.x, a1.y, a1.z, a1.w};
            float vb[8] = {b0.x, b0.y, b0.z, b0.w, b1.x, b1.y, b1.z, b1.w};
            if (col < 2 * out_chunk) {                                 // q and k sections; v passes through
                const float4* cs = reinterpret_cast<const float4*>(rope_cs + (size_t)m * half + gi * 8);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float4 t = cs[e];                            // (cos, sin) of channels 2e and 2e + 1
                    const float cc[2] = {t.x, t.z}, ss[2] = {t.y, t.w};
#pragma unroll
                    for (int f = 0; f < 2; ++f) {
                        // both channels as the stored bf16 projection, then the rotation in float32
                        const float x0 = bf16_bits_to_f32(f32_to_bf16_bits(va[2 * e + f]));
                        const float x1 = bf16_bits_to_f32(f32_to_bf16_bits(vb[2 * e + f]));
                        rope_rotate(x0, x1, cc[f], ss[f], va[2 * e + f], vb[2 * e + f]);
                    }
                }
            }
            const size_t o = (size_t)(col / out_chunk) * M * out_chunk + (size_t)m * out_chunk + col % out_chunk;
            uint4 pk;
            pk.x = pack_bf16x2(va[0], va[1]); pk.y = pack_bf16x2(va[2], va[3]);
            pk.z = pack_bf16x2(va[4], va[5]); pk.w = pack_bf16x2(va[6], va[7]);
            *reinterpret_cast<uint4*>(out + o) = pk;
            pk.x = pack_bf16x2(vb[0], vb[1]); pk.y = pack_bf16x2(vb[2], vb[3]);
            pk.z = pack_bf16x2(vb[4], vb[5]); pk.w = pack_bf16x2(vb[6], vb[7]);
            *reinterpret_cast<uint4*>(out + o + half) = pk;
        }
        return;
    }
    constexpr int CG = OUT_BN / 8;                         // 8-column groups per tile row
    for (int u = tid; u < BM * CG; u += NT) {
        const int row = u / CG, cg = u % CG;
        const int m = rt * BM + row, col = col0 + ct * OUT_BN + cg * 8;      // this launch covers columns [col0, col_end)
        if (m >= M || col >= col_end) continue;
        const float4 v0 = *reinterpret_cast<const float4*>(tile + row * LIN_PAD + cg * 8);
        const float4 v1 = *reinterpret_cast<const float4*>(tile + row * LIN_PAD + cg * 8 + 4);
        float v[8] = {v0.x, v0.y, v0.z, v0.w, v1.x, v1.y, v1.z, v1.w};
        if constexpr (EPI == LIN_PARTIAL) {
            float* po = reinterpret_cast<float*>(out) + ((size_t)blockIdx.y * M + m) * N + col;
            *reinterpret_cast<float4*>(po) = v0;
            *reinterpret_cast<float4*>(po + 4) = v1;
            continue;
        }
        const size_t o = (size_t)(col / out_chunk) * M * out_chunk + (size_t)m * out_chunk + col % out_chunk;
        if constexpr (EPI == LIN_SWIGLU) {
            const float4 u0 = *reinterpret_cast<const float4*>(tile + row * LIN_PAD + 64 + cg * 8);
            const float4 u1 = *reinterpret_cast<const float4*>(tile + row * LIN_PAD + 64 + cg * 8 + 4);
            const float up[8] = {u0.x, u0.y, u0.z, u0.w, u1.x, u1.y, u1.z, u1.w};
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] = v[e] / (1.f + expf(-v[e])) * up[e];
        }
        if constexpr (EPI == LIN_RESIDUAL) {
            const uint4 r = *reinterpret_cast<const uint4*>(residual + o);
            const uint32_t rr[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) { v[2 * e] += bf16_lo(rr[e]); v[2 * e + 1] += bf16_hi(rr[e]); }
        }
        uint4 pk;
        pk.x = pack_bf16x2(v[0], v[1]); pk.y = pack_bf16x2(v[2], v[3]);
        pk.z = pack_bf16x2(v[4], v[5]); pk.w = pack_bf16x2(v[6], v[7]);
        *reinterpret_cast<uint4*>(out + o) = pk;
    }
#endif
}

namespace {
template <int TM, int EPI>
int launch_linear(const void* a, const void* w, int M, int N, int K, const void* residual, void* out, int out_chunk,
                  int ksplit, int col0, int col_end, hipStream_t st, const float2* rope_cs = nullptr, int rope_dh = 0) {
    using C = LinCfg<TM>;
    static PerDeviceOnce lds_setup;      // per instantiation
    if (!lds_setup.run([] { return raise_dynamic_lds(linear_bf16_kernel<TM, EPI>, C::LDS); })) return D3TOM_ERR_DEVICE;
    const int out_bn = (EPI == LIN_SWIGLU) ? 64 : 128;
    const int NRT = ceil_div(M, C::BM), NCT = ceil_div(col_end - col0, out_bn);
    const int cpx = ceil_div(NCT, 8);
    int PC = 32 / NRT;
    PC = PC < 4 ? 4 : (PC > 16 ? 16 : PC);
    if (PC > cpx) PC = cpx;
    const int panels = ceil_div(cpx, PC);
    const dim3 grid(8u * (unsigned)(panels * PC * NRT), (unsigned)ksplit);
    D3TOM_LAUNCH(LINEAR, st, (linear_bf16_kernel<TM, EPI><<<grid, 512, C::LDS, st>>>(
        (const uint16_t*)a, (const uint16_t*)w, M, N, K, (const uint16_t*)residual, (uint16_t*)out, out_chunk,
        NRT, NCT, cpx, PC, col0, col_end, rope_cs, rope_dh)));
    return D3TOM_OK;
}

template <int EPI>
int launch_linear_tm(int tm, const void* a, const void* w, int M, int N, int K, const void* residual, void* out,
                     int out_chunk, int col0, int col_end, hipStream_t st, const float2* rope_cs = nullptr, int rope_dh = 0) {
    switch (tm) {
        case 1: return launch_linear<1, EPI>(a, w, M, N, K, residual, out, out_chunk, 1, col0, col_end, st, rope_cs, rope_dh);
        case 2: return launch_linear<2, EPI>(a, w, M, N, K, residual, out, out_chunk, 1, col0, col_end, st, rope_cs, rope_dh);
        default: return launch_linear<4, EPI>(a, w, M, N, K, residual, out, out_chunk, 1, col0, col_end, st, rope_cs, rope_dh);
    }
}
}  // namespace

// Row-tile height for a problem.  Taller tiles move fewer operand bytes per flop, and fewer workgroups then
// share (and ask at the same moment for) the same rows of w, which matters when w comes cold from HBM, as a
// block's weights do (read once per step).  Measured per-flop throughput of a full machine with cold weights:
// 64 rows 0.55, 128 rows 0.72 of what 256 rows reach (0.75 / 0.92 with w resident in the memory-side cache).
// But the grid runs in whole rounds of 256 workgroups (one per compute unit), so a partly filled last
// round can cost more than the tile gains.  Estimated time = rounds * rows per tile / efficiency; the
// smallest estimate wins, ties go to the smaller tile.
static double linear_estimate(int tm, int M, int n_tiles_n) {
    static const double eff[5] = {0.0, 0.55, 0.72, 0.0, 1.0};
    const long tiles = (long)ceil_div(M, tm * 64) * n_tiles_n;
    return (double)((tiles + 255) / 256) * tm / eff[tm];
}
int linear_pick_tm(int M, int n_tiles_n, double* est) {
    int best = 1;
    double best_t = 0.0;
    for (int tm = 1; tm <= 4; tm <<= 1) {
        const double t = linear_estimate(tm, M, n_tiles_n);
        if (tm == 1 || t < best_t - 1e-9) { best = tm; best_t = t; }
    }
    if (est) *est = best_t;
    return best;
}
// A last round that is mostly empty can be cut off: the leading column tiles that fill whole rounds of
// 256-row tiles go in one launch, the remaining columns in a second launch with whatever tile suits them.
// Returns the number of column tiles of the first launch (0 = one launch is as good) and both tile heights.
int linear_plan_two(int M, int n_tiles_n, int* tm_a, int* tm_b) {
    double single;
    *tm_a = linear_pick_tm(M, n_tiles_n, &single);
    *tm_b = 0;
    const int nrt4 = ceil_div(M, 256);
    const int rounds = (int)((long)nrt4 * n_tiles_n / 256);
    if (rounds < 1) return 0;
    const int cols_a = rounds * 256 / nrt4;
    if (cols_a >= n_tiles_n) return 0;
    double rest;
    const int tb = linear_pick_tm(M, n_tiles_n - cols_a, &rest);
    if (rounds * 4.0 + rest > 0.93 * single) return 0;         // not worth a second launch
    *tm_a = 4; *tm_b = tb;
    return cols_a;
}

// Number of contraction slices for a projection whose result goes through the row-wise add-and-normalise
// kernel anyway: 4 when the 256-row tiles of the whole problem fill at most a quarter of the chip and each
// slice still has a long enough k-loop, else 1 (no split).
int linear_split_plan(int M, int N, int K) {
    const long tiles = (long)ceil_div(M, 256) * ceil_div(N, LIN_BN);
    const int nkt = K / LIN_BK;
    return (K % LIN_BK == 0 && N % 8 == 0 && tiles * 4 <= 256 && nkt % 4 == 0 && nkt >= 32) ? 4 : 1;
}

// a w^T as `ksplit` float32 partial matrices [ksplit][M][N] (256-row tiles)
int linear_partial_run(const void* a, const void* w, int M, int N, int K, int ksplit, float* partial, hipStream_t st) {
    if (!a || !w || !partial || M < 1 || N < 1 || K < 1 || ksplit < 1) return D3TOM_ERR_INVALID_ARG;
    if (!aligned16(a) || !aligned16(w) || !aligned16(partial)) return D3TOM_ERR_INVALID_ARG;
    if (K % (LIN_BK * ksplit) != 0 || N % 8 != 0) return D3TOM_ERR_UNSUPPORTED;
    if ((size_t)M * K * 2 >= (1ull << 31) || (size_t)N * K * 2 >= (1ull << 31)) return D3TOM_ERR_UNSUPPORTED;
    return launch_linear<4, LIN_PARTIAL>(a, w, M, N, K, nullptr, partial, N, ksplit, 0, N, st);
}

// rope_cs != nullptr (PLAIN only, stacked q | k | v weight with out_chunk = d, head size rope_dh of 64 or 128): the
// rotary embedding of the q and k sections is applied in the epilogue; rope_cs[row * rope_dh / 2 + c] = (cos, sin)
int linear_run(const void* a, const void* w, int M, int N, int K, int epilogue, const void* residual, void* out,
               int out_chunk, int tm_override, hipStream_t st, const float2* rope_cs, int rope_dh) {
    if (!a || !w || !out || M < 1 || N < 1 || K < 1) return D3TOM_ERR_INVALID_ARG;
    if (epilogue < LIN_PLAIN || epilogue > LIN_SWIGLU) return D3TOM_ERR_INVALID_ARG;
    if (rope_cs && (epilogue != LIN_PLAIN || (rope_dh != 64 && rope_dh != 128) || out_chunk <= 0 || out_chunk % rope_dh != 0 ||
                    N != 3 * out_chunk))
        return D3TOM_ERR_INVALID_ARG;
    if (epilogue == LIN_RESIDUAL && !residual) return D3TOM_ERR_INVALID_ARG;
    if (!aligned16(a) || !aligned16(w) || !aligned16(out) || (residual && !aligned16(residual))) return D3TOM_ERR_INVALID_ARG;
    if (K % LIN_BK != 0) return D3TOM_ERR_UNSUPPORTED;
    const int n_out = (epilogue == LIN_SWIGLU) ? N / 2 : N;
    if (epilogue == LIN_SWIGLU && (N % 2 != 0)) return D3TOM_ERR_INVALID_ARG;
    if (n_out % 8 != 0) return D3TOM_ERR_UNSUPPORTED;
    if (out_chunk <= 0) out_chunk = n_out;
    if (out_chunk % 8 != 0 || n_out % out_chunk != 0) return D3TOM_ERR_INVALID_ARG;
    if (epilogue != LIN_PLAIN && out_chunk != n_out) return D3TOM_ERR_INVALID_ARG;
    // 32-bit byte offsets inside each operand
    if ((size_t)M * K * 2 >= (1ull << 31) || (size_t)N * K * 2 >= (1ull << 31)) return D3TOM_ERR_UNSUPPORTED;
    const int out_bn = (epilogue == LIN_SWIGLU) ? 64 : 128;
    auto launch = [&](int tm, int col0, int col_end) {
        switch (epilogue) {
            case LIN_PLAIN:
                if (rope_cs) return launch_linear_tm<LIN_ROPE>(tm, a, w, M, N, K, residual, out, out_chunk, col0, col_end, st, rope_cs, rope_dh);
                return launch_linear_tm<LIN_PLAIN>(tm, a, w, M, N, K, residual, out, out_chunk, col0, col_end, st);
            case LIN_RESIDUAL: return launch_linear_tm<LIN_RESIDUAL>(tm, a, w, M, N, K, residual, out, out_chunk, col0, col_end, st);
            default: return launch_linear_tm<LIN_SWIGLU>(tm, a, w, M, N, K, residual, out, out_chunk, col0, col_end, st);
        }
    };
    if (tm_override == 1 || tm_override == 2 || tm_override == 4) return launch(tm_override, 0, n_out);
    int tm_a, tm_b;
    const int cols_a = linear_plan_two(M, ceil_div(n_out, out_bn), &tm_a, &tm_b);
    if (cols_a == 0) return launch(tm_a, 0, n_out);
    const int status = launch(tm_a, 0, cols_a * out_bn);
    return status != D3TOM_OK ? status : launch(tm_b, cols_a * out_bn, n_out);
}

}  // namespace d3tom

extern "C" int d3tom_linear(const void* a, const void* w, int rows, int n_w_rows, int K, int epilogue,
                            const void* residual, void* out, int out_chunk, void* stream) {
    return d3tom::linear_run(a, w, rows, n_w_rows, K, epilogue, residual, out, out_chunk, 0, (hipStream_t)stream, nullptr, 0);
}

// Same as d3tom_linear with the row-tile height fixed (64, 128 or 256 rows: tile = 1, 2, 4); for tuning.
extern "C" int d3tom_linear_tile(const void* a, const void* w, int rows, int n_w_rows, int K, int epilogue,
                                 const void* residual, void* out, int out_chunk, int tile, void* stream) {
    if (tile != 1 && tile != 2 && tile != 4) return D3TOM_ERR_INVALID_ARG;
    return d3tom::linear_run(a, w, rows, n_w_rows, K, epilogue, residual, out, out_chunk, tile, (hipStream_t)stream, nullptr, 0);
}
