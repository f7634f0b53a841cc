// d3tom_merge: similarity-based merging (Section 3.2, "Similarity-Based Merging"; Algorithm 1, the
// FORALL block and the "Remove positions" line).
//
// Stages, all on the caller's stream:
//   norms     1 / ||row|| of every KEPT row of the similarity features (1 wave / row): the argmax over
//             kept slots of dot / (|m| |k|) does not depend on |m|, the pruned row's own norm; the same
//             waves write the ascending list of pruned visual tokens (the gaps of the ascending kept_idx)
//             and initialise the token -> (best value, slot) table
//   cosine    pruned x kept similarity GEMM on MFMA 32x32x16 bf16 with the argmax fused into the
//             epilogue: only (best value, best slot) per (pruned row, 128-slot column tile) ever
//             leaves the registers, as ONE 64-bit integer atomic max on the row's table entry (value in
//             the high word as an order-preserving integer, 2^32-1-slot in the low word: the maximum is
//             the best cosine, the lowest slot among equals, whatever order the tiles arrive in, so the
//             result is bit-reproducible); the M x k matrix is never written
//   scatter   one workgroup per OUTPUT row: a merged row scans the table for its members (ascending
//             token order), streams them with 16-byte loads and accumulates in float32 in that order,
//             other rows are copied; one store per element, no float atomics
//
// All similarities are taken on the rows as given (assignment first, aggregation afterwards).
#include "internal.hpp"
#include "direct_load.hpp"

namespace d3tom {

constexpr int COS_BN = 128;        // kept slots per column tile
constexpr int COS_BK = 64;         // contraction elements per LDS stage

// split-K partial products: at most COS_SPLIT_BLOCKS (tile, k-slice) blocks of 64 x 128 floats
constexpr int COS_SPLIT_BLOCKS = 256;
struct MergeWs {
    size_t pruned_off, rnorm_off, table_off, dots_off, total;
    int VP;                    // table entries per sample
};
__host__ inline MergeWs merge_ws_layout(int B, int max_V) {
    MergeWs w;
    w.VP = (int)align_up((size_t)max_V, 4);
    size_t o = 0;
    w.pruned_off = o; o += align_up((size_t)B * max_V * 4, 256);
    w.rnorm_off = o;  o += align_up((size_t)B * max_V * 4, 256);
    w.table_off = o;  o += align_up((size_t)B * w.VP * 8, 256);     // token -> (best value, slot) table
    w.dots_off = o;   o += (size_t)COS_SPLIT_BLOCKS * 64 * 128 * sizeof(float);
    w.total = o;
    return w;
}
size_t merge_ws_bytes(int B, int max_V) { return merge_ws_layout(B, max_V).total; }
void merge_prep_targets(void* merge_ws, int B, int max_V, MergePrep* prep) {
    const MergeWs w = merge_ws_layout(B, max_V);
    char* wsb = (char*)merge_ws;
    prep->pruned = (int32_t*)(wsb + w.pruned_off);
    prep->rnorm = (float*)(wsb + w.rnorm_off);
    prep->table = (table_t*)(wsb + w.table_off);
    prep->VP = w.VP;
}

struct SampleGeom { int tok0, N, vs, V, k, M; };
__device__ __forceinline__ SampleGeom sample_geom(int b, const int32_t* seq_off, const int32_t* vis_start,
                                                  const int32_t* vis_count, const int32_t* kept_off, int max_V, int max_keep) {
    SampleGeom s;
    s.tok0 = seq_off[b];
    s.N = seq_off[b + 1] - s.tok0;
    s.vs = min(max(vis_start[b], 0), s.N);
    s.V = min(min(vis_count[b], max_V), s.N - s.vs);
    s.k = min(min(kept_off[b + 1] - kept_off[b], max_keep), s.V);
    s.M = s.V - s.k;
    return s;
}

// ---- norms + pruned list + table init --------------------------------------------------------------
// One wave per kept slot r computes 1 / ||row|| of that slot's token.  The same wave also writes the
// piece of the ascending pruned list that lies in front of its token: kept_idx is ascending, so the
// pruned tokens j between kept_idx[r-1] and kept_idx[r] have exactly r kept tokens before them and sit
// at positions j - r of the list (the wave of the last slot also writes the piece behind its token).
// No scan, no extra workgroup.  The table entries of the same tokens are set on the way: "nothing yet"
// for the pruned ones, its own slot for the kept one.
template <typename T>
__global__ __launch_bounds__(256) void merge_norms_kernel(
    const T* __restrict__ f, int d, const int32_t* __restrict__ seq_off, const int32_t* __restrict__ vis_start,
    const int32_t* __restrict__ vis_count, const int32_t* __restrict__ kept_idx, const int32_t* __restrict__ kept_off,
    int max_V, int max_keep, float* __restrict__ rnorm, int32_t* __restrict__ pruned, table_t* __restrict__ table, int VP) {
    const int b = blockIdx.y;
    const SampleGeom s = sample_geom(b, seq_off, vis_start, vis_count, kept_off, max_V, max_keep);
    const int r = blockIdx.x * 4 + (threadIdx.x >> 6);      // kept slot
    const int lane = threadIdx.x & 63;
    if (r >= s.k) return;
    const int32_t* kp = kept_idx + kept_off[b];
    const int j = min(max(kp[r], 0), s.V - 1);
    {
        int32_t* pr = pruned + (size_t)b * max_V;
        table_t* tab = table + (size_t)b * VP;
        const int lo = (r == 0) ? -1 : min(max(kp[r - 1], 0), s.V - 1);
        // positions are >= 0 whenever kept_idx is ascending and free of repeats; the guard only keeps an
        // invalid list from writing in front of the array
        for (int t = lo + 1 + lane; t < j; t += 64) { tab[t] = 0; if (t >= r) pr[t - r] = t; }
        if (r == s.k - 1)
            for (int t = j + 1 + lane; t < s.V; t += 64) { tab[t] = 0; if (t >= s.k) pr[t - s.k] = t; }
        if (lane == 0) tab[j] = table_entry_kept(r);
    }
    const float ss = row_sum_squares(f + (size_t)(s.tok0 + s.vs + j) * d, d, lane);
    if (lane == 0) rnorm[(size_t)b * max_V + r] = reciprocal_norm(ss);
}

// ---- cosine GEMM + fused argmax, bf16 MFMA ---------------------------------------------------
// Workgroup tile: (TM*64) pruned rows x 128 kept slots; waves 0..3 compute (2 x 2, wave tile (TM*32) x 64),
// waves 4..7 only issue the loads.
//
// Operand tiles go HBM/L2 -> LDS with direct loads (buffer_load ... lds, 16 bytes per lane, no register
// staging) into a ring of COS_NS stages of 64 contraction elements; the loads of stage kt+3 are in
// flight while stage kt feeds the MFMAs, one s_barrier per stage.  A wave-load writes 1 KB of LDS
// contiguously (8 rows x 128 B), so rows cannot be padded; instead the 16-byte chunk that lands in
// position p of row r is chunk p ^ ((r >> 1) & 7) of that row (the lane picks its global address
// accordingly), which spreads the MFMA operand reads of 16 consecutive rows over all 64 banks.
//
// Workgroup ids are mapped to tiles per XCD: ids are dealt round-robin to the 8 XCDs by the hardware.  The
// tiles of a sample are numbered band by band (RB row tiles high, column-major inside a band) and that
// sequence is cut into 8 runs of equal length, one per XCD: every XCD gets the same number of tiles
// (a rectangle per XCD leaves some XCDs with more tiles than they have CUs while others idle), and a
// run covers a compact block of about RB x (run / RB) tiles, so its private L2 sees few operand rows.
// The loads are buffer loads: each lane's byte offset (row and swizzled chunk) is fixed for the whole
// sweep and the k-slice moves through the scalar offset, so a stage costs no address arithmetic.
constexpr int cos_ring_stages(int TM) { return TM >= 4 ? 3 : 4; }     // 256-row tiles: 3 stages of 48 KB fit the 160 KB of LDS
constexpr int COS_NS_MIN = 3;

template <int TM>
__global__ __launch_bounds__(512) void cos_argmax_bf16(
    const uint16_t* __restrict__ f, int d, const int32_t* __restrict__ seq_off, const int32_t* __restrict__ vis_start,
    const int32_t* __restrict__ vis_count, const int32_t* __restrict__ kept_idx, const int32_t* __restrict__ kept_off,
    int max_V, int max_keep, const int32_t* __restrict__ pruned, const float* __restrict__ rnorm,
    table_t* __restrict__ table, int VP, int per, int RB, int ksplit, float* __restrict__ dots, int nrt_launch, int nct_launch, int rn_by_token) {
#if defined(__HIP_DEVICE_COMPILE__)
    constexpr int BM = TM * 64;
    constexpr int COS_NS = cos_ring_stages(TM);
    constexpr int STAGE = (BM + COS_BN) * 128;          // bytes per ring stage (64 bf16 = 128 B per row)
    constexpr int A_LD = BM / 32;                       // direct loads per wave and stage, A tile (8 rows each)
    constexpr int B_LD = COS_BN / 32;
    constexpr int LPS = A_LD + B_LD;                    // loads per wave and stage
    extern __shared__ __attribute__((aligned(16))) char ring[];
    __shared__ float rnB[COS_BN];

    // blockIdx.x = sample * 8 * per + id; id & 7 is the XCD the hardware puts the workgroup on.  The launch is sized
    // for the largest sample (per = an eighth of its tiles); every sample numbers ITS OWN tiles and cuts that sequence
    // into 8 equal runs, so that a sample with fewer tiles still loads the 8 XCDs alike (numbered on the launch's
    // grid, the tiles of a short sample would all fall to the first XCDs).
    const int b = blockIdx.x / (8 * per);
    const int id = blockIdx.x % (8 * per);
    const SampleGeom s = sample_geom(b, seq_off, vis_start, vis_count, kept_off, max_V, max_keep);
    const int nrt_b = min((s.M + BM - 1) / BM, nrt_launch), nct_b = min((s.k + COS_BN - 1) / COS_BN, nct_launch);
    const int tiles_b = nrt_b * nct_b;
    const int per_b = (tiles_b + 7) >> 3;
    if ((id >> 3) >= per_b) return;
    const int t_lin = (id & 7) * per_b + (id >> 3);
    if (t_lin >= tiles_b) return;
    int rt, ct;
    {
        // bands about as high as a run's block is wide (RB was chosen that way for the launch's grid; a smaller
        // sample gets its own)
        int rb = RB;
        if (per_b < per) { rb = 1; while ((rb + 1) * (rb + 1) <= per_b) ++rb; }
        rb = min(rb, nrt_b);
        const int band = rb * nct_b, nfull = nrt_b / rb;
        if (t_lin < nfull * band) { const int rem = t_lin % band; rt = (t_lin / band) * rb + rem % rb; ct = rem / rb; }
        else { const int t2 = t_lin - nfull * band, rl = nrt_b - nfull * rb; rt = nfull * rb + t2 % rl; ct = t2 / rl; }
    }

    const int tid = threadIdx.x, wave = (tid >> 6) & 3, lane = tid & 63;
    const bool loader = tid >> 8;                          // waves 4..7 only move data, waves 0..3 only compute
    const int wm = wave >> 1, wn = wave & 1;
    const int c = lane & 31, g = lane >> 5;
    const int32_t* pr = pruned + (size_t)b * max_V;
    const int32_t* kp = kept_idx + kept_off[b];
    const float* rn = rnorm + (size_t)b * max_V;
    const size_t base = (size_t)(s.tok0 + s.vs) * d;

    // byte offset of this lane inside the visual block for each of its direct loads (rows past the end
    // re-read row 0; masked later); the k-slice is added through the scalar offset
    const __amdgpu_buffer_rsrc_t rsrc = make_uniform_rsrc(f + base, (uint32_t)((size_t)s.V * d * sizeof(uint16_t)));
    int a_off[A_LD], b_off[B_LD];
#pragma unroll
    for (int i = 0; i < A_LD; ++i) {
        const int row = wave * (BM / 4) + i * 8 + (lane >> 3);
        const int cg = (lane & 7) ^ ((row >> 1) & 7);
        const int p = rt * BM + row;
        const int m = min(max((p < s.M) ? pr[p] : pr[0], 0), s.V - 1);
        a_off[i] = m * d * 2 + cg * 16;
    }
#pragma unroll
    for (int i = 0; i < B_LD; ++i) {
        const int row = wave * (COS_BN / 4) + i * 8 + (lane >> 3);
        const int cg = (lane & 7) ^ ((row >> 1) & 7);
        const int r = ct * COS_BN + row;
        const int j = min(max(kp[(r < s.k) ? r : 0], 0), s.V - 1);
        b_off[i] = j * d * 2 + cg * 16;
    }
    for (int t = tid; t < COS_BN; t += 512) {
        const int r = ct * COS_BN + t;
        // 1 / norm of the kept row in slot r: stored by slot, or by token when the selection launch computed them
        rnB[t] = (r < s.k) ? rn[rn_by_token ? min(max(kp[r], 0), s.V - 1) : r] : 0.f;
    }
    // split-K: slice blockIdx.y of the contraction (ksplit slices of nkt stages each)
    const int nkt = (d / COS_BK) / ksplit;
    const int kt0 = (int)blockIdx.y * nkt;
    // LDS destinations are wave-uniform: this wave's first row of the A (B) tile, made a scalar once so
    // that a load costs one scalar add for its M0 value and no vector instruction
    const uint32_t ring0 = (uint32_t)(size_t)(lds_ptr_t)ring;
    const uint32_t a_lds = __builtin_amdgcn_readfirstlane(ring0 + wave * (BM / 4) * 128);
    const uint32_t b_lds = __builtin_amdgcn_readfirstlane(ring0 + BM * 128 + wave * (COS_BN / 4) * 128);
    // loads [n0, n1) of a stage's LPS loads (A tile first, then B tile)
    auto issue_part = [&](int kt, int stage, int n0, int n1) {
#pragma unroll
        for (int i = 0; i < A_LD; ++i)
            if (i >= n0 && i < n1)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_ptr_t)(size_t)(a_lds + stage * STAGE + i * 8 * 128), 16,
                                                         a_off[i], (kt0 + kt) * (COS_BK * 2), 0, 0);
#pragma unroll
        for (int i = 0; i < B_LD; ++i)
            if (A_LD + i >= n0 && A_LD + i < n1)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_ptr_t)(size_t)(b_lds + stage * STAGE + i * 8 * 128), 16,
                                                         b_off[i], (kt0 + kt) * (COS_BK * 2), 0, 0);
    };
    auto issue = [&](int kt, int stage) { issue_part(kt, stage, 0, LPS); };

    f32x16 acc[TM][2];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    // byte offsets of this lane's operand fragments inside a stage (k-step kk adds the swizzled chunk)
    int a_row[TM], b_row[2], a_sw[TM], b_sw[2];
#pragma unroll
    for (int i = 0; i < TM; ++i) { const int Rr = wm * (TM * 32) + i * 32 + c; a_row[i] = Rr * 128; a_sw[i] = (Rr >> 1) & 7; }
#pragma unroll
    for (int j = 0; j < 2; ++j) { const int Rr = wn * 64 + j * 32 + c; b_row[j] = BM * 128 + Rr * 128; b_sw[j] = (Rr >> 1) & 7; }

    // one stage: feed stage kt to the MFMAs
    auto stage = [&](int kt) {
        const char* sb = ring + (kt % COS_NS) * STAGE;
        // operand fragments are read one k-step ahead of the MFMAs that use them, so the LDS latency
        // of step kk + 1 is covered by the matrix work of step kk
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
        for (int kk = 0; kk < COS_BK / 16; ++kk) {
            if (kk + 1 < COS_BK / 16) read_frags(kk + 1, (kk + 1) & 1);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[kk & 1][i], bfr[kk & 1][j], acc[i][j], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    // A wave that issues a direct load waits for room in the CU's vector-memory queue; in a computing wave
    // that wait stalls the MFMA stream, so the loads have waves of their own.  One s_barrier per stage:
    // the loaders arrive once stage kt has landed, the consumers once they are done with stage kt-1,
    // whose slot the loaders then refill with stage kt+COS_NS-1.
    if (loader) {
#pragma unroll
        for (int st = 0; st < COS_NS - 1; ++st)
            if (st < nkt) issue(st, st);
        for (int kt = 0; kt < nkt; ++kt) {
            if (kt + COS_NS - 2 <= nkt - 1) wait_loads_and_barrier<(COS_NS - 2) * LPS>();
            else wait_loads_and_barrier<0>();
            if (kt + COS_NS - 1 < nkt) issue(kt + COS_NS - 1, (kt + COS_NS - 1) % COS_NS);
        }
    } else {
        for (int kt = 0; kt < nkt; ++kt) {
            wait_loads_and_barrier<0>();
            stage(kt);
        }
    }

    if (ksplit > 1) {
        // partial products of this k-slice: block (slice, tile) of BM x 128 floats, summed by cos_reduce_argmax
        const int tile_id = (b * nrt_launch + rt) * nct_launch + ct;
        const int n_tiles = (int)(gridDim.x / (8 * per)) * nrt_launch * nct_launch;
        float* blk = dots + ((size_t)blockIdx.y * n_tiles + tile_id) * (BM * COS_BN);
        if (loader) return;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int row = wm * (TM * 32) + i * 32 + (e >> 2) * 8 + g * 4 + (e & 3);
                    blk[row * COS_BN + wn * 64 + j * 32 + c] = acc[i][j][e];
                }
        return;
    }
    // epilogue: dot * rn_col (the cosine up to the row's own positive norm, which is the same for all of
    // its candidates); per row, best (value, slot) over this tile's columns.
    // The 64 candidates of a row (32 lanes x 2 wave columns) meet in LDS (the ring is free once all waves
    // are past the loop): every lane folds its two columns of a row into one candidate (branch-free; equal
    // values keep the lower slot) and stores it, then two threads per row scan 32 candidates each in
    // ascending slot order.  Rows are padded to 33 entries so that the scan of 32 different rows hits 32
    // different banks.
    __syncthreads();                                           // all waves are done with the ring
    float2* cand = reinterpret_cast<float2*>(ring);            // [BM][2][33]
    if (!loader) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int row = wm * (TM * 32) + i * 32 + (e >> 2) * 8 + g * 4 + (e & 3);
                const int col0 = wn * 64 + c, col1 = col0 + 32;
                const int s0 = ct * COS_BN + col0, s1 = s0 + 32;
                const float v0 = (s0 < s.k) ? acc[i][0][e] * rnB[col0] : -INFINITY;
                const float v1 = (s1 < s.k) ? acc[i][1][e] * rnB[col1] : -INFINITY;
                const bool t1 = v1 > v0;                       // equal values: the lower slot stays
                cand[(row * 2 + wn) * 33 + c] = make_float2(t1 ? v1 : v0, __int_as_float(t1 ? s1 : s0));
            }
    }
    __syncthreads();
    for (int t = tid; t < BM * 2; t += 512) {
        const int row = t >> 1, half = t & 1;                  // half 0: slots of wave column 0 (lower slots)
        const float2* cr = cand + (row * 2 + half) * 33;
        float best = -INFINITY; int bidx = 0x7FFFFFFF;
#pragma unroll 8
        for (int q2 = 0; q2 < 32; ++q2) {
            const float2 a = cr[q2];
            const int ia = __float_as_int(a.y);
            const bool take = (a.x > best) | ((a.x == best) & (ia < bidx));
            best = take ? a.x : best; bidx = take ? ia : bidx;
        }
        const float ov = __shfl_xor(best, 1, WAVE);
        const int oi = __shfl_xor(bidx, 1, WAVE);
        const bool take = (ov > best) | ((ov == best) & (oi < bidx));
        best = take ? ov : best; bidx = take ? oi : bidx;
        const int p = rt * BM + row;
        if (half == 0 && p < s.M) {
            const int tok = min(max(pr[p], 0), s.V - 1);
            atomicMax(table + (size_t)b * VP + tok, table_entry(best, bidx));
        }
    }
#endif
}

// ---- split-K second step: sum the k-slices, scale by the kept row's 1/norm, argmax over all slots ----
// Used when the similarity matrix has too few tiles to occupy the chip (short sequences): the GEMM is
// then cut along the contraction instead, and one wave per pruned row finishes the job here.  Slices
// are added in ascending order and slots are visited in ascending order, so the result is deterministic
// and ties go to the lowest slot.  The wave writes the row's table entry itself.
__global__ __launch_bounds__(256) void cos_reduce_argmax(
    const int32_t* __restrict__ seq_off, const int32_t* __restrict__ vis_start, const int32_t* __restrict__ vis_count,
    const int32_t* __restrict__ kept_off,
    int max_V, int max_keep, const int32_t* __restrict__ pruned, const float* __restrict__ rnorm,
    const float* __restrict__ dots, int ksplit, int n_tiles, int nrt_launch, int nct_launch,
    table_t* __restrict__ table, int VP, const int32_t* __restrict__ kept_idx /* != nullptr: rnorm is indexed by token */) {
    constexpr int BM = 64;
    const int b = blockIdx.y;
    const SampleGeom s = sample_geom(b, seq_off, vis_start, vis_count, kept_off, max_V, max_keep);
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int p = blockIdx.x * 4 + wave;
    if (s.k <= 0 || p >= s.M) return;
    const float* rn = rnorm + (size_t)b * max_V;
    const int rt = p / BM, lr = p % BM;
    const int nct = (s.k + COS_BN - 1) / COS_BN;
    float best = -INFINITY; int bidx = 0x7FFFFFFF;
    for (int ct = 0; ct < nct; ++ct) {
        const int tile_id = (b * nrt_launch + rt) * nct_launch + ct;
        // all slices of both column halves are requested before the first add (at most 16 slices)
        float v[2][16];
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            const int col = half * 64 + lane;
            const bool ok = ct * COS_BN + col < s.k;
#pragma unroll
            for (int ks = 0; ks < 16; ++ks)
                v[half][ks] = (ok && ks < ksplit) ? dots[((size_t)ks * n_tiles + tile_id) * (BM * COS_BN) + lr * COS_BN + col] : 0.f;
        }
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            const int slot = ct * COS_BN + half * 64 + lane;
            if (slot < s.k) {
                float sum = 0.f;
#pragma unroll
                for (int ks = 0; ks < 16; ++ks) sum += v[half][ks];        // ascending slices; absent ones add 0
                const float val = sum * rn[kept_idx ? min(max(kept_idx[kept_off[b] + slot], 0), s.V - 1) : slot];
                if (val > best) { best = val; bidx = slot; }
            }
        }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const float ov = __shfl_xor(best, o, WAVE);
        const int oi = __shfl_xor(bidx, o, WAVE);
        const bool take = (ov > best) | ((ov == best) & (oi < bidx));
        best = take ? ov : best; bidx = take ? oi : bidx;
    }
    if (lane == 0) {
        const int slot = min(max(bidx, 0), s.k - 1);
        const int tok = min(max(pruned[(size_t)b * max_V + p], 0), s.V - 1);
        table[(size_t)b * VP + tok] = table_entry(best, slot);
    }
}

// ---- cosine + argmax, generic: one workgroup per pruned row, waves stride over the kept slots ---
template <typename T>
__global__ __launch_bounds__(256) void cos_argmax_generic(
    const T* __restrict__ f, int d, const int32_t* __restrict__ seq_off, const int32_t* __restrict__ vis_start,
    const int32_t* __restrict__ vis_count, const int32_t* __restrict__ kept_idx, const int32_t* __restrict__ kept_off,
    int max_V, int max_keep, const int32_t* __restrict__ pruned, const float* __restrict__ rnorm,
    table_t* __restrict__ table, int VP, int rn_by_token) {
    const int p = blockIdx.x, b = blockIdx.y;
    const SampleGeom s = sample_geom(b, seq_off, vis_start, vis_count, kept_off, max_V, max_keep);
    if (p >= s.M) return;
    __shared__ float2 red[4];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int m = min(max(pruned[(size_t)b * max_V + p], 0), s.V - 1);
    const int32_t* kp = kept_idx + kept_off[b];
    const float* rn = rnorm + (size_t)b * max_V;
    const T* xm = f + (size_t)(s.tok0 + s.vs + m) * d;
    float bv = -INFINITY; int bi = 0x7FFFFFFF;
    for (int r = wave; r < s.k; r += 4) {
        const int j = min(max(kp[r], 0), s.V - 1);
        const T* xk = f + (size_t)(s.tok0 + s.vs + j) * d;
        float dot = 0.f;
        for (int cidx = lane; cidx < d; cidx += 64) dot += Elem<T>::load(xm + cidx) * Elem<T>::load(xk + cidx);
        dot = wave_sum(dot);
        const float v = dot * rn[rn_by_token ? j : r];        // the pruned row's own norm scales all its candidates alike
        if (v > bv) { bv = v; bi = r; }
    }
    if (lane == 0) red[wave] = make_float2(bv, __int_as_float(bi));
    __syncthreads();
    if (threadIdx.x == 0) {
        float2 a = red[0];
        for (int w = 1; w < 4; ++w) {
            const float2 c2 = red[w];
            if (c2.x > a.x || (c2.x == a.x && __float_as_int(c2.y) < __float_as_int(a.y))) a = c2;
        }
        table[(size_t)b * VP + m] = table_entry(a.x, min(max(__float_as_int(a.y), 0), s.k - 1));
    }
}

// ---- scatter-average + compaction ----------------------------------------------------------
// One workgroup per output row.  A merged row first finds its members: the four waves scan the
// table of the sample (a quarter each, coalesced; the low word of an entry names the slot, and the kept
// token's own entry makes it a member like the others), keep the matches in ascending token
// order (ballot + popcount, no atomics) and the four pieces are joined into one list in LDS; the
// workgroup of a slot also writes the slot into `assign` for each of its members.  The member
// rows are then streamed four at a time so that eight 16-byte loads per thread are in flight;
// accumulation order is ascending token index, so the result does not depend on the unrolling.  A slot
// with more members than the LDS list holds is processed in windows of SCAT_LIST members (re-scan).
constexpr int SCAT_LIST = 256;     // members staged per pass
constexpr int SCAT_WAVE = SCAT_LIST / 4;
template <typename T, int CPT>     // CPT: 16-byte chunks per thread per pass
__global__ __launch_bounds__(256) void merge_scatter_kernel(
    const T* __restrict__ x0, const T* __restrict__ x1, int d, const int32_t* __restrict__ seq_off, const int32_t* __restrict__ vis_start,
    const int32_t* __restrict__ vis_count, const int32_t* __restrict__ kept_idx, const int32_t* __restrict__ kept_off,
    int max_V, int max_keep, int mode, const int32_t* __restrict__ out_off, const table_t* __restrict__ table, int VP,
    const int32_t* __restrict__ vis_off, T* __restrict__ y0, T* __restrict__ y1, int32_t* __restrict__ assign_out,
    int32_t* __restrict__ counts_out, int32_t* __restrict__ src_pos_out, int nslice) {
    constexpr int EPC = 16 / sizeof(T);
    // a row may be cut into nslice column slices, one workgroup each (few output rows: more workgroups)
    const int o = blockIdx.x / nslice, slice = blockIdx.x % nslice, b = blockIdx.y;
    // blockIdx.z selects the payload (a second one shares the routing: key and value caches); the
    // index outputs are written by the first payload's workgroups only
    const T* __restrict__ x = blockIdx.z ? x1 : x0;
    T* __restrict__ y = blockIdx.z ? y1 : y0;
    int32_t* counts = (blockIdx.z || slice) ? nullptr : counts_out;
    int32_t* src_pos = (blockIdx.z || slice) ? nullptr : src_pos_out;
    int32_t* assign = (blockIdx.z || slice || !assign_out) ? nullptr : assign_out + vis_off[b];
    const SampleGeom s = sample_geom(b, seq_off, vis_start, vis_count, kept_off, max_V, max_keep);
    const int N_m = s.N - s.M;
    if (o >= N_m) return;
    __shared__ int list[SCAT_LIST];
    __shared__ int stage[4][SCAT_WAVE];
    __shared__ int wcnt[4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    T* yrow = y + (size_t)(out_off[b] + o) * d;
    const int nch = d / EPC;
    const int c_per = (nch + nslice - 1) / nslice;
    const int c_lo = slice * c_per, c_hi = min(nch, c_lo + c_per);          // this workgroup's 16-byte chunks
    int src = -1, len = 1, r = 0;
    // table of this sample, read two entries (16 bytes) per lane; a wave takes a contiguous part of it
    // (a multiple of 128 entries so that every lane takes part in each ballot)
    const uint4* tab2 = reinterpret_cast<const uint4*>(table + (size_t)b * VP);
    const int part_len = ((s.V + 511) >> 9) << 7;
    const int e0 = wave * part_len;
    const int n_it = part_len >> 7;
    int wbase = 0;                                         // members found by the waves before this one
    bool fits = true;
    uint32_t want = 0;                                     // low word of the entries of this row's slot
    // scan this wave's part: fn(token, ordinal among this wave's matches) for every match, ascending
    auto scan = [&](auto&& fn) {
        int cnt = 0;
        for (int it0 = 0; it0 < n_it; it0 += 4) {
            uint4 v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int i = e0 + (it0 + u) * 128 + lane * 2;
                v[u] = (it0 + u < n_it && i < s.V) ? tab2[i >> 1] : make_uint4(0, 0, 0, 0);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int i = e0 + (it0 + u) * 128 + lane * 2;
                const bool m0 = (v[u].x == want) && (i < s.V), m1 = (v[u].z == want) && (i + 1 < s.V);
                const unsigned long long lt = (1ull << lane) - 1ull;
                const unsigned long long b0 = __builtin_amdgcn_ballot_w64(m0), b1 = __builtin_amdgcn_ballot_w64(m1);
                int ord = cnt + __popcll(b0 & lt) + __popcll(b1 & lt);
                if (m0) fn(i, ord++);
                if (m1) fn(i + 1, ord++);
                cnt += __popcll(b0) + __popcll(b1);
            }
        }
        return cnt;
    };
    if (o < s.vs) src = o;
    else if (o >= s.vs + s.k) src = o + s.M;
    else {
        r = o - s.vs;
        want = 0xFFFFFFFFu - (uint32_t)r;
        const int cnt = scan([&](int tok, int ord) {
            if (ord < SCAT_WAVE) stage[wave][ord] = tok;
            if (assign) assign[tok] = r;
        });
        if (lane == 0) wcnt[wave] = cnt;
        __syncthreads();
        len = wcnt[0] + wcnt[1] + wcnt[2] + wcnt[3];
        fits = wcnt[0] <= SCAT_WAVE && wcnt[1] <= SCAT_WAVE && wcnt[2] <= SCAT_WAVE && wcnt[3] <= SCAT_WAVE;
        for (int w = 0; w < wave; ++w) wbase += wcnt[w];
        const int kept_tok = min(max(kept_idx[kept_off[b] + r], 0), s.V - 1);
        if (tid == 0) {
            if (src_pos) src_pos[out_off[b] + o] = s.vs + kept_tok;
            if (counts) counts[kept_off[b] + r] = len;
        }
        if (len <= 1) src = s.vs + kept_tok;               // nothing absorbed: bit-exact copy
        else if (fits) {
            if (lane < cnt) list[wbase + lane] = stage[wave][lane];
            __syncthreads();
        }
    }
    if (src >= 0) {
        if (tid == 0 && src_pos && (o < s.vs || o >= s.vs + s.k)) src_pos[out_off[b] + o] = src;
        const uint4* in = reinterpret_cast<const uint4*>(x + (size_t)(s.tok0 + src) * d);
        uint4* out = reinterpret_cast<uint4*>(yrow);
        for (int c = c_lo + tid; c < c_hi; c += 256) out[c] = in[c];
        return;
    }
    // members with ordinal in [win0, win0 + SCAT_LIST) -> list (only when the first scan did not fit)
    auto fill_window = [&](int win0) {
        scan([&](int tok, int ord) { const int pos = wbase + ord - win0; if (pos >= 0 && pos < SCAT_LIST) list[pos] = tok; });
    };
    const T* xv = x + (size_t)(s.tok0 + s.vs) * d;
    const float inv = (mode == D3TOM_MERGE_MEAN) ? (float)len : 1.0f;
    auto add_row = [&](float (&acc)[CPT][EPC], const uint4 (&w)[CPT]) {
#pragma unroll
        for (int u = 0; u < CPT; ++u) {
            if constexpr (sizeof(T) == 2) {
                acc[u][0] += bf16_lo(w[u].x); acc[u][1] += bf16_hi(w[u].x);
                acc[u][2] += bf16_lo(w[u].y); acc[u][3] += bf16_hi(w[u].y);
                acc[u][4] += bf16_lo(w[u].z); acc[u][5] += bf16_hi(w[u].z);
                acc[u][6] += bf16_lo(w[u].w); acc[u][7] += bf16_hi(w[u].w);
            } else {
                acc[u][0] += __uint_as_float(w[u].x); acc[u][1] += __uint_as_float(w[u].y);
                acc[u][2] += __uint_as_float(w[u].z); acc[u][3] += __uint_as_float(w[u].w);
            }
        }
    };
    for (int cb = c_lo; cb < c_hi; cb += 256 * CPT) {     // uniform trip count: the loop body has barriers
        const int c0 = cb + tid;
        float acc[CPT][EPC];
#pragma unroll
        for (int u = 0; u < CPT; ++u)
#pragma unroll
            for (int e = 0; e < EPC; ++e) acc[u][e] = 0.f;
        for (int l0 = 0; l0 < len; l0 += SCAT_LIST) {
            const int ln = min(SCAT_LIST, len - l0);
            if (!fits) {                                   // uniform
                __syncthreads();
                fill_window(l0);
                __syncthreads();
            }
            int t = 0;
            if constexpr (CPT == 1)                        // half-row workgroups: registers to spare for 8 rows in flight
            for (; t + 8 <= ln; t += 8) {
                uint4 w[8][CPT];
#pragma unroll
                for (int m = 0; m < 8; ++m) {
                    const uint4* row = reinterpret_cast<const uint4*>(xv + (size_t)list[t + m] * d);
#pragma unroll
                    for (int u = 0; u < CPT; ++u) { const int c = c0 + 256 * u; w[m][u] = (c < c_hi) ? row[c] : make_uint4(0, 0, 0, 0); }
                }
#pragma unroll
                for (int m = 0; m < 8; ++m) add_row(acc, w[m]);
            }
            for (; t + 4 <= ln; t += 4) {
                uint4 w[4][CPT];
#pragma unroll
                for (int m = 0; m < 4; ++m) {
                    const uint4* row = reinterpret_cast<const uint4*>(xv + (size_t)list[t + m] * d);
#pragma unroll
                    for (int u = 0; u < CPT; ++u) { const int c = c0 + 256 * u; w[m][u] = (c < c_hi) ? row[c] : make_uint4(0, 0, 0, 0); }
                }
#pragma unroll
                for (int m = 0; m < 4; ++m) add_row(acc, w[m]);
            }
            for (; t < ln; ++t) {
                uint4 w[CPT];
                const uint4* row = reinterpret_cast<const uint4*>(xv + (size_t)list[t] * d);
#pragma unroll
                for (int u = 0; u < CPT; ++u) { const int c = c0 + 256 * u; w[u] = (c < c_hi) ? row[c] : make_uint4(0, 0, 0, 0); }
                add_row(acc, w);
            }
        }
#pragma unroll
        for (int u = 0; u < CPT; ++u) {
            const int c = c0 + 256 * u;
            if (c < c_hi) {
                uint4 w;
                if constexpr (sizeof(T) == 2) {
                    w.x = pack_bf16x2(acc[u][0] / inv, acc[u][1] / inv);
                    w.y = pack_bf16x2(acc[u][2] / inv, acc[u][3] / inv);
                    w.z = pack_bf16x2(acc[u][4] / inv, acc[u][5] / inv);
                    w.w = pack_bf16x2(acc[u][6] / inv, acc[u][7] / inv);
                } else {
                    w.x = __float_as_uint(acc[u][0] / inv); w.y = __float_as_uint(acc[u][1] / inv);
                    w.z = __float_as_uint(acc[u][2] / inv); w.w = __float_as_uint(acc[u][3] / inv);
                }
                reinterpret_cast<uint4*>(yrow)[c] = w;
            }
        }
    }
}

}  // namespace d3tom

using namespace d3tom;

// Both entry points: norms + pruned list, cosine argmax, token -> slot table, scatter of one or two
// payloads that share the routing.
int d3tom::merge_run(const void* x0, void* y0, const void* x1, void* y1, const void* sim, int d, int d_sim, int dt,
                     int B, const int32_t* seq_off, const int32_t* vis_start, const int32_t* vis_count,
                     const int32_t* vis_off, const int32_t* kept_idx, const int32_t* kept_off,
                     int max_N, int max_V, int max_keep, int max_pruned, int max_out, int mode,
                     const int32_t* out_off, int32_t* assign, int32_t* counts, int32_t* src_pos,
                     void* ws, size_t ws_bytes, void* stream, bool prepared, int out_rows_hint) {
    if (!x0 || !y0 || !seq_off || !vis_start || !vis_count || !vis_off || !kept_idx || !kept_off || !out_off)
        return D3TOM_ERR_INVALID_ARG;
    if ((x1 == nullptr) != (y1 == nullptr)) return D3TOM_ERR_INVALID_ARG;
    if (B < 1 || d < 1 || max_N < 1 || max_V < 1 || max_V > max_N || max_keep < 1 || max_keep > max_V ||
        max_pruned < 0 || max_pruned > max_V || max_out < 1 || max_out > max_N)
        return D3TOM_ERR_INVALID_ARG;
    if (dt != D3TOM_F32 && dt != D3TOM_BF16) return D3TOM_ERR_INVALID_ARG;
    if (mode != D3TOM_MERGE_MEAN && mode != D3TOM_MERGE_SUM) return D3TOM_ERR_INVALID_ARG;
    const int epc = (dt == D3TOM_BF16) ? 8 : 4;
    if (!sim) { sim = x0; d_sim = d; }
    if (d_sim < 1) return D3TOM_ERR_INVALID_ARG;
    if ((d % epc) || (d_sim % epc)) return D3TOM_ERR_UNSUPPORTED;
    if (!aligned16(x0) || !aligned16(sim) || !aligned16(y0) || !aligned16(x1) || !aligned16(y1)) return D3TOM_ERR_INVALID_ARG;
    if (max_V > D3TOM_MAX_VISUAL) return D3TOM_ERR_UNSUPPORTED;
    const MergeWs w = merge_ws_layout(B, max_V);
    if (!ws) return D3TOM_ERR_INVALID_ARG;
    if (ws_bytes < w.total || (((uintptr_t)ws) & 255u)) return D3TOM_ERR_WORKSPACE_TOO_SMALL;
    hipStream_t st = (hipStream_t)stream;
    char* wsb = (char*)ws;
    int32_t* pruned = (int32_t*)(wsb + w.pruned_off);
    float* rnorm = (float*)(wsb + w.rnorm_off);
    table_t* table = (table_t*)(wsb + w.table_off);

    static PerDeviceOnce lds_setup;
    if (!lds_setup.run([] {
            return raise_dynamic_lds(cos_argmax_bf16<1>, cos_ring_stages(1) * (64 + COS_BN) * 128) &&
                   raise_dynamic_lds(cos_argmax_bf16<2>, cos_ring_stages(2) * (128 + COS_BN) * 128) &&
                   raise_dynamic_lds(cos_argmax_bf16<4>, cos_ring_stages(4) * (256 + COS_BN) * 128);
        }))
        return D3TOM_ERR_DEVICE;

    // prepared: the selection launch has left 1 / norm of every visual row (by token), the pruned list and the
    // initial table in the workspace
    const dim3 gn(ceil_div(max_keep, 4), B);
    if (prepared) {
    } else if (dt == D3TOM_BF16)
        D3TOM_LAUNCH(MERGE_NORMS, st, merge_norms_kernel<uint16_t><<<gn, 256, 0, st>>>(
            (const uint16_t*)sim, d_sim, seq_off, vis_start, vis_count, kept_idx, kept_off, max_V, max_keep, rnorm, pruned,
            table, w.VP));
    else
        D3TOM_LAUNCH(MERGE_NORMS, st, merge_norms_kernel<float><<<gn, 256, 0, st>>>(
            (const float*)sim, d_sim, seq_off, vis_start, vis_count, kept_idx, kept_off, max_V, max_keep, rnorm, pruned,
            table, w.VP));

    const bool mfma = (dt == D3TOM_BF16) && (d_sim % COS_BK == 0) && ((size_t)max_V * d_sim * 2 < ((size_t)1 << 31));
    if (mfma && max_pruned > 0) {
        const int nct = ceil_div(max_keep, COS_BN);
        // as long as the 64-row tiles still fit one round of the 256 CUs they finish sooner than half as many
        // 128-row tiles (a 64-row tile's k-loop is ~0.7 of a 128-row tile's)
        // with several rounds of 128-row tiles (large batches) 256-row tiles move a third less operand data per flop
        const int TM = ((long)nct * ceil_div(max_pruned, 128) * B > 768) ? 4 : ((long)nct * ceil_div(max_pruned, 64) * B > 256) ? 2 : 1;
        // too few 64 x 128 tiles for 256 CUs (short sequences): cut the contraction into k-slices as well
        int ksplit = 1;
        if (TM == 1) {
            const long tiles = (long)ceil_div(max_pruned, 64) * nct * B;
            const int stages = d_sim / COS_BK;
            if (tiles <= COS_SPLIT_BLOCKS / 2) {
                ksplit = 16;
                while (ksplit > 1 && (tiles * ksplit > COS_SPLIT_BLOCKS || stages % ksplit || stages / ksplit < cos_ring_stages(1))) ksplit >>= 1;
            }
        }
        const int BM = TM * 64;
        const int nrt = ceil_div(max_pruned, BM);
        // tiles of a sample in 8 equal runs (one per XCD); bands about as high as a run's block is wide
        const int per = ceil_div(nrt * nct, 8);
        int RB = 1;
        while ((RB + 1) * (RB + 1) <= per) ++RB;
        if (RB > nrt) RB = nrt;
        const dim3 g((unsigned)(8 * per * B), (unsigned)ksplit);
        float* dots = (float*)(wsb + w.dots_off);
        const size_t lds = (size_t)cos_ring_stages(TM) * (BM + COS_BN) * 128;
        const int by_token = prepared ? 1 : 0;
        if (TM == 4)
            D3TOM_LAUNCH(COS_ARGMAX, st, cos_argmax_bf16<4><<<g, 512, lds, st>>>(
                (const uint16_t*)sim, d_sim, seq_off, vis_start, vis_count, kept_idx, kept_off, max_V, max_keep, pruned,
                rnorm, table, w.VP, per, RB, 1, dots, nrt, nct, by_token));
        else if (TM == 1)
            D3TOM_LAUNCH(COS_ARGMAX, st, cos_argmax_bf16<1><<<g, 512, lds, st>>>(
                (const uint16_t*)sim, d_sim, seq_off, vis_start, vis_count, kept_idx, kept_off, max_V, max_keep, pruned,
                rnorm, table, w.VP, per, RB, ksplit, dots, nrt, nct, by_token));
        else
            D3TOM_LAUNCH(COS_ARGMAX, st, cos_argmax_bf16<2><<<g, 512, lds, st>>>(
                (const uint16_t*)sim, d_sim, seq_off, vis_start, vis_count, kept_idx, kept_off, max_V, max_keep, pruned,
                rnorm, table, w.VP, per, RB, 1, dots, nrt, nct, by_token));
        if (ksplit > 1) {
            const dim3 gr(ceil_div(max_pruned, 4), B);
            D3TOM_LAUNCH(COS_REDUCE, st, cos_reduce_argmax<<<gr, 256, 0, st>>>(
                seq_off, vis_start, vis_count, kept_off, max_V, max_keep, pruned, rnorm, dots, ksplit,
                nrt * nct * B, nrt, nct, table, w.VP, prepared ? kept_idx : nullptr));
        }
    } else if (max_pruned > 0) {
        const dim3 g(max_pruned, B);
        if (dt == D3TOM_BF16)
            D3TOM_LAUNCH(COS_ARGMAX, st, cos_argmax_generic<uint16_t><<<g, 256, 0, st>>>(
                (const uint16_t*)sim, d_sim, seq_off, vis_start, vis_count, kept_idx, kept_off, max_V, max_keep, pruned,
                rnorm, table, w.VP, prepared ? 1 : 0));
        else
            D3TOM_LAUNCH(COS_ARGMAX, st, cos_argmax_generic<float><<<g, 256, 0, st>>>(
                (const float*)sim, d_sim, seq_off, vis_start, vis_count, kept_idx, kept_off, max_V, max_keep, pruned,
                rnorm, table, w.VP, prepared ? 1 : 0));
    }

    // few output rows (short sequences): two workgroups per row, half a row each, so that more CUs stream
    const int nch = d / epc;
    // (max_out bounds the rows and sizes the grid; when it is only a loose bound, the caller's expected row count decides)
    const int rows_expected = (out_rows_hint > 0 && out_rows_hint < max_out) ? out_rows_hint : max_out;
    const int nslice = ((long)rows_expected * B * (x1 ? 2 : 1) < 768 && nch >= 512) ? 2 : 1;
    const dim3 gs(max_out * nslice, B, x1 ? 2 : 1);    // output rows (x slices) per sample x payloads; surplus workgroups exit at once
#define D3TOM_SCATTER(TYPE, CPT)                                                                                        \
    D3TOM_LAUNCH(MERGE_SCATTER, st, merge_scatter_kernel<TYPE, CPT><<<gs, 256, 0, st>>>(                                \
        (const TYPE*)x0, (const TYPE*)x1, d, seq_off, vis_start, vis_count, kept_idx, kept_off, max_V, max_keep, mode,   \
        out_off, table, w.VP, vis_off, (TYPE*)y0, (TYPE*)y1, assign, counts, src_pos, nslice))
    if (dt == D3TOM_BF16) { if (nslice == 2) D3TOM_SCATTER(uint16_t, 1); else D3TOM_SCATTER(uint16_t, 2); }
    else                  { if (nslice == 2) D3TOM_SCATTER(float, 1); else D3TOM_SCATTER(float, 2); }
#undef D3TOM_SCATTER
    return D3TOM_OK;
}

extern "C" int d3tom_merge(const void* x, const void* sim, int d, int d_sim, int dt,
                           int B, const int32_t* seq_off, const int32_t* vis_start, const int32_t* vis_count,
                           const int32_t* vis_off, const int32_t* kept_idx, const int32_t* kept_off,
                           int max_N, int max_V, int max_keep, int max_pruned, int max_out, int mode,
                           const int32_t* out_off, void* y, int32_t* assign, int32_t* counts, int32_t* src_pos,
                           void* ws, size_t ws_bytes, void* stream) {
    return merge_run(x, y, nullptr, nullptr, sim, d, d_sim, dt, B, seq_off, vis_start, vis_count, vis_off, kept_idx,
                     kept_off, max_N, max_V, max_keep, max_pruned, max_out, mode, out_off, assign, counts, src_pos, ws,
                     ws_bytes, stream);
}

extern "C" int d3tom_merge_kv(const void* k_cache, const void* v_cache, int d, int dt,
                              int B, const int32_t* seq_off, const int32_t* vis_start, const int32_t* vis_count,
                              const int32_t* vis_off, const int32_t* kept_idx, const int32_t* kept_off,
                              int max_N, int max_V, int max_keep, int max_pruned, int max_out, int mode,
                              const int32_t* out_off, void* k_out, void* v_out, int32_t* assign, int32_t* counts,
                              int32_t* src_pos, void* ws, size_t ws_bytes, void* stream) {
    if (!k_cache || !v_cache || !k_out || !v_out) return D3TOM_ERR_INVALID_ARG;
    return merge_run(k_cache, k_out, v_cache, v_out, k_cache, d, d, dt, B, seq_off, vis_start, vis_count, vis_off,
                     kept_idx, kept_off, max_N, max_V, max_keep, max_pruned, max_out, mode, out_off, assign, counts,
                     src_pos, ws, ws_bytes, stream);
}
