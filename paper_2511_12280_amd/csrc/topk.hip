// d3tom_select_topk: keep / merge partition (Section 3.2: V_kept = tokens whose score rank is at most
// the kept count; Algorithm 1, the TopK line).
//
// One 1024-thread workgroup per sample, the whole score vector resident in LDS as order-preserving
// 32-bit keys.  A most-significant-digit radix SELECT (8 bits per pass, starting below the bits that
// all keys share) finds the k-th largest key exactly (no sort), then an ordered compaction emits the
// kept positions ascending.  Equal keys at the
// threshold are taken lowest index first, which makes the selection identical to ranking by
// (score descending, index ascending).  Integer LDS atomics only: deterministic.  Scores of one sample
// share their sign and exponent bits, so the leading digits land in one or two bins; per-wave
// histograms keep those same-address updates from serialising across the whole workgroup.
//
// The selection is a chain of short dependent passes on one compute unit per sample.  Called from the one-call
// merge layer, the launch carries further workgroups (blockIdx.y > 0) that do not select anything: one wave per
// visual row, they read the rows of the similarity features front to back and store 1 / norm of each.  That
// leaves the rows in the memory-side cache for the gathers of the cosine kernel (a sequential read of cold rows
// is several times cheaper than the 128-byte gathers that kernel would otherwise send to HBM) and replaces the
// merge's norms launch; the selecting workgroup writes the pruned list and the initial token table beside the
// kept list.
#include "internal.hpp"

namespace d3tom {

constexpr int TOPK_THREADS = 1024;
constexpr int TOPK_STREAM_WGS = 96;        // streaming workgroups per launch (measured at 3645 rows of 8 KB: 32 -> 22.5 us, 64 -> 13.8,
                                           // 96 -> 13.1, 127 -> 13.5, 255 -> 14.5 us for the whole launch)

__device__ __forceinline__ uint32_t order_key(float f) {       // ascending uint order == ascending float order
    const uint32_t u = __float_as_uint(f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// exclusive prefix sum of one int per thread over the workgroup; returns the prefix, total in *total
__device__ __forceinline__ int block_excl_scan(int v, int* wsum /*[17]*/, int* total) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int inc = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int t = __shfl_up(inc, o, WAVE);
        if (lane >= o) inc += t;
    }
    __syncthreads();                       // wsum reuse
    if (lane == 63) wsum[wave] = inc;
    __syncthreads();
    if (threadIdx.x == 0) {
        int run = 0;
        for (int w = 0; w < TOPK_THREADS / 64; ++w) { const int t = wsum[w]; wsum[w] = run; run += t; }
        wsum[16] = run;
    }
    __syncthreads();
    *total = wsum[16];
    return wsum[wave] + inc - v;
}

// Kept count at a keep ratio (Section 3.2: rank at most (1 - alpha)|V|; a fractional product is rounded up):
// ceil(ratio * V - 1e-9) clamped to [1, V], in double with separately rounded product and difference, i.e.
// the same arithmetic as the host helper d3tom_keep_count.
__device__ __forceinline__ int keep_count_device(int V, double ratio) {
    double c = ceil(__dsub_rn(__dmul_rn(ratio, (double)V), 1e-9));
    if (!(c >= 1.0)) c = 1.0;
    if (c > (double)V) c = (double)V;
    return (int)c;
}

__global__ __launch_bounds__(TOPK_THREADS) void topk_select_kernel(
    const float* __restrict__ scores, const int32_t* __restrict__ score_off, const int32_t* __restrict__ keep_k,
    const int32_t* __restrict__ kept_off, int max_V, int32_t* __restrict__ kept_idx, int32_t* __restrict__ slot_of,
    const double* __restrict__ keep_ratio, const int32_t* __restrict__ seq_off, int32_t* __restrict__ keep_k_out,
    int32_t* __restrict__ kept_off_out, int32_t* __restrict__ out_off_out, MergePrep prep) {
    extern __shared__ uint32_t ukey[];                 // [max_V]
    if (blockIdx.y > 0) {
        // streaming workgroups: norms of the sample's visual rows
        stream_row_norms(prep, max_V, blockIdx.x, seq_off, (int)(blockIdx.y - 1) * (TOPK_THREADS / 64) + (int)(threadIdx.x >> 6),
                         (int)(gridDim.y - 1) * (TOPK_THREADS / 64), threadIdx.x & 63);
        return;
    }
    __shared__ int whist[16][256];        // one digit histogram per wave: same-bin updates only collide inside a wave
    __shared__ int wsum[17];
    __shared__ int sel[3];
    __shared__ uint32_t wrange[32];
    __shared__ int plan[2];               // kept count of this sample, first slot of this sample in kept_idx
    const int b = blockIdx.x;
    const int s0 = score_off[b];
    const int V = min(score_off[b + 1] - s0, max_V);
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    if (keep_ratio) {
        // kept counts from the ratios, on the device: this sample's count and the prefix sums over the samples
        // in front of it (every workgroup repeats the short loop; the last one also writes the totals)
        if (tid == 0) {
            int koff = 0, ooff = 0, kb = 1;
            for (int bb = 0; bb <= b; ++bb) {
                const int Vb = min(score_off[bb + 1] - score_off[bb], max_V);
                const int kcur = Vb > 0 ? keep_count_device(Vb, keep_ratio[bb]) : 0;
                if (bb == b) { kb = kcur; break; }
                koff += kcur;
                ooff += (seq_off[bb + 1] - seq_off[bb]) - (Vb - kcur);
            }
            plan[0] = kb; plan[1] = koff;
            keep_k_out[b] = kb; kept_off_out[b] = koff; out_off_out[b] = ooff;
            if (b == (int)gridDim.x - 1) {
                kept_off_out[b + 1] = koff + kb;
                out_off_out[b + 1] = ooff + (seq_off[b + 1] - seq_off[b]) - (V - kb);
            }
        }
        __syncthreads();
    }
    if (V <= 0) return;
    const int kk = keep_ratio ? plan[0] : min(max(keep_k[b], 1), V);

    // keys, and the range they span: bits above the highest differing bit are common to all keys
    uint32_t kmin = 0xFFFFFFFFu, kmax = 0u;
    for (int j = tid; j < V; j += TOPK_THREADS) {
        const uint32_t u = order_key(scores[s0 + j]);
        ukey[j] = u;
        kmin = min(kmin, u); kmax = max(kmax, u);
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        kmin = min(kmin, (uint32_t)__shfl_xor((int)kmin, o, WAVE));
        kmax = max(kmax, (uint32_t)__shfl_xor((int)kmax, o, WAVE));
    }
    if (lane == 0) { wrange[wave] = kmin; wrange[16 + wave] = kmax; }
    __syncthreads();
#pragma unroll
    for (int w = 0; w < 16; ++w) { kmin = min(kmin, wrange[w]); kmax = max(kmax, wrange[16 + w]); }
    const uint32_t diff = kmin ^ kmax;
    const int hi = diff ? 32 - __clz(diff) : 0;                 // number of low bits that vary
    uint32_t mask = (hi >= 32) ? 0u : ~((hi == 0) ? 0u : ((1u << hi) - 1u));
    uint32_t prefix = kmax & mask;
    int remaining = kk, tot_eq = V;
    // most-significant-digit radix select over the varying bits, 8 bits per pass
#pragma unroll 1
    for (int top = hi; top > 0; top -= 8) {
        const int shift = max(top - 8, 0);
        const uint32_t dmask = (1u << (top - shift)) - 1u;
        for (int t = tid; t < 16 * 256; t += TOPK_THREADS) (&whist[0][0])[t] = 0;
        __syncthreads();
        for (int base = 0; base < V; base += TOPK_THREADS) {
            const int j = base + tid;
            const uint32_t u = (j < V) ? ukey[j] : 0u;
            const bool match = (j < V) && ((u & mask) == prefix);
            const uint32_t dg = (u >> shift) & dmask;
            const unsigned long long mm = __ballot(match);
            if (mm) {
                // a whole wave on one digit would serialise on one LDS address: add it once instead
                const int first = __ffsll((long long)mm) - 1;
                const uint32_t d0 = (uint32_t)__shfl((int)dg, first, WAVE);
                const unsigned long long same = __ballot(match && dg == d0);
                if (same == mm) { if (lane == first) atomicAdd(&whist[wave][d0], __popcll(mm)); }
                else if (match) atomicAdd(&whist[wave][dg], 1);
            }
        }
        __syncthreads();
        if (tid < 64) {
            // lane l owns digits 255-4l .. 252-4l (descending); find the digit holding the remaining-th key
            int c[4] = {0, 0, 0, 0}, tot = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
#pragma unroll
                for (int w = 0; w < 16; ++w) c[e] += whist[w][255 - (4 * tid + e)];
                tot += c[e];
            }
            int inc = tot;
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                const int t = __shfl_up(inc, o, WAVE);
                if (tid >= o) inc += t;
            }
            int before = inc - tot;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                if (before < remaining && remaining <= before + c[e]) {
                    sel[0] = 255 - (4 * tid + e); sel[1] = remaining - before; sel[2] = c[e];
                }
                before += c[e];
            }
        }
        __syncthreads();
        prefix |= ((uint32_t)sel[0]) << shift;
        mask |= dmask << shift;
        remaining = sel[1];
        tot_eq = sel[2];
    }
    const uint32_t thr = prefix;       // k-th largest key; `remaining` of the `tot_eq` keys equal to it are kept
    const int per = (V + TOPK_THREADS - 1) / TOPK_THREADS;
    const int j0 = min(tid * per, V), j1 = min(j0 + per, V);
    int eq_before = 0;
    if (tot_eq != remaining) {         // ties straddle the threshold: lowest indices first
        int n_eq = 0;
        for (int j = j0; j < j1; ++j) n_eq += (ukey[j] == thr);
        int unused;
        eq_before = block_excl_scan(n_eq, wsum, &unused);
    }
    int n_keep = 0;
    {
        int e = eq_before;
        for (int j = j0; j < j1; ++j) {
            const uint32_t u = ukey[j];
            n_keep += (u > thr) || (u == thr && e < remaining);
            e += (u == thr);
        }
    }
    int tot_keep;
    int slot = block_excl_scan(n_keep, wsum, &tot_keep);
    const int k0 = keep_ratio ? plan[1] : kept_off[b];
    int e = eq_before;
    for (int j = j0; j < j1; ++j) {
        const uint32_t u = ukey[j];
        const bool keep = (u > thr) || (u == thr && e < remaining);
        e += (u == thr);
        slot_of[s0 + j] = keep ? slot : -1;
        if (prep.table) {
            // slot = kept tokens in front of j: a pruned token sits at position j - slot of the ascending pruned list
            prep.table[(size_t)b * prep.VP + j] = keep ? table_entry_kept(slot) : (table_t)0;
            if (!keep) prep.pruned[(size_t)b * max_V + (j - slot)] = j;
        }
        if (keep) { kept_idx[k0 + slot] = j; ++slot; }
    }
}

}  // namespace d3tom

using namespace d3tom;

int d3tom::topk_run(const float* scores, int B, const int32_t* score_off, const int32_t* keep_k, const int32_t* kept_off,
                    int max_V, int32_t* kept_idx, int32_t* slot_of, const double* keep_ratio, const int32_t* seq_off,
                    int32_t* keep_k_out, int32_t* kept_off_out, int32_t* out_off_out, void* stream, const MergePrep* prep_in,
                    bool* prepared) {
    if (prepared) *prepared = false;
    if (!scores || !score_off || !kept_idx || !slot_of) return D3TOM_ERR_INVALID_ARG;
    if (keep_ratio ? (!seq_off || !keep_k_out || !kept_off_out || !out_off_out) : (!keep_k || !kept_off)) return D3TOM_ERR_INVALID_ARG;
    if (B < 1 || max_V < 1) return D3TOM_ERR_INVALID_ARG;
    if (max_V > D3TOM_MAX_VISUAL) return D3TOM_ERR_UNSUPPORTED;
    static PerDeviceOnce lds_setup;
    if (!lds_setup.run([] { return raise_dynamic_lds(topk_select_kernel, D3TOM_MAX_VISUAL * 4); })) return D3TOM_ERR_DEVICE;
    hipStream_t st = (hipStream_t)stream;
    const bool streaming = merge_prep_usable(prep_in, B, max_V, seq_off);
    const MergePrep prep = streaming ? *prep_in : MergePrep();
    const int extra = streaming ? (B >= TOPK_STREAM_WGS ? 1 : TOPK_STREAM_WGS / B) : 0;
    D3TOM_LAUNCH(TOPK_SELECT, st, topk_select_kernel<<<dim3(B, 1 + extra), TOPK_THREADS, (size_t)max_V * 4, st>>>(
        scores, score_off, keep_k, kept_off, max_V, kept_idx, slot_of, keep_ratio, seq_off, keep_k_out, kept_off_out, out_off_out, prep));
    if (prepared) *prepared = streaming;
    return D3TOM_OK;
}

extern "C" int d3tom_select_topk(const float* scores, int B, const int32_t* score_off, const int32_t* keep_k,
                                 const int32_t* kept_off, int max_V,
                                 int32_t* kept_idx, int32_t* slot_of,
                                 void* ws, size_t ws_bytes, void* stream) {
    (void)ws; (void)ws_bytes;
    return topk_run(scores, B, score_off, keep_k, kept_off, max_V, kept_idx, slot_of, nullptr, nullptr, nullptr, nullptr,
                    nullptr, stream);
}
