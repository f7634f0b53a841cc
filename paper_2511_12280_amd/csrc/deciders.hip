// d3tom_update_deciders: the decider set of the next step (Section 3.2, "The Decider-Guided Mechanism":
// the tokens revealed in the preceding iteration, i.e. positions that hold a token now and held [MASK]
// one iteration earlier; Algorithm 1, the last line of the denoising loop).
//
// One workgroup walks the samples in order.  Per 1024-position chunk every thread tests its position,
// the flags are compacted in ascending position order (wave prefix through ballots, then a prefix over
// the 16 waves), and the running offset carries over to the next chunk and the next sample, so the list
// comes out packed exactly as d3tom_importance reads it (dec_idx + prefix-sum offsets) without a host
// round trip.  The work is a few thousand integer compares: launch-latency bound by construction.
#include "common.hpp"

namespace d3tom {

constexpr int DEC_THREADS = 1024;

__global__ __launch_bounds__(DEC_THREADS) void update_deciders_kernel(
    const int32_t* __restrict__ prev_ids, const int32_t* __restrict__ cur_ids, int mask_id, int B,
    const int32_t* __restrict__ seq_off, int max_D, int32_t* __restrict__ dec_idx, int32_t* __restrict__ dec_off,
    int32_t* __restrict__ dec_count) {
    __shared__ int wtot[DEC_THREADS / 64];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int base = 0;                                          // entries written for the samples before this one
    if (tid == 0) dec_off[0] = 0;
    for (int b = 0; b < B; ++b) {
        const int tok0 = seq_off[b];
        const int N = seq_off[b + 1] - tok0;
        int found = 0;                                     // deciders of this sample seen so far (all of them)
        for (int i0 = 0; i0 < N; i0 += DEC_THREADS) {      // uniform trip count
            const int i = i0 + tid;
            const bool f = (i < N) && (cur_ids[tok0 + i] != mask_id) && (prev_ids[tok0 + i] == mask_id);
            const unsigned long long m = __builtin_amdgcn_ballot_w64(f);
            __syncthreads();                               // wtot of the previous chunk has been read
            if (lane == 0) wtot[wave] = __popcll(m);
            __syncthreads();
            int before = 0, total = 0;
#pragma unroll
            for (int w = 0; w < DEC_THREADS / 64; ++w) {
                const int t = wtot[w];
                before += (w < wave) ? t : 0;
                total += t;
            }
            const int ord = found + before + __popcll(m & ((1ull << lane) - 1ull));
            if (f && ord < max_D) dec_idx[base + ord] = i;                    // beyond max_D: counted, not listed
            found += total;
        }
        const int kept = min(found, max_D);
        if (tid == 0) {
            dec_off[b + 1] = base + kept;
            if (dec_count) dec_count[b] = found;
        }
        base += kept;
    }
}

}  // namespace d3tom

using namespace d3tom;

extern "C" int d3tom_update_deciders(const int32_t* prev_ids, const int32_t* cur_ids, int mask_id,
                                     int B, const int32_t* seq_off, int max_D,
                                     int32_t* dec_idx, int32_t* dec_off, int32_t* dec_count, void* stream) {
    if (!prev_ids || !cur_ids || !seq_off || !dec_idx || !dec_off) return D3TOM_ERR_INVALID_ARG;
    if (B < 1 || max_D < 1) return D3TOM_ERR_INVALID_ARG;
    if (max_D > D3TOM_MAX_DECIDERS) return D3TOM_ERR_UNSUPPORTED;
    hipStream_t st = (hipStream_t)stream;
    D3TOM_LAUNCH(UPDATE_DECIDERS, st, update_deciders_kernel<<<1, DEC_THREADS, 0, st>>>(
        prev_ids, cur_ids, mask_id, B, seq_off, max_D, dec_idx, dec_off, dec_count));
    return D3TOM_OK;
}
