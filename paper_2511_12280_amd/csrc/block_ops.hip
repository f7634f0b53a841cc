// Row-wise pieces of a Llama-style block around the projections: RMSNorm and the rotary position
// embedding (the blocks that Algorithm 1 runs before and after the merge layer).  Both are pure HBM
// streaming: one workgroup per token row, 16-byte accesses, float32 arithmetic, one rounding at the store.
#include "common.hpp"

namespace d3tom {

constexpr int NORM_MAX_CHUNKS = 4;     // 16-byte chunks per thread held in registers: d <= 256 * 4 * 8

// y = x / sqrt(mean(x^2) + eps) * gain
__global__ __launch_bounds__(256) void rmsnorm_bf16_kernel(const uint16_t* __restrict__ x, const uint16_t* __restrict__ gain,
                                                           int d, float eps, uint16_t* __restrict__ y) {
    __shared__ float wsum[4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const size_t row = (size_t)blockIdx.x * d;
    const int nch = d / 8;
    uint4 v[NORM_MAX_CHUNKS];
    float ss = 0.f;
#pragma unroll
    for (int u = 0; u < NORM_MAX_CHUNKS; ++u) {
        const int c = tid + u * 256;
        v[u] = (c < nch) ? *reinterpret_cast<const uint4*>(x + row + (size_t)c * 8) : make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int u = 0; u < NORM_MAX_CHUNKS; ++u) {
        const uint32_t w[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
#pragma unroll
        for (int e = 0; e < 4; ++e) { const float a = bf16_lo(w[e]), b = bf16_hi(w[e]); ss += a * a; ss += b * b; }
    }
    ss = wave_sum(ss);
    if (lane == 0) wsum[wave] = ss;
    __syncthreads();
    const float total = (wsum[0] + wsum[1]) + (wsum[2] + wsum[3]);
    const float rinv = 1.0f / sqrtf(total / (float)d + eps);
#pragma unroll
    for (int u = 0; u < NORM_MAX_CHUNKS; ++u) {
        const int c = tid + u * 256;
        if (c >= nch) continue;
        const uint4 gq = *reinterpret_cast<const uint4*>(gain + (size_t)c * 8);
        const uint32_t w[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
        const uint32_t gw[4] = {gq.x, gq.y, gq.z, gq.w};
        uint32_t o[4];
#pragma unroll
        for (int e = 0; e < 4; ++e)
            o[e] = pack_bf16x2(bf16_lo(w[e]) * rinv * bf16_lo(gw[e]), bf16_hi(w[e]) * rinv * bf16_hi(gw[e]));
        *reinterpret_cast<uint4*>(y + row + (size_t)c * 8) = make_uint4(o[0], o[1], o[2], o[3]);
    }
}

// h = residual + sum of the float32 partial products of a split projection, rounded once to bf16 and stored;
// when a gain is given, also y = rmsnorm(h) of the stored (rounded) values: the normalisation that opens the
// next sub-block, so that it needs no launch of its own.  Slices are added in ascending order.
__global__ __launch_bounds__(256) void add_norm_bf16_kernel(const float* __restrict__ part, int nsplit, size_t split_stride,
                                                            const uint16_t* residual, const uint16_t* __restrict__ gain,
                                                            int d, float eps, uint16_t* h, uint16_t* __restrict__ y) {
    __shared__ float wsum[4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const size_t row = (size_t)blockIdx.x * d;
    const int nch = d / 8;
    uint32_t hv[NORM_MAX_CHUNKS][4];
    float ss = 0.f;
#pragma unroll
    for (int u = 0; u < NORM_MAX_CHUNKS; ++u) {
        const int c = tid + u * 256;
        if (c >= nch) { hv[u][0] = hv[u][1] = hv[u][2] = hv[u][3] = 0; continue; }
        const uint4 r = *reinterpret_cast<const uint4*>(residual + row + (size_t)c * 8);
        const uint32_t rr[4] = {r.x, r.y, r.z, r.w};
        float acc[8];
#pragma unroll
        for (int e = 0; e < 4; ++e) { acc[2 * e] = bf16_lo(rr[e]); acc[2 * e + 1] = bf16_hi(rr[e]); }
        float sum[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        for (int s = 0; s < nsplit; ++s) {
            const float* p = part + (size_t)s * split_stride + row + (size_t)c * 8;
            const float4 a = *reinterpret_cast<const float4*>(p), b = *reinterpret_cast<const float4*>(p + 4);
            sum[0] += a.x; sum[1] += a.y; sum[2] += a.z; sum[3] += a.w;
            sum[4] += b.x; sum[5] += b.y; sum[6] += b.z; sum[7] += b.w;
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            hv[u][e] = pack_bf16x2(acc[2 * e] + sum[2 * e], acc[2 * e + 1] + sum[2 * e + 1]);
            const float lo = bf16_lo(hv[u][e]), hi = bf16_hi(hv[u][e]);
            ss += lo * lo; ss += hi * hi;
        }
        *reinterpret_cast<uint4*>(h + row + (size_t)c * 8) = make_uint4(hv[u][0], hv[u][1], hv[u][2], hv[u][3]);
    }
    if (!gain) return;
    ss = wave_sum(ss);
    if (lane == 0) wsum[wave] = ss;
    __syncthreads();
    const float total = (wsum[0] + wsum[1]) + (wsum[2] + wsum[3]);
    const float rinv = 1.0f / sqrtf(total / (float)d + eps);
#pragma unroll
    for (int u = 0; u < NORM_MAX_CHUNKS; ++u) {
        const int c = tid + u * 256;
        if (c >= nch) continue;
        const uint4 gq = *reinterpret_cast<const uint4*>(gain + (size_t)c * 8);
        const uint32_t gw[4] = {gq.x, gq.y, gq.z, gq.w};
        uint32_t o[4];
#pragma unroll
        for (int e = 0; e < 4; ++e)
            o[e] = pack_bf16x2(bf16_lo(hv[u][e]) * rinv * bf16_lo(gw[e]), bf16_hi(hv[u][e]) * rinv * bf16_hi(gw[e]));
        *reinterpret_cast<uint4*>(y + row + (size_t)c * 8) = make_uint4(o[0], o[1], o[2], o[3]);
    }
}

// Rotary embedding, in place on q and k [rows, H, dh]: channel c < dh/2 of every head is paired with
// channel c + dh/2 and the pair is turned by pos * theta^(-2c/dh).  The dh/2 angles of a token are the
// same for all heads and for q and k: the first dh/2 threads evaluate them once, in double precision
// (positions reach the thousands, where a float32 angle would already be off by 1e-4), the workgroup
// then streams the row.
__global__ __launch_bounds__(256) void rope_bf16_kernel(uint16_t* __restrict__ q, uint16_t* __restrict__ k,
                                                        const int32_t* __restrict__ pos, int H, int dh, double log2_theta) {
    __shared__ float cs[128], sn[128];
    const int tid = threadIdx.x;
    const int half = dh >> 1;
    const int p = pos[blockIdx.x];
    if (tid < half) {
        const double inv_freq = exp2(-2.0 * (double)tid / (double)dh * log2_theta);
        double s, c;
        sincos((double)p * inv_freq, &s, &c);
        cs[tid] = (float)c; sn[tid] = (float)s;
    }
    __syncthreads();
    const int cpp = half / 8;                        // 16-byte chunks per half head
    const int units = H * cpp;                       // per tensor
    const size_t row = (size_t)blockIdx.x * H * dh;
    for (int u = tid; u < 2 * units; u += 256) {
        uint16_t* t = (u < units) ? q : k;
        const int uu = (u < units) ? u : u - units;
        const int h = uu / cpp, cc = uu % cpp;
        uint16_t* pa = t + row + (size_t)h * dh + cc * 8;
        const uint4 A = *reinterpret_cast<const uint4*>(pa);
        const uint4 Bv = *reinterpret_cast<const uint4*>(pa + half);
        const uint32_t aw[4] = {A.x, A.y, A.z, A.w}, bw[4] = {Bv.x, Bv.y, Bv.z, Bv.w};
        uint32_t ao[4], bo[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int c0 = cc * 8 + 2 * e;
            const float a0 = bf16_lo(aw[e]), a1 = bf16_hi(aw[e]), b0 = bf16_lo(bw[e]), b1 = bf16_hi(bw[e]);
            float ra0, rb0, ra1, rb1;
            rope_rotate(a0, b0, cs[c0], sn[c0], ra0, rb0);
            rope_rotate(a1, b1, cs[c0 + 1], sn[c0 + 1], ra1, rb1);
            ao[e] = pack_bf16x2(ra0, ra1);
            bo[e] = pack_bf16x2(rb0, rb1);
        }
        *reinterpret_cast<uint4*>(pa) = make_uint4(ao[0], ao[1], ao[2], ao[3]);
        *reinterpret_cast<uint4*>(pa + half) = make_uint4(bo[0], bo[1], bo[2], bo[3]);
    }
}

// (cos, sin) of every token's dh/2 rotary angles, the float32 values the kernel above uses: for the projection
// epilogue that applies the rotation itself (one table per step instead of one rotary launch per block)
__global__ __launch_bounds__(256) void rope_table_kernel(const int32_t* __restrict__ pos, int rows, int dh, double log2_theta,
                                                         float2* __restrict__ table) {
    const int half = dh >> 1;
    const int t = blockIdx.x * 256 + threadIdx.x;
    if (t >= rows * half) return;
    const int r = t / half, c = t - r * half;
    const double inv_freq = exp2(-2.0 * (double)c / (double)dh * log2_theta);
    double s, co;
    sincos((double)pos[r] * inv_freq, &s, &co);
    table[t] = make_float2((float)co, (float)s);
}

int rope_table_run(const int32_t* pos, int rows, int dh, float theta, float2* table, hipStream_t st) {
    if (!pos || !table || rows < 1 || dh < 2) return D3TOM_ERR_INVALID_ARG;
    if (!(theta > 1.f) || !(theta < 3.0e38f)) return D3TOM_ERR_INVALID_ARG;
    D3TOM_LAUNCH(ROPE, st, (rope_table_kernel<<<ceil_div(rows * (dh >> 1), 256), 256, 0, st>>>(pos, rows, dh, log2((double)theta), table)));
    return D3TOM_OK;
}

int rmsnorm_run(const void* x, const void* gain, int rows, int d, float eps, void* y, hipStream_t st) {
    if (!x || !gain || !y || rows < 1 || d < 1) return D3TOM_ERR_INVALID_ARG;
    if (!aligned16(x) || !aligned16(gain) || !aligned16(y)) return D3TOM_ERR_INVALID_ARG;
    if (!(eps >= 0.f)) return D3TOM_ERR_INVALID_ARG;
    if (d % 8 != 0 || d > 256 * NORM_MAX_CHUNKS * 8) return D3TOM_ERR_UNSUPPORTED;
    D3TOM_LAUNCH(RMSNORM, st, (rmsnorm_bf16_kernel<<<rows, 256, 0, st>>>((const uint16_t*)x, (const uint16_t*)gain, d, eps,
                                                                          (uint16_t*)y)));
    return D3TOM_OK;
}

// h (may be the residual buffer itself) and, when gain is not null, y = rmsnorm(h)
int add_norm_run(const float* part, int nsplit, const void* residual, const void* gain, int rows, int d, float eps,
                 void* h, void* y, hipStream_t st) {
    if (!part || !residual || !h || rows < 1 || d < 1 || nsplit < 1 || (gain && !y)) return D3TOM_ERR_INVALID_ARG;
    if (d % 8 != 0 || d > 256 * NORM_MAX_CHUNKS * 8) return D3TOM_ERR_UNSUPPORTED;
    D3TOM_LAUNCH(RMSNORM, st, (add_norm_bf16_kernel<<<rows, 256, 0, st>>>(part, nsplit, (size_t)rows * d, (const uint16_t*)residual,
                                                                           (const uint16_t*)gain, d, eps, (uint16_t*)h, (uint16_t*)y)));
    return D3TOM_OK;
}

int rope_run(void* q, void* k, const int32_t* pos, int rows, int H, int dh, float theta, hipStream_t st) {
    if (!q || !k || !pos || rows < 1 || H < 1 || dh < 1) return D3TOM_ERR_INVALID_ARG;
    if (!aligned16(q) || !aligned16(k)) return D3TOM_ERR_INVALID_ARG;
    if (!(theta > 1.f) || !(theta < 3.0e38f)) return D3TOM_ERR_INVALID_ARG;
    if (dh % 16 != 0 || dh > 256) return D3TOM_ERR_UNSUPPORTED;
    D3TOM_LAUNCH(ROPE, st, (rope_bf16_kernel<<<rows, 256, 0, st>>>((uint16_t*)q, (uint16_t*)k, pos, H, dh, log2((double)theta))));
    return D3TOM_OK;
}

}  // namespace d3tom

extern "C" int d3tom_rmsnorm(const void* x, const void* gain, int rows, int d, float eps, void* y, void* stream) {
    return d3tom::rmsnorm_run(x, gain, rows, d, eps, y, (hipStream_t)stream);
}

extern "C" int d3tom_rope(void* q, void* k, const int32_t* pos, int rows, int H, int dh, float theta, void* stream) {
    return d3tom::rope_run(q, k, pos, rows, H, dh, theta, (hipStream_t)stream);
}
