// Internal helpers shared by the gfx950 kernels of libd3tom (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <mutex>
#include "../../include/d3tom.h"

namespace d3tom {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;

constexpr int WAVE = 64;
constexpr float LOG2E = 1.4426950408889634f;

// ---- bf16 <-> f32 -------------------------------------------------------------------------
__device__ __forceinline__ float bf16_bits_to_f32(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }
// round-to-nearest-even; inputs are finite by contract
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f) {
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    return (uint32_t)f32_to_bf16_bits(lo) | ((uint32_t)f32_to_bf16_bits(hi) << 16);
}
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

// element load as float for the generic (untuned) kernels
template <typename T> struct Elem;
template <> struct Elem<float> {
    static __device__ __forceinline__ float load(const float* p) { return *p; }
    static __device__ __forceinline__ void store(float* p, float v) { *p = v; }
};
template <> struct Elem<uint16_t> {   // bf16 storage
    static __device__ __forceinline__ float load(const uint16_t* p) { return bf16_bits_to_f32(*p); }
    static __device__ __forceinline__ void store(uint16_t* p, float v) { *p = f32_to_bf16_bits(v); }
};

// ---- wave / block reductions ----------------------------------------------------------------
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, WAVE);
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, WAVE));
    return v;
}
__device__ __forceinline__ int wave_sum_i(int v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, WAVE);
    return v;
}

// Reductions over the 16 lanes of a DPP row (lanes 16 i .. 16 i + 15), every lane ends with the result.
// Four data-parallel-primitive steps inside the vector ALU (no LDS traffic): swap neighbours, swap
// pairs, mirror inside each half row, mirror the whole row.
template <int CTRL>
__device__ __forceinline__ float dpp_move(float x) {
    return __uint_as_float((uint32_t)__builtin_amdgcn_update_dpp(0, (int)__float_as_uint(x), CTRL, 0xF, 0xF, true));
}
__device__ __forceinline__ float row16_max(float v) {
    v = fmaxf(v, dpp_move<0xB1>(v));     // quad_perm [1,0,3,2]
    v = fmaxf(v, dpp_move<0x4E>(v));     // quad_perm [2,3,0,1]
    v = fmaxf(v, dpp_move<0x141>(v));    // row_half_mirror
    v = fmaxf(v, dpp_move<0x140>(v));    // row_mirror
    return v;
}
__device__ __forceinline__ float row16_sum(float v) {
    v += dpp_move<0xB1>(v);
    v += dpp_move<0x4E>(v);
    v += dpp_move<0x141>(v);
    v += dpp_move<0x140>(v);
    return v;
}

// Combine two (running max, running sum of exp2) pairs.  -inf max means "empty".
__device__ __forceinline__ void lse2_combine(float& m, float& z, float m2, float z2) {
    float mn = fmaxf(m, m2);
    float a = (m == -INFINITY) ? 0.f : z * exp2f(m - mn);
    float b = (m2 == -INFINITY) ? 0.f : z2 * exp2f(m2 - mn);
    m = mn; z = a + b;
}

// One rotary pair (a, b) turned by the angle with cosine c and sine s.  The fused multiply-adds are spelled out so
// that every kernel that rotates (the rotary kernel, the q | k | v projection's epilogue) rounds the same way.
__device__ __forceinline__ void rope_rotate(float a, float b, float c, float s, float& ra, float& rb) {
    ra = __builtin_fmaf(a, c, -(b * s));
    rb = __builtin_fmaf(b, c, a * s);
}

// The same with the hardware exponential (one instruction, about 1 ulp, results below the normal range flush to
// zero): for the MFMA kernels, whose workgroups combine hundreds of pairs each.
__device__ __forceinline__ void lse2_combine_fast(float& m, float& z, float m2, float z2) {
    float mn = fmaxf(m, m2);
    float a = (m == -INFINITY) ? 0.f : z * __builtin_amdgcn_exp2f(m - mn);
    float b = (m2 == -INFINITY) ? 0.f : z2 * __builtin_amdgcn_exp2f(m2 - mn);
    m = mn; z = a + b;
}

__host__ __device__ __forceinline__ int ceil_div(int a, int b) { return (a + b - 1) / b; }
__host__ __device__ __forceinline__ size_t align_up(size_t a, size_t b) { return (a + b - 1) / b * b; }

// host-side argument checks
inline bool aligned16(const void* p) { return (((uintptr_t)p) & 15u) == 0; }

// One-time set-up per device (raising a kernel's dynamic LDS limit): safe when several host threads enter
// the same entry point at once, and repeated for every device the library is used on.
struct PerDeviceOnce {
    static constexpr int MAX_DEVICES = 64;
    std::once_flag flag[MAX_DEVICES];
    bool ok[MAX_DEVICES] = {};
    template <typename Fn>
    bool run(Fn&& fn) {
        int dev = -1;
        if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return false;
        std::call_once(flag[dev], [&] { ok[dev] = fn(); });
        return ok[dev];
    }
};
template <typename K>
inline bool raise_dynamic_lds(K kernel, int bytes) {
    return hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes) == hipSuccess;
}

// ---- optional per-kernel timing (d3tom_profile_*): HIP events around each launch when enabled ----
namespace prof {
enum Kernel {
    IMP_STATS = 0, IMP_SCORES, IMP_FINISH, TOPK_SELECT, MERGE_NORMS, COS_ARGMAX, MERGE_ASSIGN, MERGE_SCATTER, ATTEND,
    UPDATE_DECIDERS, COS_REDUCE, LINEAR, RMSNORM, ROPE, STACK_META,
    NUM_KERNELS
};
extern bool g_enabled;
void mark_begin(int kernel, hipStream_t st);
void mark_end(int kernel, hipStream_t st);
struct Scope {
    int kernel; hipStream_t st;
    Scope(int k, hipStream_t s) : kernel(k), st(s) { if (g_enabled) mark_begin(k, s); }
    ~Scope() { if (g_enabled) mark_end(kernel, st); }
};
}  // namespace prof

#define D3TOM_LAUNCH_CHECK()                                         \
    do {                                                             \
        if (hipGetLastError() != hipSuccess) return D3TOM_ERR_DEVICE; \
    } while (0)

// launch one kernel (timed when profiling is on) and turn a rejected launch into a status
#define D3TOM_LAUNCH(KERNEL_ID, STREAM, ...)                         \
    do {                                                             \
        {                                                            \
            prof::Scope _scope(prof::KERNEL_ID, STREAM);             \
            __VA_ARGS__;                                             \
        }                                                            \
        D3TOM_LAUNCH_CHECK();                                        \
    } while (0)

}  // namespace d3tom
