// Internal helpers shared by the libfate translation units (host + device).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include "../../include/fate.h"

namespace fate {

void set_error(const char* fmt, ...);

#define FATE_FAIL(code, ...)            \
    do {                                \
        ::fate::set_error(__VA_ARGS__); \
        return (code);                  \
    } while (0)

#define FATE_HIP(expr)                                                                   \
    do {                                                                                 \
        hipError_t _e = (expr);                                                          \
        if (_e != hipSuccess) {                                                          \
            ::fate::set_error("%s failed: %s (%s:%d)", #expr, hipGetErrorString(_e),     \
                              __FILE__, __LINE__);                                       \
            return FATE_EHIP;                                                            \
        }                                                                                \
    } while (0)

static inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

#define FATE_CHECK_PTR(p)                                                     \
    do {                                                                      \
        if ((p) == nullptr) FATE_FAIL(FATE_EINVAL, "%s is NULL", #p);         \
        if (!::fate::aligned16(p)) FATE_FAIL(FATE_EALIGN, "%s is not 16-byte aligned", #p); \
    } while (0)

#define FATE_CHECK_PTR_OPT(p)                                                 \
    do {                                                                      \
        if ((p) != nullptr && !::fate::aligned16(p))                          \
            FATE_FAIL(FATE_EALIGN, "%s is not 16-byte aligned", #p);          \
    } while (0)

constexpr int kWave = 64;
constexpr int kMaxE = 256;
constexpr int kMaxM = 64;

#ifdef __HIPCC__
__device__ __forceinline__ float bf16_bits_to_f32(uint32_t v16) { return __uint_as_float(v16 << 16); }
__device__ __forceinline__ float bf16_lo(uint32_t pair) { return __uint_as_float(pair << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t pair) { return __uint_as_float(pair & 0xffff0000u); }

// round-to-nearest-even fp32 -> bf16 bits (finite inputs)
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;   // NaN stays NaN
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}

// Wave-wide all-reduce on the data-parallel-primitive (DPP) path: four
// exchange steps inside each row of 16 lanes (no LDS crossbar), then the four
// row results are combined through scalar lane reads.  Result is uniform.
// ---- data handed between workgroups of one launch ---------------------------
// Relaxed atomics at device scope: the accesses go past the per-XCD L2 to the
// point where all compute dies agree, so no cache-wide write-back or
// invalidate is needed around them.  Ordering comes from the producer waiting
// for its stores before it bumps a counter, and from the consumer reading the
// counter before the data.  A workgroup barrier alone does not wait for a
// wave's outstanding global stores (waves of one workgroup share their vector
// cache, so a workgroup-scope release needs no such wait): every wave calls
// wait_own_stores() before the barrier that precedes the counter update, or
// the data validates itself (values tagged with the call's epoch).
__device__ __forceinline__ void wait_own_stores() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }
__device__ __forceinline__ void st_dev(int32_t* p, int32_t v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_dev(uint32_t* p, uint32_t v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_dev(float* p, float v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ int32_t ld_dev(const int32_t* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float ld_dev(const float* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ unsigned long long ld_dev(const unsigned long long* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

template <int CTRL>
__device__ __forceinline__ float dpp_f32(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, false));
}
__device__ __forceinline__ float read_lane_f32(float v, int lane) {
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), lane));
}
__device__ __forceinline__ float wave_sum(float v) {
    v += dpp_f32<0xB1>(v);    // quad_perm [1,0,3,2]
    v += dpp_f32<0x4E>(v);    // quad_perm [2,3,0,1]
    v += dpp_f32<0x141>(v);   // row_half_mirror
    v += dpp_f32<0x140>(v);   // row_mirror
    return (read_lane_f32(v, 0) + read_lane_f32(v, 16)) + (read_lane_f32(v, 32) + read_lane_f32(v, 48));
}
__device__ __forceinline__ float wave_max(float v) {
    v = fmaxf(v, dpp_f32<0xB1>(v));
    v = fmaxf(v, dpp_f32<0x4E>(v));
    v = fmaxf(v, dpp_f32<0x141>(v));
    v = fmaxf(v, dpp_f32<0x140>(v));
    return fmaxf(fmaxf(read_lane_f32(v, 0), read_lane_f32(v, 16)),
                 fmaxf(read_lane_f32(v, 32), read_lane_f32(v, 48)));
}
#endif

}  // namespace fate
