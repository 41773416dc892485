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

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}
#endif

}  // namespace fate
