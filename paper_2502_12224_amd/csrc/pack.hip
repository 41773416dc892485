// Canonical [rows, K] codes -> device-native 1 KiB tiles (see qformat.h).
#include "common.h"
#include "qformat.h"

namespace fate {

// one thread per output dword
__global__ __launch_bounds__(256) void pack_weight_kernel(const uint32_t* __restrict__ src,
                                                          uint32_t* __restrict__ dst, int rows, int K,
                                                          int bits, long long ndw) {
    long long o = (long long)blockIdx.x * 256 + threadIdx.x;
    if (o >= ndw) return;
    const int d = (int)(o & 3);
    const int lane = (int)((o >> 2) & 63);
    const long long tile = o >> 8;
    const int n = lane & 31, half = lane >> 5;
    if (bits == 2) {
        const int tiles_k = K / 128;
        const int rb = (int)(tile / tiles_k), kb = (int)(tile % tiles_k);
        const long long row = (long long)rb * 32 + n;
        const int k0 = kb * 128 + half * 64 + 16 * d;               // 16 fields = one canonical dword
        const uint32_t s = src[(row * K + k0) >> 4];
        uint32_t r = 0;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            r |= ((s >> (4 * i)) & 0x3u) << (2 * i);                // column 2i   -> bits 2i
            r |= ((s >> (4 * i + 2)) & 0x3u) << (2 * i + 16);       // column 2i+1 -> bits 16 + 2i
        }
        dst[o] = r;
    } else if (bits == 4) {
        const int tiles_k = K / 64;
        const int rb = (int)(tile / tiles_k), kb = (int)(tile % tiles_k);
        const long long row = (long long)rb * 32 + n;
        const int k0 = kb * 64 + half * 32 + 8 * d;                 // 8 codes = one canonical dword
        const uint32_t s = src[(row * K + k0) >> 3];
        uint32_t r = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            r |= ((s >> (8 * i)) & 0xfu) << (4 * i);                // column 2i   -> nibble i
            r |= ((s >> (8 * i + 4)) & 0xfu) << (4 * i + 16);       // column 2i+1 -> nibble i+4
        }
        dst[o] = r;
    } else {
        const int tiles_k = K / 32;
        const int rb = (int)(tile / tiles_k), kb = (int)(tile % tiles_k);
        const long long row = (long long)rb * 32 + n;
        const int k0 = kb * 32 + half * 16 + 4 * d;
        dst[o] = src[(row * K + k0) >> 2] ^ 0x80808080u;            // two's complement -> offset binary
    }
}

// [rows, groups] -> [groups, rows], one thread per element
__global__ __launch_bounds__(256) void pack_scales_kernel(const uint16_t* __restrict__ src,
                                                          uint16_t* __restrict__ dst, int rows, int groups) {
    const long long o = (long long)blockIdx.x * 256 + threadIdx.x;
    if (o >= (long long)rows * groups) return;
    const int g = (int)(o / rows), r = (int)(o - (long long)g * rows);
    dst[o] = src[(long long)r * groups + g];
}

}  // namespace fate

using namespace fate;

extern "C" fate_status fate_pack_scales(void* stream, const void* canonical_dev, int rows, int groups,
                                        void* packed_dev) {
    if (rows < 1 || groups < 1) FATE_FAIL(FATE_ESHAPE, "rows = %d, groups = %d must be positive", rows, groups);
    FATE_CHECK_PTR(canonical_dev);
    FATE_CHECK_PTR(packed_dev);
    if (canonical_dev == packed_dev) FATE_FAIL(FATE_EINVAL, "packing is out of place");
    const long long n = (long long)rows * groups;
    const long long grid = (n + 255) / 256;
    if (grid > 0x7fffffffLL) FATE_FAIL(FATE_ESHAPE, "matrix too large");
    pack_scales_kernel<<<(unsigned)grid, 256, 0, static_cast<hipStream_t>(stream)>>>(
        static_cast<const uint16_t*>(canonical_dev), static_cast<uint16_t*>(packed_dev), rows, groups);
    FATE_HIP(hipGetLastError());
    return FATE_OK;
}

extern "C" fate_status fate_pack_weight(void* stream, const void* canonical_dev, int rows, int K, int bits,
                                        void* packed_dev) {
    if (bits != 2 && bits != 4 && bits != 8) FATE_FAIL(FATE_EINVAL, "bits = %d (2, 4 or 8 supported)", bits);
    if (rows < 32 || rows % 32 != 0) FATE_FAIL(FATE_ESHAPE, "rows = %d must be a positive multiple of 32", rows);
    const int kt = bits == 2 ? 128 : 64;
    if (K < kt || K % kt != 0) FATE_FAIL(FATE_ESHAPE, "K = %d must be a positive multiple of %d", K, kt);
    FATE_CHECK_PTR(canonical_dev);
    FATE_CHECK_PTR(packed_dev);
    if (canonical_dev == packed_dev) FATE_FAIL(FATE_EINVAL, "packing is out of place");
    const long long ndw = (long long)rows * K * bits / 32;
    const long long grid = (ndw + 255) / 256;
    if (grid > 0x7fffffffLL) FATE_FAIL(FATE_ESHAPE, "matrix too large");
    pack_weight_kernel<<<(unsigned)grid, 256, 0, static_cast<hipStream_t>(stream)>>>(
        static_cast<const uint32_t*>(canonical_dev), static_cast<uint32_t*>(packed_dev), rows, K, bits, ndw);
    FATE_HIP(hipGetLastError());
    return FATE_OK;
}
